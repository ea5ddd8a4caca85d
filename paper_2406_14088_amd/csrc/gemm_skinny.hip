// Skinny-M GEMM for the decode step: C[M, N] = A[M, K] * W[N, K]^T with M <= 256 (A half, W bf16).
//
// A decode step multiplies a few rows of activations (one per sequence) with every weight matrix, so
// the step is bound by streaming the weights from HBM exactly once.  Design for gfx950:
//   * one workgroup = 8 wavefronts = 4 column groups x 2 K halves: wavefront (ng, kg) owns 32 output
//     columns and all (<= 256) rows, and multiplies the half kg of every 128-wide K chunk; the two K
//     halves are added through LDS at the end (inside the workgroup, fixed order);
//   * weights go global -> VGPR directly in MFMA operand layout (lane = (row of W, 8 consecutive k)),
//     through an 8-fragment register ring that is refilled fragment by fragment two K chunks ahead,
//     never touching LDS; eight wavefronts per compute unit keep enough loads in flight;
//   * each weight fragment is widened bf16 -> half in registers (3 VALU ops per pair, exact for normal
//     halves) and fed to v_mfma_f32_32x32x16_f16 with fp32 accumulators: half activations keep 11
//     significant bits where bf16 would keep 8, at the same matrix-core rate;
//   * the activation chunk [M, 128] is staged once per workgroup in LDS (padded rows, conflict-free
//     ds_read_b128), shared by the eight wavefronts and read one k-step ahead of the MFMAs;
//   * split-K over workgroups (grid.y) gives enough workgroups to fill 256 CUs; each split writes its
//     fp32 partial tile and the consumer kernel adds the partials in a fixed order (deterministic).
// Buffer loads with a range-checked descriptor return 0 outside a matrix, so ragged N and K need no
// per-load branches; the activation tile is zero-filled beyond K.
#include <type_traits>

#include "kernels.h"

#define SK_BK 128            // K elements per chunk
#define SK_LDS_STRIDE 136    // half elements per LDS row (128 + 8 pad -> 272 B, conflict-free b128 reads)
#define SK_THREADS 512
#define SK_OOB 0x80000000u   // byte offset beyond every descriptor: such a load returns zeros, touches no memory

struct SkinnyParams {
    const f16_t *A;
    const bf16_t *W[3];
    int rows[3];
    int tile_begin[4];  // first n-tile of each matrix (prefix sums), tile_begin[3] = total
    int col_off[3];
    int lda_bytes;      // row stride of A in bytes
    uint32_t a_bytes;   // size of A in bytes (range check)
    int M, K, chunks, splits, epilogue;
    void *out;
    int64_t ldc;
    size_t split_stride;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

template <int MT>
__global__ __launch_bounds__(SK_THREADS, 2) void gemm_skinny_kernel(SkinnyParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    f16_t *xs = reinterpret_cast<f16_t *>(smem);  // [2][MT*32][SK_LDS_STRIDE]
    constexpr int BM = MT * 32;
    constexpr int XLOADS = MT;  // 16-byte loads per thread per chunk: BM*128*2 B / (512 thr * 16 B)
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);  // wavefront id as a scalar: descriptors stay in SGPRs
    const int ng = w & 3, kg = w >> 2;                      // column group, K half
    const int K = p.K;

    // ---- which weight rows does this wavefront own?
    int tile = blockIdx.x;
    int seg = tile >= p.tile_begin[2] ? 2 : (tile >= p.tile_begin[1] ? 1 : 0);
    int n_base, out_col;  // first W row of this wavefront / first output column
    if (p.epilogue == EPI_SWIGLU) {
        seg = ng >> 1;                       // column groups 0,1: gate; 2,3: up
        n_base = tile * 64 + (ng & 1) * 32;
        out_col = n_base;
    } else {
        n_base = (tile - p.tile_begin[seg]) * 128 + ng * 32;
        out_col = p.col_off[seg] + n_base;
    }
    const int rows = seg == 0 ? p.rows[0] : (seg == 1 ? p.rows[1] : p.rows[2]);
    const bf16_t *Wp = seg == 0 ? p.W[0] : (seg == 1 ? p.W[1] : p.W[2]);
    __amdgpu_buffer_rsrc_t wr = make_rsrc(Wp, (uint32_t)((size_t)rows * K * 2));
    __amdgpu_buffer_rsrc_t ar = make_rsrc(p.A, p.a_bytes);
    int wrow = n_base + (lane & 31);
    // rows past the matrix read row 0 instead (always in bounds); their columns are never stored
    const uint32_t w_off = (uint32_t)(wrow < rows ? wrow : 0) * (uint32_t)K * 2u + (uint32_t)(lane >> 5) * 16u +
                           (uint32_t)kg * 128u;

    // ---- K range of this split
    const int c0 = (int)(((int64_t)blockIdx.y * p.chunks) / p.splits);
    const int c1 = (int)(((int64_t)(blockIdx.y + 1) * p.chunks) / p.splits);

    // activation loader: thread -> (row r0 + 32*i, 16-byte column group c16); rows >= M and columns >= K
    // get an offset outside the descriptor's range, for which the hardware returns zeros
    const int c16 = t & 15, r0 = t >> 4;
    uint32_t x_off[XLOADS];
#pragma unroll
    for (int i = 0; i < XLOADS; ++i) {
        int row = r0 + 32 * i;
        x_off[i] = row < p.M ? (uint32_t)row * (uint32_t)p.lda_bytes + (uint32_t)c16 * 16u : SK_OOB;
    }
    u32x4_t xr[XLOADS];
    u32x4_t wq[8];  // raw bf16 weight fragments of two consecutive chunks (ring buffer): 4 k-steps each
    f32x16_t acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

    // Loads that are not needed (past the K range of this split) get an offset outside the descriptor's
    // range: the hardware answers with zeros and touches no memory, and the number of outstanding loads
    // stays the same on every trip, so the compiler's wait counters stay exact.
    auto load_x = [&](int c, bool wanted) {
        bool ok = wanted && (c * SK_BK + c16 * 8 < K);
        uint32_t cb = (uint32_t)c * (SK_BK * 2);
#pragma unroll
        for (int i = 0; i < XLOADS; ++i)
            xr[i] = __builtin_amdgcn_raw_buffer_load_b128(ar, (int)(ok ? x_off[i] + cb : SK_OOB), 0, 0);
    };
    auto store_x = [&](int buf) {
        f16_t *dst = xs + (size_t)buf * BM * SK_LDS_STRIDE;
#pragma unroll
        for (int i = 0; i < XLOADS; ++i) {
            int row = r0 + 32 * i;
            *reinterpret_cast<u32x4_t *>(dst + row * SK_LDS_STRIDE + c16 * 8) = xr[i];
        }
    };
#define SK_ISSUE_W(OFF, S, SLOT) wq[SLOT] = __builtin_amdgcn_raw_buffer_load_b128(wr, (int)((OFF) + (uint32_t)((S) * 32)), 0, 0)

    // One chunk: every weight fragment is consumed by MT MFMAs and its register is refilled at once with
    // the same fragment of the chunk after next.  Activation fragments are read from LDS one k-step
    // ahead of the MFMAs that use them.  The loop body is two such chunks back to back with no branch
    // inside (a chunk past the end of the split multiplies zeros): static ring indices, exact wait counts.
    auto body = [&](int c, auto par_tag) {
        constexpr int PAR = decltype(par_tag)::value;
        __syncthreads();  // activation tile of chunk c is in LDS buffer PAR; buffer PAR^1 is free
        const f16_t *src = xs + (size_t)PAR * BM * SK_LDS_STRIDE + (lane & 31) * SK_LDS_STRIDE + (lane >> 5) * 8 + kg * 64;
        const uint32_t off2 = c + 2 < c1 ? w_off + (uint32_t)(c + 2) * (SK_BK * 2) : SK_OOB;
        f16x8_t a[2][MT];
        f16x8_t wf[2];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[0][mt] = *reinterpret_cast<const f16x8_t *>(src + mt * 32 * SK_LDS_STRIDE);
        wf[0] = __builtin_bit_cast(f16x8_t, bf16x8_to_f16x8(wq[PAR * 4]));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s + 1 < 4) {  // operands of step s+1 are requested before the MFMAs of step s are issued ...
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    a[(s + 1) & 1][mt] = *reinterpret_cast<const f16x8_t *>(src + mt * 32 * SK_LDS_STRIDE + (s + 1) * 16);
                wf[(s + 1) & 1] = __builtin_bit_cast(f16x8_t, bf16x8_to_f16x8(wq[PAR * 4 + s + 1]));
            }
            __builtin_amdgcn_sched_barrier(0);
            // ... so that the LDS latency hides behind MT matrix instructions
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[s & 1][mt], wf[s & 1], acc[mt], 0, 0, 0);
            SK_ISSUE_W(off2, s, PAR * 4 + s);
            __builtin_amdgcn_sched_barrier(0);
        }
        store_x(PAR ^ 1);  // activation tile of chunk c+1 (loaded one chunk ago; zeros past the end)
        load_x(c + 2, c + 2 < c1);
        __builtin_amdgcn_sched_barrier(0);
    };

    if (c0 < c1) {
        load_x(c0, true);
        {
            const uint32_t off0 = w_off + (uint32_t)c0 * (SK_BK * 2);
            const uint32_t off1 = c0 + 1 < c1 ? w_off + (uint32_t)(c0 + 1) * (SK_BK * 2) : SK_OOB;
#pragma unroll
            for (int s = 0; s < 4; ++s) SK_ISSUE_W(off0, s, s);
#pragma unroll
            for (int s = 0; s < 4; ++s) SK_ISSUE_W(off1, s, 4 + s);
        }
        store_x(0);
        load_x(c0 + 1, c0 + 1 < c1);
        __builtin_amdgcn_sched_barrier(0);
        for (int c = c0; c < c1; c += 2) {
            body(c, std::integral_constant<int, 0>{});
            body(c + 1, std::integral_constant<int, 1>{});
        }
    }
#undef SK_ISSUE_W

    // ---- add the two K halves: wavefronts kg = 1 hand their accumulators to kg = 0 through LDS
    float *ex = reinterpret_cast<float *>(smem);  // [4 column groups][MT*16][64]
    __syncthreads();                              // every wavefront is done reading the activation tiles
    if (kg == 1) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 16; ++j) ex[(ng * MT * 16 + mt * 16 + j) * 64 + lane] = acc[mt][j];
    }
    __syncthreads();
    if (kg == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[mt][j] += ex[(ng * MT * 16 + mt * 16 + j) * 64 + lane];
    }

    // ---- epilogue.  Lane holds column (lane & 31); register j of tile mt is row
    //      mt*32 + (j/4)*8 + (lane>>5)*4 + (j%4).
    const int col_local = lane & 31;
    if (p.epilogue != EPI_SWIGLU) {
        float *out = reinterpret_cast<float *>(p.out) + (size_t)blockIdx.y * p.split_stride;
        const bool accumulate = p.epilogue == EPI_F32_ACC;
        if (kg == 0 && n_base + col_local < rows) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    int m = mt * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
                    if (m < p.M) {
                        float *dst = out + (size_t)m * p.ldc + out_col + col_local;
                        *dst = accumulate ? *dst + acc[mt][j] : acc[mt][j];
                    }
                }
        }
    } else {
        // SwiGLU: column groups 2,3 (up) hand their sums to column groups 0,1 (gate) through LDS.
        __syncthreads();  // the K-half exchange above has been read
        if (kg == 0 && ng >= 2) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 16; ++j) ex[((ng - 2) * MT * 16 + mt * 16 + j) * 64 + lane] = acc[mt][j];
        }
        __syncthreads();
        if (kg == 0 && ng < 2 && n_base + col_local < rows) {
            f16_t *out = reinterpret_cast<f16_t *>(p.out);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    int m = mt * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
                    float g = acc[mt][j], u = ex[(ng * MT * 16 + mt * 16 + j) * 64 + lane];
                    float a = g / (1.0f + expf(-g)) * u;
                    if (m < p.M) out[(size_t)m * p.ldc + out_col + col_local] = f32_to_f16(a);
                }
        }
    }
}

int gemm_skinny_default_splits(int M, int N, int K) {
    (void)M;
    int tiles = ceil_div(N, 128);
    int chunks = ceil_div(K, SK_BK);
    int s = 512 / (tiles > 0 ? tiles : 1);  // aim at two workgroups per compute unit
    if (s < 1) s = 1;
    if (s > chunks / 4) s = chunks / 4 > 0 ? chunks / 4 : 1;  // keep at least 4 chunks per split
    if (s > 16) s = 16;
    return s;
}

template <int MT>
static void launch_mt(const SkinnyParams &p, int tiles, hipStream_t st) {
    size_t lds = (size_t)2 * MT * 32 * SK_LDS_STRIDE * sizeof(f16_t);
    size_t ex = (size_t)4 * MT * 16 * 64 * sizeof(float);  // exchange area of the K-half reduction
    if (ex > lds) lds = ex;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_skinny_kernel<MT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        attr_set = true;
    }
    gemm_skinny_kernel<MT><<<dim3(tiles, p.splits), SK_THREADS, lds, st>>>(p);
}

void launch_gemm_skinny(const GemmArgs &a, hipStream_t st) {
    if (a.M <= 0) return;
    SkinnyParams p;
    p.A = a.A;
    p.lda_bytes = (int)(a.lda * 2);
    p.a_bytes = (uint32_t)((((size_t)a.M - 1) * a.lda + a.K) * 2);
    p.M = a.M;
    p.K = a.K;
    p.chunks = ceil_div(a.K, SK_BK);
    p.epilogue = a.epilogue;
    p.splits = a.epilogue != EPI_F32 ? 1 : (a.splits < 1 ? 1 : a.splits);
    if (p.splits > p.chunks) p.splits = p.chunks;
    p.out = a.out;
    p.ldc = a.ldc;
    p.split_stride = a.split_stride;
    int tiles = 0, col = 0;
    for (int i = 0; i < 3; ++i) {
        p.W[i] = a.W[i] ? a.W[i] : a.W[0];
        p.rows[i] = a.W[i] ? a.rows[i] : 0;
        p.tile_begin[i] = tiles;
        p.col_off[i] = col;
        if (a.epilogue == EPI_SWIGLU) continue;
        tiles += ceil_div(p.rows[i], 128);
        col += p.rows[i];
    }
    if (a.epilogue == EPI_SWIGLU) tiles = ceil_div(a.rows[0], 64);
    p.tile_begin[3] = tiles;
    if (tiles <= 0) return;
    if (a.M <= 32) launch_mt<1>(p, tiles, st);
    else if (a.M <= 64) launch_mt<2>(p, tiles, st);
    else if (a.M <= 128) launch_mt<4>(p, tiles, st);
    else launch_mt<8>(p, tiles, st);
}
