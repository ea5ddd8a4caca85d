// Skinny-M GEMM for the decode step: C[M, N] = A[M, K] * W[N, K]^T with M <= 256 (A half, W bf16).
//
// A decode step multiplies a few rows of activations (one per sequence) with every weight matrix, so
// the step is bound by streaming the weights from HBM exactly once.  What limits a compute unit here
// is not the matrix cores but its vector-memory pipeline: a load instruction whose 64 lanes touch 32
// different rows costs several times more issue time than one whose lanes cover whole 128-byte lines.
// Design for gfx950:
//   * one workgroup = 8 wavefronts = 4 column groups x 2 K halves: wavefront (ng, kg) owns 32 weight
//     rows (= output columns) and multiplies the half kg (64 elements = one 128-byte line per row) of
//     every 128-wide K chunk; the two K halves are added through LDS at the end (fixed order);
//   * weights are fetched with fully coalesced loads (8 lanes x 16 B = one line of one row, 8 rows per
//     instruction), kept in flight in an 8-register ring two chunks ahead, widened bf16 -> half in
//     registers (exact for normal halves), parked in a wavefront-private, XOR-swizzled LDS strip and read
//     back as MFMA fragments (lane = weight row, 8 consecutive k) without bank conflicts; the strip is
//     private to the wavefront, so this needs no barrier;
//   * the activation chunk [M, 128] is staged once per workgroup in LDS (padded rows, conflict-free
//     ds_read_b128), shared by the eight wavefronts and read one k-step ahead of the MFMAs;
//   * v_mfma_f32_32x32x16_f16 with fp32 accumulators: half activations keep 11 significant bits where
//     bf16 would keep 8, at the same matrix-core rate;
//   * results leave through an LDS tile so that global stores are whole 512-byte rows (float4 per lane);
//   * split-K over workgroups (grid.y) gives enough workgroups to fill 256 CUs; each split writes its
//     fp32 partial tile and the consumer kernel adds the partials in a fixed order (deterministic).
// Buffer loads with a range-checked descriptor return 0 outside a matrix, so ragged N and K need no
// per-load branches; the activation tile is zero-filled beyond K.
#include <type_traits>

#include "kernels.h"

#define SK_BK 128            // K elements per chunk
#define SK_LDS_STRIDE 136    // half elements per LDS row of the activation tile (128 + 8 pad -> 272 B)
#define SK_THREADS 512
#define SK_BM 128            // activation rows per workgroup (grid.z walks taller batches)
#define SK_MT 4              // 32-row MFMA tiles per workgroup
#define SK_OOB 0xFFFFFF00u   // byte offset beyond every descriptor (< 4 GiB - 256): such a load returns zeros, touches no memory
#define SK_X_BYTES (2 * SK_BM * SK_LDS_STRIDE * 2)   // two activation buffers
#define SK_W_BYTES (8 * 2 * 4096)                    // per wavefront: two strips of 32 rows x 128 B
#define SK_CT_STRIDE 132                             // floats per row of the fp32 output tile in LDS

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

__global__ __launch_bounds__(SK_THREADS, 2) void gemm_skinny_kernel(SkinnyParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int MT = SK_MT, BM = SK_BM;
    f16_t *xs = reinterpret_cast<f16_t *>(smem);  // [2][BM][SK_LDS_STRIDE]
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);  // wavefront id as a scalar: descriptors stay in SGPRs
    const int ng = w & 3, kg = w >> 2;                      // column group, K half
    const int K = p.K;
    const int m0 = blockIdx.z * BM;                         // first activation row of this workgroup
    const int Mloc = p.M - m0 < BM ? p.M - m0 : BM;

    // ---- which weight rows does this wavefront own?
    int tile = blockIdx.x;
    int seg = tile >= p.tile_begin[2] ? 2 : (tile >= p.tile_begin[1] ? 1 : 0);
    int n_base, tile_col;  // first W row of this wavefront / first output column of the workgroup
    if (p.epilogue == EPI_SWIGLU) {
        seg = ng >> 1;                       // column groups 0,1: gate; 2,3: up
        n_base = tile * 64 + (ng & 1) * 32;
        tile_col = tile * 64;
    } else {
        n_base = (tile - p.tile_begin[seg]) * 128 + ng * 32;
        tile_col = p.col_off[seg] + (tile - p.tile_begin[seg]) * 128;
    }
    const int rows = seg == 0 ? p.rows[0] : (seg == 1 ? p.rows[1] : p.rows[2]);
    const bf16_t *Wp = seg == 0 ? p.W[0] : (seg == 1 ? p.W[1] : p.W[2]);
    __amdgpu_buffer_rsrc_t wr = make_rsrc(Wp, (uint32_t)((size_t)rows * K * 2));
    __amdgpu_buffer_rsrc_t ar = make_rsrc(p.A, p.a_bytes);

    // weight loader: instruction i fetches rows 8i + lane/8 of the strip, 16-byte piece lane%8 of the 128-byte half
    uint32_t w_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = n_base + 8 * i + (lane >> 3);
        // rows past the matrix read row 0 instead (always in bounds); their columns are never stored
        w_off[i] = (uint32_t)(r < rows ? r : 0) * (uint32_t)K * 2u + (uint32_t)kg * 128u + (uint32_t)(lane & 7) * 16u;
    }
    // wavefront-private LDS strip, [2][32 rows][8 pieces of 16 B]; piece j of row r sits in slot j ^ ((r >> 1) & 7):
    // 64 banks = 256 bytes = two rows per clock, and a fragment read has 16 consecutive rows in the 16 lanes served
    // together, so the slot changes every second row
    unsigned char *wl = smem + SK_X_BYTES + w * 8192;
    int wst[4];  // store address of instruction i (row = lane/8 + 8i)
#pragma unroll
    for (int i = 0; i < 4; ++i) wst[i] = (lane >> 3) * 128 + (((lane & 7) ^ (((8 * i + (lane >> 3)) >> 1) & 7)) << 4);
    int wld[4];                                                             // fragment address of k-step s
#pragma unroll
    for (int s = 0; s < 4; ++s) wld[s] = (lane & 31) * 128 + (((2 * s + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);

    // ---- K range of this split
    const int c0 = (int)(((int64_t)blockIdx.y * p.chunks) / p.splits);
    const int c1 = (int)(((int64_t)(blockIdx.y + 1) * p.chunks) / p.splits);

    // activation loader: thread -> (row r0 + 32*i, 16-byte column group c16); rows >= M and columns >= K
    // get an offset outside the descriptor's range, for which the hardware returns zeros
    const int c16 = t & 15, r0 = t >> 4;
    uint32_t x_off[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        int row = r0 + 32 * i;
        x_off[i] = (uint32_t)(m0 + row) * (uint32_t)p.lda_bytes + (uint32_t)c16 * 16u;
    }
    u32x4_t xr[2][MT];  // activation pieces in flight: xr[i & 1] belongs to chunk c0 + i
    const bool stream_w = gridDim.z == 1;
    u32x4_t wq[8];      // raw bf16 weight pieces in flight: slots (i & 1) * 4 .. + 3 belong to chunk c0 + i
    f32x16_t acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;

    // Loads that are not needed (past the K range of this split) get an offset outside the descriptor's
    // range: the hardware answers with zeros and touches no memory, and the number of outstanding loads
    // stays the same on every trip, so the compiler's wait counters stay exact.
    auto load_x = [&](int c, int set) {
        bool ok = c < c1 && (c * SK_BK + c16 * 8 < K);
        uint32_t cb = (uint32_t)c * (SK_BK * 2);
#pragma unroll
        for (int i = 0; i < MT; ++i)
            xr[set][i] = __builtin_amdgcn_raw_buffer_load_b128(ar, (int)(ok && r0 + 32 * i < Mloc ? x_off[i] + cb : SK_OOB), 0, 0);
    };
    auto store_x1 = [&](int set, int buf, int i) {
        f16_t *dst = xs + (size_t)buf * BM * SK_LDS_STRIDE;
        *reinterpret_cast<u32x4_t *>(dst + (r0 + 32 * i) * SK_LDS_STRIDE + c16 * 8) = xr[set][i];
    };
    auto load_w1 = [&](int c, int slot, int i) {  // piece i of chunk c -> ring slot
        uint32_t cb = (uint32_t)c * (SK_BK * 2);
        // one row block: every weight byte is used once and is loaded non-temporally (streams faster than a cached load)
        if (stream_w) wq[slot] = __builtin_amdgcn_raw_buffer_load_b128(wr, (int)(c < c1 ? w_off[i] + cb : SK_OOB), 0, 3);
        else wq[slot] = __builtin_amdgcn_raw_buffer_load_b128(wr, (int)(c < c1 ? w_off[i] + cb : SK_OOB), 0, 0);
    };
    auto stage_w1 = [&](int slot, int buf, int i) {  // ring slot -> half -> LDS strip `buf`
        *reinterpret_cast<u32x4_t *>(wl + buf * 4096 + i * 1024 + wst[i]) = bf16x8_to_f16x8(wq[slot]);
    };

    // One chunk (index i relative to c0, PAR = i & 1): MFMAs on the strip/tile staged one chunk ago.
    // Interleaved with its four k-steps, piece by piece: the next chunk's activations move registers ->
    // LDS tile, the next chunk's weights move ring -> half -> LDS strip, and the ring is refilled three
    // chunks ahead, so that the matrix cores, the LDS and the memory pipeline work at the same time.
    // The hardware counts outstanding loads in issue order: all (short-latency, L2) activation loads of a
    // trip are issued before its weight loads, so waiting for them never waits for young weight loads.
    auto body = [&](int c, auto par_tag) {
        constexpr int PAR = decltype(par_tag)::value;
        __syncthreads();  // activation tile of chunk c is in LDS buffer PAR; buffer PAR^1 is free
        load_x(c + 2, PAR);
        const f16_t *src = xs + (size_t)PAR * BM * SK_LDS_STRIDE + (lane & 31) * SK_LDS_STRIDE + (lane >> 5) * 8 + kg * 64;
        const unsigned char *wsrc = wl + PAR * 4096;
        f16x8_t a[2][MT];
        f16x8_t wf[2];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[0][mt] = *reinterpret_cast<const f16x8_t *>(src + mt * 32 * SK_LDS_STRIDE);
        wf[0] = *reinterpret_cast<const f16x8_t *>(wsrc + wld[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s + 1 < 4) {  // operands of step s+1 are requested before the MFMAs of step s are issued
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    a[(s + 1) & 1][mt] = *reinterpret_cast<const f16x8_t *>(src + mt * 32 * SK_LDS_STRIDE + (s + 1) * 16);
                wf[(s + 1) & 1] = *reinterpret_cast<const f16x8_t *>(wsrc + wld[s + 1]);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[s & 1][mt], wf[s & 1], acc[mt], 0, 0, 0);
            store_x1(PAR ^ 1, PAR ^ 1, s);               // activation piece s of chunk c+1 (loaded one chunk ago)
            stage_w1((PAR ^ 1) * 4 + s, PAR ^ 1, s);     // weight piece s of chunk c+1: ring -> strip
            load_w1(c + 3, (PAR ^ 1) * 4 + s, s);        // and refill its ring slot
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (c0 < c1) {
        load_x(c0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_w1(c0, i, i);
#pragma unroll
        for (int i = 0; i < MT; ++i) store_x1(0, 0, i);
        load_x(c0 + 1, 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_w1(c0 + 1, 4 + i, i);
#pragma unroll
        for (int i = 0; i < 4; ++i) stage_w1(i, 0, i);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_w1(c0 + 2, i, i);
        __builtin_amdgcn_sched_barrier(0);
        for (int c = c0; c < c1; c += 2) {
            body(c, std::integral_constant<int, 0>{});
            body(c + 1, std::integral_constant<int, 1>{});
        }
    }

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
    __syncthreads();  // the exchange area is free again

    // ---- epilogue through an LDS tile.  Lane holds column (lane & 31) of its group; register j of tile mt
    //      is row mt*32 + (j/4)*8 + (lane>>5)*4 + (j%4).
    if (p.epilogue != EPI_SWIGLU) {
        float *ct = reinterpret_cast<float *>(smem);  // [BM][SK_CT_STRIDE]
        if (kg == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    int m = mt * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
                    ct[m * SK_CT_STRIDE + ng * 32 + (lane & 31)] = acc[mt][j];
                }
        }
        __syncthreads();
        // 32 lanes x float4 = one 512-byte output row; 16 rows per pass
        float *out = reinterpret_cast<float *>(p.out) + (size_t)blockIdx.y * p.split_stride;
        const bool accumulate = p.epilogue == EPI_F32_ACC;
        const int c4 = (t & 31) * 4, rr = t >> 5;
        const int n_tile0 = (tile - p.tile_begin[seg]) * 128;  // first weight row of the tile inside its matrix
        const int ncols = rows - n_tile0;                      // valid columns of this tile (may exceed 128)
#pragma unroll
        for (int i = 0; i < BM / 16; ++i) {
            int m = rr + 16 * i;
            if (m < Mloc && c4 < ncols) {
                f32x4_t v = *reinterpret_cast<const f32x4_t *>(ct + m * SK_CT_STRIDE + c4);
                float *dst = out + (size_t)(m0 + m) * p.ldc + tile_col + c4;
                if (c4 + 4 <= ncols && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
                    if (accumulate) v += *reinterpret_cast<const f32x4_t *>(dst);
                    *reinterpret_cast<f32x4_t *>(dst) = v;
                } else {
                    for (int e = 0; e < 4 && c4 + e < ncols; ++e) dst[e] = accumulate ? dst[e] + v[e] : v[e];
                }
            }
        }
    } else {
        // SwiGLU: column groups 2,3 (up) hand their sums to column groups 0,1 (gate); the gate side combines
        // and parks half results in an LDS tile; then whole 128-byte rows go out.
        if (kg == 0 && ng >= 2) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 16; ++j) ex[((ng - 2) * MT * 16 + mt * 16 + j) * 64 + lane] = acc[mt][j];
        }
        __syncthreads();
        f16_t *ht = reinterpret_cast<f16_t *>(smem + 2 * MT * 16 * 64 * 4);  // [BM][72] halves, after the exchange area
        if (kg == 0 && ng < 2) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    int m = mt * 32 + (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
                    float g = acc[mt][j], u = ex[(ng * MT * 16 + mt * 16 + j) * 64 + lane];
                    ht[m * 72 + ng * 32 + (lane & 31)] = f32_to_f16(g / (1.0f + expf(-g)) * u);
                }
        }
        __syncthreads();
        f16_t *out = reinterpret_cast<f16_t *>(p.out);
        const int c8 = (t & 7) * 8, rr = t >> 3;  // 8 lanes x 16 B = one 128-byte output row; 64 rows per pass
        const int ncols = rows - tile * 64;
#pragma unroll
        for (int i = 0; i < BM / 64; ++i) {
            int m = rr + 64 * i;
            if (m < Mloc && c8 < ncols) {
                f16_t *dst = out + (size_t)(m0 + m) * p.ldc + tile_col + c8;
                const f16_t *srcp = ht + m * 72 + c8;
                if (c8 + 8 <= ncols && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
                    *reinterpret_cast<u32x4_t *>(dst) = *reinterpret_cast<const u32x4_t *>(srcp);
                } else {
                    for (int e = 0; e < 8 && c8 + e < ncols; ++e) dst[e] = srcp[e];
                }
            }
        }
    }
}

int gemm_skinny_default_splits(int M, int N, int K) {
    (void)M;
    int tiles = ceil_div(N, 128);
    int chunks = ceil_div(K, SK_BK);
    int s = 256 / (tiles > 0 ? tiles : 1);  // aim at one 8-wavefront workgroup per compute unit
    if (s < 1) s = 1;
    if (s > chunks / 4) s = chunks / 4 > 0 ? chunks / 4 : 1;  // keep at least 4 chunks per split
    if (s > 16) s = 16;
    return s;
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
    size_t lds = SK_X_BYTES + SK_W_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_skinny_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        attr_set = true;
    }
    gemm_skinny_kernel<<<dim3(tiles, p.splits, ceil_div(a.M, SK_BM)), SK_THREADS, lds, st>>>(p);
}
