// Large-M GEMM for prefill: C[M, N] = A[M, K] * W[N, K]^T (A half, W bf16), both operands tiled
// through LDS, v_mfma_f32_32x32x16_f16 with fp32 accumulators.  Weights are widened bf16 -> half
// (exact for normal halves) once, on their way from registers into LDS.
//
// Prefill multiplies all prompt tokens of a chunk of sequences (thousands of rows) with every weight
// matrix: a dense contraction, bound by the matrix cores.  Design for gfx950:
//   * workgroup = 4 wavefronts in a 2 x 2 grid; each wavefront owns (WM*32) x (WN*32) of the tile
//     (WM = WN = 4: a 256 x 256 tile, 128 x 128 per wavefront, 256 accumulator registers), so that
//     each 1 KB LDS fragment read feeds four MFMAs;
//   * K chunks of 64, register-staged global -> LDS copies, double-buffered LDS (one barrier per chunk);
//   * LDS rows padded to 72 elements: ds_read_b128 of MFMA fragments is bank-conflict free;
//   * workgroup ids are remapped so that the workgroups resident on one XCD (ids congruent mod 8)
//     work on neighbouring tiles and share their operand panels in that XCD's L2;
//   * fused epilogues: fp32 store, fp32 accumulate (residual add: read-modify-write of whole rows, 16 bytes per
//     lane, staged through LDS, all reads of a band requested before its first write), SwiGLU (wavefront column 0
//     holds the gate tile, column 1 the up tile of the same outputs; exchanged through LDS).
#include <type_traits>

#include "kernels.h"

#define TG_BK 64
#define TG_LDS_STRIDE 72
#define TG_THREADS 256

struct TiledParams {
    const f16_t *A;
    const bf16_t *W[3];
    int rows[3];
    int tile_begin[4];
    int col_off[3];
    int64_t lda;
    uint32_t a_bytes;  // size of A (both terms) in bytes (range check)
    uint32_t lo_delta;  // byte distance from the first to the second activation term (0: one term)
    int M, K, chunks, terms, epilogue;
    int tiles_m, tiles_n;
    void *out;
    f16_t *out_lo;      // EPI_SWIGLU, optional: second half term of the result
    int64_t ldc;
    RopeEpilogue rope;  // EPI_ROPE
    const f16_t *P[3];  // fragment-order copies of W[0..2] (gemm_tiled_dma_kernel), or all NULL
    int ksteps;         // 16-element k-steps of a packed weight row: ceil(K / 16)
};

// EPI (GemmEpilogue) is a template parameter: each epilogue gets a kernel of its own, so that the registers one of them
// needs after the loop do not change the allocation inside the loop of the others.
// Which tile a workgroup computes, and where its two column halves come from.
struct TileCtx {
    int m0;                                 // first activation row
    int seg_h[2], nbase_h[2], ocol_h[2];    // per column half: weight matrix, first weight row, first output column
};

template <int WM, int WN, int EPI>
__device__ __forceinline__ TileCtx tile_setup(const TiledParams &p) {
    constexpr int BM = 2 * WM * 32, BN = 2 * WN * 32, HALF_N = WN * 32;
    // ---- XCD-aware tile order: consecutive logical ids live on one XCD; walk tiles in groups of 8 rows
    int nwg = p.tiles_m * p.tiles_n;
    int bid = blockIdx.x;
    int per_xcd = (nwg + 7) / 8;
    int logical = (bid % 8) * per_xcd + bid / 8;
    if (nwg % 8 != 0) logical = bid;  // ragged grids keep the plain order
    constexpr int GROUP_M = 8;
    int group = logical / (GROUP_M * p.tiles_n);
    int first_m = group * GROUP_M;
    int gsize = p.tiles_m - first_m < GROUP_M ? p.tiles_m - first_m : GROUP_M;
    int in_group = logical % (GROUP_M * p.tiles_n);
    int tile_m = first_m + in_group % gsize;
    int tile_n = in_group / gsize;

    // ---- weight rows of each half of the B tile (half h belongs to wavefront column h)
    TileCtx c;
    if (EPI == EPI_SWIGLU) {
        for (int h = 0; h < 2; ++h) { c.seg_h[h] = h; c.nbase_h[h] = tile_n * HALF_N; c.ocol_h[h] = tile_n * HALF_N; }
    } else {
        int seg = tile_n >= p.tile_begin[2] ? 2 : (tile_n >= p.tile_begin[1] ? 1 : 0);
        for (int h = 0; h < 2; ++h) {
            c.seg_h[h] = seg;
            c.nbase_h[h] = (tile_n - p.tile_begin[seg]) * BN + h * HALF_N;
            c.ocol_h[h] = p.col_off[seg] + c.nbase_h[h];
        }
    }
    c.m0 = tile_m * BM;
    return c;

}

// Epilogue shared by the main-loop variants.  The four wavefronts form a 2 x 2 grid (wm, wn); acc[i][j] is the 32 x 32
// tile (wm * WM + i, wn * WN + j) of the workgroup's output.
template <int WM, int WN, int EPI>
__device__ __forceinline__ void tiled_epilogue(const TiledParams &p, const TileCtx &c, f32x16_t (&acc)[WM][WN], unsigned char *smem) {
    const int t = threadIdx.x, lane = t & 63, w = t >> 6, wm = w >> 1, wn = w & 1;
    const int m0 = c.m0;
    const int *seg_h = c.seg_h, *nbase_h = c.nbase_h, *ocol_h = c.ocol_h;
    // ---- epilogue.  Lane holds column (lane & 31) of each 32x32 tile; register e is row
    //      (e/4)*8 + (lane>>5)*4 + (e%4).
    const int rows_w = p.rows[seg_h[wn]];
    const int nb = nbase_h[wn], oc = ocol_h[wn];
    constexpr int CT = WN * 32 + 8;  // floats per row of a 32-row band in LDS (4 rows apart = 32 banks apart: no conflicts)
    constexpr bool ROPE = EPI == EPI_ROPE || EPI == EPI_ROPE_BS;
    constexpr bool BS = EPI == EPI_ROPE_BS;  // cache rows as 16-bit block-scaled fixed point, q with its low half term
    if (EPI == EPI_F32_ACC || ROPE) __syncthreads();  // every wavefront is done with the operand tiles
    if (ROPE) {
        // The wavefront's 128 columns are one head of q, k or v.  Element e pairs with e + 64: accumulator tiles j and
        // j + 2 of the same lane.  The arithmetic is that of rope_append_kernel, operation for operation, so both paths
        // store the same bits.  Rows leave through a per-wavefront LDS band as whole 256-byte head rows.
        const RopeEpilogue &rp = p.rope;
        const int seg = seg_h[wn];          // 0: q, 1: k, 2: v
        const int head = nb >> 7;           // head within its matrix
        const bool head_ok = nb < rows_w;   // (whole heads: the 128 columns exist or none does)
        constexpr int HT = 128 + 8;         // halves per row of the band
        f16_t *ht = reinterpret_cast<f16_t *>(smem) + w * 32 * HT;
        float *hs = reinterpret_cast<float *>(smem + 4 * 32 * HT * 2) + w * 32;  // row scales of the band (block-scaled cache)
        f16_t *hl = reinterpret_cast<f16_t *>(smem + 4 * 32 * HT * 2 + 4 * 32 * 4) + w * 32 * HT;  // low half terms of q rows
        if (head_ok) {
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                const int mb = m0 + (wm * WM + i) * 32;  // first row of the band (uniform over the wavefront)
                const int pos_b = mb % rp.T, seq_b = rp.b0 + mb / rp.T;
                // KIND 0: half rows; 1: half rows and their low terms (q next to a block-scaled cache); 2: block-scaled k/v rows.
                // One fully unrolled copy of the band per kind (accumulators must be indexed with constants), chosen per wavefront.
                auto band = [&](auto kind_tag) {
                    constexpr int KIND = decltype(kind_tag)::value;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int r = (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                        int pos = pos_b + r;
                        if (pos >= rp.T) pos -= rp.T;  // T >= 32: at most one wrap inside a band
                        pos = pos < rp.S ? pos : rp.S - 1;
                        const float *tab = rp.rope_tab + (size_t)pos * 128;
                        float va[2], vc2[2];
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const int rr = j * 32 + (lane & 31);
                            float a = acc[i][j][e], c = acc[i][j + 2][e];
                            if (seg != 2) {
                                const float cs = tab[2 * rr], sn = tab[2 * rr + 1];
                                const float ra = __fmaf_rn(a, cs, -__fmul_rn(c, sn));
                                const float rb = __fmaf_rn(c, cs, __fmul_rn(a, sn));
                                a = ra; c = rb;
                            }
                            va[j] = a; vc2[j] = c;
                        }
                        if (KIND == 2) {
                            // the 32 lanes of a half-wavefront hold the 128 elements of row r: row maximum by xor shuffles
                            float am = fmaxf(fmaxf(fabsf(va[0]), fabsf(va[1])), fmaxf(fabsf(vc2[0]), fabsf(vc2[1])));
                            am = fmaxf(am, __shfl_xor(am, 1, 64));
                            am = fmaxf(am, __shfl_xor(am, 2, 64));
                            am = fmaxf(am, __shfl_xor(am, 4, 64));
                            am = fmaxf(am, __shfl_xor(am, 8, 64));
                            am = fmaxf(am, __shfl_xor(am, 16, 64));
                            const float inv = kv_inv_of(am);
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                const int rr = j * 32 + (lane & 31);
                                ht[r * HT + rr] = (f16_t)(kv_quant(va[j], inv) & 0xffff);
                                ht[r * HT + rr + 64] = (f16_t)(kv_quant(vc2[j], inv) & 0xffff);
                            }
                            if ((lane & 31) == 0) hs[r] = kv_scale_of(am);
                        } else {
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                const int rr = j * 32 + (lane & 31);
                                const f16_t ha = f32_to_f16(va[j]), hc = f32_to_f16(vc2[j]);
                                ht[r * HT + rr] = ha;
                                ht[r * HT + rr + 64] = hc;
                                if (KIND == 1) {
                                    hl[r * HT + rr] = f32_to_f16(va[j] - f16_to_f32(ha));
                                    hl[r * HT + rr + 64] = f32_to_f16(vc2[j] - f16_to_f32(hc));
                                }
                            }
                        }
                    }
                };
                if (!BS) band(std::integral_constant<int, 0>{});
                else if (seg == 0) band(std::integral_constant<int, 1>{});
                else band(std::integral_constant<int, 2>{});
                // 16 lanes per row (16 bytes each), 4 rows per instruction
                const int c8 = (lane & 15) * 8;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int r = k * 4 + (lane >> 4), m = mb + r;
                    if (m >= p.M) continue;
                    int pos = pos_b + r, seq = seq_b;
                    if (pos >= rp.T) { pos -= rp.T; seq += 1; }
                    const u32x4_t v = *reinterpret_cast<const u32x4_t *>(ht + r * HT + c8);
                    if (seg == 0) {
                        *reinterpret_cast<u32x4_t *>(rp.q_f16 + ((size_t)m * rp.Hq + head) * 128 + c8) = v;
                        if (BS && rp.q_f16_lo) {  // second half term of q, from the band of low terms
                            const u32x4_t vl = *reinterpret_cast<const u32x4_t *>(hl + r * HT + c8);
                            *reinterpret_cast<u32x4_t *>(rp.q_f16_lo + ((size_t)m * rp.Hq + head) * 128 + c8) = vl;
                        }
                    } else {
                        bool store_kv = pos < rp.S;
                        if (rp.d_valid) {
                            int nv = rp.d_valid[seq];
                            nv = nv < 1 ? 1 : (nv > rp.T ? rp.T : nv);
                            store_kv = store_kv && pos < nv;
                        }
                        if (store_kv) {
                            const size_t rowi = kv_row_index(rp.map, seq, head, rp.Hkv, rp.S, pos);
                            f16_t *dst = (seg == 1 ? rp.kc : rp.vc) + rowi * 128 + c8;
                            *reinterpret_cast<u32x4_t *>(dst) = v;
                            if (BS && (lane & 15) == 0) (seg == 1 ? rp.map.kscale : rp.map.vscale)[rowi] = hs[r];
                        }
                    }
                }
            }
        }
    } else if (EPI == EPI_F32) {
        // plain stores: a wavefront store instruction writes two runs of 128 bytes, which the memory system takes as
        // well as whole rows; no detour through LDS
        float *out = reinterpret_cast<float *>(p.out);
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            int n = j * 32 + (lane & 31);
            if (nb + n >= rows_w) continue;
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    int m = m0 + (wm * WM + i) * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                    if (m < p.M) out[(size_t)m * p.ldc + oc + n] = acc[i][j][e];
                }
        }
    } else if (EPI == EPI_F32_ACC) {
        // read-modify-write of the residual: whole rows, 16 bytes per lane, and all reads of a band are requested
        // before its first write (the compiler may not move a load of `out` above a store to it)
        float *out = reinterpret_cast<float *>(p.out);
        float *ct = reinterpret_cast<float *>(smem) + w * 32 * CT;  // private to the wavefront: no barriers below
        constexpr int LPR = WN * 8;        // lanes per row (4 floats each)
        constexpr int RPI = 64 / LPR;      // rows per store instruction
        constexpr int NK = 32 / RPI;
        const int c4 = (lane % LPR) * 4, r_in = lane / LPR;
        const int ncols = rows_w - nb < WN * 32 ? rows_w - nb : WN * 32;
        const bool vec = c4 + 4 <= ncols && ((p.ldc | oc) & 3) == 0;  // 16-byte aligned whole group
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int mb = m0 + (wm * WM + i) * 32;
            f32x4_t old[NK];
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                const int m = mb + k * RPI + r_in;
                old[k] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                if (vec && m < p.M) old[k] = *reinterpret_cast<const f32x4_t *>(out + (size_t)m * p.ldc + oc + c4);
            }
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    ct[((e >> 2) * 8 + (lane >> 5) * 4 + (e & 3)) * CT + j * 32 + (lane & 31)] = acc[i][j][e];
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                const int r = k * RPI + r_in, m = mb + r;
                if (m >= p.M || c4 >= ncols) continue;
                f32x4_t v = *reinterpret_cast<const f32x4_t *>(ct + r * CT + c4);
                float *dst = out + (size_t)m * p.ldc + oc + c4;
                if (vec) {
                    v.x += old[k].x; v.y += old[k].y; v.z += old[k].z; v.w += old[k].w;
                    *reinterpret_cast<f32x4_t *>(dst) = v;
                } else {
                    float vv[4] = {v.x, v.y, v.z, v.w};
                    for (int q = 0; q < 4 && c4 + q < ncols; ++q) dst[q] += vv[q];
                }
            }
        }
    } else {
        // wavefront column 1 (up) hands its band to wavefront column 0 (gate) of the same rows through LDS
        float *ex = reinterpret_cast<float *>(smem) + wm * (WN * 16 * 64);                // [WN][16][64] floats per wavefront row
        f16_t *ht = reinterpret_cast<f16_t *>(smem + 2 * WN * 16 * 64 * 4) + wm * 32 * (2 * CT);  // [32][2 CT] halves
        f16_t *out = reinterpret_cast<f16_t *>(p.out);
        constexpr int LPR = WN * 4;        // lanes per row (8 halves each)
        constexpr int RPI = 64 / LPR;
        const int c8 = (lane % LPR) * 8, r_in = lane / LPR;
        const int ncols = rows_w - nb < WN * 32 ? rows_w - nb : WN * 32;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            __syncthreads();  // the previous band has been read
            if (wn == 1) {
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) ex[(j * 16 + e) * 64 + lane] = acc[i][j][e];
            }
            __syncthreads();
            if (wn == 0) {
                // the band is private to this wavefront: the high term leaves first, then the band is refilled with the
                // low term half(y - half(y)) when the caller asked for it
                for (int tm = 0; tm < (p.out_lo ? 2 : 1); ++tm) {
#pragma unroll
                    for (int j = 0; j < WN; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            float g = acc[i][j][e], u = ex[(j * 16 + e) * 64 + lane];
                            float a = g / (1.0f + expf(-g)) * u;
                            const f16_t hi = f32_to_f16(a);
                            ht[((e >> 2) * 8 + (lane >> 5) * 4 + (e & 3)) * (2 * CT) + j * 32 + (lane & 31)] =
                                tm == 0 ? hi : f32_to_f16(a - f16_to_f32(hi));
                        }
                    f16_t *outp = tm == 0 ? out : p.out_lo;
                    const int mb = m0 + (wm * WM + i) * 32;
#pragma unroll
                    for (int k = 0; k < 32 / RPI; ++k) {
                        const int r = k * RPI + r_in, m = mb + r;
                        if (m >= p.M || c8 >= ncols) continue;
                        u32x4_t v = *reinterpret_cast<const u32x4_t *>(ht + r * (2 * CT) + c8);
                        f16_t *dst = outp + (size_t)m * p.ldc + oc + c8;
                        if (c8 + 8 <= ncols && (((size_t)m * p.ldc + oc) & 7) == 0) {
                            *reinterpret_cast<u32x4_t *>(dst) = v;
                        } else {
                            const f16_t *src = ht + r * (2 * CT) + c8;
                            for (int q = 0; q < 8 && c8 + q < ncols; ++q) dst[q] = src[q];
                        }
                    }
                }
            }
        }
    }
}

template <int WM, int WN, int EPI>
__global__ __launch_bounds__(TG_THREADS, 1) void gemm_tiled_kernel(TiledParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int BM = 2 * WM * 32, BN = 2 * WN * 32, HALF_N = WN * 32;
    constexpr int A_LOADS = BM / 32, B_LOADS = BN / 32;  // 16-byte loads per thread per chunk
    f16_t *as = reinterpret_cast<f16_t *>(smem);                    // [2][BM][72]
    f16_t *bs = as + 2 * BM * TG_LDS_STRIDE;                         // [2][BN][72]
    const int t = threadIdx.x, lane = t & 63, w = t >> 6, wm = w >> 1, wn = w & 1;
    const int K = p.K;

    const TileCtx ctx = tile_setup<WM, WN, EPI>(p);
    const int m0 = ctx.m0;
    const int *seg_h = ctx.seg_h, *nbase_h = ctx.nbase_h;

    // loader mapping: thread -> (row t/8 + 32*i, 16-byte group t%8).  Range-checked buffer loads: rows past
    // the matrix and K columns past the end get an offset outside the descriptor and come back as zeros,
    // so the loop needs no branches and the count of outstanding loads is the same on every trip.
    const int lc = t & 7, lr = t >> 3;
    constexpr uint32_t OOB = 0xFFFFFF00u;
    __amdgpu_buffer_rsrc_t a_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<f16_t *>(p.A), 0, (int)p.a_bytes, 0x00020000);
    uint32_t a_off[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        int row = m0 + lr + 32 * i;
        a_off[i] = row < p.M ? (uint32_t)((size_t)row * p.lda * 2) + (uint32_t)lc * 16u : OOB;
    }
    // B rows of the two halves may come from different matrices: one descriptor per half
    __amdgpu_buffer_rsrc_t b_rs[2];
    uint32_t b_off[B_LOADS];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
        b_rs[hh] = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(p.W[seg_h[hh]]), 0,
                                                      (int)(uint32_t)((size_t)p.rows[seg_h[hh]] * K * 2), 0x00020000);
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        int r = lr + 32 * i;
        int hh = r / HALF_N;
        int row = nbase_h[hh] + (r - hh * HALF_N);
        int rows = p.rows[seg_h[hh]];
        b_off[i] = (uint32_t)(row < rows ? row : 0) * (uint32_t)K * 2u + (uint32_t)lc * 16u;  // clamped rows are never stored
    }
    u32x4_t ar[A_LOADS], br[B_LOADS];
    f32x16_t acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Trip c covers K chunk c % chunks of activation term c / chunks: with two terms the contraction runs over
    // [A | A_lo] against [W | W], so both products land in the same accumulators.
    const int trips = p.chunks * p.terms;
    auto load_a1 = [&](int c, int i) {
        int term = c >= p.chunks ? 1 : 0, ck = c - term * p.chunks;
        uint32_t kb = (uint32_t)ck * (TG_BK * 2) + (term ? p.lo_delta : 0u);
        bool kok = c < trips && ck * TG_BK + lc * 8 < K;
        ar[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rs, (int)(kok && a_off[i] != OOB ? a_off[i] + kb : OOB), 0, 0);
    };
    auto load_b1 = [&](int c, int i) {
        int ck = c >= p.chunks ? c - p.chunks : c;
        uint32_t kb = (uint32_t)ck * (TG_BK * 2);
        bool kok = c < trips && ck * TG_BK + lc * 8 < K;
        // piece i belongs to half (32 i) / HALF_N: a compile-time choice of descriptor
        br[i] = __builtin_amdgcn_raw_buffer_load_b128((32 * i) / HALF_N == 0 ? b_rs[0] : b_rs[1], (int)(kok ? b_off[i] + kb : OOB), 0, 0);
    };
    auto store_a1 = [&](int buf, int i) {
        *reinterpret_cast<u32x4_t *>(as + buf * BM * TG_LDS_STRIDE + (lr + 32 * i) * TG_LDS_STRIDE + lc * 8) = ar[i];
    };
    auto store_b1 = [&](int buf, int i) {
        *reinterpret_cast<u32x4_t *>(bs + buf * BN * TG_LDS_STRIDE + (lr + 32 * i) * TG_LDS_STRIDE + lc * 8) = bf16x8_to_f16x8(br[i]);
    };

    // One K chunk: 4 k-steps of WM*WN MFMAs on the tiles staged one chunk ago.  Interleaved with them, piece by
    // piece: LDS fragments of the next k-step, the next chunk's operands registers -> LDS (weights widened on the
    // way), and the loads of the chunk after next into the registers just freed -- so the matrix cores, the LDS
    // and the memory pipeline overlap although only one wavefront runs per SIMD.
    constexpr int APS = A_LOADS / 4, BPS = B_LOADS / 4;  // pieces staged per k-step
    auto body = [&](int c, auto par_tag) {
        constexpr int PAR = decltype(par_tag)::value;
        __syncthreads();  // tiles of chunk c are in LDS buffer PAR; buffer PAR^1 is free
        const f16_t *ap = as + PAR * BM * TG_LDS_STRIDE + (wm * WM * 32 + (lane & 31)) * TG_LDS_STRIDE + (lane >> 5) * 8;
        const f16_t *bp = bs + PAR * BN * TG_LDS_STRIDE + (wn * WN * 32 + (lane & 31)) * TG_LDS_STRIDE + (lane >> 5) * 8;
        f16x8_t af[2][WM], bf[2][WN];
#pragma unroll
        for (int i = 0; i < WM; ++i) af[0][i] = *reinterpret_cast<const f16x8_t *>(ap + i * 32 * TG_LDS_STRIDE);
#pragma unroll
        for (int j = 0; j < WN; ++j) bf[0][j] = *reinterpret_cast<const f16x8_t *>(bp + j * 32 * TG_LDS_STRIDE);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s + 1 < 4) {
#pragma unroll
                for (int i = 0; i < WM; ++i)
                    af[(s + 1) & 1][i] = *reinterpret_cast<const f16x8_t *>(ap + i * 32 * TG_LDS_STRIDE + (s + 1) * 16);
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    bf[(s + 1) & 1][j] = *reinterpret_cast<const f16x8_t *>(bp + j * 32 * TG_LDS_STRIDE + (s + 1) * 16);
            }
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[s & 1][i], bf[s & 1][j], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < APS; ++q) { store_a1(PAR ^ 1, s * APS + q); load_a1(c + 2, s * APS + q); }
#pragma unroll
            for (int q = 0; q < BPS; ++q) { store_b1(PAR ^ 1, s * BPS + q); load_b1(c + 2, s * BPS + q); }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) load_a1(0, i);
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) load_b1(0, i);
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) { store_a1(0, i); load_a1(1, i); }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) { store_b1(0, i); load_b1(1, i); }
    __builtin_amdgcn_sched_barrier(0);
    for (int c = 0; c < trips; c += 2) {
        body(c, std::integral_constant<int, 0>{});
        body(c + 1, std::integral_constant<int, 1>{});  // past the end: multiplies zero tiles
    }

    tiled_epilogue<WM, WN, EPI>(p, ctx, acc, smem);
}

// ---------------------------------------------------------------------------------------------------------------------
// The same tile computation with both operands copied global -> LDS by the load unit itself (buffer_load ... lds): no
// staging registers, no ds_write, no bf16 -> half conversion in the loop.  Needs the weights as half in matrix-core
// fragment order (the copies the decode step streams): a B fragment is then 1 KB of consecutive bytes in memory and in
// LDS.  K is walked in stages of 32 through a ring of four stages (three in flight while one is consumed): a wavefront
// waits on its own load counter for the oldest stage, the barrier then makes every wavefront's part of it visible.
// Activation rows are 64 bytes per stage; their 16-byte pieces are stored XOR-permuted (piece ^ (row / 4 & 3)), so a fragment
// read -- 16 consecutive rows, same piece, in the 16 lanes served together -- covers all 64 banks.
#define TD_STAGES 4
#define TD_SK 32
#define TD_A_BYTES (256 * TD_SK * 2)
#define TD_STAGE_BYTES (2 * TD_A_BYTES)
#define TD_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

template <int EPI>
__global__ __launch_bounds__(TG_THREADS, 1) void gemm_tiled_dma_kernel(TiledParams p) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    constexpr int WM = 4, WN = 4;
    const int t = threadIdx.x, lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w >> 1, wn = w & 1;
    const int K = p.K;
    const TileCtx ctx = tile_setup<WM, WN, EPI>(p);
    // A voffset at or above 2^31 is out of range for every descriptor used here (the launcher keeps them below 2 GB) and
    // stays so with any scalar offset added: such a copy writes zeros.
    constexpr uint32_t OOB = 0x80000000u;

    // ---- copy plan.  A stage holds A[256 rows][32 k] (16 KB) and B as 8 column blocks x 2 k-steps of 1 KB fragments (16 KB).
    //      Wavefront w issues copy instructions 4 w .. 4 w + 3 of each operand.  Per lane and instruction a fixed byte
    //      offset (voffset); what moves with the stage is a scalar offset, the same for the whole wavefront.
    __amdgpu_buffer_rsrc_t a_rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<f16_t *>(p.A), 0, (int)p.a_bytes, 0x00020000);
    uint32_t a_vo[4];  // this lane's 16-byte piece of its row, chunk 0, term 0
    int a_lim[4];      // the piece holds data while 32 * chunk < a_lim (0 for rows past M: never)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = 16 * (4 * w + q) + (lane >> 2);  // row of the tile
        const int piece = (lane & 3) ^ ((r >> 2) & 3);
        a_vo[q] = (uint32_t)((size_t)(ctx.m0 + r) * p.lda * 2) + (uint32_t)piece * 16u;
        a_lim[q] = ctx.m0 + r < p.M ? K - piece * 8 : 0;

    }
    // B: fragment f = 4 w + q of a stage is column block f / 2 of the tile (blocks 0..3: half 0, 4..7: half 1), k-step f % 2
    __amdgpu_buffer_rsrc_t b_rs[4];
    uint32_t b_vo[4];
    int b_ks[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int f = 4 * w + q, blk = f >> 1, hh = blk >> 2;
        const int seg = ctx.seg_h[hh];
        const int nblk = ctx.nbase_h[hh] / 32 + (blk & 3);  // 32-row block within its matrix
        const int nblocks = (p.rows[seg] + 31) / 32;
        // (the descriptor must sit in scalar registers: say so, or every copy instruction is wrapped in a loop over distinct values)
        const uint64_t pa = (uint64_t)p.P[seg];
        const uint32_t pa_lo = __builtin_amdgcn_readfirstlane((uint32_t)pa), pa_hi = __builtin_amdgcn_readfirstlane((uint32_t)(pa >> 32));
        const uint32_t pbytes = __builtin_amdgcn_readfirstlane((uint32_t)((size_t)nblocks * p.ksteps * 1024));
        b_rs[q] = __builtin_amdgcn_make_buffer_rsrc((void *)(((uint64_t)pa_hi << 32) | pa_lo), 0, (int)pbytes, 0x00020000);
        b_ks[q] = f & 1;
        b_vo[q] = nblk < nblocks ? (uint32_t)(((size_t)nblk * p.ksteps + b_ks[q]) * 1024) + (uint32_t)lane * 16u : OOB;

    }
    const int chunks = (K + TD_SK - 1) / TD_SK;  // stages per activation term
    const int trips = chunks * p.terms;
    // what a stage's copies share: computed once per stage in scalar registers
    struct StageScalars { int k32; int ks2; uint32_t a_so, b_so; };
    auto stage_scalars = [&](int c) {
        StageScalars z;
        const int term = c >= chunks ? 1 : 0, ck = c - term * chunks;
        const bool live = c < trips;
        z.k32 = live ? ck * TD_SK : 0x7fffffff;   // past the last stage: every piece is "beyond K"
        z.ks2 = live ? 2 * ck : 0x3fffffff;
        z.a_so = live ? (uint32_t)ck * (TD_SK * 2) + (term ? p.lo_delta : 0u) : 0u;
        z.b_so = live ? (uint32_t)ck * 2048u : 0u;
        return z;
    };
    auto issue_a = [&](const StageScalars &z, int stage, int q) {
        unsigned char *ad = smem + stage * TD_STAGE_BYTES + (4 * w + q) * 1024;
        const uint32_t vo = z.k32 < a_lim[q] ? a_vo[q] : OOB;
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass does not know this builtin
        __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rs, TD_LDS_PTR(ad), 16, (int)vo, (int)z.a_so, 0, 0);
#else
        (void)ad; (void)vo;
#endif
    };
    auto issue_b = [&](const StageScalars &z, int stage, int q) {
        unsigned char *bd = smem + stage * TD_STAGE_BYTES + TD_A_BYTES + (4 * w + q) * 1024;
        const uint32_t vo = z.ks2 + b_ks[q] < p.ksteps ? b_vo[q] : OOB;
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rs[q], TD_LDS_PTR(bd), 16, (int)vo, (int)z.b_so, 0, 0);
#else
        (void)bd; (void)vo;
#endif
    };
    auto issue = [&](int c, int stage) {
        const StageScalars z = stage_scalars(c);
#pragma unroll
        for (int q = 0; q < 4; ++q) { issue_a(z, stage, q); issue_b(z, stage, q); }
    };

    // ---- fragment addresses within a stage
    int a_ld[WM][2];  // row tile i, k-step s: row wm * 128 + 32 i + (lane & 31), piece 2 s + (lane >> 5)
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const int row = wm * 128 + 32 * i + (lane & 31);
            a_ld[i][s2] = row * 64 + (((2 * s2 + (lane >> 5)) ^ ((row >> 2) & 3)) << 4);
        }
    const int b_ld = TD_A_BYTES + wn * 8 * 1024 + lane * 16;  // column tile j, k-step s: + (2 j + s) * 1024

    f32x16_t acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // One wavefront per SIMD: whatever it issues that is not a matrix-core instruction delays the next one, unless it sits
    // in the shadow of one (32 cycles each).  So the loop is written as the instruction order it should have: after each
    // of the 16 matrix instructions of a k-step one small piece of other work -- a fragment read for the next k-step (into
    // the other half of a register ping-pong), or one copy instruction of the stage three ahead -- with scheduling
    // fences between, so that the compiler keeps the order.
    f16x8_t af[2][WM], bf[2][WN];
    auto read_a = [&](int stage, int s2, int buf, int i) {
        af[buf][i] = *reinterpret_cast<const f16x8_t *>(smem + stage * TD_STAGE_BYTES + a_ld[i][s2]);
    };
    auto read_b = [&](int stage, int s2, int buf, int j) {
        bf[buf][j] = *reinterpret_cast<const f16x8_t *>(smem + stage * TD_STAGE_BYTES + b_ld + (2 * j + s2) * 1024);
    };
    auto multiply = [&](int buf, int n) {
        const int i = n >> 2, j = n & 3;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[buf][i], bf[buf][j], acc[i][j], 0, 0, 0);
    };
    // (a bare barrier instruction: the workgroup barrier of the language also waits for every outstanding load, which
    //  would end the overlap of the copies with the arithmetic; the explicit counter wait says what has to have landed)
    constexpr int YOUNGER = 8 * (TD_STAGES - 2);  // copy instructions of the two stages younger than the one waited for
    constexpr int WAIT_STAGE = (YOUNGER & 15) | (7 << 4) | (0 << 8) | ((YOUNGER >> 4) << 14);  // vmcnt(YOUNGER), lgkmcnt(0)
#pragma unroll
    for (int k = 0; k < TD_STAGES - 1; ++k) issue(k, k);
    __builtin_amdgcn_s_waitcnt(WAIT_STAGE);
    __builtin_amdgcn_s_barrier();  // chunk 0 is in stage 0 for every wavefront
    issue(TD_STAGES - 1, TD_STAGES - 1);
#pragma unroll
    for (int n = 0; n < 4; ++n) { read_b(0, 0, 0, n); read_a(0, 0, 0, n); }
    __builtin_amdgcn_sched_barrier(0);
    for (int c0 = 0; c0 < trips; c0 += TD_STAGES) {
#pragma unroll
        for (int k = 0; k < TD_STAGES; ++k) {  // unrolled: stage offsets become immediates
            if (c0 + k < trips) {               // uniform over the workgroup
                // k-step 0 of stage k (fragments: ping), reading k-step 1 (pong)
#pragma unroll
                for (int n = 0; n < 16; ++n) {
                    multiply(0, n);
                    __builtin_amdgcn_sched_barrier(0);
                    if (n < 4) read_b(k, 1, 1, n);
                    else if (n < 8) read_a(k, 1, 1, n - 4);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // chunk c0 + k + 1 has landed for this wavefront, and its own reads of stage k are complete ...
                __builtin_amdgcn_s_waitcnt(WAIT_STAGE);
                __builtin_amdgcn_s_barrier();  // ... and for every wavefront: stage k is free, stage k + 1 is readable
                __builtin_amdgcn_sched_barrier(0);
                // k-step 1 (pong), reading k-step 0 of stage k + 1 (ping) and refilling stage k with chunk c0 + k + 4
                const StageScalars z = stage_scalars(c0 + k + TD_STAGES);
#pragma unroll
                for (int n = 0; n < 16; ++n) {
                    multiply(1, n);
                    __builtin_amdgcn_sched_barrier(0);
                    if (n < 4) read_b((k + 1) % TD_STAGES, 0, 0, n);
                    else if (n < 8) read_a((k + 1) % TD_STAGES, 0, 0, n - 4);
                    else if (n < 12) issue_a(z, k, n - 8);
                    else issue_b(z, k, n - 12);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
    __builtin_amdgcn_s_waitcnt((0 & 15) | (7 << 4) | (15 << 8) | (0 << 14));  // no copy may still be writing LDS
    __syncthreads();
    tiled_epilogue<WM, WN, EPI>(p, ctx, acc, smem);
}

template <int WM, int WN, int EPI>
static void launch_t(TiledParams &p, const GemmArgs &a, hipStream_t st) {
    constexpr int BM = 2 * WM * 32, BN = 2 * WN * 32;
    int tiles = 0, col = 0;
    for (int i = 0; i < 3; ++i) {
        p.tile_begin[i] = tiles;
        p.col_off[i] = col;
        if (a.epilogue == EPI_SWIGLU) continue;
        tiles += ceil_div(p.rows[i], BN);
        col += p.rows[i];
    }
    if (a.epilogue == EPI_SWIGLU) tiles = ceil_div(a.rows[0], BN / 2);
    p.tile_begin[3] = tiles;
    p.tiles_n = tiles;
    p.tiles_m = ceil_div(a.M, BM);
    if (tiles <= 0 || p.tiles_m <= 0) return;
    size_t lds = (size_t)2 * (BM + BN) * TG_LDS_STRIDE * sizeof(f16_t);
    size_t ex = (size_t)2 * WM * 16 * 64 * sizeof(float);
    if (ex > lds) lds = ex;
    size_t bands = (size_t)4 * 32 * (WN * 32 + 8) * sizeof(float);  // accumulate epilogue: one 32-row band per wavefront
    if (bands > lds) lds = bands;
    // SwiGLU epilogue: two exchange areas plus two half bands
    size_t sw = (size_t)2 * WN * 16 * 64 * sizeof(float) + (size_t)2 * 32 * 2 * (WN * 32 + 8) * sizeof(f16_t);
    if (sw > lds) lds = sw;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tiled_kernel<WM, WN, EPI>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        attr_set = true;
    }
    if (WM == 4 && WN == 4 && p.P[0]) {
        size_t dlds = (size_t)TD_STAGES * TD_STAGE_BYTES;
        if (lds > dlds) dlds = lds;
        static bool dma_attr_set = false;
        if (!dma_attr_set) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tiled_dma_kernel<EPI>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            dma_attr_set = true;
        }
        gemm_tiled_dma_kernel<EPI><<<p.tiles_m * p.tiles_n, TG_THREADS, dlds, st>>>(p);
        return;
    }
    gemm_tiled_kernel<WM, WN, EPI><<<p.tiles_m * p.tiles_n, TG_THREADS, lds, st>>>(p);
}

static void launch_one(const GemmArgs &a, hipStream_t st) {
    TiledParams p = {};
    p.A = a.A;
    p.lda = a.lda;
    p.a_bytes = (uint32_t)((((size_t)a.M - 1) * a.lda + a.K) * 2);
    p.lo_delta = 0;
    p.terms = 1;
    if (a.A_lo) {  // the caller has checked that A_lo lies above A and both fit one descriptor
        p.lo_delta = (uint32_t)((a.A_lo - a.A) * sizeof(f16_t));
        p.a_bytes += p.lo_delta;
        p.terms = 2;
    }
    p.M = a.M;
    p.K = a.K;
    p.chunks = ceil_div(a.K, TG_BK);
    p.epilogue = a.epilogue;
    p.out = a.out;
    p.out_lo = a.epilogue == EPI_SWIGLU ? a.out_lo : nullptr;
    p.ldc = a.ldc;
    int n_total = 0;
    bool have_p = a.P[0] != nullptr;
    for (int i = 0; i < 3; ++i) {
        p.W[i] = a.W[i] ? a.W[i] : a.W[0];
        p.rows[i] = a.W[i] ? a.rows[i] : 0;
        n_total += p.rows[i];
        if (a.W[i] && !a.P[i]) have_p = false;
    }
    p.ksteps = ceil_div(a.K, 16);
    if (p.a_bytes >= 0x80000000u) have_p = false;
    for (int i = 0; i < 3; ++i) {
        // fragment-order copies are used when every matrix has one and every operand stays below 2 GB (the kernel marks
        // a copy as out of range with bit 31 of its offset)
        if (a.W[i] && have_p && (size_t)ceil_div(p.rows[i], 32) * p.ksteps * 1024 >= 0x80000000ull) have_p = false;
    }
    for (int i = 0; i < 3; ++i) p.P[i] = have_p ? (a.P[i] ? a.P[i] : a.P[0]) : nullptr;
    // big tiles only when they still give every compute unit work
    long big_tiles = (long)ceil_div(a.M, 256) * ceil_div(n_total, 256);
    const bool big = a.M >= 1024 && big_tiles >= 256;
    if (a.epilogue == EPI_SWIGLU) { if (big) launch_t<4, 4, EPI_SWIGLU>(p, a, st); else launch_t<2, 2, EPI_SWIGLU>(p, a, st); }
    else if (a.epilogue == EPI_F32_ACC) { if (big) launch_t<4, 4, EPI_F32_ACC>(p, a, st); else launch_t<2, 2, EPI_F32_ACC>(p, a, st); }
    else if (a.epilogue == EPI_ROPE) {  // 128-column wavefronts only
        p.rope = *a.rope;
        if (p.rope.map.kscale) { p.epilogue = EPI_ROPE_BS; launch_t<4, 4, EPI_ROPE_BS>(p, a, st); }
        else launch_t<4, 4, EPI_ROPE>(p, a, st);
    }
    else { if (big) launch_t<4, 4, EPI_F32>(p, a, st); else launch_t<2, 2, EPI_F32>(p, a, st); }
}

// Can launch_gemm_tiled run EPI_ROPE on this problem?  (Whole heads of 128 per matrix, bands that wrap at most once,
// enough tiles for the 256 x 256 kernel, operands that need no cutting.)
bool gemm_tiled_rope_supported(int M, int K, int64_t lda, int Hq, int Hkv, int hd, int rope_style, int T, bool two_terms) {
    if (hd != 128 || rope_style != 1 || T < 32 || M < 1024) return false;
    const long n_total = (long)(Hq + 2 * Hkv) * 128;
    if ((long)ceil_div(M, 256) * ceil_div((int)n_total, 256) < 256) return false;
    const size_t a_bytes = (((size_t)M - 1) * lda + K) * 2 * (two_terms ? 2 : 1) + (two_terms ? (size_t)M * lda * 2 : 0);
    if (a_bytes >= 0xF0000000ull || (size_t)Hq * 128 * K * 2 >= 0xF0000000ull) return false;
    return true;
}

// The kernel addresses each operand through a buffer descriptor with 32-bit byte offsets: operands of
// TG_MAX_BYTES or more are cut into row blocks (of A) or into per-matrix row blocks (of W) here.
#define TG_MAX_BYTES 0xF0000000ull

void launch_gemm_tiled(const GemmArgs &a, hipStream_t st) {
    if (a.M <= 0) return;
    const size_t out_elem = a.epilogue == EPI_SWIGLU ? sizeof(f16_t) : sizeof(float);
    size_t a_bytes = (((size_t)a.M - 1) * a.lda + a.K) * 2;
    if (a.A_lo) a_bytes += (size_t)(a.A_lo - a.A) * 2;
    if (a_bytes >= TG_MAX_BYTES && a.A_lo && (size_t)(a.A_lo - a.A) * 2 >= TG_MAX_BYTES / 2) {
        // the two terms are too far apart for one descriptor: two passes, the second accumulating (fp32 outputs only)
        GemmArgs s = a;
        s.A_lo = nullptr;
        launch_gemm_tiled(s, st);
        s.A = a.A_lo;
        s.epilogue = EPI_F32_ACC;
        launch_gemm_tiled(s, st);
        return;
    }
    if (a_bytes >= TG_MAX_BYTES) {
        int rows_max = (int)((TG_MAX_BYTES / ((size_t)a.lda * 2)) / 256 * 256);
        for (int m = 0; m < a.M; m += rows_max) {
            GemmArgs s = a;
            s.A = a.A + (size_t)m * a.lda;
            if (a.A_lo) s.A_lo = a.A_lo + (size_t)m * a.lda;
            s.M = a.M - m < rows_max ? a.M - m : rows_max;
            s.out = static_cast<char *>(a.out) + (size_t)m * a.ldc * out_elem;
            if (a.out_lo) s.out_lo = a.out_lo + (size_t)m * a.ldc;
            launch_gemm_tiled(s, st);
        }
        return;
    }
    bool w_big = false;
    for (int i = 0; i < 3; ++i)
        if (a.W[i] && (size_t)a.rows[i] * a.K * 2 >= TG_MAX_BYTES) w_big = true;
    if (!w_big) { launch_one(a, st); return; }
    int rows_max = (int)((TG_MAX_BYTES / ((size_t)a.K * 2)) / 256 * 256);
    if (a.epilogue == EPI_SWIGLU) {  // gate and up blocks of the same output columns go together
        for (int n = 0; n < a.rows[0]; n += rows_max) {
            GemmArgs s = a;
            s.P[0] = s.P[1] = s.P[2] = nullptr;  // row blocks of the weights: the fragment-order copies are not cut along
            int r = a.rows[0] - n < rows_max ? a.rows[0] - n : rows_max;
            s.W[0] = a.W[0] + (size_t)n * a.K;
            s.W[1] = a.W[1] + (size_t)n * a.K;
            s.rows[0] = s.rows[1] = r;
            s.out = static_cast<char *>(a.out) + (size_t)n * out_elem;
            if (a.out_lo) s.out_lo = a.out_lo + n;
            launch_one(s, st);
        }
        return;
    }
    int col = 0;
    for (int i = 0; i < 3; ++i) {
        if (!a.W[i] || a.rows[i] <= 0) continue;
        for (int n = 0; n < a.rows[i]; n += rows_max) {
            GemmArgs s = a;
            s.P[0] = s.P[1] = s.P[2] = nullptr;
            s.W[0] = a.W[i] + (size_t)n * a.K;
            s.rows[0] = a.rows[i] - n < rows_max ? a.rows[i] - n : rows_max;
            s.W[1] = s.W[2] = nullptr;
            s.rows[1] = s.rows[2] = 0;
            s.out = static_cast<char *>(a.out) + (size_t)(col + n) * out_elem;
            launch_one(s, st);
        }
        col += a.rows[i];
    }
}
