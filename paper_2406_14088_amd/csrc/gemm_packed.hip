// Skinny-M GEMM over weights re-laid-out once in matrix-core fragment order (the decode step).
//
// A decode step multiplies one row of activations per sequence with every weight matrix: each weight
// is used for only M (<= 128 per workgroup) multiply-adds, so the step lives off streaming the weights
// from HBM exactly once, and whatever a compute unit has to do per weight byte besides the multiply
// (widening bf16, transposing row-major rows into the lane = row layout the matrix cores want) costs
// throughput.  The weights of a generation phase do not change, so that work is done once:
//
//   pack:   W [N, K] bf16 row-major  ->  P [ceil(N/32)][ceil(K/16)][64 lanes][8] IEEE half, where lane l of
//           fragment (nb, ks) holds W[32 nb + (l & 31), 16 ks + 8 (l >> 5) + 0..7] (zero outside W).
//           One fragment is exactly the B operand of one v_mfma_f32_32x32x16_f16 and is 1 KB of
//           consecutive memory; the fragments of one 32-row block follow each other along K.
//
//   gemm:   a wavefront owns NB 32-row blocks (= 32 NB output columns) and walks along K: one
//           16-byte-per-lane load (a whole, contiguous KB) fetches a fragment straight into the
//           registers the MFMA reads -- no LDS, no conversion, no shuffle on the weight side.  Loads
//           run two or four K chunks (4 NB fragments each) ahead in a register ring.
//           The activation chunk [128 rows, 64 k] is shared by the four wavefronts of a workgroup: it is
//           copied global -> LDS by the load unit itself (buffer loads with the LDS bit: no registers,
//           no ds_write), in an XOR-swizzled layout whose fragment reads are free of bank conflicts, two
//           chunks ahead in a three-deep buffer ring.
//           TERMS = 2 multiplies the same weight fragment with two activation tiles (the two-term split
//           of the normalised activations) into the same accumulators.
//           Split-K over workgroups (grid.y) fills the chip; every split writes its own fp32 partial tile
//           and the consumer adds the partials in a fixed order (deterministic).
//           Epilogues: fp32 partials / fp32 accumulate through an LDS tile (whole 512-byte rows per
//           store instruction); SwiGLU with gate block and up block of the same columns held by the same
//           wavefront, so the nonlinearity needs no exchange.
#include <type_traits>

#include "kernels.h"

#define PK_BK 64             // K elements per chunk (4 MFMA k-steps)
#define PK_THREADS 256
#define PK_OOB 0xFFFFFF00u   // byte offset beyond every descriptor: such a load returns zeros, touches no memory
#define PK_CT_STRIDE 132     // floats per row of the fp32 output tile in LDS
#define PK_HT_STRIDE 136     // halves per row of the SwiGLU output tile in LDS
#define PK_MAX_BYTES 0xF0000000ull

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// ---------------------------------------------------------------------------------------------------
// pack
// ---------------------------------------------------------------------------------------------------
// One workgroup converts one (32-row block, 64-wide K chunk) = 4 fragments: rows are read as whole
// 128-byte lines (8 lanes x 16 B per row), widened, transposed through LDS, written as 4 contiguous KB.
__global__ __launch_bounds__(256) void pack_weights_kernel(const bf16_t *W, f16_t *P, int N, int K, int ksteps) {
    __shared__ __attribute__((aligned(16))) uint32_t tile[32][36];  // 32 rows x 64 halves (+ pad)
    const int t = threadIdx.x;
    const int nb = blockIdx.y, kc = blockIdx.x;
    const int r = t >> 3, g = t & 7;  // row of the block, 16-byte piece of the 128-byte chunk
    const int n = nb * 32 + r, k = kc * 64 + g * 8;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (n < N && k < K) v = bf16x8_to_f16x8(*reinterpret_cast<const u32x4_t *>(W + (size_t)n * K + k));  // K % 8 == 0
    *reinterpret_cast<u32x4_t *>(&tile[r][g * 4]) = v;
    __syncthreads();
    // thread t writes lane (t & 63) of fragment ks = 4 kc + t / 64
    const int s = t >> 6, l = t & 63;
    const int ks = kc * 4 + s;
    if (ks < ksteps) {
        u32x4_t o = *reinterpret_cast<const u32x4_t *>(&tile[l & 31][s * 8 + (l >> 5) * 4]);
        *reinterpret_cast<u32x4_t *>(P + (((size_t)nb * ksteps + ks) * 64 + l) * 8) = o;
    }
}

size_t packed_weight_bytes(int N, int K) { return (size_t)ceil_div(N, 32) * ceil_div(K, 16) * 1024; }

void launch_pack_weights(const bf16_t *W, f16_t *P, int N, int K, hipStream_t st) {
    if (N <= 0 || K <= 0) return;
    int ksteps = ceil_div(K, 16);
    // grid.y is limited to 65535 blocks: walk taller matrices in slabs
    const int max_nb = 65535;
    int nblocks = ceil_div(N, 32);
    for (int b0 = 0; b0 < nblocks; b0 += max_nb) {
        int nbl = nblocks - b0 < max_nb ? nblocks - b0 : max_nb;
        int rows_left = N - b0 * 32;
        pack_weights_kernel<<<dim3(ceil_div(K, 64), nbl), 256, 0, st>>>(W + (size_t)b0 * 32 * K, P + (size_t)b0 * ksteps * 512,
                                                                     rows_left, K, ksteps);
    }
}

// ---------------------------------------------------------------------------------------------------
// gemm
// ---------------------------------------------------------------------------------------------------
struct PackedParams {
    const f16_t *A;     // first-term activations [M, K], row stride lda
    const f16_t *A_lo;  // second-term activations (TERMS == 2), same shape and stride
    const f16_t *P[3];  // packed matrices
    int rows[3];
    int tile_begin[4];  // first n-tile of each matrix (prefix sums), tile_begin[3] = total
    int col_off[3];
    int lda_bytes;
    uint32_t a_bytes;   // size of each activation matrix in bytes (range check)
    int M, K, ksteps, chunks, splits, epilogue;
    int tiles, zblocks;  // n-tiles, row blocks
    void *out;
    f16_t *out_lo;       // SwiGLU epilogue, optional: second half term of the result, half(y - half(y)), same layout as out
    int64_t ldc;
    size_t split_stride;
    // plain fp32 epilogue of a single matrix, optional (the LM head): per output row and per pass of 128 columns the largest
    // value and its (lowest) column, NaN if the pass holds one -- cand_val / cand_idx [M][cand_tiles]; no_store: out is not written
    float *cand_val;
    int32_t *cand_idx;
    int cand_tiles;
    int no_store;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t pk_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// registers a lane needs, roughly: accumulators + weight ring + two sets of activation fragments + addressing
constexpr int pk_regs(int NB, int MT, int RC) { return NB * MT * 16 + RC * NB * 16 + MT * 8 + 40; }
constexpr int pk_wgs_per_cu(int NB, int MT, int RC) { return pk_regs(NB, MT, RC) <= 128 ? 4 : (pk_regs(NB, MT, RC) <= 168 ? 3 : 2); }

// SW: the weights are loaded non-temporally (one row block: every weight byte is used once).  A template parameter,
// because the cache policy is an immediate of the load instruction and a branch per load would cut the loop into pieces.
// CAND: the plain-store epilogue also leaves the candidates of a greedy choice (PackedParams::cand_val); a template
// parameter so that the projections that never ask for them keep their code and registers.
template <int NB, int TERMS, int MT, int RC, bool SW, bool CAND = false>
__global__ __launch_bounds__(PK_THREADS, pk_wgs_per_cu(NB, MT, RC)) void gemm_packed_kernel(PackedParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int BM = 32 * MT;               // activation rows per workgroup
    constexpr int NBUF = TERMS == 1 ? 3 : 2;  // activation buffers: the copy of chunk c + NBUF - 1 runs during chunk c
    constexpr int NBF = 4 * NB;               // weight fragments per chunk and wavefront
    constexpr int HS = 4 * TERMS;             // (k-step, term) pairs per chunk
    constexpr int XTILE = BM * PK_BK * 2;     // bytes of one activation tile in LDS
    constexpr int XBUF = TERMS * XTILE;       // bytes of one activation buffer
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int K = p.K;

    // ---- workgroup id -> (n-tile, K split, row block).  Workgroups whose ids are congruent mod 8 share an
    //      XCD and its L2: the row blocks of one (tile, split) -- which stream the same weights -- get ids
    //      8 apart, so the weights come from HBM once and from that L2 for the other row blocks.
    const int ts_total = p.tiles * p.splits;
    const int id = blockIdx.x;
    const int ts = (id / (8 * p.zblocks)) * 8 + (id & 7);
    const int zb = (id % (8 * p.zblocks)) >> 3;
    if (ts >= ts_total) return;  // padding of the id space (whole workgroup, before any barrier)
    const int tile = ts % p.tiles, split = ts / p.tiles;
    const int m0 = zb * BM;
    const int Mloc = p.M - m0 < BM ? p.M - m0 : BM;

    // ---- which 32-row blocks does this wavefront own?  Slot j of wavefront w:
    //      fp32 epilogues: block 4 NB tile + 4 j + w of its matrix (pass j of the epilogue covers 128 adjacent columns);
    //      SwiGLU:         j = 0 gate block, j = 1 up block, both number 4 tile + w.
    int seg = tile >= p.tile_begin[2] ? 2 : (tile >= p.tile_begin[1] ? 1 : 0);
    const bool swiglu = p.epilogue == EPI_SWIGLU;
    if (swiglu) seg = 0;
    const int ltile = tile - p.tile_begin[seg];
    const int rows = seg == 0 ? p.rows[0] : (seg == 1 ? p.rows[1] : p.rows[2]);
    const int nblocks = (rows + 31) >> 5;
    __amdgpu_buffer_rsrc_t wr[NB];
    uint32_t w_off[NB];
    bool w_ok[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        int nb = swiglu ? ltile * 4 + w : (ltile * NB + j) * 4 + w;
        const f16_t *P = swiglu ? (j == 0 ? p.P[0] : p.P[1]) : (seg == 0 ? p.P[0] : (seg == 1 ? p.P[1] : p.P[2]));
        wr[j] = pk_rsrc(P, (uint32_t)((size_t)nblocks * p.ksteps * 1024));
        w_ok[j] = nb < nblocks;
        w_off[j] = ((uint32_t)nb * (uint32_t)p.ksteps * 64u + (uint32_t)lane) * 16u;
    }

    // ---- K range of this split
    const int c0 = (int)(((int64_t)split * p.chunks) / p.splits);
    const int c1 = (int)(((int64_t)(split + 1) * p.chunks) / p.splits);
    const int ks_end = c1 * 4 < p.ksteps ? c1 * 4 : p.ksteps;

    // ---- activation copy global -> LDS.  Instruction i of wavefront w fills the 1 KB block of rows
    //      8 (MT w + i) .. + 7 of a tile: lane l lands at byte 16 l of the block, i.e. row l / 8, slot l % 8.
    //      Piece g (16 bytes) of row r is kept in slot g ^ ((r >> 1) & 7): the LDS has 64 banks (256 bytes per
    //      clock), a 16-byte-per-lane read is served 16 lanes at a time, and a fragment read has 16 consecutive
    //      rows of one piece in those lanes -- two rows per 256 bytes, so the slot must change every second row.
    __amdgpu_buffer_rsrc_t ar[TERMS];
    ar[0] = pk_rsrc(p.A, p.a_bytes);
    if (TERMS == 2) ar[TERMS - 1] = pk_rsrc(p.A_lo, p.a_bytes);
    uint32_t x_off[MT];
    int x_piece[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        int row = (w * MT + i) * 8 + (lane >> 3);
        x_piece[i] = (lane & 7) ^ ((row >> 1) & 7);
        x_off[i] = row < Mloc ? (uint32_t)(m0 + row) * (uint32_t)p.lda_bytes + (uint32_t)x_piece[i] * 16u : PK_OOB;
    }
    auto copy_x = [&](int c, int buf) {
        uint32_t cb = (uint32_t)c * (PK_BK * 2);
#pragma unroll
        for (int tm = 0; tm < TERMS; ++tm)
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                unsigned char *dst = smem + buf * XBUF + tm * XTILE + (w * MT + i) * 1024;
                bool ok = c < c1 && (c * PK_BK + x_piece[i] * 8 < K);
                uint32_t off = ok && x_off[i] != PK_OOB ? x_off[i] + cb : PK_OOB;
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass does not know this builtin
                __builtin_amdgcn_raw_ptr_buffer_load_lds(ar[tm], LDS_PTR(dst), 16, (int)off, 0, 0, 0);
#else
                (void)dst; (void)off;
#endif
            }
    };
    // fragment of k-step s, tile mt: row 32 mt + (lane & 31), pieces 2 s + (lane >> 5)
    int xld[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) xld[s] = (lane & 31) * 128 + (((2 * s + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);

    u32x4_t ring[RC * NBF];  // weight fragments in flight: slots (i % RC) * NBF + s * NB + j belong to chunk c0 + i
    auto load_w = [&](int c, int s, int j, int slot) {
        int ks = c * 4 + s;
        uint32_t off = (ks < ks_end && w_ok[j]) ? w_off[j] + (uint32_t)ks * 1024u : PK_OOB;
        // With one row block every weight byte is used once: a streaming (non-temporal) load, which this part's memory
        // system moves faster than a cached one (7.05 against 6.2 TB/s on plain streaming).  With more row blocks the
        // other blocks of the tile are meant to find the fragment in L2.
        ring[slot] = __builtin_amdgcn_raw_buffer_load_b128(wr[j], (int)off, 0, SW ? 3 : 0);
    };

    f32x16_t acc[NB][MT];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

    // One chunk (PAR = parity of its index relative to c0): all activation copies of a trip are issued
    // before its weight loads -- the hardware retires loads in issue order, so waiting for the (short, L2)
    // activation copy never waits for younger weight loads.
    auto body = [&](int c, int buf, auto par_tag) {
        constexpr int PAR = decltype(par_tag)::value;
        // The copy of chunk c was issued NBUF - 1 trips ago.  Loads retire in issue order, so it has landed once at
        // most the loads issued after it are still outstanding: the weight loads of that trip and everything of
        // the trips in between.  The barrier orders only what each wavefront has waited for itself, and the
        // compiler does not wait for another wavefront's benefit: the wait is spelled out.
        constexpr int YOUNGER = NBF + (NBUF - 2) * (TERMS * MT + NBF);
        static_assert(YOUNGER < 64, "vmcnt is a 6-bit counter");
        __builtin_amdgcn_s_waitcnt((YOUNGER & 15) | (7 << 4) | (15 << 8) | ((YOUNGER >> 4) << 14));  // vmcnt(YOUNGER) only
        // (the bare barrier instruction: before the language's workgroup barrier the compiler waits for every copy into LDS
        //  still in flight, i.e. also for the younger ones and for the weight loads issued before them, which would cut
        //  the distance the loads run ahead to one trip)
        __builtin_amdgcn_s_barrier();  // the tile of chunk c has landed for every wavefront; buffer of chunk c-1 is free
        int nbuf = buf + NBUF - 1;
        if (nbuf >= NBUF) nbuf -= NBUF;
        copy_x(c + NBUF - 1, nbuf);
        __builtin_amdgcn_sched_barrier(0);  // the copies stay ahead of this trip's weight loads in issue order
        const unsigned char *xb = smem + buf * XBUF;
        f16x8_t a[2][MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[0][mt] = *reinterpret_cast<const f16x8_t *>(xb + xld[0] + mt * 4096);
#pragma unroll
        for (int hs = 0; hs < HS; ++hs) {
            const int s = hs / TERMS, tm = hs % TERMS;
            if (hs + 1 < HS) {
                const int s2 = (hs + 1) / TERMS, tm2 = (hs + 1) % TERMS;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    a[(hs + 1) & 1][mt] = *reinterpret_cast<const f16x8_t *>(xb + tm2 * XTILE + xld[s2] + mt * 4096);
            }
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[j][mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[hs & 1][mt], __builtin_bit_cast(f16x8_t, ring[PAR * NBF + s * NB + j]),
                                                                      acc[j][mt], 0, 0, 0);
            if (tm == TERMS - 1) {
#pragma unroll
                for (int j = 0; j < NB; ++j) load_w(c + RC, s, j, PAR * NBF + s * NB + j);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (c0 < c1) {
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) copy_x(c0 + i, i);
#pragma unroll
        for (int i = 0; i < RC; ++i)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int j = 0; j < NB; ++j) load_w(c0 + i, s, j, i * NBF + s * NB + j);
        __builtin_amdgcn_sched_barrier(0);
        int buf = 0;
        for (int c = c0; c < c1; c += RC) {  // trips past the end multiply zero tiles
            body(c, buf, std::integral_constant<int, 0>{});
            buf = buf + 1 == NBUF ? 0 : buf + 1;
            body(c + 1, buf, std::integral_constant<int, 1>{});
            buf = buf + 1 == NBUF ? 0 : buf + 1;
            if constexpr (RC == 4) {
                body(c + 2, buf, std::integral_constant<int, 2>{});
                buf = buf + 1 == NBUF ? 0 : buf + 1;
                body(c + 3, buf, std::integral_constant<int, 3>{});
                buf = buf + 1 == NBUF ? 0 : buf + 1;
            }
        }
    }
    // The copies issued for chunks past the end write zeros into the buffers: they must have landed before
    // the epilogue reuses that memory.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // every wavefront is done reading the activation buffers

    // ---- epilogues.  Lane holds column (lane & 31) of its block; register e of tile mt is row
    //      32 mt + 8 (e / 4) + 4 (lane >> 5) + (e % 4).
    if (!swiglu) {
        float *ct = reinterpret_cast<float *>(smem);  // [BM][PK_CT_STRIDE]
        float *out = reinterpret_cast<float *>(p.out) + (size_t)split * p.split_stride;
        const bool accumulate = p.epilogue == EPI_F32_ACC;
        const int c4 = (t & 31) * 4, rr = t >> 5;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if (j > 0) __syncthreads();
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    int m = mt * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                    ct[m * PK_CT_STRIDE + w * 32 + (lane & 31)] = acc[j][mt][e];
                }
            __syncthreads();
            const int n_first = (ltile * NB + j) * 128;  // first weight row of this pass inside its matrix
            const int ncols = rows - n_first;             // valid columns (may exceed 128, may be <= 0)
            if constexpr (CAND) {
                // The greedy choice starts here: thread (row m, half hs) scans 64 of the row's 128 values of this pass in
                // ascending columns, the two halves meet by one shuffle; the best value (lowest column on ties; NaN if the
                // pass holds one) goes to the candidate list that argmax_merge finishes.
                const int m = t >> 1, hs = t & 1;
                float bv = -INFINITY;
                int bi = 0x7fffffff;
                int nan = 0;
                if (m < BM) {
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const int c = hs * 64 + 4 * k;
                        const f32x4_t v = *reinterpret_cast<const f32x4_t *>(ct + m * PK_CT_STRIDE + c);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (c + e < ncols) {
                                nan |= (v[e] != v[e]);
                                if (v[e] > bv) { bv = v[e]; bi = n_first + c + e; }
                            }
                    }
                }
                const float ov = __shfl_xor(bv, 1, 64);
                const int oi = __shfl_xor(bi, 1, 64);
                nan |= __shfl_xor(nan, 1, 64);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
                if (hs == 0 && m < Mloc) {
                    const size_t at = (size_t)(m0 + m) * p.cand_tiles + (ltile * NB + j);
                    p.cand_val[at] = nan ? __builtin_nanf("") : bv;
                    p.cand_idx[at] = bi;
                }
            }
            // 32 lanes x float4 = one 512-byte output row; 8 rows per pass
#pragma unroll
            for (int i = 0; i < BM / 8; ++i) {
                int m = rr + 8 * i;
                if (m < Mloc && c4 < ncols && !(CAND && p.no_store)) {
                    f32x4_t v = *reinterpret_cast<const f32x4_t *>(ct + m * PK_CT_STRIDE + c4);
                    float *dst = out + (size_t)(m0 + m) * p.ldc + p.col_off[seg] + n_first + c4;
                    if (c4 + 4 <= ncols && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
                        if (accumulate) v += *reinterpret_cast<const f32x4_t *>(dst);
                        *reinterpret_cast<f32x4_t *>(dst) = v;
                    } else {
                        for (int e = 0; e < 4 && c4 + e < ncols; ++e) dst[e] = accumulate ? dst[e] + v[e] : v[e];
                    }
                }
            }
        }
    } else if (NB == 2) {
        f16_t *ht = reinterpret_cast<f16_t *>(smem);  // [BM][PK_HT_STRIDE], and a second tile for the low term
        const bool two_out = p.out_lo != nullptr;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int m = mt * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                float g = acc[0][mt][e], u = acc[NB - 1][mt][e];
                const float y = g / (1.0f + expf(-g)) * u;
                const f16_t hi = f32_to_f16(y);
                ht[m * PK_HT_STRIDE + w * 32 + (lane & 31)] = hi;
                if (two_out) ht[(BM + m) * PK_HT_STRIDE + w * 32 + (lane & 31)] = f32_to_f16(y - f16_to_f32(hi));
            }
        __syncthreads();
        const int c8 = (t & 15) * 8, rr = t >> 4;  // 16 lanes x 16 B = one 256-byte output row; 16 rows per pass
        const int ncols = rows - ltile * 128;
        for (int tm = 0; tm < (two_out ? 2 : 1); ++tm) {
            f16_t *out = tm == 0 ? reinterpret_cast<f16_t *>(p.out) : p.out_lo;
#pragma unroll
            for (int i = 0; i < BM / 16; ++i) {
                int m = rr + 16 * i;
                if (m < Mloc && c8 < ncols) {
                    f16_t *dst = out + (size_t)(m0 + m) * p.ldc + ltile * 128 + c8;
                    const f16_t *srcp = ht + (tm * BM + m) * PK_HT_STRIDE + c8;
                    if (c8 + 8 <= ncols && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0)) {
                        *reinterpret_cast<u32x4_t *>(dst) = *reinterpret_cast<const u32x4_t *>(srcp);
                    } else {
                        for (int e = 0; e < 8 && c8 + e < ncols; ++e) dst[e] = srcp[e];
                    }
                }
            }
        }
    }
}

template <int NB, int TERMS, int MT, int RC, bool SW>
static void launch_p2(PackedParams &p, hipStream_t st) {
    constexpr int NBUF = TERMS == 1 ? 3 : 2;
    constexpr int BM = 32 * MT;
    size_t lds = (size_t)NBUF * TERMS * BM * PK_BK * 2;
    size_t epi = (size_t)BM * PK_CT_STRIDE * sizeof(float);
    if (epi > lds) lds = epi;
    if (p.out_lo && (size_t)2 * BM * PK_HT_STRIDE * sizeof(f16_t) > lds) lds = (size_t)2 * BM * PK_HT_STRIDE * sizeof(f16_t);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_packed_kernel<NB, TERMS, MT, RC, SW>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        attr_set = true;
    }
    p.zblocks = ceil_div(p.M, BM);
    int ids = ceil_div(p.tiles * p.splits, 8) * 8 * p.zblocks;
    if constexpr (NB == 1 && RC == 2) {
        if (p.cand_val) {  // the LM head with a fused greedy choice
            static bool cand_attr_set = false;
            if (!cand_attr_set) {
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_packed_kernel<NB, TERMS, MT, RC, SW, true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
                cand_attr_set = true;
            }
            gemm_packed_kernel<NB, TERMS, MT, RC, SW, true><<<ids, PK_THREADS, lds, st>>>(p);
            return;
        }
    }
    gemm_packed_kernel<NB, TERMS, MT, RC, SW><<<ids, PK_THREADS, lds, st>>>(p);
}

template <int NB, int TERMS, int MT, int RC>
static void launch_p(PackedParams &p, hipStream_t st) {
    if (p.M <= 32 * MT) launch_p2<NB, TERMS, MT, RC, true>(p, st);   // one row block
    else launch_p2<NB, TERMS, MT, RC, false>(p, st);                 // the other row blocks of a tile read the weights from L2
}

// Weight chunks in flight per wavefront: 2, or 4 on request where the registers allow it (trips are rounded up
// to the ring depth).
template <int NB, int TERMS>
static void launch_pm(PackedParams &p, int mt, int depth, hipStream_t st) {
    const bool deep = depth == 4;  // no gain measured so far: not chosen by default
    if (mt == 1) {
        if (deep) launch_p<NB, TERMS, 1, 4>(p, st);
        else launch_p<NB, TERMS, 1, 2>(p, st);
    } else if (mt == 2) {
        if (deep) launch_p<NB, TERMS, 2, 4>(p, st);
        else launch_p<NB, TERMS, 2, 2>(p, st);
    } else {
        if (deep && NB == 1) launch_p<NB, TERMS, 4, (NB == 1 ? 4 : 2)>(p, st);
        else launch_p<NB, TERMS, 4, 2>(p, st);
    }
}

// ---------------------------------------------------------------------------------------------------
// Fused gate/up projection for few rows, K halves on separate wavefronts
// ---------------------------------------------------------------------------------------------------
// out[M, F] = silu(A Wg^T) * (A Wu^T) for M <= 128 rows per workgroup, from the fragment-order copies.  The row-major
// kernel of the same projection (gemm_skinny.hip) spends its time in LDS: every weight passes through a wavefront-private
// LDS strip and every activation fragment is read by four wavefronts -- 224 KB of LDS traffic per 128-wide K chunk and
// workgroup.  Here a workgroup of four wavefronts owns 64 gate + 64 up columns as (column half cw) x (K half kg):
// wavefront (cw, kg) holds the gate block and the up block of columns 32 cw .. 32 cw + 31, takes their fragments straight
// from memory and multiplies the half kg (64 elements) of every 128-wide K chunk; the activation chunk is copied
// global -> LDS by the load unit and each half is read by two wavefronts: 96 KB per chunk.  At the end the kg = 1
// wavefronts hand their sums to kg = 0 through LDS, which applies the SwiGLU.  The order of every sum -- the K half of
// each chunk in ascending chunks, then half 0 + half 1 -- is that of the row-major kernel, and so are the results, bit for
// bit.  One workgroup per compute unit (the register ring holds RC chunks of weight fragments: 8 KB each).
#define PS_BK 128
template <int RC, bool SW>
__global__ __launch_bounds__(PK_THREADS, 1) void gemm_packed_swiglu_halves_kernel(PackedParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int MT = 4, BM = 128, NBUF = 3;
    constexpr int XTILE = BM * 64 * 2;   // one 64-wide half of an activation chunk
    constexpr int XBUF = 2 * XTILE;
    const int t = threadIdx.x, lane = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int cw = w & 1, kg = w >> 1;
    const int K = p.K;

    // workgroup id -> (column tile, row block): ids congruent mod 8 share an XCD, the row blocks of a tile get ids 8 apart
    const int id = blockIdx.x;
    const int tile = (id / (8 * p.zblocks)) * 8 + (id & 7);
    const int zb = (id % (8 * p.zblocks)) >> 3;
    if (tile >= p.tiles) return;  // padding of the id space (whole workgroup, before any barrier)
    const int m0 = zb * BM;
    const int Mloc = p.M - m0 < BM ? p.M - m0 : BM;
    const int rows = p.rows[0];
    const int nblocks = (rows + 31) >> 5;
    const int nb = tile * 2 + cw;  // 32-row block of gate and of up
    __amdgpu_buffer_rsrc_t wr[2];
    wr[0] = pk_rsrc(p.P[0], (uint32_t)((size_t)nblocks * p.ksteps * 1024));
    wr[1] = pk_rsrc(p.P[1], (uint32_t)((size_t)nblocks * p.ksteps * 1024));
    const bool w_ok = nb < nblocks;
    const uint32_t w_off = ((uint32_t)nb * (uint32_t)p.ksteps * 64u + (uint32_t)lane) * 16u;
    const int trips = (K + PS_BK - 1) / PS_BK;

    // activation copy: instruction i of wavefront w fills rows 8 (4 w + i) .. + 7 of one half; piece g of row r sits in
    // slot g ^ ((r >> 1) & 7), as in gemm_packed_kernel
    __amdgpu_buffer_rsrc_t ar = pk_rsrc(p.A, p.a_bytes);
    uint32_t x_off[MT];
    int x_piece[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        int row = (w * MT + i) * 8 + (lane >> 3);
        x_piece[i] = (lane & 7) ^ ((row >> 1) & 7);
        x_off[i] = row < Mloc ? (uint32_t)(m0 + row) * (uint32_t)p.lda_bytes + (uint32_t)x_piece[i] * 16u : PK_OOB;
    }
    auto copy_x = [&](int c, int buf) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                unsigned char *dst = smem + buf * XBUF + hf * XTILE + (w * MT + i) * 1024;
                bool ok = c < trips && (c * PS_BK + hf * 64 + x_piece[i] * 8 < K);
                uint32_t off = ok && x_off[i] != PK_OOB ? x_off[i] + (uint32_t)c * (PS_BK * 2) + (uint32_t)hf * 128u : PK_OOB;
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass does not know this builtin
                __builtin_amdgcn_raw_ptr_buffer_load_lds(ar, LDS_PTR(dst), 16, (int)off, 0, 0, 0);
#else
                (void)dst; (void)off;
#endif
            }
    };
    int xld[4];
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) xld[s2] = (lane & 31) * 128 + (((2 * s2 + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4);

    u32x4_t ring[RC * 8];  // slots (c % RC) * 8 + 2 s + j: k-step s of this wavefront's half of chunk c, j = 0 gate, 1 up
    auto load_w = [&](int c, int s2, int j, int slot) {
        int ks = c * 8 + kg * 4 + s2;
        uint32_t off = (ks < p.ksteps && w_ok) ? w_off + (uint32_t)ks * 1024u : PK_OOB;
        ring[slot] = __builtin_amdgcn_raw_buffer_load_b128(wr[j], (int)off, 0, SW ? 3 : 0);
    };

    f32x16_t acc[2][MT];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][i][e] = 0.f;

    auto body = [&](int c, int buf, auto slot_tag) {
        constexpr int SLOT = decltype(slot_tag)::value;
        // the copy of chunk c was issued two trips ago, before that trip's 8 weight loads and the 16 loads of the last trip
        constexpr int YOUNGER = 8 + 16;
        __builtin_amdgcn_s_waitcnt((YOUNGER & 15) | (7 << 4) | (15 << 8) | ((YOUNGER >> 4) << 14));  // vmcnt(YOUNGER) only
        __builtin_amdgcn_s_barrier();  // chunk c has landed for every wavefront; the buffer of chunk c - 1 is free
        int nbuf = buf + NBUF - 1;
        if (nbuf >= NBUF) nbuf -= NBUF;
        copy_x(c + NBUF - 1, nbuf);
        __builtin_amdgcn_sched_barrier(0);  // the copies stay ahead of this trip's weight loads in issue order
        const unsigned char *xb = smem + buf * XBUF + kg * XTILE;
        f16x8_t a[2][MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[0][mt] = *reinterpret_cast<const f16x8_t *>(xb + xld[0] + mt * 4096);
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) {
            if (s2 + 1 < 4) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) a[(s2 + 1) & 1][mt] = *reinterpret_cast<const f16x8_t *>(xb + xld[s2 + 1] + mt * 4096);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[j][mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[s2 & 1][mt], __builtin_bit_cast(f16x8_t, ring[SLOT * 8 + 2 * s2 + j]),
                                                                      acc[j][mt], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 2; ++j) load_w(c + RC, s2, j, SLOT * 8 + 2 * s2 + j);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (trips > 0) {
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) copy_x(i, i);
#pragma unroll
        for (int i = 0; i < RC; ++i)
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
                for (int j = 0; j < 2; ++j) load_w(i, s2, j, i * 8 + 2 * s2 + j);
        __builtin_amdgcn_sched_barrier(0);
        int buf = 0;
        for (int c = 0; c < trips; c += RC) {  // trips past the end multiply zero tiles
            body(c, buf, std::integral_constant<int, 0>{});
            buf = buf + 1 == NBUF ? 0 : buf + 1;
            body(c + 1, buf, std::integral_constant<int, 1 % RC>{});
            buf = buf + 1 == NBUF ? 0 : buf + 1;
            if constexpr (RC == 4) {
                body(c + 2, buf, std::integral_constant<int, 2 % RC>{});
                buf = buf + 1 == NBUF ? 0 : buf + 1;
                body(c + 3, buf, std::integral_constant<int, 3 % RC>{});
                buf = buf + 1 == NBUF ? 0 : buf + 1;
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);  // copies issued for chunks past the end (zeros) must have landed before the memory is reused
    __syncthreads();

    // ---- half 0 + half 1: kg = 1 hands its sums to kg = 0 (same operand order as the row-major kernel)
    float *ex = reinterpret_cast<float *>(smem);  // [2 column halves][2 MT 16][64 lanes]
    if (kg == 1) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int e = 0; e < 16; ++e) ex[((cw * 2 + j) * MT * 16 + mt * 16 + e) * 64 + lane] = acc[j][mt][e];
    }
    __syncthreads();
    f16_t *ht = reinterpret_cast<f16_t *>(smem + 2 * 2 * MT * 16 * 64 * 4);  // 2 x [BM][72] halves (both terms), after the exchange area
    const bool two_out = p.out_lo != nullptr;
    if (kg == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float g = acc[0][mt][e], u = acc[1][mt][e];
                g += ex[((cw * 2 + 0) * MT * 16 + mt * 16 + e) * 64 + lane];
                u += ex[((cw * 2 + 1) * MT * 16 + mt * 16 + e) * 64 + lane];
                int m = mt * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const float y = g / (1.0f + expf(-g)) * u;
                const f16_t hi = f32_to_f16(y);
                ht[m * 72 + cw * 32 + (lane & 31)] = hi;
                if (two_out) ht[(BM + m) * 72 + cw * 32 + (lane & 31)] = f32_to_f16(y - f16_to_f32(hi));
            }
    }
    __syncthreads();
    const int c8 = (t & 7) * 8, rr = t >> 3;  // 8 lanes x 16 B = one 128-byte output row; 32 rows per pass
    const int ncols = rows - tile * 64;
    f16_t *const outs[2] = {reinterpret_cast<f16_t *>(p.out), p.out_lo};
#pragma unroll
    for (int i = 0; i < BM / 32; ++i) {
        int m = rr + 32 * i;
        if (m < Mloc && c8 < ncols) {
            const size_t at = (size_t)(m0 + m) * p.ldc + tile * 64 + c8;
            const bool vec = c8 + 8 <= ncols && ((at * sizeof(f16_t)) & 15) == 0 && ((reinterpret_cast<uintptr_t>(outs[0]) | reinterpret_cast<uintptr_t>(outs[1])) & 15) == 0;
            // both terms of a row piece leave together: their LDS reads first, then the two stores
            const f16_t *src0 = ht + m * 72 + c8, *src1 = ht + (BM + m) * 72 + c8;
            if (vec) {
                const u32x4_t v0 = *reinterpret_cast<const u32x4_t *>(src0);
                u32x4_t v1 = v0;
                if (two_out) v1 = *reinterpret_cast<const u32x4_t *>(src1);
                *reinterpret_cast<u32x4_t *>(outs[0] + at) = v0;
                if (two_out) *reinterpret_cast<u32x4_t *>(outs[1] + at) = v1;
            } else {
                for (int e = 0; e < 8 && c8 + e < ncols; ++e) {
                    outs[0][at + e] = src0[e];
                    if (two_out) outs[1][at + e] = src1[e];
                }
            }
        }
    }
}

template <int RC, bool SW>
static void launch_halves(PackedParams &p, hipStream_t st) {
    size_t lds = (size_t)3 * 2 * 128 * 64 * 2;  // three chunk buffers; the epilogue's exchange area and first tile fit inside
    const size_t epi = (size_t)2 * 2 * 4 * 16 * 64 * 4 + (size_t)2 * 128 * 72 * 2;  // exchange area + both output tiles
    if (epi > lds) lds = epi;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_packed_swiglu_halves_kernel<RC, SW>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        attr_set = true;
    }
    int ids = ceil_div(p.tiles, 8) * 8 * p.zblocks;
    gemm_packed_swiglu_halves_kernel<RC, SW><<<ids, PK_THREADS, lds, st>>>(p);
}

bool gemm_packed_swiglu_halves_supported(int F, int K) {
    return F > 0 && K > 0 && (size_t)ceil_div(F, 32) * ceil_div(K, 16) * 1024 < PK_MAX_BYTES;
}

void launch_gemm_packed_swiglu_halves(const PackedGemmArgs &a, hipStream_t st) {
    if (a.M <= 0) return;
    PackedParams p = {};
    p.A = a.A;
    p.A_lo = nullptr;
    p.lda_bytes = (int)(a.lda * 2);
    p.a_bytes = (uint32_t)((((size_t)a.M - 1) * a.lda + a.K) * 2);
    p.M = a.M;
    p.K = a.K;
    p.ksteps = ceil_div(a.K, 16);
    p.chunks = ceil_div(a.K, PK_BK);
    p.epilogue = EPI_SWIGLU;
    p.splits = 1;
    p.out = a.out;
    p.out_lo = a.out_lo;
    p.ldc = a.ldc;
    p.P[0] = a.P[0]; p.P[1] = a.P[1]; p.P[2] = a.P[0];
    p.rows[0] = a.rows[0]; p.rows[1] = a.rows[0]; p.rows[2] = 0;
    p.tiles = ceil_div(a.rows[0], 64);
    p.zblocks = ceil_div(a.M, 128);
    if (p.tiles <= 0) return;
    const bool deep = a.depth != 2;
    if (p.zblocks == 1) { if (deep) launch_halves<4, true>(p, st); else launch_halves<2, true>(p, st); }
    else { if (deep) launch_halves<4, false>(p, st); else launch_halves<2, false>(p, st); }
}

// Decomposition of a projection with fp32 partial outputs.  Measured inside whole decode steps of the 7B shape,
// one 128-row workgroup per column tile and split-K up to about one workgroup per compute unit was as fast as
// any mix of 64-row workgroups, two column blocks per wavefront and deeper splits (all within 3 %).
void gemm_packed_plan(int N, int K, int M, int *nb, int *rows_per_wg, int *splits) {
    int chunks = ceil_div(K, PK_BK);
    *nb = 1;
    *rows_per_wg = M <= 32 ? 32 : (M <= 64 ? 64 : 128);
    int wgs = ceil_div(N, 128) * ceil_div(M, *rows_per_wg);
    if (wgs < 1) wgs = 1;  // empty input
    int s = 256 / wgs;
    if (s > chunks / 8) s = chunks / 8;  // at least 8 chunks per split
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    *splits = s;
}

// whether launch_gemm_packed serves a matrix in one launch (what the fused greedy choice needs)
bool gemm_packed_single_launch(int N, int K) {
    return (size_t)ceil_div(N, 32) * 32 * ((size_t)ceil_div(K, 16) * 32) < PK_MAX_BYTES;
}

void launch_gemm_packed(const PackedGemmArgs &a, hipStream_t st) {
    if (a.M <= 0) return;
    // 32-bit byte offsets inside the kernel: a packed matrix of PK_MAX_BYTES or more is walked in row slabs
    const size_t row_bytes = (size_t)ceil_div(a.K, 16) * 32;  // packed bytes per weight row
    bool big = false;
    for (int i = 0; i < 3; ++i)
        if (a.P[i] && (size_t)ceil_div(a.rows[i], 32) * 32 * row_bytes >= PK_MAX_BYTES) big = true;
    if (big) {
        const int rows_max = (int)((PK_MAX_BYTES / row_bytes) / 256 * 256);
        const size_t out_elem = a.epilogue == EPI_SWIGLU ? sizeof(f16_t) : sizeof(float);
        int col = 0;
        for (int i = 0; i < (a.epilogue == EPI_SWIGLU ? 1 : 3); ++i) {
            if (!a.P[i] || a.rows[i] <= 0) continue;
            for (int n = 0; n < a.rows[i]; n += rows_max) {
                PackedGemmArgs s = a;
                const size_t skip = (size_t)(n / 32) * ceil_div(a.K, 16) * 512;  // halves
                s.P[0] = a.P[i] + skip;
                s.rows[0] = a.rows[i] - n < rows_max ? a.rows[i] - n : rows_max;
                s.P[1] = s.P[2] = nullptr;
                s.rows[1] = s.rows[2] = 0;
                if (a.epilogue == EPI_SWIGLU) { s.P[1] = a.P[1] + skip; s.rows[1] = s.rows[0]; }
                s.out = static_cast<char *>(a.out) + (size_t)(col + n) * out_elem;
                if (a.out_lo) s.out_lo = a.out_lo + (col + n);
                launch_gemm_packed(s, st);
            }
            col += a.rows[i];
        }
        return;
    }
    PackedParams p;
    p.A = a.A;
    p.A_lo = a.A_lo;
    p.lda_bytes = (int)(a.lda * 2);
    p.a_bytes = (uint32_t)((((size_t)a.M - 1) * a.lda + a.K) * 2);
    p.M = a.M;
    p.K = a.K;
    p.ksteps = ceil_div(a.K, 16);
    p.chunks = ceil_div(a.K, PK_BK);
    p.epilogue = a.epilogue;
    p.splits = a.epilogue != EPI_F32 ? 1 : (a.splits < 1 ? 1 : a.splits);
    if (p.splits > p.chunks) p.splits = p.chunks;
    p.out = a.out;
    p.out_lo = a.epilogue == EPI_SWIGLU ? a.out_lo : nullptr;
    p.ldc = a.ldc;
    p.split_stride = a.split_stride;
    // candidates of a fused greedy choice: one matrix, the plain store epilogue, no K split (the caller has checked)
    const bool cand = a.cand_val && a.cand_idx && a.epilogue == EPI_F32 && p.splits == 1 && !a.P[1] && !a.P[2] && a.nb != 2 &&
                      a.depth != 4;
    p.cand_val = cand ? a.cand_val : nullptr;
    p.cand_idx = cand ? a.cand_idx : nullptr;
    p.cand_tiles = ceil_div(a.rows[0], 128);
    p.no_store = cand && a.no_store ? 1 : 0;
    const bool swiglu = a.epilogue == EPI_SWIGLU;
    const int nb = swiglu ? 2 : (a.nb == 2 ? 2 : 1);
    int tiles = 0, col = 0;
    for (int i = 0; i < 3; ++i) {
        p.P[i] = a.P[i] ? a.P[i] : a.P[0];
        p.rows[i] = a.P[i] ? a.rows[i] : 0;
        p.tile_begin[i] = tiles;
        p.col_off[i] = col;
        if (swiglu) continue;
        tiles += ceil_div(p.rows[i], 128 * nb);
        col += p.rows[i];
    }
    if (swiglu) tiles = ceil_div(a.rows[0], 128);
    p.tile_begin[3] = tiles;
    p.tiles = tiles;
    if (tiles <= 0) return;
    const bool two = a.A_lo != nullptr;
    int mt = a.rows_per_wg >= 128 ? 4 : (a.rows_per_wg >= 64 ? 2 : (a.rows_per_wg >= 32 ? 1 : 4));
    while (mt > 1 && 32 * (mt / 2) >= a.M) mt /= 2;  // no point in row tiles the batch does not fill
    if (nb == 2) {
        if (two) launch_pm<2, 2>(p, mt, a.depth, st);
        else launch_pm<2, 1>(p, mt, a.depth, st);
    } else {
        if (two) launch_pm<1, 2>(p, mt, a.depth, st);
        else launch_pm<1, 1>(p, mt, a.depth, st);
    }
}
