// Decode attention for grouped-query models (4 or 8 query heads per kv head, head_dim 128) on the matrix cores.
//
// With one query head per kv head, decode attention is a pure HBM stream and plain vector arithmetic keeps up
// (attention_decode.hip).  With 8 query heads sharing every cache row, the vector units become the limit: each
// 512 bytes of K and V cost 8 dot products and 8 weighted sums of 128 elements.  Here the group of heads is the
// small dimension of two real matrix products per tile of 16 cache rows,
//     S^T[16 keys x 16 columns] = K[16 x 128] * Q^T[128 x 16],     O^T[128 x 16 columns] += V^T[128 x 16 keys] * P^T[16 x 16],
// where the 16 columns are the high and the low half-precision term of up to 8 heads (columns c and c + 8 belong to head
// c): q and the probabilities enter the matrix cores as two-term sums, so the products carry fp32-grade operands and only
// K and V are half, as stored.  Computing S transposed leaves a lane with 4 keys of one column, which already is the
// register layout P^T needs as the second operand of the second product.
//
// Memory path: one wavefront per (sequence, kv head, group of 8 heads, sequence split).  K and V tiles travel from HBM
// straight into the wavefront's own LDS ring (buffer loads with the LDS destination, 1 KB per instruction, three tiles in
// flight) -- no registers, no barriers: a wavefront waits on its own load counter.  The 16-byte pieces of a row are
// stored XOR-permuted so that both read patterns are bank-conflict free: K rows as 16-byte operand fragments (piece ^ row),
// V transposed through 16-bit reads (piece ^ 4 * (row / 4)).  Rows past the end are cut off by the buffer descriptor
// (they arrive as zeros) and masked to weight 0.
//
// I16: the cache rows are block-scaled 16-bit fixed point (int16 elements times one fp32 scale per row, KvMap::kscale /
// vscale).  An int16 n is split exactly into two integer-valued halves, n = (n & ~31) + (n & 31): a multiple of 32 of
// magnitude <= 32768 and an integer in [0, 31] are both IEEE half values, so K and V enter the matrix cores without any
// rounding at the price of a second matrix instruction per operand.  The row scales travel with their tile (two more
// copy instructions into the stage) and are applied to the scores (K) and to the probabilities (V).
#include "kernels.h"

#define GA_TILE 16                 // cache rows per tile
#ifndef GA_STAGES
#define GA_STAGES 3                // LDS ring: two tiles in flight while one is consumed (24 KB: six wavefronts per compute unit)
#endif
#define GA_TILE_BYTES (GA_TILE * 256)  // one K (or V) tile of head_dim 128 in half
#define GA_STAGE_BYTES (2 * GA_TILE_BYTES)

#define GA_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

#define GA_SCALE_BYTES 512              // I16: K scales at +0, V scales at +256 behind the two tiles of a stage (16 floats each in use)

typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float ga_ror8(float v) {  // lane l of a row of 16 receives lane (l + 8) % 16
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, true));
}

template <bool PAGED, bool I16>
__global__ __launch_bounds__(64) void decode_attention_gqa_kernel(const float *__restrict__ q, const f16_t *__restrict__ kc,
                                                                  const f16_t *__restrict__ vc,
                                                                  const int32_t *__restrict__ d_len, f16_t *__restrict__ out,
                                                                  f16_t *__restrict__ out_lo,
                                                                  float *__restrict__ ws, int Hq, int Hkv, int S, int nsplit,
                                                                  int len_stride, KvMap map,
                                                                  const int32_t *__restrict__ d_done) {
    constexpr int HD = 128;
    constexpr int STAGE = GA_STAGE_BYTES + (I16 ? GA_SCALE_BYTES : 0);
    __shared__ __attribute__((aligned(1024))) unsigned char ring[GA_STAGES * STAGE];
    const int lane = threadIdx.x;
    const int c = lane & 15, j = lane >> 4;  // column (head and term) / group of 4 keys
    const int g = Hq / Hkv;
    const int G8 = g < 8 ? g : 8;            // heads of this wavefront
    const int hgs = g / G8;
    int item = blockIdx.x;
    const int split = item % nsplit; item /= nsplit;
    const int hg = item % hgs; item /= hgs;
    const int kvh = item % Hkv;
    const int b = item / Hkv;
    const int head0 = kvh * g + hg * G8;
    if (d_done && d_done[b]) return;  // an ended sequence: its cache is not read any more (its output row keeps old values)

    const int pos = __builtin_amdgcn_readfirstlane(d_len[(size_t)b * len_stride]);
    int n = pos + 1;  // visible cache rows
    if (n > S) n = S;
    int chunk = (n + nsplit - 1) / nsplit;
    chunk = (chunk + GA_TILE - 1) / GA_TILE * GA_TILE;
    const int j0 = split * chunk;
    const int j1 = j0 + chunk < n ? j0 + chunk : n;
    const int ntiles = j1 > j0 ? (j1 - j0 + GA_TILE - 1) / GA_TILE : 0;

    // ---- Q^T operand: column c = head (c & 7), term (c >> 3); k-step s covers head_dim 32 s + 8 j + 0..7
    const int head = c & 7;
    const bool col_ok = head < G8;
    f16x8_t qf[4];
    {
        const float *qp = q + ((size_t)b * Hq + head0 + (col_ok ? head : 0)) * HD + 8 * j;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            f32x4_t a = *reinterpret_cast<const f32x4_t *>(qp + 32 * s);
            f32x4_t bb = *reinterpret_cast<const f32x4_t *>(qp + 32 * s + 4);
            float x[8] = {a.x, a.y, a.z, a.w, bb.x, bb.y, bb.z, bb.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = col_ok ? x[e] : 0.f;  // columns without a head contribute nothing
                const _Float16 hi = (_Float16)__builtin_amdgcn_fmed3f(v, -65504.f, 65504.f);  // saturating, like every half here
                const _Float16 lo = (_Float16)__builtin_amdgcn_fmed3f(v - (float)hi, -65504.f, 65504.f);
                qf[s][e] = c < 8 ? hi : lo;
            }
        }
    }

    // ---- every tile gets its own buffer descriptor (scalar registers): base = the tile's first row -- in a paged cache a
    //      tile never straddles pages, which hold a multiple of 16 rows and start at multiples of 16 -- and size = its
    //      visible rows, so rows at and beyond j1 are out of range.
    const bool stream_kv = hgs == 1;
    const int32_t *pages = PAGED ? map.table + (size_t)b * map.table_stride : nullptr;
    // copy instruction i (0..3) of a tile moves rows 4 i .. 4 i + 3; this lane fills slot (lane & 15) of row 4 i + j
    uint32_t ksrc[4], vsrc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 4 * i + j;
        ksrc[i] = (uint32_t)r * 256u + (uint32_t)((c ^ r) & 15) * 16u;
        vsrc[i] = (uint32_t)r * 256u + (uint32_t)((c ^ (4 * i)) & 15) * 16u;
    }
    auto issue_tile = [&](int tile, int stage) {
        const bool live = tile < ntiles;
        const int row0 = live ? j0 + tile * GA_TILE : 0;
        const int rows = live ? (j1 - row0 < GA_TILE ? j1 - row0 : GA_TILE) : 0;  // 0: every lane is out of range
        size_t first;  // row index of the tile's first row within the layer's K (or V) area
        if (PAGED) {
            const int page = __builtin_amdgcn_readfirstlane(pages[row0 >> map.page_shift]);
            first = (((size_t)page * Hkv + kvh) << map.page_shift) + (row0 & ((1 << map.page_shift) - 1));
        } else {
            first = ((size_t)b * Hkv + kvh) * S + row0;
        }
        __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<f16_t *>(kc + first * HD), 0, rows * (HD * 2), 0x00020000);
        __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc(const_cast<f16_t *>(vc + first * HD), 0, rows * (HD * 2), 0x00020000);
        if (I16) {  // the scales of the tile's rows: lane r < rows fetches scale r, every other lane is out of range (zero)
            __amdgpu_buffer_rsrc_t ksr = __builtin_amdgcn_make_buffer_rsrc(map.kscale + first, 0, rows * 4, 0x00020000);
            __amdgpu_buffer_rsrc_t vsr = __builtin_amdgcn_make_buffer_rsrc(map.vscale + first, 0, rows * 4, 0x00020000);
            unsigned char *sd = ring + stage * STAGE + GA_STAGE_BYTES;
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ksr, GA_LDS_PTR(sd), 4, lane * 4, 0, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(vsr, GA_LDS_PTR(sd + 256), 4, lane * 4, 0, 0, 0);
#else
            (void)sd; (void)ksr; (void)vsr;
#endif
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned char *kd = ring + stage * STAGE + i * 1024;
            unsigned char *vd = kd + GA_TILE_BYTES;
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass does not know this builtin
            if (stream_kv) {  // the only reader of these rows: non-temporal copies (they stream faster than cached ones)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, GA_LDS_PTR(kd), 16, (int)ksrc[i], 0, 0, 3);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, GA_LDS_PTR(vd), 16, (int)vsrc[i], 0, 0, 3);
            } else {          // 16 heads per kv head: the second wavefront of the kv head finds the rows in L2
                __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, GA_LDS_PTR(kd), 16, (int)ksrc[i], 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, GA_LDS_PTR(vd), 16, (int)vsrc[i], 0, 0, 0);
            }
#else
            (void)kd; (void)vd; (void)kr; (void)vr;
#endif
        }
    };

    // ---- LDS read addresses (relative to a stage)
    int kaddr[4];  // K operand of k-step s: row c of the tile, piece 4 s + j, stored at slot piece ^ row
#pragma unroll
    for (int s = 0; s < 4; ++s) kaddr[s] = c * 256 + (((4 * s + j) ^ c) << 4);
    int vaddr[8];  // V^T operand of head_dim tile t: element 16 t + c of rows 4 j + 0..3
#pragma unroll
    for (int t = 0; t < 8; ++t) vaddr[t] = GA_TILE_BYTES + 4 * j * 256 + (((2 * t + (c >> 3)) ^ (4 * j)) << 4) + (c & 7) * 2;

    f32x4_t oacc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) oacc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float mrun = -INFINITY, den = 0.f;
    const float scale = rsqrtf((float)HD);

#pragma unroll
    for (int k = 0; k < GA_STAGES - 1; ++k) issue_tile(k, k);
    __builtin_amdgcn_sched_barrier(0);

    auto consume = [&](int tile, const unsigned char *st) {
        // scores of 16 keys x 16 columns
        f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (I16) {
                const u32x4_t kw = *reinterpret_cast<const u32x4_t *>(st + kaddr[s]);
                const u32x4_t wh = {kw.x & 0xFFE0FFE0u, kw.y & 0xFFE0FFE0u, kw.z & 0xFFE0FFE0u, kw.w & 0xFFE0FFE0u};
                const u32x4_t wl = {kw.x & 0x001F001Fu, kw.y & 0x001F001Fu, kw.z & 0x001F001Fu, kw.w & 0x001F001Fu};
                const f16x8_t kh = __builtin_convertvector(__builtin_bit_cast(s16x8_t, wh), f16x8_t);
                const f16x8_t kl = __builtin_convertvector(__builtin_bit_cast(s16x8_t, wl), f16x8_t);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, qf[s], sacc, 0, 0, 0);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kl, qf[s], sacc, 0, 0, 0);
            } else {
                f16x8_t kf = *reinterpret_cast<const f16x8_t *>(st + kaddr[s]);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf, qf[s], sacc, 0, 0, 0);
            }
        }
        // I16: the scales of keys 4 j + 0..3 (K) and of the same rows of V
        f32x4_t ksc = {1.f, 1.f, 1.f, 1.f}, vsc = {1.f, 1.f, 1.f, 1.f};
        if (I16) {
            ksc = *reinterpret_cast<const f32x4_t *>(st + GA_STAGE_BYTES + 16 * j);
            vsc = *reinterpret_cast<const f32x4_t *>(st + GA_STAGE_BYTES + 256 + 16 * j);
        }
        // register i: key 4 j + i of the tile, column c.  High and low term of a head sit 8 columns apart.
        float sc[4];
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = sacc[i] + ga_ror8(sacc[i]);
            if (I16) v *= ksc[i];
            const int key = j0 + tile * GA_TILE + 4 * j + i;
            sc[i] = key < j1 ? v * scale : -INFINITY;
            tmax = fmaxf(tmax, sc[i]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float mnew = fmaxf(mrun, tmax);  // finite: every tile holds at least one visible key
        if (__any(mnew > mrun)) {  // once the running maxima have settled, most tiles change none of them
            const float alpha = mrun == -INFINITY ? 0.f : __expf(mrun - mnew);
            mrun = mnew;
            den *= alpha;
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) oacc[t][i] *= alpha;
        }
        f16x4_t pf;
        float wref = 1.f;  // I16: what the weights of this tile are measured in
        if (I16) {
            // The row scale of V rides on the probability: weight = p * scale.  A scale is of order 1e-5 .. 1e-4, below the
            // normal range of a half, so the tile's weights are normalised by their largest (per column) before they are
            // split into half terms, and the tile's product is accumulated times that factor.
            float w[4];
            float wmax = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = __expf(sc[i] - mnew);  // 0 for keys past the end
                den += p;
                w[i] = p * vsc[i];
                wmax = fmaxf(wmax, w[i]);
            }
            wmax = fmaxf(wmax, __shfl_xor(wmax, 16, 64));
            wmax = fmaxf(wmax, __shfl_xor(wmax, 32, 64));
            const float inv = wmax > 0.f ? 1.0f / wmax : 0.f;
            wref = wmax;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float x = w[i] * inv;  // in [0, 1]
                const _Float16 hi = (_Float16)x;
                pf[i] = c < 8 ? hi : (_Float16)(x - (float)hi);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = __expf(sc[i] - mnew);  // 0 for keys past the end
                den += p;
                const _Float16 hi = (_Float16)p;
                pf[i] = c < 8 ? hi : (_Float16)(p - (float)hi);
            }
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (I16) {
                s16x4_t nh, nl;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint16_t n = *reinterpret_cast<const uint16_t *>(st + vaddr[t] + i * 256);
                    nh[i] = (short)(n & 0xFFE0u);
                    nl[i] = (short)(n & 0x001Fu);
                }
                f32x4_t part = {0.f, 0.f, 0.f, 0.f};
                part = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_convertvector(nh, f16x4_t), pf, part, 0, 0, 0);
                part = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_convertvector(nl, f16x4_t), pf, part, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i) oacc[t][i] = fmaf(wref, part[i], oacc[t][i]);
            } else {
                f16x4_t vf;
#pragma unroll
                for (int i = 0; i < 4; ++i) vf[i] = __builtin_bit_cast(_Float16, *reinterpret_cast<const uint16_t *>(st + vaddr[t] + i * 256));
                oacc[t] = __builtin_amdgcn_mfma_f32_16x16x16f16(vf, pf, oacc[t], 0, 0, 0);
            }
        }
    };

    // tile t has landed once at most the GA_STAGES - 2 younger tiles (8 copy instructions each, 10 with scales) are pending
    constexpr int YOUNGER = (I16 ? 10 : 8) * (GA_STAGES - 2);
    static_assert(YOUNGER < 64, "vmcnt is a 6-bit counter");
    for (int tile0 = 0; tile0 < ntiles; tile0 += GA_STAGES) {
#pragma unroll
        for (int k = 0; k < GA_STAGES; ++k) {  // unrolled: the stage offsets become immediates of the LDS reads
            if (tile0 + k < ntiles) {
                __builtin_amdgcn_s_waitcnt((YOUNGER & 15) | (7 << 4) | (15 << 8) | ((YOUNGER >> 4) << 14));  // vmcnt(YOUNGER) only
                __builtin_amdgcn_sched_barrier(0);
                issue_tile(tile0 + k + GA_STAGES - 1, (k + GA_STAGES - 1) % GA_STAGES);  // into the stage consumed one step ago
                __builtin_amdgcn_sched_barrier(0);
                consume(tile0 + k, ring + k * STAGE);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt((0 & 15) | (7 << 4) | (15 << 8) | (0 << 14));  // no copy may outlive the wavefront's LDS

    // ---- totals: the lane groups j hold disjoint keys (den), the columns c and c + 8 the two terms of a head (oacc)
    den += __shfl_xor(den, 16, 64);
    den += __shfl_xor(den, 32, 64);
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) oacc[t][i] += ga_ror8(oacc[t][i]);
    if (c < G8) {  // lane (j, c): head c, head_dim elements 16 t + 4 j + 0..3
        const int hq = head0 + c;
        if (nsplit == 1) {
            const float inv = 1.0f / den;
            f16_t *op = out + ((size_t)b * Hq + hq) * HD + 4 * j;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                u32x2_t o2;
                o2.x = pack_f16x2(oacc[t][0] * inv, oacc[t][1] * inv);
                o2.y = pack_f16x2(oacc[t][2] * inv, oacc[t][3] * inv);
                *reinterpret_cast<u32x2_t *>(op + 16 * t) = o2;
                if (out_lo) {  // second half term of the output (two-term output projection)
                    u32x2_t l2;
                    l2.x = pack_f16x2_lo(oacc[t][0] * inv, oacc[t][1] * inv, o2.x);
                    l2.y = pack_f16x2_lo(oacc[t][2] * inv, oacc[t][3] * inv, o2.y);
                    *reinterpret_cast<u32x2_t *>(out_lo + ((size_t)b * Hq + hq) * HD + 4 * j + 16 * t) = l2;
                }
            }
        } else {
            float *p = ws + (((size_t)b * Hq + hq) * nsplit + split) * (HD + 2);
            if (j == 0) { p[0] = mrun; p[1] = den; }
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) p[2 + 16 * t + 4 * j + i] = oacc[t][i];
        }
    }
}

bool decode_attention_gqa_supported(int Hq, int Hkv, int hd) {
    if (hd != 128 || Hkv <= 0 || Hq % Hkv) return false;
    const int g = Hq / Hkv;
    return g == 4 || (g >= 8 && g % 8 == 0);
}

// Block-scaled rows are served when 8 heads share a cache row; with 4 the integer conversions outweigh what the matrix
// cores save and the vector kernel is faster (32/8 heads, 1536 cached rows, batch 128: 190-200 us here).
bool decode_attention_gqa_takes(int Hq, int Hkv, int hd, bool block_scaled) {
    return decode_attention_gqa_supported(Hq, Hkv, hd) && (!block_scaled || Hq / Hkv >= 8);
}

int decode_attention_gqa_default_splits(int B, int Hq, int Hkv, int S, bool block_scaled) {
    const int g = Hq / Hkv;
    long items = (long)B * Hkv * (g < 8 ? 1 : g / 8);
    // one wavefront per SIMD over 256 compute units, at least; block-scaled rows: three per two SIMDs (the conversions make a
    // tile's critical path longer, and six wavefronts per compute unit is what the LDS ring allows: batch 64, 64/8 heads, 1536
    // rows: 126 us with 2 splits, 101 with 3, 123 with 4)
    const long want = block_scaled ? 1536 : 1024;
    int s = (int)((want + items - 1) / items);
    int cap = S / 128;                          // but keep >= 128 positions per split at full length
    if (s > cap) s = cap;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    return s;
}

void launch_decode_attention_gqa(const float *q, const f16_t *kc, const f16_t *vc, const int32_t *d_len, int len_stride,
                                 f16_t *out, float *ws, int B, int Hq, int Hkv, int S, int nsplit, hipStream_t st, KvMap map,
                                 const int32_t *d_done, f16_t *out_lo) {
    if (B <= 0) return;
    const int g = Hq / Hkv;
    const int items = B * Hkv * (g < 8 ? 1 : g / 8) * nsplit;
#define GA_LAUNCH(PAGEDV, I16V) \
    decode_attention_gqa_kernel<PAGEDV, I16V><<<items, 64, 0, st>>>(q, kc, vc, d_len, out, out_lo, ws, Hq, Hkv, S, nsplit, len_stride, map, d_done)
    if (map.table && map.kscale) GA_LAUNCH(true, true);
    else if (map.table) GA_LAUNCH(true, false);
    else if (map.kscale) GA_LAUNCH(false, true);
    else GA_LAUNCH(false, false);
#undef GA_LAUNCH
    if (nsplit > 1) launch_decode_attention_merge(ws, out, B, Hq, 128, nsplit, st, out_lo);
}
