// Decode attention: one new query per (sequence, query head) against the KV cache.
//
// Every decode step re-reads the whole cache (the paper, Section 8.5 (strong scaling trend), calls this iterative KV-cache
// loading the irreducible overhead of generation), so this kernel is a pure HBM stream: each cache
// element is used once per query head that shares it.  Design for gfx950:
//   * one WAVEFRONT per (sequence, kv head, group of GT query heads, sequence split); no LDS and no
//     barriers on the streaming path;
//   * the cache slab of one (sequence, kv head) is contiguous [position][head_dim], so a wavefront
//     load instruction fetches 1 KB of consecutive bytes (64 lanes x 16 B = 4 rows of head_dim 128);
//   * a lane owns 8 consecutive head_dim elements; q.k is finished by a 16-lane DPP reduction;
//   * each of the 64/LPR lane groups runs its own online softmax (running max / sum / weighted V) over
//     the rows it sees; groups are merged once at the end by wavefront shuffles;
//   * grouped-query attention: the GT query heads that share a kv head are processed by the same
//     wavefront, so K and V are read once for all of them;
//   * paged cache (PAGED = true): the cache is a pool of pages of 2^k positions and a per-sequence page list says
//     where each run of positions lives; a page of one kv head is still a contiguous run of rows, and the page
//     numbers of the next iteration are fetched while the current rows are in flight;
//   * optional split over the sequence axis (more wavefronts for long contexts / small batches):
//     splits write (max, sum, unnormalised output) partials that a small merge kernel combines.
//   * fused form (FUSED = true): the wavefront takes the new token's q, k and v straight from the split-K
//     partials of the QKV projection -- it adds the partials, rotates q and k at the token's position, uses
//     the half-rounded k/v row in place of the cache row of that position, and one wavefront per
//     (sequence, kv head) stores that row into the cache.  No separate rotary/append kernel and no q buffer.
// All arithmetic is fp32; only the cache elements and the output are half.
#include "kernels.h"

#define DA_THREADS 256
#define DA_U 4  // cache rows-per-lane-group in flight per iteration (x2 for K and V)

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// sum over the LPR lanes that share a cache row; every lane of the group receives the total
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
    v += dpp_f<0xB1>(v);               // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);               // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);              // row_half_mirror: joins the two quads of 8 lanes
    if (LPR == 16) v += dpp_f<0x140>(v);  // row_mirror: joins the two halves of 16 lanes
    return v;
}

// what the fused form needs to build q and the new cache row itself
struct FusedQkv {
    const float *part;    // split-K partials of the QKV projection, each [B, (Hq + 2 Hkv) * HD] laid out q | k | v
    int nsplit;
    size_t split_stride;  // elements between partials
    const float *rope_tab;  // [S, HD/2, 2] (cos, sin)
    int rope_style;
};

// Sum of the partials of 8 consecutive columns starting at `col` of row `row`.
__device__ __forceinline__ void sum_partials8(const FusedQkv &f, size_t row_off, int col, float x[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.f;
    for (int s = 0; s < f.nsplit; ++s) {
        const f32x4_t *p = reinterpret_cast<const f32x4_t *>(f.part + (size_t)s * f.split_stride + row_off + col);
        f32x4_t a = p[0], b = p[1];
        x[0] += a.x; x[1] += a.y; x[2] += a.z; x[3] += a.w;
        x[4] += b.x; x[5] += b.y; x[6] += b.z; x[7] += b.w;
    }
}

// Rotates the 8 head elements c*8 .. c*8+7 a lane holds (the 16 or 8 lanes of a group hold one head vector).
// Style 1 pairs element e with e + HD/2: the partner sits in lane c ^ (LPR/2) of the same group.
template <int HD>
__device__ __forceinline__ void rotate8(float x[8], int c, const float *tab /* row of the position */, int style) {
    constexpr int LPR = HD / 8, HALF = HD / 2;
    if (style == 0) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int r = c * 4 + k;
            float cs = tab[2 * r], sn = tab[2 * r + 1];
            float a = x[2 * k], b = x[2 * k + 1];
            x[2 * k] = a * cs - b * sn;
            x[2 * k + 1] = a * sn + b * cs;
        }
    } else {
        const bool low = c < LPR / 2;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float other = __shfl_xor(x[i], LPR / 2, 64);
            int r = (c * 8 + i) % HALF;
            float cs = tab[2 * r], sn = tab[2 * r + 1];
            float a = low ? x[i] : other, b = low ? other : x[i];
            x[i] = low ? a * cs - b * sn : a * sn + b * cs;
        }
    }
}

// I16: the cache rows are 16-bit block-scaled fixed point (KvMap::kscale / vscale) instead of half: the elements are
// widened from integers and the row's scale multiplies the finished dot product (K) or the probability (V).
// out_lo (optional): second half term of the output, half(o - half(o)), for a two-term output projection.
template <int HD, int GT, bool FUSED, bool PAGED, bool I16>
__global__ __launch_bounds__(DA_THREADS) void decode_attention_kernel(
    const float *__restrict__ q, f16_t *kc, f16_t *vc, const int32_t *__restrict__ d_len, f16_t *__restrict__ out,
    f16_t *__restrict__ out_lo, float *__restrict__ ws, int n_items, int Hq, int Hkv, int S, int nsplit, int len_stride,
    FusedQkv fq, KvMap map, const int32_t *__restrict__ d_done) {
    static_assert(!(FUSED && PAGED), "the fused form addresses contiguous slabs only");
    static_assert(!(FUSED && I16), "the fused form stores half rows");
    constexpr int LPR = HD / 8;     // lanes per cache row
    constexpr int RPW = 64 / LPR;   // rows per wavefront load instruction
    const int lane = threadIdx.x & 63;
    const int item = blockIdx.x * (DA_THREADS / 64) + (threadIdx.x >> 6);
    if (item >= n_items) return;
    const int g = Hq / Hkv, hgs = g / GT;
    int split = item % nsplit;
    int rest = item / nsplit;
    int hg = rest % hgs; rest /= hgs;
    int kvh = rest % Hkv;
    int b = rest / Hkv;
    const int head0 = kvh * g + hg * GT;  // first query head of this wavefront
    if (d_done && d_done[b]) return;  // an ended sequence: its cache is not read any more (its output row keeps old values)

    const int pos = d_len[(size_t)b * len_stride];  // position of the new token (len_stride 0: one length for all sequences)
    if (FUSED && pos >= S) return;  // capacity is checked on the host; never write outside the cache
    int n = pos + 1;  // visible cache rows: positions 0 .. len
    if (n > S) n = S;
    const int chunk = (n + nsplit - 1) / nsplit;
    const int j0 = split * chunk;
    const int j1 = j0 + chunk < n ? j0 + chunk : n;

    const int c = lane % LPR, r = lane / LPR;
    float qr[GT][8];
    u32x4_t k_new = {0u, 0u, 0u, 0u}, v_new = {0u, 0u, 0u, 0u};  // FUSED: the cache row of position `pos`, as stored
    if (FUSED) {
        const size_t row_off = (size_t)b * (Hq + 2 * Hkv) * HD;
        const float *tab = fq.rope_tab + (size_t)pos * HD;
#pragma unroll
        for (int gh = 0; gh < GT; ++gh) {
            sum_partials8(fq, row_off, (head0 + gh) * HD + c * 8, qr[gh]);
            rotate8<HD>(qr[gh], c, tab, fq.rope_style);
        }
        if (j0 <= pos && pos < j1) {  // wavefront-uniform
            float x[8];
            sum_partials8(fq, row_off, (Hq + kvh) * HD + c * 8, x);
            rotate8<HD>(x, c, tab, fq.rope_style);
            k_new.x = pack_f16x2(x[0], x[1]); k_new.y = pack_f16x2(x[2], x[3]);
            k_new.z = pack_f16x2(x[4], x[5]); k_new.w = pack_f16x2(x[6], x[7]);
            sum_partials8(fq, row_off, (Hq + Hkv + kvh) * HD + c * 8, x);
            v_new.x = pack_f16x2(x[0], x[1]); v_new.y = pack_f16x2(x[2], x[3]);
            v_new.z = pack_f16x2(x[4], x[5]); v_new.w = pack_f16x2(x[6], x[7]);
            if (hg == 0 && r == 0) {  // one wavefront per (sequence, kv head) appends the row
                *reinterpret_cast<u32x4_t *>(kc + (((size_t)b * Hkv + kvh) * S + pos) * HD + c * 8) = k_new;
                *reinterpret_cast<u32x4_t *>(vc + (((size_t)b * Hkv + kvh) * S + pos) * HD + c * 8) = v_new;
            }
        }
    } else {
#pragma unroll
        for (int gh = 0; gh < GT; ++gh) {
            const f32x4_t *qp = reinterpret_cast<const f32x4_t *>(q + ((size_t)b * Hq + head0 + gh) * HD + c * 8);
            f32x4_t a = qp[0], bb = qp[1];
            qr[gh][0] = a.x; qr[gh][1] = a.y; qr[gh][2] = a.z; qr[gh][3] = a.w;
            qr[gh][4] = bb.x; qr[gh][5] = bb.y; qr[gh][6] = bb.z; qr[gh][7] = bb.w;
        }
    }
    const float scale = rsqrtf((float)HD);
    // contiguous: the slab of this (sequence, kv head); paged: the pool, rows found through the sequence's page list
    const f16_t *kb = kc + (PAGED ? (size_t)0 : ((size_t)b * Hkv + kvh) * S * HD) + c * 8;
    const f16_t *vb = vc + (PAGED ? (size_t)0 : ((size_t)b * Hkv + kvh) * S * HD) + c * 8;
    const float *ksb = I16 ? map.kscale + (PAGED ? (size_t)0 : ((size_t)b * Hkv + kvh) * S) : nullptr;
    const float *vsb = I16 ? map.vscale + (PAGED ? (size_t)0 : ((size_t)b * Hkv + kvh) * S) : nullptr;
    const int32_t *pages = PAGED ? map.table + (size_t)b * map.table_stride : nullptr;
    const int pmask = (1 << map.page_shift) - 1;
    // page numbers are fetched one iteration ahead, so the cache loads never wait for the page list
    int pg[DA_U];
    if (PAGED) {
#pragma unroll
        for (int u = 0; u < DA_U; ++u) {
            int j = j0 + u * RPW + r;
            int jc = j < j1 ? j : j1 - 1;
            pg[u] = pages[jc >> map.page_shift];
        }
    }

    float mx[GT], den[GT], acc[GT][8];
#pragma unroll
    for (int gh = 0; gh < GT; ++gh) {
        mx[gh] = -INFINITY; den[gh] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[gh][i] = 0.f;
    }

    for (int base = j0; base < j1; base += RPW * DA_U) {
        u32x4_t kr[DA_U], vr[DA_U];
        float ksc[DA_U], vsc[DA_U];
        int jj[DA_U];
        bool is_new[DA_U];
        // Contiguous block-scaled rows: the RPW * DA_U scales of this trip are consecutive floats, so one load per
        // wavefront (lane l takes the scale of row base + l mod rows-per-trip) fetches them all and a lane picks its rows'
        // scales by shuffles -- a per-row load would add one memory request per row-load instruction.
        float ks_l = 1.f, vs_l = 1.f;
        if (I16 && !PAGED) {
            const int j = base + lane % (RPW * DA_U);
            const int jc = j < j1 ? j : j1 - 1;
            ks_l = ksb[jc];
            vs_l = vsb[jc];
        }
#pragma unroll
        for (int u = 0; u < DA_U; ++u) {
            int j = base + u * RPW + r;
            jj[u] = j;
            int jc = j < j1 ? j : j1 - 1;  // rows past the end re-read the last valid row; their weight is 0
            is_new[u] = FUSED && jc == pos;
            const size_t row = PAGED ? (((size_t)pg[u] * Hkv + kvh) << map.page_shift) + (jc & pmask) : (size_t)jc;
            // every cache row is used once per step: non-temporal loads stream it past the caches (measured on plain
            // streaming of 8 GiB: 7.05 TB/s against 6.2 TB/s with ordinary loads)
            kr[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(kb + row * HD));
            vr[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(vb + row * HD));
            if (I16 && PAGED) { ksc[u] = ksb[row]; vsc[u] = vsb[row]; }
            else if (I16) { ksc[u] = __shfl(ks_l, u * RPW + r, 64); vsc[u] = __shfl(vs_l, u * RPW + r, 64); }
            else { ksc[u] = 1.f; vsc[u] = 1.f; }
        }
        if (PAGED) {
#pragma unroll
            for (int u = 0; u < DA_U; ++u) {
                int j = base + RPW * DA_U + u * RPW + r;
                int jc = j < j1 ? j : j1 - 1;
                pg[u] = pages[jc >> map.page_shift];
            }
        }
        if (FUSED) {  // the row of the new position comes from registers: the cache may not hold it yet
#pragma unroll
            for (int u = 0; u < DA_U; ++u)
                if (is_new[u]) { kr[u] = k_new; vr[u] = v_new; }
        }
        float kf[DA_U][8];
#pragma unroll
        for (int u = 0; u < DA_U; ++u) {
            if (I16) {
                kf[u][0] = i16lo_to_f32(kr[u].x); kf[u][1] = i16hi_to_f32(kr[u].x);
                kf[u][2] = i16lo_to_f32(kr[u].y); kf[u][3] = i16hi_to_f32(kr[u].y);
                kf[u][4] = i16lo_to_f32(kr[u].z); kf[u][5] = i16hi_to_f32(kr[u].z);
                kf[u][6] = i16lo_to_f32(kr[u].w); kf[u][7] = i16hi_to_f32(kr[u].w);
            } else {
                kf[u][0] = f16lo_to_f32(kr[u].x); kf[u][1] = f16hi_to_f32(kr[u].x);
                kf[u][2] = f16lo_to_f32(kr[u].y); kf[u][3] = f16hi_to_f32(kr[u].y);
                kf[u][4] = f16lo_to_f32(kr[u].z); kf[u][5] = f16hi_to_f32(kr[u].z);
                kf[u][6] = f16lo_to_f32(kr[u].w); kf[u][7] = f16hi_to_f32(kr[u].w);
            }
        }
        float sc[GT][DA_U];
#pragma unroll
        for (int gh = 0; gh < GT; ++gh)
#pragma unroll
            for (int u = 0; u < DA_U; ++u) {
                float d = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) d = fmaf(qr[gh][i], kf[u][i], d);
                d = group_sum<LPR>(d) * scale;
                if (I16) d *= ksc[u];
                sc[gh][u] = jj[u] < j1 ? d : -INFINITY;
            }
        float vf[DA_U][8];
#pragma unroll
        for (int u = 0; u < DA_U; ++u) {
            if (I16) {
                vf[u][0] = i16lo_to_f32(vr[u].x); vf[u][1] = i16hi_to_f32(vr[u].x);
                vf[u][2] = i16lo_to_f32(vr[u].y); vf[u][3] = i16hi_to_f32(vr[u].y);
                vf[u][4] = i16lo_to_f32(vr[u].z); vf[u][5] = i16hi_to_f32(vr[u].z);
                vf[u][6] = i16lo_to_f32(vr[u].w); vf[u][7] = i16hi_to_f32(vr[u].w);
            } else {
                vf[u][0] = f16lo_to_f32(vr[u].x); vf[u][1] = f16hi_to_f32(vr[u].x);
                vf[u][2] = f16lo_to_f32(vr[u].y); vf[u][3] = f16hi_to_f32(vr[u].y);
                vf[u][4] = f16lo_to_f32(vr[u].z); vf[u][5] = f16hi_to_f32(vr[u].z);
                vf[u][6] = f16lo_to_f32(vr[u].w); vf[u][7] = f16hi_to_f32(vr[u].w);
            }
        }
#pragma unroll
        for (int gh = 0; gh < GT; ++gh) {
            float mnew = mx[gh];
#pragma unroll
            for (int u = 0; u < DA_U; ++u) mnew = fmaxf(mnew, sc[gh][u]);
            if (mnew == -INFINITY) continue;  // this lane group has seen no valid row yet
            float alpha = mx[gh] == -INFINITY ? 0.f : __expf(mx[gh] - mnew);
            mx[gh] = mnew;
            den[gh] *= alpha;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[gh][i] *= alpha;
#pragma unroll
            for (int u = 0; u < DA_U; ++u) {
                float p = __expf(sc[gh][u] - mnew);  // exp(-inf) = 0 for rows past the end
                den[gh] += p;
                const float pv = I16 ? p * vsc[u] : p;  // the row's scale rides on the probability
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[gh][i] = fmaf(pv, vf[u][i], acc[gh][i]);
            }
        }
    }

    // ---- merge the RPW lane groups (lanes with equal c) of the wavefront
#pragma unroll
    for (int gh = 0; gh < GT; ++gh) {
        float m = mx[gh];
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
        float wgt = mx[gh] == -INFINITY ? 0.f : __expf(mx[gh] - m);
        float l = den[gh] * wgt;
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) l += __shfl_xor(l, o, 64);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float a = acc[gh][i] * wgt;
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) a += __shfl_xor(a, o, 64);
            acc[gh][i] = a;
        }
        if (r == 0) {
            int head = head0 + gh;
            if (nsplit == 1) {
                float inv = 1.0f / l;
                u32x4_t o4;
                o4.x = pack_f16x2(acc[gh][0] * inv, acc[gh][1] * inv);
                o4.y = pack_f16x2(acc[gh][2] * inv, acc[gh][3] * inv);
                o4.z = pack_f16x2(acc[gh][4] * inv, acc[gh][5] * inv);
                o4.w = pack_f16x2(acc[gh][6] * inv, acc[gh][7] * inv);
                *reinterpret_cast<u32x4_t *>(out + ((size_t)b * Hq + head) * HD + c * 8) = o4;
                if (out_lo) {
                    u32x4_t l4;
                    l4.x = pack_f16x2_lo(acc[gh][0] * inv, acc[gh][1] * inv, o4.x);
                    l4.y = pack_f16x2_lo(acc[gh][2] * inv, acc[gh][3] * inv, o4.y);
                    l4.z = pack_f16x2_lo(acc[gh][4] * inv, acc[gh][5] * inv, o4.z);
                    l4.w = pack_f16x2_lo(acc[gh][6] * inv, acc[gh][7] * inv, o4.w);
                    *reinterpret_cast<u32x4_t *>(out_lo + ((size_t)b * Hq + head) * HD + c * 8) = l4;
                }
            } else {
                float *p = ws + (((size_t)b * Hq + head) * nsplit + split) * (HD + 2);
                if (c == 0) { p[0] = m; p[1] = l; }
                float *ps = p + 2 + c * 8;
#pragma unroll
                for (int i = 0; i < 8; ++i) ps[i] = acc[gh][i];
            }
        }
    }
}

// Combines the split partials: o = sum_s o_s e^(m_s - M) / sum_s l_s e^(m_s - M)
__global__ __launch_bounds__(128) void decode_attention_merge_kernel(const float *__restrict__ ws, f16_t *__restrict__ out,
                                                                     f16_t *__restrict__ out_lo, int hd, int nsplit) {
    int bh = blockIdx.x, e = threadIdx.x;
    if (e >= hd) return;
    const float *p = ws + (size_t)bh * nsplit * (hd + 2);
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[s * (hd + 2)]);
    float L = 0.f, o = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        float m = p[s * (hd + 2)];
        float wgt = m == -INFINITY ? 0.f : __expf(m - M);
        L += p[s * (hd + 2) + 1] * wgt;
        o += p[s * (hd + 2) + 2 + e] * wgt;
    }
    const float y = o / L;
    const f16_t hi = f32_to_f16(y);
    out[(size_t)bh * hd + e] = hi;
    if (out_lo) out_lo[(size_t)bh * hd + e] = f32_to_f16(y - f16_to_f32(hi));
}

size_t decode_attention_ws_floats(int B, int Hq, int hd, int nsplit) {
    return nsplit > 1 ? (size_t)B * Hq * nsplit * (hd + 2) : 0;
}

// Query heads of one kv head that a wavefront processes together (they share every cache row it loads).  At most 4:
// with 8 the per-head state fills the register file and one wavefront per SIMD cannot hide the cache latency;
// the second wavefront of a kv head finds the rows in L2.
int decode_attention_group(int g) { return g % 4 == 0 ? 4 : (g % 2 == 0 ? 2 : 1); }

int decode_attention_default_splits(int B, int Hkv, int S) {
    long items = (long)B * Hkv;
    int s = (int)((2048 + items - 1) / items);  // aim at >= 2 wavefronts per SIMD over 256 compute units
    int cap = S / 128;                          // but keep >= 128 positions per split at full length
    if (s > cap) s = cap;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    return s;
}

template <int HD, int GT>
static void launch_da(const float *q, f16_t *kc, f16_t *vc, const int32_t *d_len, int len_stride, f16_t *out, f16_t *out_lo, float *ws,
                      int B, int Hq, int Hkv, int S, int nsplit, const FusedQkv *fq, const KvMap &map, const int32_t *d_done,
                      hipStream_t st) {
    int g = Hq / Hkv;
    int n_items = B * Hkv * (g / GT) * nsplit;
    int blocks = ceil_div(n_items, DA_THREADS / 64);
    const bool i16 = map.kscale != nullptr;
#define DA_LAUNCH(FUSEDV, PAGEDV, I16V, QV, FQV, MAPV, DONEV)                                                                   \
    decode_attention_kernel<HD, GT, FUSEDV, PAGEDV, I16V><<<blocks, DA_THREADS, 0, st>>>(QV, kc, vc, d_len, out, out_lo, ws, n_items, \
                                                                                         Hq, Hkv, S, nsplit, len_stride, FQV, MAPV, DONEV)
    if (fq) DA_LAUNCH(true, false, false, nullptr, *fq, KvMap(), nullptr);
    else if (map.table && i16) DA_LAUNCH(false, true, true, q, FusedQkv{}, map, d_done);
    else if (map.table) DA_LAUNCH(false, true, false, q, FusedQkv{}, map, d_done);
    else if (i16) DA_LAUNCH(false, false, true, q, FusedQkv{}, map, d_done);
    else DA_LAUNCH(false, false, false, q, FusedQkv{}, KvMap(), d_done);
#undef DA_LAUNCH
}

static void dispatch_da(const float *q, f16_t *kc, f16_t *vc, const int32_t *d_len, int len_stride, f16_t *out, f16_t *out_lo, float *ws,
                        int B, int Hq, int Hkv, int hd, int S, int nsplit, const FusedQkv *fq, const KvMap &map, const int32_t *d_done,
                        hipStream_t st) {
    if (B <= 0) return;
    int g = Hq / Hkv;
    int gt = decode_attention_group(g);
#define DA_CASE(HDV, GTV) \
    if (hd == HDV && gt == GTV) { launch_da<HDV, GTV>(q, kc, vc, d_len, len_stride, out, out_lo, ws, B, Hq, Hkv, S, nsplit, fq, map, d_done, st); }
    DA_CASE(128, 1) DA_CASE(128, 2) DA_CASE(128, 4)
    DA_CASE(64, 1) DA_CASE(64, 2) DA_CASE(64, 4)
#undef DA_CASE
    if (nsplit > 1) launch_decode_attention_merge(ws, out, B, Hq, hd, nsplit, st, out_lo);
}

void launch_decode_attention(const float *q, const f16_t *kc, const f16_t *vc, const int32_t *d_len, int len_stride, f16_t *out,
                             float *ws, int B, int Hq, int Hkv, int hd, int S, int nsplit, hipStream_t st, KvMap map,
                             const int32_t *d_done, f16_t *out_lo) {
    // many query heads per cache row: the matrix-core kernel (half and block-scaled rows)
    if (decode_attention_gqa_takes(Hq, Hkv, hd, map.kscale != nullptr)) {
        launch_decode_attention_gqa(q, kc, vc, d_len, len_stride, out, ws, B, Hq, Hkv, S, nsplit, st, map, d_done, out_lo);
        return;
    }
    dispatch_da(q, const_cast<f16_t *>(kc), const_cast<f16_t *>(vc), d_len, len_stride, out, out_lo, ws, B, Hq, Hkv, hd, S, nsplit,
                nullptr, map, d_done, st);
}

void launch_decode_attention_fused(const float *qkv, int nsplit_qkv, size_t split_stride, const float *rope_tab, int rope_style,
                                   f16_t *kc, f16_t *vc, const int32_t *d_len, int len_stride, f16_t *out, float *ws, int B, int Hq,
                                   int Hkv, int hd, int S, int nsplit, hipStream_t st) {
    FusedQkv fq;
    fq.part = qkv; fq.nsplit = nsplit_qkv; fq.split_stride = split_stride; fq.rope_tab = rope_tab; fq.rope_style = rope_style;
    dispatch_da(nullptr, kc, vc, d_len, len_stride, out, nullptr, ws, B, Hq, Hkv, hd, S, nsplit, &fq, KvMap(), nullptr, st);
}

void launch_decode_attention_merge(const float *ws, f16_t *out, int B, int Hq, int hd, int nsplit, hipStream_t st, f16_t *out_lo) {
    decode_attention_merge_kernel<<<B * Hq, 128, 0, st>>>(ws, out, out_lo, hd, nsplit);
}
