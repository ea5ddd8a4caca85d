// Bandwidth-trivial steps of the generation path: embedding gather, residual add + RMSNorm, rotary
// embedding + KV-cache append, greedy argmax.  fp32 VALU arithmetic, wavefront (64-lane) reductions.
#include "kernels.h"

// ------------------------------------------------------------------------------------------------
// Embedding gather: the first step of a forward pass (paper Section 2.1: prompt tokens, or the latest
// generated token, enter the model).  One workgroup per token row.
__global__ __launch_bounds__(256) void embed_kernel(const int32_t *__restrict__ tokens, const bf16_t *__restrict__ emb,
                                                    float *__restrict__ x, int d, int vocab) {
    int m = blockIdx.x;
    int tok = tokens[m];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
    const u32x4_t *src = reinterpret_cast<const u32x4_t *>(emb + (size_t)tok * d);
    f32x4_t *dst = reinterpret_cast<f32x4_t *>(x + (size_t)m * d);
    for (int i = threadIdx.x; i < d / 8; i += blockDim.x) {
        u32x4_t v = src[i];
        f32x4_t a = {bf16lo_to_f32(v.x), bf16hi_to_f32(v.x), bf16lo_to_f32(v.y), bf16hi_to_f32(v.y)};
        f32x4_t b = {bf16lo_to_f32(v.z), bf16hi_to_f32(v.z), bf16lo_to_f32(v.w), bf16hi_to_f32(v.w)};
        dst[2 * i] = a;
        dst[2 * i + 1] = b;
    }
}

void launch_embed(const int32_t *tokens, const bf16_t *emb, float *x, int M, int d, int vocab, hipStream_t st) {
    if (M <= 0) return;
    embed_kernel<<<M, 256, 0, st>>>(tokens, emb, x, d, vocab);
}

// ------------------------------------------------------------------------------------------------
// Residual add of split-K partial sums, then RMSNorm: y = g * x / sqrt(mean(x^2) + eps).
// The residual stream stays fp32; only the normalised copy that feeds the next projection is half.
// One workgroup per row; each thread keeps its slice of the row in registers (hidden <= 8192).
#define RN_MAX_SPLITS 16
template <int THREADS, int MAXV>
__global__ __launch_bounds__(THREADS) void add_rmsnorm_kernel(float *__restrict__ x, const float *__restrict__ part,
                                                              int nsplit, size_t part_stride,
                                                              const bf16_t *__restrict__ gain, float eps,
                                                              f16_t *__restrict__ h, f16_t *__restrict__ h_lo, int d) {
    __shared__ float red[THREADS / RL_WAVE];
    int m = blockIdx.x, t = threadIdx.x;
    f32x4_t v[MAXV];
    float ss = 0.f;
    f32x4_t *xr = reinterpret_cast<f32x4_t *>(x + (size_t)m * d);
    const f32x4_t *pr = reinterpret_cast<const f32x4_t *>(part + (size_t)m * d);
    const size_t ps4 = part_stride / 4;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        int e4 = t + i * THREADS;
        if (e4 * 4 < d) {
            f32x4_t a = xr[e4];
            // partials are added in split order (fixed, so results are reproducible); eight, then four loads in flight
            int s = 0;
            for (; s + 8 <= nsplit; s += 8) {
                f32x4_t q[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) q[u] = pr[(size_t)(s + u) * ps4 + e4];
#pragma unroll
                for (int u = 0; u < 8; ++u) a += q[u];
            }
            for (; s + 4 <= nsplit; s += 4) {
                f32x4_t p0 = pr[(size_t)s * ps4 + e4], p1 = pr[(size_t)(s + 1) * ps4 + e4];
                f32x4_t p2 = pr[(size_t)(s + 2) * ps4 + e4], p3 = pr[(size_t)(s + 3) * ps4 + e4];
                a += p0; a += p1; a += p2; a += p3;
            }
            for (; s < nsplit; ++s) a += pr[(size_t)s * ps4 + e4];
            if (nsplit > 0) xr[e4] = a;
            v[i] = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
    ss = wave_sum(ss);
    if ((t & 63) == 0) red[t >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < THREADS / RL_WAVE; ++w) tot += red[w];
    float inv = 1.0f / sqrtf(tot / (float)d + eps);
    u32x2_t *hr = reinterpret_cast<u32x2_t *>(h + (size_t)m * d);
    u32x2_t *lr = h_lo ? reinterpret_cast<u32x2_t *>(h_lo + (size_t)m * d) : nullptr;
    const u32x2_t *gr = reinterpret_cast<const u32x2_t *>(gain);
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        int e4 = t + i * THREADS;
        if (e4 * 4 < d) {
            u32x2_t g = gr[e4];
            float y0 = bf16lo_to_f32(g.x) * v[i].x * inv, y1 = bf16hi_to_f32(g.x) * v[i].y * inv;
            float y2 = bf16lo_to_f32(g.y) * v[i].z * inv, y3 = bf16hi_to_f32(g.y) * v[i].w * inv;
            u32x2_t o;
            o.x = pack_f16x2(y0, y1);
            o.y = pack_f16x2(y2, y3);
            hr[e4] = o;
            if (lr) {  // second half-precision term: what the first rounding lost (y = hi + lo up to 2^-22 relative)
                u32x2_t r;
                r.x = pack_f16x2(y0 - f16lo_to_f32(o.x), y1 - f16hi_to_f32(o.x));
                r.y = pack_f16x2(y2 - f16lo_to_f32(o.y), y3 - f16hi_to_f32(o.y));
                lr[e4] = r;
            }
        }
    }
}

void launch_add_rmsnorm(float *x, const float *part, int nsplit, size_t part_stride, const bf16_t *gain, float eps,
                        f16_t *h, f16_t *h_lo, int M, int d, hipStream_t st) {
    if (M <= 0) return;
    // few rows (decode): many threads per row so that every row streams with many loads in flight;
    // many rows (prefill): fewer threads per row, more rows per compute unit
    if (M <= 1024 && d > 1024)
        add_rmsnorm_kernel<1024, 2><<<M, 1024, 0, st>>>(x, part, nsplit, part_stride, gain, eps, h, h_lo, d);
    else
        add_rmsnorm_kernel<256, 8><<<M, 256, 0, st>>>(x, part, nsplit, part_stride, gain, eps, h, h_lo, d);
}

// ------------------------------------------------------------------------------------------------
// Rotary embedding of q and k at the token's absolute position, and KV-cache append.
// Pair r of a head turns by the angle pos * base^(-2r/hd); cos/sin come from a table built in fp64.
// One thread per (token row, head, pair) item.
__global__ __launch_bounds__(256) void rope_append_kernel(const float *__restrict__ qkv, int nsplit, size_t split_stride,
                                                          int T, int b0, const int32_t *__restrict__ d_pos0, int pos_stride,
                                                          const float *__restrict__ rope_tab, int rope_style, int Hq,
                                                          int Hkv, int hd, int S, float *__restrict__ q_f32,
                                                          f16_t *__restrict__ q_f16, f16_t *__restrict__ kc,
                                                          f16_t *__restrict__ vc, KvMap map,
                                                          const int32_t *__restrict__ d_valid,
                                                          const int32_t *__restrict__ d_done, f16_t *__restrict__ q_f16_lo) {
    int m = blockIdx.x;
    int b = b0 + m / T;
    bool store_kv = true;  // rows past a sequence's own length never reach the cache
    if (d_valid) {
        int nv = d_valid[b];
        nv = nv < 1 ? 1 : (nv > T ? T : nv);
        store_kv = m % T < nv;
    }
    if (d_done && d_done[b]) store_kv = false;  // an ended sequence is fed its end token again: nothing new to keep
    int pos = d_pos0[(size_t)(m / T) * pos_stride] + m % T;  // pos_stride 0: one start for all rows; 1: one per sequence
    if (pos >= S) return;  // capacity is checked on the host; never write outside the cache
    int half = hd >> 1;
    int nq = Hq * half, nk = Hkv * half;
    int ld = (Hq + 2 * Hkv) * hd;
    const float *row = qkv + (size_t)m * ld;
    const float *tab = rope_tab + (size_t)pos * hd;  // [half][2]
    int it = blockIdx.y * blockDim.x + threadIdx.x;
    const bool valid = it < nq + 2 * nk;
    int kind = 0, head = 0, r = 0, ia = 0, ib = 1;
    float a = 0.f, c = 0.f;
    if (valid) {
        kind = it < nq ? 0 : (it < nq + nk ? 1 : 2);
        int local = kind == 0 ? it : (kind == 1 ? it - nq : it - nq - nk);
        head = local / half;
        r = local % half;
        int col0 = (kind == 0 ? 0 : (kind == 1 ? Hq * hd : (Hq + Hkv) * hd)) + head * hd;
        if (kind == 2 || rope_style == 0) { ia = 2 * r; ib = 2 * r + 1; } else { ia = r; ib = r + half; }
        for (int s = 0; s < nsplit; ++s) {
            a += row[(size_t)s * split_stride + col0 + ia];
            c += row[(size_t)s * split_stride + col0 + ib];
        }
        if (kind != 2) {
            float cs = tab[2 * r], sn = tab[2 * r + 1];
            float ra = a * cs - c * sn, rb = a * sn + c * cs;
            a = ra; c = rb;
        }
        if (kind == 0) {
            size_t o = (size_t)m * Hq * hd + (size_t)head * hd;
            if (q_f32) { q_f32[o + ia] = a; q_f32[o + ib] = c; }
            if (q_f16) {
                const f16_t ha = f32_to_f16(a), hc = f32_to_f16(c);
                q_f16[o + ia] = ha; q_f16[o + ib] = hc;
                if (q_f16_lo) { q_f16_lo[o + ia] = f32_to_f16(a - f16_to_f32(ha)); q_f16_lo[o + ib] = f32_to_f16(c - f16_to_f32(hc)); }
            }
        }
    }
    const bool kv_item = valid && kind != 0 && store_kv;
    if (map.kscale) {
        // 16-bit block-scaled rows: the hd / 2 threads of a head are consecutive lanes (hd is 64 or 128 here and every
        // offset of the item space is a multiple of hd / 2), so the row maximum is an xor-shuffle reduction among them
        float am = valid && kind != 0 ? fmaxf(fabsf(a), fabsf(c)) : 0.f;
        for (int o = 1; o < half; o <<= 1) am = fmaxf(am, __shfl_xor(am, o, 64));
        if (kv_item) {
            const size_t rowi = kv_row_index(map, b, head, Hkv, S, pos);
            const float inv = kv_inv_of(am);
            int16_t *dst = reinterpret_cast<int16_t *>(kind == 1 ? kc : vc) + rowi * hd;
            dst[ia] = (int16_t)kv_quant(a, inv);
            dst[ib] = (int16_t)kv_quant(c, inv);
            if (r == 0) (kind == 1 ? map.kscale : map.vscale)[rowi] = kv_scale_of(am);
        }
    } else if (kv_item) {
        f16_t *dst = (kind == 1 ? kc : vc) + kv_row_index(map, b, head, Hkv, S, pos) * hd;
        dst[ia] = f32_to_f16(a);
        dst[ib] = f32_to_f16(c);
    }
}

void launch_rope_append(const float *qkv, int nsplit, size_t split_stride, int M, int T, int b0, const int32_t *d_pos0,
                        int pos_stride, const float *rope_tab, int rope_style, int Hq, int Hkv, int hd, int S, float *q_f32,
                        f16_t *q_f16, f16_t *kc, f16_t *vc, hipStream_t st, KvMap map, const int32_t *d_valid,
                        const int32_t *d_done, f16_t *q_f16_lo) {
    if (M <= 0) return;
    int items = (Hq + 2 * Hkv) * (hd / 2);
    dim3 grid(M, ceil_div(items, 256));
    rope_append_kernel<<<grid, 256, 0, st>>>(qkv, nsplit, split_stride, T, b0, d_pos0, pos_stride, rope_tab, rope_style, Hq, Hkv, hd, S,
                                          q_f32, q_f16, kc, vc, map, d_valid, d_done, q_f16_lo);
}

// ------------------------------------------------------------------------------------------------
// What follows the choice of a token (one thread per sequence): a sequence that had already ended keeps returning the
// end token and does not grow; otherwise the sequence grows by the token it was just fed, and ends if the new token is
// the end token.  lens / done may be NULL (no bookkeeping), eos < 0 means no end token.
__device__ __forceinline__ int finish_token(int tok, int b, int32_t *lens, int32_t *done, int eos) {
    if (done && done[b]) return eos;
    if (lens) lens[b] += 1;
    if (done && eos >= 0 && tok == eos) done[b] = 1;
    return tok;
}

// Greedy token: index of the largest logit, lowest index on ties; -1 if the row holds a NaN.
#define AM_THREADS 1024
__global__ __launch_bounds__(AM_THREADS) void argmax_kernel(const float *__restrict__ logits, int V,
                                                            int32_t *__restrict__ next, int32_t *lens, int32_t *done, int eos) {
    __shared__ float sv[AM_THREADS / RL_WAVE];
    __shared__ int si[AM_THREADS / RL_WAVE];
    __shared__ int snan;
    int b = blockIdx.x, t = threadIdx.x;
    if (t == 0) snan = 0;
    __syncthreads();
    const float *row = logits + (size_t)b * V;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    bool nan = false;
    for (int i = t; i < V; i += AM_THREADS) {
        float v = row[i];
        nan |= (v != v);
        if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(bv, o, 64);
        int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (nan) snan = 1;
    if ((t & 63) == 0) { sv[t >> 6] = bv; si[t >> 6] = bi; }
    __syncthreads();
    if (t == 0) {
        for (int w = 1; w < AM_THREADS / RL_WAVE; ++w)
            if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
        next[b] = finish_token((snan || bi == 0x7fffffff) ? -1 : bi, b, lens, done, eos);
    }
}

void launch_argmax(const float *logits, int B, int V, int32_t *next, int32_t *lens, int32_t *done, int eos, hipStream_t st) {
    if (B <= 0) return;
    argmax_kernel<<<B, AM_THREADS, 0, st>>>(logits, V, next, lens, done, eos);
}

// The greedy token from per-tile candidates (written by the LM-head projection's epilogue): one wavefront per row.
__global__ __launch_bounds__(RL_WAVE) void argmax_merge_kernel(const float *__restrict__ cand_val, const int32_t *__restrict__ cand_idx,
                                                               int tiles, int32_t *__restrict__ next, int32_t *lens, int32_t *done,
                                                               int eos) {
    const int b = blockIdx.x, t = threadIdx.x;
    const float *cv = cand_val + (size_t)b * tiles;
    const int32_t *ci = cand_idx + (size_t)b * tiles;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    int nan = 0;
    for (int i = t; i < tiles; i += RL_WAVE) {
        const float v = cv[i];
        const int idx = ci[i];
        nan |= (v != v);
        if (v > bv || (v == bv && idx < bi)) { bv = v; bi = idx; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        nan |= __shfl_xor(nan, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (t == 0) next[b] = finish_token((nan || bi == 0x7fffffff) ? -1 : bi, b, lens, done, eos);
}
void launch_argmax_merge(const float *cand_val, const int32_t *cand_idx, int B, int tiles, int32_t *next, int32_t *lens, int32_t *done,
                         int eos, hipStream_t st) {
    if (B <= 0) return;
    argmax_merge_kernel<<<B, RL_WAVE, 0, st>>>(cand_val, cand_idx, tiles, next, lens, done, eos);
}

// lens[b] = clamp(lens_in[b], 1, T) (T when lens_in is NULL), done[b] = 0: the sequence state a prefill leaves behind.
__global__ void init_state_kernel(int32_t *lens, int32_t *done, int B, const int32_t *lens_in, int T) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int n = lens_in ? lens_in[b] : T;
    lens[b] = n < 1 ? 1 : (n > T ? T : n);
    done[b] = 0;
}
void launch_init_state(int32_t *lens, int32_t *done, int B, const int32_t *lens_in, int T, hipStream_t st) {
    if (B <= 0) return;
    init_state_kernel<<<ceil_div(B, 256), 256, 0, st>>>(lens, done, B, lens_in, T);
}

// out[i, :] = h[i * T + clamp(lens[b0 + i], 1, T) - 1, :]: the last valid position of every sequence (half rows of d elements)
__global__ __launch_bounds__(256) void gather_last_rows_kernel(const f16_t *__restrict__ h, const int32_t *__restrict__ lens, int b0,
                                                               int T, int d, f16_t *__restrict__ out) {
    int i = blockIdx.x;
    int n = lens[b0 + i];
    n = n < 1 ? 1 : (n > T ? T : n);
    const u32x4_t *src = reinterpret_cast<const u32x4_t *>(h + ((size_t)i * T + n - 1) * d);
    u32x4_t *dst = reinterpret_cast<u32x4_t *>(out + (size_t)i * d);
    for (int k = threadIdx.x; k < d / 8; k += 256) dst[k] = src[k];
}
void launch_gather_last_rows(const f16_t *h, const int32_t *lens, int b0, int nb, int T, int d, f16_t *out, hipStream_t st) {
    if (nb <= 0) return;
    gather_last_rows_kernel<<<nb, 256, 0, st>>>(h, lens, b0, T, d, out);
}

// ------------------------------------------------------------------------------------------------
// Log-probability of the following token: out[g] = x[target] - log sum_v exp(x[v]) for the logit row of global row
// g = m_first + blockIdx.x, target = tokens[g + 1]; rows that end a sequence (g % T == T - 1) have no following
// token and get 0.  One pass: every thread keeps a running (max, sum of exp(x - max)) over its strided share, the
// pairs are merged across the wavefront and the workgroup.
#define LP_THREADS 512
__device__ __forceinline__ void lse_merge(float &m, float &s, float m2, float s2) {
    float mn = fmaxf(m, m2);
    if (mn == -INFINITY) { m = mn; s = 0.f; return; }
    s = s * expf(m - mn) + s2 * expf(m2 - mn);
    m = mn;
}
__global__ __launch_bounds__(LP_THREADS) void logprob_gather_kernel(const float *__restrict__ logits, int64_t ld, int V,
                                                                    const int32_t *__restrict__ tokens, int T, int64_t m_first,
                                                                    float *__restrict__ out) {
    __shared__ float sm[LP_THREADS / RL_WAVE], ss[LP_THREADS / RL_WAVE];
    const int t = threadIdx.x;
    const int64_t g = m_first + blockIdx.x;
    if (g % T == T - 1) {
        if (t == 0) out[g] = 0.f;
        return;
    }
    const float *row = logits + (size_t)blockIdx.x * ld;
    float m = -INFINITY, s = 0.f;
    for (int i = t; i < V; i += LP_THREADS) {
        float x = row[i];
        if (x > m) { s = s * expf(m - x) + 1.f; m = x; }  // exp(-inf) = 0 on the first element
        else s += expf(x - m);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lse_merge(m, s, __shfl_xor(m, o, 64), __shfl_xor(s, o, 64));
    if ((t & 63) == 0) { sm[t >> 6] = m; ss[t >> 6] = s; }
    __syncthreads();
    if (t == 0) {
        for (int w = 1; w < LP_THREADS / RL_WAVE; ++w) lse_merge(m, s, sm[w], ss[w]);
        int target = tokens[g + 1];
        target = target < 0 ? 0 : (target >= V ? V - 1 : target);  // ids outside the vocabulary are clamped, as in the embedding
        out[g] = row[target] - (m + logf(s));
    }
}

void launch_logprob_gather(const float *logits, int64_t ld, int M, int V, const int32_t *tokens, int T, int64_t m_first,
                           float *out, hipStream_t st) {
    if (M <= 0) return;
    logprob_gather_kernel<<<M, LP_THREADS, 0, st>>>(logits, ld, V, tokens, T, m_first, out);
}

// ------------------------------------------------------------------------------------------------
// Scalar head: out[m] = sum_k h[m, k] * w[k] (h half, w bf16 or fp32, fp32 accumulation), one wavefront per row.
__global__ __launch_bounds__(256) void rowdot_kernel(const f16_t *__restrict__ h, const f16_t *__restrict__ h_lo,
                                                     const void *__restrict__ w, int w_is_f32, int M, int d, float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const f16_t *row = h + (size_t)m * d;
    const f16_t *row_lo = h_lo ? h_lo + (size_t)m * d : nullptr;  // second half term of the rows (two-term activations)
    float acc = 0.f;
    for (int k = lane; k < d; k += 64) {
        float wk = w_is_f32 ? reinterpret_cast<const float *>(w)[k] : bf16_to_f32(reinterpret_cast<const bf16_t *>(w)[k]);
        float x = f16_to_f32(row[k]);
        if (row_lo) x += f16_to_f32(row_lo[k]);
        acc = fmaf(x, wk, acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) out[m] = acc;
}
void launch_rowdot(const f16_t *h, const f16_t *h_lo, const void *w, int w_is_f32, int M, int d, float *out, hipStream_t st) {
    if (M <= 0) return;
    rowdot_kernel<<<ceil_div(M, 4), 256, 0, st>>>(h, h_lo, w, w_is_f32, M, d, out);
}

// ------------------------------------------------------------------------------------------------
// Temperature sampling by inversion: e_v = exp((x_v - max) / temperature), next = smallest v with
// e_0 + ... + e_v > u * sum(e); -1 if the row holds a NaN.  One workgroup per row.  Every thread owns a contiguous
// segment of the row, the segment sums are scanned in thread order (fixed summation order: deterministic), and the
// first thread (with weight) whose prefix exceeds the target walks its segment.
#define SP_THREADS 1024
__global__ __launch_bounds__(SP_THREADS) void sample_kernel(const float *__restrict__ logits, int V, float inv_temp,
                                                            const float *__restrict__ u, int32_t *__restrict__ next,
                                                            int32_t *lens, int32_t *done, int eos) {
    __shared__ float red[SP_THREADS / RL_WAVE];
    __shared__ float bcast;
    __shared__ float pre[SP_THREADS];
    __shared__ int snan, stoken, sowner;
    const int b = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const float *row = logits + (size_t)b * V;
    const int seg = (V + SP_THREADS - 1) / SP_THREADS;
    const int i0 = t * seg < V ? t * seg : V, i1 = i0 + seg < V ? i0 + seg : V;
    if (t == 0) { snan = 0; stoken = -1; sowner = SP_THREADS; }
    __syncthreads();
    // ---- row maximum
    float m = -INFINITY;
    bool nan = false;
    for (int i = i0; i < i1; ++i) { float x = row[i]; nan |= (x != x); m = fmaxf(m, x); }
    m = wave_max(m);
    if (nan) snan = 1;
    if (lane == 0) red[wv] = m;
    __syncthreads();
    if (t == 0) {
        float mm = red[0];
        for (int w = 1; w < SP_THREADS / RL_WAVE; ++w) mm = fmaxf(mm, red[w]);
        bcast = mm;
    }
    __syncthreads();
    const float mx = bcast;
    const bool bad = snan != 0;
    __syncthreads();
    // ---- segment sums and their inclusive scan in thread order
    float s = 0.f;
    for (int i = i0; i < i1; ++i) s += expf((row[i] - mx) * inv_temp);
    float incl = s;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        float up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    if (lane == 63) red[wv] = incl;
    __syncthreads();
    float base = 0.f;
    for (int w = 0; w < wv; ++w) base += red[w];
    float total = 0.f;
    for (int w = 0; w < SP_THREADS / RL_WAVE; ++w) total += red[w];
    incl += base;
    pre[t] = incl;
    __syncthreads();
    // A thread's range starts exactly where its predecessor's ends (the stored prefix, not incl - s, which differs from it
    // by rounding): the ranges tile [0, last prefix) without gaps.  The prefixes come out of a tree-shaped scan and may
    // step back by an ulp, so the owner is the FIRST thread with weight whose prefix exceeds the target.
    const float excl = t == 0 ? 0.f : pre[t - 1];
    const float target = u[b] * total;
    if (!bad && s > 0.f && incl > target) atomicMin(&sowner, t);
    __syncthreads();
    if (t == sowner) {
        float run = excl;
        int tok = -1, last = i0;
        for (int i = i0; i < i1; ++i) {
            float e = expf((row[i] - mx) * inv_temp);
            if (e > 0.f) last = i;
            run += e;
            if (e > 0.f && run > target) { tok = i; break; }
        }
        stoken = tok >= 0 ? tok : last;  // the serial walk may round below the scanned prefix: the segment's last weighted index
    }
    __syncthreads();
    if (t == 0) {
        int tok = stoken;
        if (!bad && tok < 0) {  // u * total rounded up to the total: the last index that carries weight
            for (int i = V - 1; i >= 0; --i)
                if (expf((row[i] - mx) * inv_temp) > 0.f) { tok = i; break; }
        }
        next[b] = finish_token(bad ? -1 : tok, b, lens, done, eos);
    }
}

void launch_sample(const float *logits, int B, int V, float temperature, const float *u, int32_t *next, int32_t *lens,
                   int32_t *done, int eos, hipStream_t st) {
    if (B <= 0) return;
    sample_kernel<<<B, SP_THREADS, 0, st>>>(logits, V, 1.0f / temperature, u, next, lens, done, eos);
}

// dst[i * dst_stride] = src[i * src_stride] for i < n (32-bit words of any type)
__global__ void copy_strided_kernel(const uint32_t *__restrict__ src, int64_t src_stride, uint32_t *__restrict__ dst,
                                    int64_t dst_stride, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[(size_t)i * dst_stride] = src[(size_t)i * src_stride];
}
void launch_copy_strided(const void *src, int64_t src_stride, void *dst, int64_t dst_stride, int n, hipStream_t st) {
    if (n <= 0) return;
    copy_strided_kernel<<<ceil_div(n, 256), 256, 0, st>>>(reinterpret_cast<const uint32_t *>(src), src_stride,
                                                          reinterpret_cast<uint32_t *>(dst), dst_stride, n);
}

// Batch compaction: row i of the compacted batch is row kept[i] of the old one (kept ascending, kept[i] >= i).  One
// workgroup; every thread reads all of its values before anyone writes, so the arrays are permuted in place.
#define CS_THREADS 1024
#define CS_PER_THREAD 8
__global__ __launch_bounds__(CS_THREADS) void compact_state_kernel(int32_t *lens, int32_t *done, int32_t *tokens,
                                                                 const int32_t *__restrict__ kept, int n) {
    int32_t l[CS_PER_THREAD], t[CS_PER_THREAD];
#pragma unroll
    for (int k = 0; k < CS_PER_THREAD; ++k) {
        const int i = threadIdx.x + k * CS_THREADS;
        l[k] = 0; t[k] = 0;
        if (i < n) {
            const int src = kept[i];
            l[k] = lens[src];
            if (tokens) t[k] = tokens[src];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < CS_PER_THREAD; ++k) {
        const int i = threadIdx.x + k * CS_THREADS;
        if (i < n) {
            lens[i] = l[k];
            done[i] = 0;  // only sequences that have not ended are kept
            if (tokens) tokens[i] = t[k];
        }
    }
}
int compact_state_max_batch() { return CS_THREADS * CS_PER_THREAD; }
void launch_compact_state(int32_t *lens, int32_t *done, int32_t *tokens, const int32_t *kept, int n, hipStream_t st) {
    if (n <= 0) return;
    compact_state_kernel<<<1, CS_THREADS, 0, st>>>(lens, done, tokens, kept, n);
}

// One sequence's cache rows (contiguous cache) move to another sequence slot: for every (layer, K|V, kv head) the first
// `rows` rows of slab src are copied to slab dst -- 16-bit elements, and the fp32 row scales when the rows are block-scaled.
// Source and destination slabs are different sequences, so the ranges never overlap.
__global__ __launch_bounds__(256) void kv_move_kernel(f16_t *kv, float *scales, size_t area_elems, int Hkv, int S, int hd, int src,
                                                      int dst, int rows) {
    const int area = blockIdx.y;               // 2 * layer + (0: K, 1: V)
    const int kvh = blockIdx.x;
    f16_t *base = kv + (size_t)area * area_elems;
    const u32x4_t *from = reinterpret_cast<const u32x4_t *>(base + ((size_t)src * Hkv + kvh) * S * hd);
    u32x4_t *to = reinterpret_cast<u32x4_t *>(base + ((size_t)dst * Hkv + kvh) * S * hd);
    const size_t n16 = (size_t)rows * hd / 8;  // hd is 64 or 128: whole 16-byte pieces
    for (size_t i = threadIdx.x; i < n16; i += 256) to[i] = from[i];
    if (scales) {
        const size_t area_rows = area_elems / hd;
        const float *sf = scales + (size_t)area * area_rows + ((size_t)src * Hkv + kvh) * S;
        float *sd = scales + (size_t)area * area_rows + ((size_t)dst * Hkv + kvh) * S;
        for (int i = threadIdx.x; i < rows; i += 256) sd[i] = sf[i];
    }
}
void launch_kv_move(f16_t *kv, float *scales, size_t area_elems, int n_areas, int Hkv, int S, int hd, int src, int dst, int rows,
                    hipStream_t st) {
    if (rows <= 0 || n_areas <= 0 || src == dst) return;
    kv_move_kernel<<<dim3(Hkv, n_areas), 256, 0, st>>>(kv, scales, area_elems, Hkv, S, hd, src, dst, rows);
}

__global__ void set_i32_kernel(int32_t *p, int32_t v) { p[0] = v; }
void launch_set_i32(int32_t *p, int32_t v, hipStream_t st) { set_i32_kernel<<<1, 1, 0, st>>>(p, v); }

__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float *__restrict__ src, bf16_t *__restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = f32_to_bf16(src[i]);
}
void launch_f32_to_bf16(const float *src, bf16_t *dst, size_t n, hipStream_t st) {
    if (n == 0) return;
    size_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    f32_to_bf16_kernel<<<(unsigned)blocks, 256, 0, st>>>(src, dst, n);
}

// Plain device copy, 16 bytes per lane: a kernel of exactly known traffic (n bytes read, n written) that the
// benchmark runs next to the real kernels so that profiler byte counters can be scaled.
__global__ __launch_bounds__(256) void copy_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}
void launch_copy(const void *src, void *dst, size_t bytes, hipStream_t st) {
    size_t n16 = bytes / 16;
    if (n16 == 0) return;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    copy_kernel<<<(unsigned)blocks, 256, 0, st>>>(reinterpret_cast<const u32x4_t *>(src), reinterpret_cast<u32x4_t *>(dst), n16);
}
