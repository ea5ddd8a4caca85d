// Prefill attention: causal attention of all prompt positions of a sequence against the K/V rows that
// the same prefill pass has just written into the cache (tiled, online softmax, f16 MFMA).
//
// Layout of the computation for gfx950 (wavefront = 64 lanes, v_mfma_f32_32x32x16_f16):
//   * workgroup = 4 wavefronts = 128 consecutive query positions of one (sequence, query head);
//     wavefront w owns 32 of them and keeps its Q fragments in registers for the whole kernel;
//   * key tiles of 32 positions are staged once per workgroup in LDS (K and V, padded rows);
//   * scores are computed TRANSPOSED, S^T = K Q^T, so that in the accumulator layout a lane holds one
//     query column and 16 key rows: the softmax statistics of a query are lane-local (one shuffle
//     joins the two half-wavefronts), and the probabilities already sit in the register layout of the
//     B operand of the second product O^T += V^T P^T -- no shuffle or LDS round trip for P;
//   * V^T fragments are gathered from the LDS tile with 16-bit reads (the transpose happens there).
// Softmax and accumulation are fp32; probabilities are rounded to half for the matrix cores.
#include "kernels.h"

#define PA_THREADS 256
#define PA_KT 32          // keys per tile
#define PA_STRIDE(HD) ((HD) + 8)

// I16: the cache rows are 16-bit block-scaled fixed point (KvMap::kscale / vscale).  A row element q * scale has more
// significant bits than a half holds, so it enters the matrix cores as a two-term half sum hi + lo, and so do the
// probabilities and -- when q_lo is given -- the queries: each of the two products of a tile becomes three matrix
// instructions (hi x hi, lo x hi, hi x lo; lo x lo is below fp32 resolution) and no operand carries a single half rounding.
// q_lo (optional, I16 only): second half term of q, laid out like q.
// out_lo (optional): half(o - half(o)), the second term of the output for a two-term output projection.
template <int HD, bool I16>
__global__ __launch_bounds__(PA_THREADS) void prefill_attention_kernel(const f16_t *__restrict__ q,
                                                                      const f16_t *__restrict__ q_lo,
                                                                      const f16_t *__restrict__ kc,
                                                                      const f16_t *__restrict__ vc,
                                                                      f16_t *__restrict__ out, f16_t *__restrict__ out_lo,
                                                                      int b0, int T, int Hq,
                                                                      int Hkv, int S, KvMap map,
                                                                      const int32_t *__restrict__ d_valid) {
    constexpr int KS = HD / 16;   // k16 steps of the QK product
    constexpr int ET = HD / 32;   // 32-row tiles of O^T
    constexpr int STR = PA_STRIDE(HD);
    constexpr int NT = I16 ? 2 : 1;  // half terms per cache element
    __shared__ __attribute__((aligned(16))) f16_t ks[NT * PA_KT * STR];
    __shared__ __attribute__((aligned(16))) f16_t vs[NT * PA_KT * STR];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6, half = lane >> 5, l32 = lane & 31;
    const int qt = blockIdx.x;          // query tile (128 positions)
    const int u = blockIdx.y;           // query head
    const int bl = blockIdx.z;          // sequence within the chunk
    const int kvh = u / (Hq / Hkv);
    const int q0 = qt * 128 + w * 32;   // first query position of this wavefront
    const int qpos = q0 + l32;          // this lane's query column
    const size_t ldq = (size_t)Hq * HD;

    // Q fragments (B operand of S^T = K Q^T): lane = (query column l32, hd slice half*8 + 16*s)
    f16x8_t qf[KS], ql[I16 ? KS : 1];
    const bool two_q = I16 && q_lo != nullptr;  // uniform
    {
        int qrow = qpos < T ? qpos : T - 1;
        const size_t qoff = ((size_t)bl * T + qrow) * ldq + (size_t)u * HD + half * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const f16x8_t *>(q + qoff + s * 16);
        if (I16) {
#pragma unroll
            for (int s = 0; s < KS; ++s)
                ql[s] = two_q ? *reinterpret_cast<const f16x8_t *>(q_lo + qoff + s * 16) : f16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    int n_keys = T;  // keys this sequence really has in the cache
    if (d_valid) {
        int nv = d_valid[b0 + bl];
        n_keys = nv < 1 ? 1 : (nv > T ? T : nv);
    }

    f32x16_t oacc[ET];
#pragma unroll
    for (int e = 0; e < ET; ++e)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[e][i] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;  // running max (shared by both halves) and this half's partial sum
    const float scale = rsqrtf((float)HD);

    int last_q = qt * 128 + 127;
    if (last_q > T - 1) last_q = T - 1;
    const int n_tiles = last_q / PA_KT + 1;  // key tiles any wavefront of the workgroup needs
    for (int kt = 0; kt < n_tiles; ++kt) {
        __syncthreads();  // previous tile fully consumed
        // stage K and V rows kt*32 .. +31: 32 rows x HD*2 bytes each = HD/8 16-byte pieces per row
        for (int idx = t; idx < PA_KT * (HD / 8); idx += PA_THREADS) {
            int row = idx / (HD / 8), piece = idx % (HD / 8);
            int key = kt * PA_KT + row;
            u32x4_t kv = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
            float ksc = 0.f, vsc = 0.f;
            if (key < n_keys) {  // rows past the prompt may hold arbitrary bits: keep them out (0 * NaN)
                const size_t rowi = kv_row_index(map, b0 + bl, kvh, Hkv, S, key);
                const size_t at = rowi * HD + piece * 8;
                kv = *reinterpret_cast<const u32x4_t *>(kc + at);
                vv = *reinterpret_cast<const u32x4_t *>(vc + at);
                if (I16) { ksc = map.kscale[rowi]; vsc = map.vscale[rowi]; }
            }
            if (I16) {
                u32x4_t hi, lo;
                auto split = [](u32x4_t w, float sc, u32x4_t &h, u32x4_t &l) {
                    const uint32_t in[4] = {w.x, w.y, w.z, w.w};
                    uint32_t ho[4], lo_[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float x0 = i16lo_to_f32(in[i]) * sc, x1 = i16hi_to_f32(in[i]) * sc;
                        ho[i] = pack_f16x2(x0, x1);
                        lo_[i] = pack_f16x2_lo(x0, x1, ho[i]);
                    }
                    h = u32x4_t{ho[0], ho[1], ho[2], ho[3]};
                    l = u32x4_t{lo_[0], lo_[1], lo_[2], lo_[3]};
                };
                split(kv, ksc, hi, lo);
                *reinterpret_cast<u32x4_t *>(ks + row * STR + piece * 8) = hi;
                *reinterpret_cast<u32x4_t *>(ks + (PA_KT + row) * STR + piece * 8) = lo;
                split(vv, vsc, hi, lo);
                *reinterpret_cast<u32x4_t *>(vs + row * STR + piece * 8) = hi;
                *reinterpret_cast<u32x4_t *>(vs + (PA_KT + row) * STR + piece * 8) = lo;
            } else {
                *reinterpret_cast<u32x4_t *>(ks + row * STR + piece * 8) = kv;
                *reinterpret_cast<u32x4_t *>(vs + row * STR + piece * 8) = vv;
            }
        }
        __syncthreads();
        if (kt * PA_KT > q0 + 31) continue;  // tile entirely above this wavefront's diagonal (uniform per wavefront)

        // S^T tile: rows = keys, columns = queries
        f32x16_t sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int tm = 0; tm < NT; ++tm) {
                f16x8_t kf = *reinterpret_cast<const f16x8_t *>(ks + (tm * PA_KT + l32) * STR + half * 8 + s * 16);
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[s], sacc, 0, 0, 0);
                if (I16 && tm == 0 && two_q) sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, ql[s], sacc, 0, 0, 0);
            }
        }
        // register i holds key row (i/4)*8 + half*4 + (i%4) of the tile, query column l32
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int key = kt * PA_KT + (i >> 2) * 8 + half * 4 + (i & 3);
            float sv = key <= qpos ? sacc[i] * scale : -INFINITY;  // causal mask
            sacc[i] = sv;
            tmax = fmaxf(tmax, sv);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        float mnew = fmaxf(mrun, tmax);  // finite: key 0 is visible to every query
        float alpha = mrun == -INFINITY ? 0.f : __expf(mrun - mnew);
        mrun = mnew;
        lrun *= alpha;
#pragma unroll
        for (int e = 0; e < ET; ++e)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[e][i] *= alpha;
        f16x8_t pf[2], pl[I16 ? 2 : 1];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float p = __expf(sacc[i] - mnew);
            lrun += p;
            const _Float16 ph = (_Float16)p;
            pf[i >> 3][i & 7] = ph;
            if (I16) pl[i >> 3][i & 7] = (_Float16)(p - (float)ph);
        }
        // O^T += V^T P^T.  Slot j of k-step s in lane-half h stands for key (2s + j/4)*8 + h*4 + j%4 -- the
        // key that accumulator register s*8 + j already holds, so P needs no data movement.
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int e = 0; e < ET; ++e) {
#pragma unroll
                for (int tm = 0; tm < NT; ++tm) {
                    f16x8_t vf;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        int krow = (2 * s + (j >> 2)) * 8 + half * 4 + (j & 3);
                        vf[j] = __builtin_bit_cast(_Float16, vs[(tm * PA_KT + krow) * STR + e * 32 + l32]);
                    }
                    oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[s], oacc[e], 0, 0, 0);
                    if (I16 && tm == 0) oacc[e] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pl[s], oacc[e], 0, 0, 0);
                }
            }
        }
    }

    // normalise and store: lane = query column; register i of tile e is head_dim row e*32 + (i/4)*8 + half*4 + i%4
    float ltot = lrun + __shfl_xor(lrun, 32, 64);
    if (qpos < T) {
        float inv = 1.0f / ltot;
        f16_t *op = out + ((size_t)bl * T + qpos) * ldq + (size_t)u * HD;
#pragma unroll
        for (int e = 0; e < ET; ++e)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                u32x2_t o2;
                o2.x = pack_f16x2(oacc[e][i4 * 4 + 0] * inv, oacc[e][i4 * 4 + 1] * inv);
                o2.y = pack_f16x2(oacc[e][i4 * 4 + 2] * inv, oacc[e][i4 * 4 + 3] * inv);
                *reinterpret_cast<u32x2_t *>(op + e * 32 + i4 * 8 + half * 4) = o2;
                if (out_lo) {
                    u32x2_t l2;
                    l2.x = pack_f16x2_lo(oacc[e][i4 * 4 + 0] * inv, oacc[e][i4 * 4 + 1] * inv, o2.x);
                    l2.y = pack_f16x2_lo(oacc[e][i4 * 4 + 2] * inv, oacc[e][i4 * 4 + 3] * inv, o2.y);
                    *reinterpret_cast<u32x2_t *>(out_lo + (op - out) + e * 32 + i4 * 8 + half * 4) = l2;
                }
            }
    }
}

void launch_prefill_attention(const f16_t *q, const f16_t *kc, const f16_t *vc, f16_t *out, int nb, int b0, int T,
                              int Hq, int Hkv, int hd, int S, hipStream_t st, KvMap map, const int32_t *d_valid, f16_t *out_lo,
                              const f16_t *q_lo) {
    if (nb <= 0 || T <= 0) return;
    dim3 grid(ceil_div(T, 128), Hq, nb);
    const bool i16 = map.kscale != nullptr;
    if (hd == 128 && i16) prefill_attention_kernel<128, true><<<grid, PA_THREADS, 0, st>>>(q, q_lo, kc, vc, out, out_lo, b0, T, Hq, Hkv, S, map, d_valid);
    else if (hd == 128) prefill_attention_kernel<128, false><<<grid, PA_THREADS, 0, st>>>(q, nullptr, kc, vc, out, out_lo, b0, T, Hq, Hkv, S, map, d_valid);
    else if (i16) prefill_attention_kernel<64, true><<<grid, PA_THREADS, 0, st>>>(q, q_lo, kc, vc, out, out_lo, b0, T, Hq, Hkv, S, map, d_valid);
    else prefill_attention_kernel<64, false><<<grid, PA_THREADS, 0, st>>>(q, nullptr, kc, vc, out, out_lo, b0, T, Hq, Hkv, S, map, d_valid);
}
