/*
 * rl_gen_ops.h -- single-kernel entry points of the generation library (C ABI).
 *
 * Each call enqueues exactly one step of the hot path (the rows of the decoder that the paper's
 * "Generation" function call -- Section 2.1 -- runs for every prompt / generated token) on the
 * given stream, so that every kernel can be checked against the CPU oracle in isolation and be
 * timed on its own.  All pointers are DEVICE pointers borrowed for the duration of the enqueued
 * work; 16-bit tensors are passed as uint16_t bit patterns -- weights (emb, gain, W_i) are bf16,
 * activations and cache slabs (h, A, q_f16, kc, vc, attention outputs) are IEEE half, called "f16"
 * below; `hip_stream` is a hipStream_t (NULL =
 * default stream).  Return: 0, or a negative rl_gen_status (rl_gen.h); nothing is enqueued on error.
 *
 * Two optional argument groups recur (both follow rl_gen_shape.precision, rl_gen.h):
 *   kscale, vscale (both or neither; NULL = the cache rows are IEEE half): fp32 row scales of a block-scaled cache.  kc / vc
 *     then hold int16 elements, element e of row i standing for kc[i][e] * kscale[i]; a row is one (position, kv head)
 *     vector of hd elements and the scales are indexed like the rows ([n_seq][Hkv][S], or [n_pages][Hkv][page_size]).
 *     A writer sets scale = max|x| / 32767 over the row and stores round(x / scale).
 *   out_lo (NULL = not wanted): second term of a two-term half output, out_lo = f16(y - f16(y)) where out = f16(y), laid out
 *     like out; a projection that multiplies both terms sees y with about 22 significant bits.
 */
#ifndef RL_GEN_OPS_H
#define RL_GEN_OPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Embedding gather: x[m, :] = tok_emb[tokens[m], :] widened to fp32.  tokens int32 [M], emb bf16
 * [vocab, d], x fp32 [M, d]; d % 8 == 0.  Ids outside [0, vocab) are clamped. */
int rl_op_embed(const int32_t *tokens, const uint16_t *emb, float *x, int32_t M, int32_t d, int32_t vocab,
                void *hip_stream);

/* Residual add + RMSNorm: x[m,:] += sum_{s<nsplit} part[s*part_stride + m*d + :] (x is updated in
 * place when nsplit > 0; part may be NULL when nsplit == 0), then
 * y = gain * x / sqrt(mean(x^2) + eps), h[m,:] = f16(y).  x fp32 [M, d], gain bf16 [d], h f16 [M, d];
 * d % 4 == 0 and d <= 8192.  If h_lo is not NULL it receives the second term of a two-term split,
 * h_lo[m,:] = f16(y - h[m,:]) (f16 [M, d]): a projection fed with the stacked rows [h; h_lo] and summed
 * over the two row blocks sees the activation with ~22 instead of 11 significant bits. */
int rl_op_add_rmsnorm(float *x, const float *part, int32_t nsplit, size_t part_stride, const uint16_t *gain, float eps,
                      uint16_t *h, uint16_t *h_lo, int32_t M, int32_t d, void *hip_stream);

/* Projection: out[m, off_i + n] = sum_k A[m,k] * W_i[n,k] for up to three bf16 matrices W_i
 * [rows_i, K] placed side by side along the output columns (unused: NULL / 0 rows).
 * A f16 [M, K] with row stride lda; K % 8 == 0, lda % 8 == 0.  Weights are widened bf16 -> f16 in the
 * kernel (exact for |w| >= 2^-14) and multiplied on the f16 matrix cores with fp32 accumulation.
 * epilogue 0: fp32 out, row stride ldc; split s (0 <= s < splits) writes its partial sum at
 *             out + s*split_stride (the consumer adds the partials);
 * epilogue 1: SwiGLU, W_0 = gate, W_1 = up (equal shapes): out f16 [m*ldc + n] = silu(gate)*up;
 * epilogue 2: fp32 out[m*ldc + col] += result (residual add).
 * splits applies to the skinny kernel with epilogue 0 only.  kernel: 0 = choose by M, 1 = skinny
 * (weights streamed once through registers; M <= 256), 2 = tiled (both operands through LDS).
 * A_lo (kernel 2, epilogues 0 and 2; else NULL): second term of the activations, f16 [M, K] with the same stride,
 * located above A in the same allocation: out = (A + A_lo) W^T as one contraction over [A | A_lo] x [W | W].
 * out_lo (kernel 2 with epilogue 1; else NULL): second half term of the SwiGLU result. */
int rl_op_gemm(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *W0, const uint16_t *W1, const uint16_t *W2,
               int32_t rows0, int32_t rows1, int32_t rows2, int32_t M, int32_t K, void *out, int64_t ldc, size_t split_stride,
               int32_t splits, int32_t epilogue, int32_t kernel, uint16_t *out_lo, void *hip_stream);

/* The large-M projection kernel fed fragment-order copies of its weights as well (P_i = rl_op_pack_weights of W_i, one per
 * W_i): tiles of 256 x 256 then copy both operands global -> LDS with the load unit (no staging registers, no conversion in
 * the loop); smaller problems run as rl_op_gemm with kernel 2 does.  epilogue 0, 1 or 2 as in rl_op_gemm; out as there.
 * The products are the same; sums over K are formed in the same order, so results equal rl_op_gemm's bit for bit. */
int rl_op_gemm_tiled_packed(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *W0, const uint16_t *W1,
                            const uint16_t *W2, const uint16_t *P0, const uint16_t *P1, const uint16_t *P2, int32_t rows0, int32_t rows1,
                            int32_t rows2, int32_t M, int32_t K, void *out, int64_t ldc, int32_t epilogue, void *hip_stream);

/* QKV projection of a prefill with the rotary embedding and the cache append in its epilogue (what a prefill of a model
 * with head_dim 128 and rotary style 1 runs): [q | k | v] = (A + A_lo) [Wq; Wk; Wv]^T by the large-M kernel, row m being
 * sequence b0 + m / T at position m % T; q and k rotated with rope_tab (fp32 [S, 64, 2]); q stored as half [M, Hq*128],
 * k and v rows rounded to half and stored into kc / vc (half [n_seq][Hkv][S][128]).  Bit for bit what rl_op_gemm (fp32
 * output) followed by rl_op_rope_append stores.  RL_GEN_E_SHAPE where the fused form does not apply (head_dim, style,
 * T < 32, fewer than 256 tiles of 256 x 256).  Pq, Pk, Pv: optional fragment-order copies of the three matrices (all or
 * none): with them both operands are copied global -> LDS directly, as in rl_op_gemm_tiled_packed; same stored bits.
 * q_f16_lo (optional): second half term of q, f16(q - f16(q)), laid out like q_f16. */
int rl_op_gemm_rope(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *Wq, const uint16_t *Wk, const uint16_t *Wv,
                    const uint16_t *Pq, const uint16_t *Pk, const uint16_t *Pv, int32_t Hq, int32_t Hkv, int32_t hd, int32_t M, int32_t K, int32_t T, int32_t b0, const float *rope_tab,
                    int32_t rope_style, int32_t S, uint16_t *q_f16, uint16_t *kc, uint16_t *vc, float *kscale, float *vscale,
                    uint16_t *q_f16_lo, void *hip_stream);

/* Weights in matrix-core fragment order.  rl_op_pack_weights converts W bf16 [N, K] row-major (K % 8 == 0)
 * into P, rl_op_packed_weight_bytes(N, K) bytes of f16: P[ceil(N/32)][ceil(K/16)][64][8], where element e of
 * lane l of fragment (nb, ks) is W[32 nb + (l & 31), 16 ks + 8 (l >> 5) + e], widened bf16 -> f16 (exact for
 * |w| >= 2^-14), zero outside W.  A fragment is the B operand of one 32x32x16 f16 MFMA and 1 KB of consecutive
 * memory, so the projection below fetches weights straight into the registers the matrix cores read. */
size_t rl_op_packed_weight_bytes(int32_t N, int32_t K);
int rl_op_pack_weights(const uint16_t *W, uint16_t *P, int32_t N, int32_t K, void *hip_stream);

/* Projection over packed weights (the decode step's form of rl_op_gemm; same meaning of rows_i, M, K, lda,
 * out, ldc, split_stride, splits and epilogue).  A_lo: optional second term of the activations (f16 [M, K],
 * same stride, or NULL): out = (A + A_lo) W^T with both products accumulated in fp32, which is how the
 * two-term split of rl_op_add_rmsnorm reaches the QKV projection.  nb: 32-column blocks per wavefront,
 * 1 or 2 (0: chosen from the number of columns); epilogue 1 (SwiGLU) always uses gate block + up block.
 * rows_per_wg: activation rows per workgroup, 32, 64 or 128 (0: 128): smaller row blocks give more workgroups
 * without split-K partials; the row blocks of one column tile stream the same weights (HBM once, L2 after).
 * depth: 64-wide K chunks of weights each wavefront keeps in flight, 2 or 4 (0: 2).
 * out_lo (epilogue 1 only; else NULL): second half term of the SwiGLU result. */
int rl_op_gemm_packed(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *P0, const uint16_t *P1,
                      const uint16_t *P2, int32_t rows0, int32_t rows1, int32_t rows2, int32_t M, int32_t K, void *out,
                      int64_t ldc, size_t split_stride, int32_t splits, int32_t epilogue, int32_t nb, int32_t rows_per_wg,
                      int32_t depth, uint16_t *out_lo, void *hip_stream);

/* The LM head with the greedy choice fused into it (the last two steps of a decode step as the generator runs them):
 * logits[M, V] = (A + A_lo) P^T as rl_op_gemm_packed computes it for one matrix, and next[m] = the column of the largest
 * logit of row m -- lowest column on ties, -1 if the row holds a NaN -- i.e. exactly rl_op_argmax of those logits.  The
 * projection's epilogue leaves the best logit of every pass of 128 columns in ws, a second small kernel picks among them:
 * the logits are never re-read, and with logits == NULL never written.  A f16 [M, K] (row stride lda), A_lo f16 or NULL,
 * P f16 fragment-order copy of the [V, K] matrix, logits fp32 (row stride ldc >= V) or NULL, next int32 [M], ws fp32
 * [rl_op_lm_head_argmax_ws_floats(M, V)]; all DEVICE.  RL_GEN_E_SHAPE when the packed matrix reaches 3.75 GB. */
size_t rl_op_lm_head_argmax_ws_floats(int32_t M, int32_t V);
int rl_op_lm_head_argmax(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *P, int32_t V, int32_t M, int32_t K,
                         float *logits, int64_t ldc, float *ws, int32_t *next, void *hip_stream);

/* Fused gate/up projection of few rows from fragment-order copies, the two 64-wide halves of every 128-wide K chunk on
 * separate wavefronts: out[M, F] (DEVICE half, row stride ldc) = silu(A Pg^T) * (A Pu^T), A DEVICE half [M, K] with row stride lda,
 * Pg and Pu = rl_op_pack_weights of the gate and up matrices [F, K].  The sums are formed in the order of rl_op_gemm's kernel 1 with
 * epilogue 1, so the two calls store the same bits.  depth: 128-wide weight chunks in flight per wavefront, 2 or 4 (0: 4).
 * K % 8 == 0, lda % 8 == 0, each packed matrix below 3.75 GB; RL_GEN_E_SHAPE otherwise. */
int rl_op_gemm_packed_swiglu_halves(const uint16_t *A, int64_t lda, const uint16_t *Pg, const uint16_t *Pu, int32_t F, int32_t M,
                                    int32_t K, uint16_t *out, int64_t ldc, int32_t depth, uint16_t *out_lo, void *hip_stream);

/* Builds the rotary table the library uses: tab fp32 [max_seq, head_dim/2, 2] = (cos, sin) of
 * pos * base^(-2r/head_dim), evaluated in fp64 on the host and copied (synchronously) to `tab`. */
int rl_op_build_rope_table(float *tab, int32_t max_seq, int32_t head_dim, float base);

/* Rotary embedding + KV-cache append.  qkv fp32: nsplit partials, each [M, (Hq+2Hkv)*hd] laid out
 * q | k | v per row, split_stride elements apart.  Row m is sequence b0 + m / T at position
 * d_pos0[(m / T) * pos_stride] + m % T (d_pos0: DEVICE int32; pos_stride 0: one start position, 1: one per sequence).  Writes q_f32 and/or q_f16 ([M, Hq*hd], either may
 * be NULL) and the cache rows of kc / vc (f16 [n_seq][Hkv][S][hd], or block-scaled rows with their scales in kscale / vscale:
 * then hd must be 64 or 128).  q_f16_lo (optional, needs q_f16): second half term of q.  Positions >= S are skipped. */
int rl_op_rope_append(const float *qkv, int32_t nsplit, size_t split_stride, int32_t M, int32_t T, int32_t b0,
                      const int32_t *d_pos0, int32_t pos_stride, const float *rope_tab, int32_t rope_style, int32_t Hq, int32_t Hkv,
                      int32_t hd, int32_t S, float *q_f32, uint16_t *q_f16, uint16_t *kc, uint16_t *vc, float *kscale, float *vscale,
                      uint16_t *q_f16_lo, void *hip_stream);

/* Decode attention: for each sequence b < B and query head u, softmax(q_u . k_j / sqrt(hd)) v_j over
 * cache rows j = 0 .. d_len[b * len_stride] of kv head u / (Hq/Hkv) (len_stride 0: one length for all, 1: per sequence).  q fp32 [B, Hq*hd]; kc, vc f16; out f16 [B, Hq*hd].
 * nsplit >= 1 splits the rows over wavefronts; ws must then hold rl_op_decode_attention_ws_floats
 * floats (may be NULL for nsplit == 1).  hd in {64, 128}.  d_done: DEVICE int32 [B] or NULL; sequences with a non-zero
 * flag (ended, Section 2.1) are skipped: their cache is not read and their rows of out are left as they are.
 * With kscale / vscale the matrix-core kernel serves head_dim 128 with a multiple of 8 query heads per kv head, the vector
 * kernel everything else. */
int rl_op_decode_attention(const float *q, const uint16_t *kc, const uint16_t *vc, const int32_t *d_len, int32_t len_stride,
                           uint16_t *out, float *ws, int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit,
                           const int32_t *d_done, const float *kscale, const float *vscale, uint16_t *out_lo, void *hip_stream);
size_t rl_op_decode_attention_ws_floats(int32_t B, int32_t Hq, int32_t hd, int32_t nsplit);

/* rl_op_decode_attention for callers that cannot allocate or pass a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same operation, same kernels and same results; the split partials (the `ws` of
 * rl_op_decode_attention) live in a scratch array of RL_OP_NOALLOC_SCRATCH_BYTES that is part of the library's code object on
 * every GPU (held until the process ends).  The call allocates nothing and calls no allocating routine; on its first use
 * on a device it looks the array's address up (hipGetSymbolAddress) -- make that first call outside a stream capture.
 * RL_GEN_E_CAPACITY (text in rl_gen_last_error(NULL)) when rl_op_decode_attention_ws_floats(B, Hq, hd, nsplit) * 4 exceeds the
 * scratch size.  All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (different streams
 * or host threads) race on it; calls that follow each other on one stream do not. */
#define RL_OP_NOALLOC_SCRATCH_BYTES (16u << 20)
int rl_op_decode_attention_noalloc(const float *q, const uint16_t *kc, const uint16_t *vc, const int32_t *d_len, int32_t len_stride,
                                   uint16_t *out, int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit,
                                   const int32_t *d_done, const float *kscale, const float *vscale, uint16_t *out_lo,
                                   void *hip_stream);

/* The same attention over a paged cache (Section 7 names paged attention as a technique the generation backend can
 * take in).  k_pool / v_pool: DEVICE f16 [n_pages][Hkv][page_size][hd]; table: DEVICE int32 [B, table_stride], entry
 * (b, i) = pool page that holds positions i*page_size .. of sequence b; page_size a power of two in [16, 4096],
 * table_stride * page_size >= S.  Entries for positions 0 .. d_len[b] are read and must name pages inside the pool:
 * they are not checked.  The result equals rl_op_decode_attention on the same rows bit for bit. */
int rl_op_decode_attention_paged(const float *q, const uint16_t *k_pool, const uint16_t *v_pool, const int32_t *table,
                                 int32_t table_stride, int32_t page_size, const int32_t *d_len, int32_t len_stride, uint16_t *out,
                                 float *ws, int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit,
                                 const float *kscale, const float *vscale, void *hip_stream);

/* Rotary embedding + KV-cache append + decode attention in one kernel (what a decode step runs): q, k and v of the
 * new token of every sequence are taken from qkv -- nsplit_qkv fp32 partials, each [B, (Hq+2Hkv)*hd] laid out
 * q | k | v per row, split_stride elements apart (multiple of 4) -- added, q and k rotated at position d_len[b * len_stride] with
 * rope_tab, the k/v rows rounded to f16 and stored at that position of kc / vc (f16 [n_seq][Hkv][S][hd], WRITTEN),
 * and attention runs over positions 0 .. d_len[0] with the new row taken from registers.  out, ws, nsplit as in
 * rl_op_decode_attention.  d_len[0] >= S: nothing is written (the host checks capacity before a step). */
int rl_op_decode_attention_fused(const float *qkv, int32_t nsplit_qkv, size_t split_stride, const float *rope_tab,
                                 int32_t rope_style, uint16_t *kc, uint16_t *vc, const int32_t *d_len, int32_t len_stride,
                                 uint16_t *out, float *ws,
                                 int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit, void *hip_stream);

/* Prefill attention: causal attention of positions 0..T-1 of nb sequences; sequence i reads cache
 * sequence b0 + i.  q f16 [nb*T, Hq*hd] (rotated), kc, vc f16 (or block-scaled: each element then enters the matrix cores
 * as a two-term half sum, and so do the probabilities; q_lo, optional and for block-scaled rows only, is the second half term
 * of q, laid out like q), out f16 [nb*T, Hq*hd].  hd in {64, 128}. */
int rl_op_prefill_attention(const uint16_t *q, const uint16_t *kc, const uint16_t *vc, uint16_t *out, int32_t nb,
                            int32_t b0, int32_t T, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, const float *kscale,
                            const float *vscale, uint16_t *out_lo, const uint16_t *q_lo, void *hip_stream);

/* Greedy token: next[b] = lowest index of the largest of logits[b, 0..V-1]; -1 if the row has a NaN. */
int rl_op_argmax(const float *logits, int32_t B, int32_t V, int32_t *next, void *hip_stream);

/* Temperature sampling by inversion: next[b] = smallest v with sum_{i<=v} e_i > u[b] * sum_i e_i, e_i = exp((logits[b,i] -
 * max_i logits[b,i]) / temperature); u fp32 [B] in [0, 1); temperature > 0; -1 if the row has a NaN.  fp32 sums in a fixed
 * order (deterministic); a draw within rounding distance of a step of the cumulative distribution may land on either side. */
int rl_op_sample(const float *logits, int32_t B, int32_t V, float temperature, const float *u, int32_t *next, void *hip_stream);

/* Log-probability of the following token (Section 2.1, inference call): for the M rows g = m_first .. m_first+M-1 of
 * a flattened [n_seq, T] token grid, out[g] = logits[g - m_first, tokens[g+1]] - log sum_v exp(logits[g - m_first, v]);
 * rows with g % T == T-1 (no following token) get 0.  logits fp32 [M, V] with row stride ld; tokens int32, indexed
 * up to m_first + M (ids outside [0, V) are clamped); out fp32, indexed by g. */
int rl_op_logprob_gather(const float *logits, int64_t ld, int32_t M, int32_t V, const int32_t *tokens, int32_t T,
                         int64_t m_first, float *out, void *hip_stream);

/* Plain device-to-device copy of `bytes` bytes (multiple of 16; 16-byte aligned pointers), 16 bytes per
 * lane.  Not a step of the method: a kernel of exactly known traffic that the benchmark profiles next
 * to the real kernels to scale hardware byte counters. */
int rl_op_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RL_GEN_OPS_H */
