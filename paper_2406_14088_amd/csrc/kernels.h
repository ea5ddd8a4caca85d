// Host-side launch wrappers of the gfx950 kernels (one per step of the generation hot path).
// All pointers are device pointers; every launcher only enqueues work on `st`.
#pragma once
#include "common.h"

// ---- elementwise.hip -------------------------------------------------------------------------
// x[m, :] = widen(emb[clamp(tokens[m]), :])                      tokens int32 [M], emb bf16 [vocab, d], x fp32 [M, d]
void launch_embed(const int32_t *tokens, const bf16_t *emb, float *x, int M, int d, int vocab, hipStream_t st);
// x[m, :] += sum_s part[s*part_stride + m*d + :]  (nsplit may be 0);  y = gain * x / sqrt(mean(x^2) + eps);
// h[m, :] = half(y); if h_lo is given, h_lo[m, :] = half(y - h[m, :]) (two-term split: h + h_lo carries ~22 bits of y)
void launch_add_rmsnorm(float *x, const float *part, int nsplit, size_t part_stride, const bf16_t *gain, float eps,
                        f16_t *h, f16_t *h_lo, int M, int d, hipStream_t st);
// Sums the split partials of the fused QKV projection, rotates q and k heads at their positions and
// writes q (fp32 and/or half, [M, Hq*hd]) and the cache rows.  Row m is sequence b0 + m / T at
// position d_pos0[(m / T) * pos_stride] + m % T (pos_stride 0: one start position for all; 1: one per sequence).  rope_tab: fp32 [max_seq, hd/2, 2] (cos, sin).
// kc / vc: this layer's K and V areas (half), laid out as `map` says (default: slabs [max_batch][Hkv][S][hd]).
// d_valid (optional, indexed by sequence): only the first clamp(d_valid[b], 1, T) rows of a sequence reach the cache.
// d_done (optional, indexed by sequence): sequences with a non-zero flag store no cache row (q is still written).
void launch_rope_append(const float *qkv, int nsplit, size_t split_stride, int M, int T, int b0, const int32_t *d_pos0,
                        int pos_stride, const float *rope_tab, int rope_style, int Hq, int Hkv, int hd, int S, float *q_f32,
                        f16_t *q_f16, f16_t *kc, f16_t *vc, hipStream_t st, KvMap map = KvMap(),
                        const int32_t *d_valid = nullptr, const int32_t *d_done = nullptr,
                        f16_t *q_f16_lo = nullptr);  // optional: second half term of q, half(q - half(q)), laid out like q_f16
// next[b] = lowest index of the largest logit of row b (-1 if the row holds a NaN).  Optional bookkeeping per sequence
// (lens, done may be NULL; eos < 0: no end token): a sequence with done[b] returns eos and does not grow; otherwise
// lens[b] += 1 and done[b] = (next[b] == eos).
void launch_argmax(const float *logits, int B, int V, int32_t *next, int32_t *lens, int32_t *done, int eos, hipStream_t st);
// lens[b] = clamp(lens_in[b], 1, T) (T if lens_in is NULL), done[b] = 0
void launch_init_state(int32_t *lens, int32_t *done, int B, const int32_t *lens_in, int T, hipStream_t st);
// out[i, :] = h[i * T + clamp(lens[b0 + i], 1, T) - 1, :]  (half rows of d elements, d % 8 == 0)
// Batch compaction (ended sequences leave the batch): the per-sequence state and, optionally, a token buffer permuted in
// place (row i <- row kept[i], kept ascending), and one sequence's cache rows copied to another slot of a contiguous cache.
int compact_state_max_batch();
void launch_compact_state(int32_t *lens, int32_t *done, int32_t *tokens, const int32_t *kept, int n, hipStream_t st);
void launch_kv_move(f16_t *kv, float *scales, size_t area_elems, int n_areas, int Hkv, int S, int hd, int src, int dst, int rows,
                    hipStream_t st);
// Second half of the fused greedy choice: token of row b = column of the largest candidate (lowest column on ties, -1 if a
// candidate is NaN), then the same end-token and length bookkeeping as launch_argmax.
void launch_argmax_merge(const float *cand_val, const int32_t *cand_idx, int B, int tiles, int32_t *next, int32_t *lens, int32_t *done,
                         int eos, hipStream_t st);
void launch_gather_last_rows(const f16_t *h, const int32_t *lens, int b0, int nb, int T, int d, f16_t *out, hipStream_t st);
// next[b] = smallest v with cumulative softmax(logits[b] / temperature) above u[b] (-1 on NaN); bookkeeping as launch_argmax.
void launch_sample(const float *logits, int B, int V, float temperature, const float *u, int32_t *next, int32_t *lens,
                   int32_t *done, int eos, hipStream_t st);
void launch_set_i32(int32_t *p, int32_t v, hipStream_t st);
// dst[i * dst_stride] = src[i * src_stride] for i < n; 32-bit elements of any type, strides in elements
void launch_copy_strided(const void *src, int64_t src_stride, void *dst, int64_t dst_stride, int n, hipStream_t st);
// out[m] = sum_k h[m, k] * w[k]   (h half [M, d]; w bf16 or fp32 [d]; fp32 accumulation)
void launch_rowdot(const f16_t *h, const f16_t *h_lo, const void *w, int w_is_f32, int M, int d, float *out, hipStream_t st);
// Rows m_first .. m_first + M - 1 of a [n_seq * T] token grid: out[g] = log softmax(logits[g - m_first, :])[tokens[g + 1]],
// 0 for the last position of a sequence.  logits fp32 [M, V] with row stride ld.
void launch_logprob_gather(const float *logits, int64_t ld, int M, int V, const int32_t *tokens, int T, int64_t m_first,
                           float *out, hipStream_t st);
// dst[i] = bf16(src[i])  (round to nearest even)
void launch_f32_to_bf16(const float *src, bf16_t *dst, size_t n, hipStream_t st);

// dst[0 .. bytes) = src[0 .. bytes)  (bytes rounded down to a multiple of 16)
void launch_copy(const void *src, void *dst, size_t bytes, hipStream_t st);

// ---- gemm_skinny.hip / gemm_tiled.hip ----------------------------------------------------------
// C[m, off_i + n] = sum_k A[m, k] * W_i[n, k]  for up to three weight matrices W_i ([rows_i, K] bf16,
// row-major) laid side by side along the output columns (off_0 = 0, off_1 = rows_0, ...).
// Activations A are half; weights are widened bf16 -> half inside the kernels (exact for normal halves)
// and multiplied on the f16 matrix cores with fp32 accumulation.
enum GemmEpilogue {
    EPI_F32 = 0,    // out fp32: split s writes out + s*split_stride, element [m*ldc + col]
    EPI_SWIGLU = 1, // W_0 = gate, W_1 = up (same shape): out half [m*ldc + n] = silu(gate) * up; splits must be 1
    EPI_F32_ACC = 2, // out fp32 [m*ldc + col] += result (residual add); splits must be 1
    EPI_ROPE = 3,    // tiled kernel only: W_0, W_1, W_2 = Wq, Wk, Wv; the result is rotated and stored as launch_rope_append
                     // would store it (q half, cache rows), without the fp32 round trip; see RopeEpilogue
    EPI_ROPE_BS = 4  // chosen by the launcher for EPI_ROPE when RopeEpilogue::map names row scales: block-scaled cache rows, and
                     // q with its low half term
};
// What the EPI_ROPE epilogue needs: row m of the product is sequence b0 + m / T at position m % T (a prefill from
// position 0).  head_dim 128 and rotary style 1 (element e pairs with e + 64) only; every W_i holds whole heads.
struct RopeEpilogue {
    const float *rope_tab;  // [S, 64, 2] (cos, sin)
    int T, b0, Hq, Hkv, S;
    f16_t *q_f16;           // [M, Hq * 128]
    f16_t *q_f16_lo = nullptr;  // optional: second half term of q, half(q - half(q)), same layout
    f16_t *kc, *vc;         // this layer's K and V areas, laid out as `map` says
    KvMap map;
    const int32_t *d_valid; // optional, as in launch_rope_append
};
struct GemmArgs {
    const f16_t *A;       // [M, K] half, row stride lda (elements)
    const f16_t *A_lo = nullptr;  // tiled kernel only: second term of the activations (same shape and stride, above A within
                                  // 3.75 GB): out = (A + A_lo) W^T, computed as one contraction over [A | A_lo] x [W | W]
    int64_t lda;
    const bf16_t *W[3];
    int rows[3];          // rows of each W_i (0 for unused)
    int M, K;
    void *out;
    int64_t ldc;          // row stride of out (elements)
    size_t split_stride;  // elements between split partials (EPI_F32)
    int splits;           // split-K factor (>= 1)
    int epilogue;
    const RopeEpilogue *rope = nullptr;  // EPI_ROPE
    // tiled kernel only, optional: fragment-order half copies of W[0..2] (as written by launch_pack_weights).  When every
    // W_i has one, large tiles copy both operands global -> LDS directly instead of staging them through registers.
    const f16_t *P[3] = {nullptr, nullptr, nullptr};
    f16_t *out_lo = nullptr;  // EPI_SWIGLU of the tiled kernel, optional: second half term of the result, laid out like out
};
// M <= 256: weights stream through registers exactly once, activations are staged in LDS.
void launch_gemm_skinny(const GemmArgs &a, hipStream_t st);
// any M: both operands tiled through LDS (the prefill path).
void launch_gemm_tiled(const GemmArgs &a, hipStream_t st);
int gemm_skinny_default_splits(int M, int N, int K);
bool gemm_tiled_rope_supported(int M, int K, int64_t lda, int Hq, int Hkv, int hd, int rope_style, int T, bool two_terms);

// ---- gemm_packed.hip -----------------------------------------------------------------------------
// Weights re-laid-out once in matrix-core fragment order: P[ceil(N/32)][ceil(K/16)][64 lanes][8] halves, lane l of
// fragment (nb, ks) = W[32 nb + (l & 31), 16 ks + 8 (l >> 5) + 0..7], zero outside W.
size_t packed_weight_bytes(int N, int K);
void launch_pack_weights(const bf16_t *W, f16_t *P, int N, int K, hipStream_t st);  // K % 8 == 0
struct PackedGemmArgs {
    const f16_t *A;       // [M, K] half, row stride lda (elements)
    const f16_t *A_lo;    // optional second term of the activations (same shape and stride): out = (A + A_lo) W^T
    int64_t lda;
    const f16_t *P[3];    // packed matrices, side by side along the output columns as in GemmArgs
    int rows[3];
    int M, K;
    void *out;
    int64_t ldc;
    size_t split_stride;
    int splits;
    int epilogue;         // GemmEpilogue; EPI_SWIGLU: P[0] = gate, P[1] = up
    int nb;               // 32-column blocks per wavefront, 1 or 2 (fp32 epilogues; SwiGLU always uses 2)
    int depth;            // weight chunks in flight per wavefront: 2 or 4 (0: 2)
    int rows_per_wg;      // activation rows per workgroup: 32, 64 or 128 (0: 128); the row blocks of one tile re-read its weights from L2
    f16_t *out_lo = nullptr;  // EPI_SWIGLU, optional: second half term of the result, half(y - half(y)), laid out like out
    // EPI_F32 of one matrix without K split, optional (the LM head with a fused greedy choice): per row and per pass of 128
    // columns the largest value and its lowest column (NaN if the pass holds a NaN), [M][ceil(rows[0] / 128)] each;
    // launch_argmax_merge turns them into tokens.  no_store: the fp32 result itself is not written.
    float *cand_val = nullptr;
    int32_t *cand_idx = nullptr;
    bool no_store = false;
};
bool gemm_packed_single_launch(int N, int K);  // the matrix is served by one launch (no row slabs): candidates are possible
// M of any size (row blocks of 128 re-stream the weights; meant for M <= 256).
void launch_gemm_packed(const PackedGemmArgs &a, hipStream_t st);
// Fused gate/up projection (EPI_SWIGLU) of few rows from the copies, K halves on separate wavefronts: the sums are
// formed in the order of launch_gemm_skinny's and equal them bit for bit.  a.P[0] = gate, a.P[1] = up, a.rows[0] = F;
// a.depth: weight chunks (128 wide) in flight per wavefront, 2 or 4 (0: 4).
bool gemm_packed_swiglu_halves_supported(int F, int K);
void launch_gemm_packed_swiglu_halves(const PackedGemmArgs &a, hipStream_t st);
void gemm_packed_plan(int N, int K, int M, int *nb, int *rows_per_wg, int *splits);

// ---- attention_decode.hip ------------------------------------------------------------------------
// One new query per (sequence, query head) against cache rows 0 .. d_len[b * len_stride] (inclusive).
// q fp32 [B, Hq*hd] (already rotated); kc/vc this layer's K and V areas (half) laid out as `map` says; out half
// [B, Hq*hd].  ws: fp32 workspace of decode_attention_ws_floats(...) elements when nsplit > 1.
void launch_decode_attention(const float *q, const f16_t *kc, const f16_t *vc, const int32_t *d_len, int len_stride, f16_t *out,
                             float *ws, int B, int Hq, int Hkv, int hd, int S, int nsplit, hipStream_t st, KvMap map = KvMap(),
                             const int32_t *d_done = nullptr,   // d_done (optional): sequences with a non-zero flag are skipped
                             f16_t *out_lo = nullptr);          // out_lo (optional): half(o - half(o)), second term of the output
// Fused form: q, k, v of the new token are taken from the split-K partials of the QKV projection (each
// [B, (Hq+2Hkv)*hd], q | k | v per row): partials added, q and k rotated at position *d_len, the k/v row appended to
// the cache (kc/vc are written) and used from registers.  Replaces launch_rope_append + launch_decode_attention.
void launch_decode_attention_fused(const float *qkv, int nsplit_qkv, size_t split_stride, const float *rope_tab, int rope_style,
                                   f16_t *kc, f16_t *vc, const int32_t *d_len, int len_stride, f16_t *out, float *ws, int B, int Hq,
                                   int Hkv, int hd, int S, int nsplit, hipStream_t st);
// ---- attention_decode_gqa.hip: the same operation on the matrix cores for grouped-query shapes (head_dim 128 and 4, 8, 16,
// ... query heads per kv head); launch_decode_attention forwards to it when decode_attention_gqa_supported().
bool decode_attention_gqa_supported(int Hq, int Hkv, int hd);
bool decode_attention_gqa_takes(int Hq, int Hkv, int hd, bool block_scaled);  // supported, and faster than the vector kernel
int decode_attention_gqa_default_splits(int B, int Hq, int Hkv, int S, bool block_scaled);
void launch_decode_attention_gqa(const float *q, const f16_t *kc, const f16_t *vc, const int32_t *d_len, int len_stride,
                                 f16_t *out, float *ws, int B, int Hq, int Hkv, int S, int nsplit, hipStream_t st,
                                 KvMap map = KvMap(), const int32_t *d_done = nullptr, f16_t *out_lo = nullptr);
void launch_decode_attention_merge(const float *ws, f16_t *out, int B, int Hq, int hd, int nsplit, hipStream_t st,
                                   f16_t *out_lo = nullptr);
size_t decode_attention_ws_floats(int B, int Hq, int hd, int nsplit);
int decode_attention_default_splits(int B, int Hkv, int S);
int decode_attention_group(int g);  // query heads per wavefront for Hq/Hkv = g

// ---- attention_prefill.hip -----------------------------------------------------------------------
// Causal attention over the T prompt positions of nb sequences whose K/V already sit in the cache.
// q half [nb*T, Hq*hd] (rotated); sequence i of the chunk is cache sequence b0 + i; out half [nb*T, Hq*hd].
// d_valid (optional, indexed by cache sequence): only keys below clamp(d_valid[b], 1, T) exist; later keys count as
// zero rows with zero weight, and the output rows of later queries are unspecified (finite).
void launch_prefill_attention(const f16_t *q, const f16_t *kc, const f16_t *vc, f16_t *out, int nb, int b0, int T,
                              int Hq, int Hkv, int hd, int S, hipStream_t st, KvMap map = KvMap(),
                              const int32_t *d_valid = nullptr, f16_t *out_lo = nullptr, const f16_t *q_lo = nullptr);
