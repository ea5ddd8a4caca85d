/*
 * rl_gen.h -- C ABI of the MI355X (gfx950) library for the actor's batched autoregressive
 * generation: prefill plus per-token decode of a LLaMA-architecture decoder with a KV cache.
 *
 * The operation is the "Generation" model function call of the paper (Section 2.1, RLHF workflow):
 * a prefill forward pass over all prompt tokens yields the first generated token; the decode phase
 * then feeds the single latest token of every sequence and yields the next one, repeatedly.
 * The workload is fixed-length (Appendix A, experiment details): all sequences of a batch have the
 * same prompt length and generation never stops early.  The weight inventory follows the paper's
 * model-configuration table: untied input/output embeddings, bias-free projections, NumKVHeads may
 * be smaller than NumAttentionHeads (grouped-query attention).
 *
 * Conventions
 *   - Every pointer marked DEVICE is HIP device memory of the current device, allocated by the
 *     caller (for example through torch) and BORROWED: it must stay valid while the handle lives.
 *     The library allocates no device memory except bf16 copies of fp32 weights (weight_dtype 0).
 *   - `hip_stream` is a hipStream_t passed as void*; NULL is the default stream.  Calls enqueue work
 *     on that stream and return without synchronising; results are ready when the stream reaches
 *     that point.  One handle must not be used from two streams or two host threads at once.
 *   - Return value: RL_GEN_OK (0) or a negative rl_gen_status.  A failed call leaves the sequence
 *     state (batch, length) unchanged.  No exception crosses this boundary.
 *   - Number formats: weights are bf16 (as given) and are widened to IEEE half inside the kernels, or
 *     once per generation phase into the fragment-order copies of rl_gen_pack_weights (exact for
 *     |w| >= 2^-14); activations that feed a projection are IEEE half (same size as bf16, 11 instead of
 *     8 significant bits), as one term or as a two-term sum hi + lo (see rl_gen_shape.precision); the KV
 *     cache holds 16-bit elements, IEEE half or block-scaled fixed point (see rl_gen_shape.precision);
 *     the residual stream, normalisation statistics, softmax, accumulators and logits are fp32.
 *   - Range: fp32 -> half conversions saturate at +-65504 (never inf).  Activations that feed a
 *     projection (normalised rows times gain, attention outputs, SwiGLU outputs) are exact to half
 *     precision while their magnitude stays below 65504 and saturate beyond; NaN is never produced from
 *     finite inputs.  Block-scaled cache rows have no such limit (the scale is fp32).
 *   - Matrices are row-major [out_features, in_features]; token ids are int32 in [0, vocab) --
 *     ids outside that range are clamped on the device (no fault), the result is then unspecified.
 */
#ifndef RL_GEN_H
#define RL_GEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rl_gen rl_gen_t; /* opaque, library-owned */

typedef enum {
    RL_GEN_OK = 0,
    RL_GEN_E_NULL = -1,     /* a required pointer is NULL */
    RL_GEN_E_SHAPE = -2,    /* inconsistent or unsupported model shape / argument value */
    RL_GEN_E_CAPACITY = -3, /* batch, sequence length or an arena exceeds what was reserved */
    RL_GEN_E_STATE = -4,    /* call order violated (decode before prefill, ...) */
    RL_GEN_E_HIP = -5       /* a HIP runtime call failed; text in rl_gen_last_error() */
} rl_gen_status;

typedef struct {
    int32_t n_layers, hidden, n_heads, n_kv_heads, head_dim, ffn, vocab;
    float rope_base; /* rotary base, 10000 for the benchmark shapes */
    float rms_eps;   /* added to the mean square inside the square root */
    int32_t rope_style;   /* 0: pairs (2r, 2r+1) of a head rotate together; 1: pairs (r, r + head_dim/2) */
    int32_t weight_dtype; /* 0: fp32 (converted once to bf16 at create), 1: bf16 */
    int32_t max_batch;    /* KV capacity in sequences */
    int32_t max_seq;      /* KV capacity in tokens per sequence (prompt + generated) */
    int32_t precision;    /* which 16-bit roundings the path keeps; the logit error against an fp64 evaluation grows with
                           * depth and width, and the stated tolerance (max-abs 3e-2) needs more care for deeper models:
                           *  1  activations enter the QKV projection as a two-term half sum; everything else that is
                           *     stored in 16 bits is one IEEE half; KV cache IEEE half
                           *  2  as 1, and the attention output enters the O projection and the SwiGLU output the down
                           *     projection as two-term sums; the KV cache rows are 16-bit block-scaled fixed point
                           *     (int16 elements, one fp32 scale per position and kv head: about 15 significant bits at the
                           *     same 2 bytes per element); grouped-query shapes that the matrix-core decode attention
                           *     serves (head_dim 128 with 4 or a multiple of 8 query heads per kv head) keep IEEE half
                           *  3  as 2, and the FFN-norm output enters gate/up and the final-norm output the LM head as
                           *     two-term sums; block-scaled KV cache for every shape
                           *  0  automatic: 3 for more than 32 layers or hidden above 4096, else 2 */
} rl_gen_shape;

/* The level a shape's `precision` field resolves to (1, 2 or 3; negative status on an invalid shape), and whether the KV
 * cache of such a handle holds block-scaled rows (1) or IEEE half rows (0). */
int rl_gen_precision_level(const rl_gen_shape *shape);
int rl_gen_kv_block_scaled(const rl_gen_shape *shape);

/* Supported shapes: hidden == n_heads*head_dim, n_heads % n_kv_heads == 0, n_heads/n_kv_heads <= 16,
 * head_dim in {64, 128}, hidden % 8 == 0, ffn % 8 == 0, all counts positive (n_layers may be 0). */

typedef struct {                 /* all DEVICE, borrowed, dtype given by weight_dtype */
    const void *tok_emb;         /* [vocab, hidden] */
    const void *const *attn_norm; /* HOST array of n_layers DEVICE pointers, each [hidden] */
    const void *const *wq;       /* each [n_heads*head_dim, hidden] */
    const void *const *wk;       /* each [n_kv_heads*head_dim, hidden] */
    const void *const *wv;       /* each [n_kv_heads*head_dim, hidden] */
    const void *const *wo;       /* each [hidden, n_heads*head_dim] */
    const void *const *ffn_norm; /* each [hidden] */
    const void *const *w_gate;   /* each [ffn, hidden] */
    const void *const *w_up;     /* each [ffn, hidden] */
    const void *const *w_down;   /* each [hidden, ffn] */
    const void *final_norm;      /* [hidden] */
    const void *lm_head;         /* [vocab, hidden] */
} rl_gen_weights;

/* Closed forms (host only, no GPU needed).  Return 0 / negative on an invalid shape. */
int64_t rl_gen_param_count(const rl_gen_shape *shape); /* parameters of the model-configuration table's inventory */
size_t rl_gen_kv_bytes(const rl_gen_shape *shape);     /* bytes of the KV arena: 2*L*max_batch*Hkv*max_seq*head_dim*2, plus 4
                                                          per cache row (head_dim elements) when rows are block-scaled */
size_t rl_gen_work_bytes(const rl_gen_shape *shape);   /* bytes of the activation workspace arena */
int rl_gen_validate_shape(const rl_gen_shape *shape);  /* RL_GEN_OK or RL_GEN_E_SHAPE */

/* Creates a handle.  kv_arena / work_arena: DEVICE, 256-byte aligned, at least rl_gen_kv_bytes /
 * rl_gen_work_bytes long (else RL_GEN_E_CAPACITY), contents need not be initialised.  The host
 * arrays inside `weights` are copied; the device tensors they point to are borrowed.
 * KV layout inside the arena: [layer][K|V][sequence][kv_head][position][head_dim], 16-bit elements (IEEE half or int16);
 * block-scaled caches keep their fp32 row scales behind all rows, [layer][K|V][sequence][kv_head][position]. */
int rl_gen_create(const rl_gen_shape *shape, const rl_gen_weights *weights, void *kv_arena, size_t kv_bytes,
                  void *work_arena, size_t work_bytes, rl_gen_t **out);

/* Fragment-order copies of the projection matrices for the decode step.  A decode step multiplies only one
 * row per sequence with every weight matrix, so it lives off streaming the weights once; rl_gen_pack_weights
 * re-lays the borrowed matrices Wq, Wk, Wv, Wo, down of every layer and the LM head into packed_arena
 * (DEVICE, 256-byte aligned, at least rl_gen_packed_bytes long, caller-owned, borrowed while the handle
 * lives) in the order the matrix cores read them (IEEE half; layout in rl_gen_ops.h), enqueued on
 * hip_stream.  Afterwards steps of at most 256 rows (decode, short prefills) read the copies of these
 * matrices instead of the row-major weights; prefills of 1024 rows or more read them as the B operand of the large
 * tile kernel (copied global -> LDS directly; same bits as without).  Call it again after the weights changed (a training step
 * between two generation phases); packed_arena == NULL detaches the copies.  Results are the same to fp32
 * summation order with and without the copies.  Use the same stream as for the following steps, or
 * synchronise in between. */
size_t rl_gen_packed_bytes(const rl_gen_shape *shape);
/* The same plus copies of the gate/up pair of every layer.  Whatever an arena holds beyond rl_gen_packed_bytes goes
 * to gate/up pairs, layer by layer from layer 0 ((full - base) / n_layers bytes each; rl_gen_packed_gate_up_layers tells
 * how many the last rl_gen_pack_weights re-laid).  Every step then runs the fused gate/up projection of those layers
 * from the copies: up to 128 rows and FFN widths up to 16384 with a kernel whose sums are formed in the order of the
 * row-major kernel's (the same bits as without copies), otherwise (more rows, wider FFNs, prefills) with the kernel of
 * the other projections (the same values to fp32 summation order).  rl_gen_prefers_packed_gate_up: 1 when the copies
 * pay for this shape (always: they cost their memory, nothing else), else 0. */
size_t rl_gen_packed_bytes_full(const rl_gen_shape *shape);
int rl_gen_prefers_packed_gate_up(const rl_gen_shape *shape);
int rl_gen_packed_gate_up_layers(const rl_gen_t *h);
int rl_gen_pack_weights(rl_gen_t *h, void *packed_arena, size_t packed_bytes, void *hip_stream);

/* Prefill (Section 2.1: one forward pass that consumes all prompt tokens and yields the first
 * generated token).  tokens: DEVICE int32 [B, T] row-major, 1 <= B <= max_batch, 1 <= T <= max_seq.
 * logits: DEVICE fp32 [B, vocab] of the LAST prompt position, or NULL.  next: DEVICE int32 [B],
 * greedy token = lowest index of the largest logit.  Replaces any previous sequence state:
 * afterwards every sequence has length T. */
int rl_gen_prefill(rl_gen_t *h, const int32_t *tokens, int32_t B, int32_t T, float *logits, int32_t *next,
                   void *hip_stream);

/* Prefill of prompts of different lengths (Appendix A notes that prompt and generation lengths vary in practice; the
 * benchmark pads to the maximum).  tokens: DEVICE int32 [B, T], sequence b holds lens[b] prompt tokens followed by
 * padding (any valid ids).  lens: DEVICE int32 [B], values clamped to [1, T] on the device.  logits / next are those of
 * each sequence's own last prompt position.  Afterwards sequence b has length lens[b] and decode steps append at each
 * sequence's own position; rl_gen_state reports T, the upper bound the capacity check uses.  All B*T rows are
 * computed; padded positions reach neither the cache nor a later result.  On a paged generator the call first reads
 * lens back (one stream synchronisation). */
int rl_gen_prefill_ragged(rl_gen_t *h, const int32_t *tokens, const int32_t *lens, int32_t B, int32_t T, float *logits,
                          int32_t *next, void *hip_stream);

/* ---- Paged KV cache -----------------------------------------------------------------------------------------------
 * Section 5.1 counts the KV cache as memory that a call holds only while it runs, and Section 7 names paged attention
 * as a technique the generation backend can take in: the cache becomes a pool of fixed-size pages, and a per-sequence
 * page list says where each run of positions lives, so a batch of sequences of different lengths occupies pool memory
 * in proportion to what each one needs rather than max_batch * max_seq.
 *
 * rl_gen_page_bytes: bytes one page takes across all layers, K and V (0 for an invalid shape or page size; page_size is
 * a power of two in [16, 4096] positions).
 * rl_gen_create_paged: as rl_gen_create, but the kv arena is a pool of floor(kv_bytes / page bytes) >= 1 pages
 * (rl_gen_pool_pages returns the count).  Before the first prefill / inference call the caller hands over the page
 * lists with rl_gen_set_block_table. */
size_t rl_gen_page_bytes(const rl_gen_shape *shape, int32_t page_size);
int rl_gen_create_paged(const rl_gen_shape *shape, const rl_gen_weights *weights, void *kv_arena, size_t kv_bytes,
                        void *work_arena, size_t work_bytes, int32_t page_size, rl_gen_t **out);
int rl_gen_pool_pages(const rl_gen_t *h);

/* Page lists.  table: HOST int32 [B, pages_per_seq], entry (b, i) = pool page holding positions i*page .. (i+1)*page-1
 * of sequence b; capacity: HOST int32 [B], positions reserved for sequence b (0 .. max_seq): only the first
 * ceil(capacity[b] / page) entries of row b are read.  Every entry read must lie in [0, pool pages) and no page may be
 * named twice, else RL_GEN_E_CAPACITY / RL_GEN_E_SHAPE and the previous lists stay.  The lists are copied to the device
 * on `hip_stream`, which is synchronised; no other call on this handle may be in flight.  Cache contents are not
 * touched, so a caller may extend a sequence (append pages, raise its capacity) or hand the pages of an ended sequence
 * to another between steps.  The calls that store cache rows check capacity on the host: prefill and the inference
 * calls need capacity[b] >= the sequence's length, a decode step needs room for one more row in every sequence the host
 * does not know to have ended (it learns about ended sequences and exact lengths in rl_gen_read_state; until then it
 * counts every sequence as growing).  A violated check returns RL_GEN_E_CAPACITY before anything is launched. */
int rl_gen_set_block_table(rl_gen_t *h, const int32_t *table, const int32_t *capacity, int32_t B, int32_t pages_per_seq,
                           void *hip_stream);

/* Host-only helper (no device work): fills table (HOST int32 [B, pages_per_seq]) with consecutive pool pages, sequence
 * after sequence, ceil(capacity[b] / page_size) each, -1 in unused entries.  Returns the number of pages used, or
 * RL_GEN_E_CAPACITY if they exceed n_pages or a sequence needs more than pages_per_seq, RL_GEN_E_SHAPE for a bad argument. */
int32_t rl_gen_plan_pages(const int32_t *capacity, int32_t B, int32_t page_size, int32_t n_pages, int32_t pages_per_seq,
                          int32_t *table);

/* End token (Section 2.1: generation runs until termination).  eos >= 0: a sequence whose returned token is eos has ended:
 * from the next step on it returns eos, its length stays, and what is fed for it is ignored (its logits are not
 * meaningful).  eos < 0 (default): sequences never end, as in the fixed-length benchmark.  Applies from the next step. */
int rl_gen_set_eos(rl_gen_t *h, int32_t eos);

/* Copies the per-sequence lengths and end flags (HOST int32 [batch] each, either may be NULL) after waiting for the
 * stream. */
int rl_gen_read_state(rl_gen_t *h, int32_t *lens, int32_t *done, void *hip_stream);

/* Batch compaction after early termination (Appendix A: prompt and generation lengths vary; Section 2.1: a sequence is
 * generated until it terminates).  Sequences that have produced the end token (rl_gen_set_eos) leave the batch; the others
 * move up, in their order, to rows 0 .. n-1, and every later rl_gen_decode_step works on n rows: an ended sequence then
 * costs nothing any more.  kept: HOST int32 [current batch], receives the old row of every new row (ascending);
 * n_kept: HOST, receives n.  tokens: DEVICE int32 [current batch] or NULL -- a buffer of per-sequence values (typically the
 * `next` of the last step) permuted in place along with the batch, so that it can feed the next step.  Synchronises the
 * stream (it has to read the end flags).  A contiguous cache moves the rows of every sequence that changes its slot
 * (bytes of its tokens so far); a paged cache moves nothing: the page lists move, the caller's own copy of them has to follow
 * `kept`, and the pages of the dropped sequences are the caller's again.  With n == current batch nothing changes; with
 * n == 0 the generator is left without sequences, as after rl_gen_reset.  Per-sequence results of later steps are
 * the same as without compaction (rows of a batch do not interact).
 * Errors: RL_GEN_E_NULL, RL_GEN_E_STATE (no sequences), RL_GEN_E_CAPACITY (more than 8192 sequences), RL_GEN_E_HIP. */
int rl_gen_compact(rl_gen_t *h, int32_t *tokens, int32_t *kept, int32_t *n_kept, void *hip_stream);

/* One decode step (Section 2.1: input the single latest token of each sequence, produce the next).
 * tokens: DEVICE int32 [B] with B as given to the last prefill -- the caller chooses what to feed
 * (the previous `next` buffer for free-running greedy generation, or reference tokens for teacher
 * forcing).  logits: DEVICE fp32 [B, vocab] or NULL.  next: DEVICE int32 [B].  tokens and next may
 * be the same buffer.  Appends one position to every sequence; RL_GEN_E_CAPACITY once length
 * would exceed max_seq, RL_GEN_E_STATE before a prefill. */
int rl_gen_decode_step(rl_gen_t *h, const int32_t *tokens, float *logits, int32_t *next, void *hip_stream);

/* The whole generation call (Section 2.1: prefill, then decode steps that feed each sequence its own latest token),
 * with the batch cut into sequential portions when it is larger than the generator (Section 4: a call may process its
 * data in several sequential micro-batches so that its active memory -- here the KV cache -- fits the device).
 * prompts: DEVICE int32 [B, P].  out: DEVICE int32 [B, G], row b = the G tokens generated for sequence b (the first by
 * the prefill, the others by G-1 decode steps; after an end token the row repeats it).  Sequences b0 .. b0+max_batch-1
 * form a portion; each portion runs prefill and all its decode steps before the next one starts, in the same cache.
 * u: DEVICE fp32 [G, B] uniform draws in [0, 1), entry (g, b) chooses token g of sequence b -- required while sampling
 * is on (rl_gen_set_sampling with a positive temperature; that call's own draw buffer is not used here), ignored
 * otherwise.  Needs P + G - 1 <= max_seq (on a paged generator: that many positions reserved for each of the first
 * min(B, max_batch) sequences).  Everything is enqueued on hip_stream; afterwards the state is that of the last portion. */
int rl_gen_generate(rl_gen_t *h, const int32_t *prompts, int32_t B, int32_t P, int32_t G, const float *u, int32_t *out,
                    void *hip_stream);

/* Inference call (Section 2.1: one forward pass over prompt + response that scores every generated token; the
 * next call after generation in the RLHF dataflow).  tokens: DEVICE int32 [B, T] row-major.  logp: DEVICE fp32
 * [B, T]: logp[b, i] = log softmax(logits of position i)[tokens[b, i+1]] for i < T-1 -- the log-probability the
 * model assigns to the token that follows position i -- and logp[b, T-1] = 0.  The [B, T, vocab] logits are never
 * handed out: the LM head runs over blocks of rows into the workspace and a gather kernel reduces each block.
 * Same limits and errors as rl_gen_prefill, and like a prefill it replaces the sequence state (afterwards every
 * sequence has length T and decode steps may follow). */
int rl_gen_logprobs(rl_gen_t *h, const int32_t *tokens, int32_t B, int32_t T, float *logp, void *hip_stream);

/* Inference call with a scalar head (Section 2.1: the Critic and Reward models score every token of prompt +
 * response with one number).  head: DEVICE [hidden], of the handle's weight dtype (bf16 bits, or fp32 when
 * weight_dtype is 0), borrowed for the call.  values: DEVICE fp32 [B, T]: values[b, i] = head . (final RMSNorm of
 * the residual stream at position i), the normalised row rounded to half as for the LM head.  The decoder
 * weights are the handle's; limits, errors and the effect on the sequence state are those of rl_gen_logprobs. */
int rl_gen_values(rl_gen_t *h, const int32_t *tokens, int32_t B, int32_t T, const void *head, float *values, void *hip_stream);

/* Whether decode steps are replayed as one captured HIP graph (1, default) or launched kernel by
 * kernel (0).  Both produce identical results. */
int rl_gen_set_graph(rl_gen_t *h, int32_t enabled);

/* Sampling instead of the greedy choice (Section 2.1: the generation call samples the next token).  temperature > 0:
 * prefill and decode steps return next[b] = the smallest v whose cumulative softmax(logits[b] / temperature) exceeds
 * u[b], with u: DEVICE fp32 [max_batch] of uniform draws in [0, 1), borrowed until the next call of this function;
 * the caller refreshes its contents between steps (in stream order) -- the library draws no random numbers.
 * temperature <= 0 (u may be NULL): back to greedy.  Takes effect from the next step. */
int rl_gen_set_sampling(rl_gen_t *h, float temperature, const float *u);

/* Number of half-precision terms in which the normalised activations reach the QKV projection: 2 (default;
 * the projection runs on the stacked rows [h; h - half(h)] and k, v, q carry ~22-bit activations) or 1 (faster,
 * less accurate: the projection that feeds the KV cache is the rounding the logits are most sensitive to).
 * Takes effect from the next prefill / decode step. */
int rl_gen_set_qkv_terms(rl_gen_t *h, int32_t terms);

/* Forgets all sequences (weights and arenas stay).  Host-side only. */
int rl_gen_reset(rl_gen_t *h);
/* Current state: number of sequences and tokens per sequence (0, 0 before a prefill). */
int rl_gen_state(const rl_gen_t *h, int32_t *batch, int32_t *length);
/* Waits for the handle's pending work and releases library-owned memory.  NULL is accepted. */
void rl_gen_destroy(rl_gen_t *h);
/* Text of the last error of this handle (or of the last failed create when h is NULL).
 * Static storage, not thread-safe. */
const char *rl_gen_last_error(const rl_gen_t *h);

/* ---- per-kernel timing (used by the benchmark to report the roofline of single kernels) --------
 * While profiling is on, every kernel launch of prefill/decode is bracketed by HIP events on the
 * caller's stream and decode steps are not graph-replayed.  rl_gen_profile_read synchronises the
 * stream, then fills, for each kernel class id < RL_GEN_N_KERNEL_CLASSES, the number of launches
 * and the summed duration in milliseconds since profiling was switched on, and clears the sums. */
enum {
    RL_GEN_K_EMBED = 0, RL_GEN_K_ADD_RMSNORM, RL_GEN_K_GEMM_QKV, RL_GEN_K_ROPE_APPEND, RL_GEN_K_DECODE_ATTN,
    RL_GEN_K_ATTN_MERGE, RL_GEN_K_PREFILL_ATTN, RL_GEN_K_GEMM_O, RL_GEN_K_GEMM_GATE_UP, RL_GEN_K_GEMM_DOWN,
    RL_GEN_K_GEMM_LM_HEAD, RL_GEN_K_ARGMAX, RL_GEN_K_MISC, RL_GEN_N_KERNEL_CLASSES
};
int rl_gen_profile(rl_gen_t *h, int32_t enabled);
int rl_gen_profile_read(rl_gen_t *h, int32_t *launches /*HOST [N_KERNEL_CLASSES]*/,
                        float *milliseconds /*HOST [N_KERNEL_CLASSES]*/, void *hip_stream);
const char *rl_gen_kernel_class_name(int32_t id);

#ifdef __cplusplus
}
#endif
#endif /* RL_GEN_H */
