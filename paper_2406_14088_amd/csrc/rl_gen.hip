// Host side of the C ABI (include/rl_gen.h, include/rl_gen_ops.h): argument validation, arena
// carving, kernel sequencing of prefill / decode steps, HIP-graph replay of decode steps and
// per-kernel event timing.  All arithmetic of the method runs in the kernels this file launches.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "../../include/rl_gen.h"
#include "../../include/rl_gen_ops.h"
#include "kernels.h"

// Scratch memory of the entry point that allocates nothing (rl_op_decode_attention_noalloc): one array per GPU, part of the
// library's code object, held until the process ends.  In host code the array's name is a stand-in, not a device address:
// the address on the current device comes from hipGetSymbolAddress (scratch_of_current_device) and only that pointer is
// handed to kernels.
static __device__ __align__(256) unsigned char scratch[RL_OP_NOALLOC_SCRATCH_BYTES];

namespace {

char g_create_error[512] = "";

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, looked up once per device.
int scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RL_GEN_E_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return RL_GEN_E_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return RL_GEN_OK;
}

constexpr int kPrefillChunkTokens = 16384;  // prompt tokens pushed through the layers at once
constexpr int kSkinnyMaxM = 256;
constexpr int kMaxSplits = 16;
constexpr size_t kAlign = 256;
constexpr int kMinPage = 16, kMaxPage = 4096;  // positions per page of a paged cache (powers of two)

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct WorkPlan {
    size_t x, h, part, qf32, qbf, attn, act, attn_ws, logits, next, draws, rope, state, table, kept, total;
    size_t part_elems;  // floats in the split-K partial area
    int rows;  // activation rows the workspace can hold
};

int validate(const rl_gen_shape *s) {
    if (!s) return RL_GEN_E_NULL;
    if (s->n_layers < 0 || s->hidden <= 0 || s->n_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0 || s->ffn <= 0 ||
        s->vocab <= 0 || s->max_batch <= 0 || s->max_seq <= 0)
        return RL_GEN_E_SHAPE;
    if ((int64_t)s->n_heads * s->head_dim != s->hidden) return RL_GEN_E_SHAPE;
    if (s->n_heads % s->n_kv_heads != 0 || s->n_heads / s->n_kv_heads > 16) return RL_GEN_E_SHAPE;
    if (s->head_dim != 64 && s->head_dim != 128) return RL_GEN_E_SHAPE;
    if (s->hidden % 8 != 0 || s->ffn % 8 != 0 || s->hidden > 8192) return RL_GEN_E_SHAPE;
    if (s->rope_style != 0 && s->rope_style != 1) return RL_GEN_E_SHAPE;
    if (s->weight_dtype != 0 && s->weight_dtype != 1) return RL_GEN_E_SHAPE;
    if (!(s->rope_base > 0.f) || !(s->rms_eps >= 0.f)) return RL_GEN_E_SHAPE;
    if (s->precision < 0 || s->precision > 3) return RL_GEN_E_SHAPE;
    // every weight matrix is addressed through a 32-bit range-checked buffer descriptor
    const uint64_t lim = 0xffffffffull;
    if ((uint64_t)s->vocab * s->hidden * 2 > lim || (uint64_t)s->ffn * s->hidden * 2 > lim) return RL_GEN_E_SHAPE;
    return RL_GEN_OK;
}

// Which 16-bit roundings the path keeps (rl_gen_shape.precision).  The logit error against an fp64 evaluation grows
// roughly with the square root of the depth and with the width (measured, random-init weights: rms 4.7e-3 at 32 layers
// x 4096, 7.5e-3 at 40 x 5120, 2.0e-2 at 80 x 8192 on level 1; on level 2: 2.7e-3, 4.6e-3 -- the latter with a worst logit
// of 2.8e-2 --), so models deeper or wider than the 7B shape default to the most careful level.
int prec_level(const rl_gen_shape *s) {
    if (s->precision != 0) return s->precision;
    return s->n_layers > 32 || s->hidden > 4096 ? 3 : 2;
}
// Level 2 keeps half rows for the grouped-query shapes that the matrix-core decode attention serves (with 4 heads per kv
// head block-scaled rows would move them to the slower vector kernel); level 3 asks for the more exact cache everywhere.
bool kv_block_scaled(const rl_gen_shape *s) {
    const int p = prec_level(s);
    return p >= 3 || (p == 2 && !decode_attention_gqa_supported(s->n_heads, s->n_kv_heads, s->head_dim));
}
size_t kv_row_bytes(const rl_gen_shape *s) { return (size_t)s->head_dim * sizeof(f16_t) + (kv_block_scaled(s) ? sizeof(float) : 0); }

int page_shift_of(int page_size) {
    for (int sh = 4; (1 << sh) <= kMaxPage; ++sh)
        if ((1 << sh) == page_size) return sh;
    return 0;
}

int attn_splits(const rl_gen_shape *s) {
    if (decode_attention_gqa_takes(s->n_heads, s->n_kv_heads, s->head_dim, kv_block_scaled(s)))
        return decode_attention_gqa_default_splits(s->max_batch, s->n_heads, s->n_kv_heads, s->max_seq, kv_block_scaled(s));
    int g = s->n_heads / s->n_kv_heads;
    int gt = decode_attention_group(g);
    return decode_attention_default_splits(s->max_batch, s->n_kv_heads * (g / gt), s->max_seq);
}

WorkPlan plan_work(const rl_gen_shape *s) {
    WorkPlan p;
    int64_t all = (int64_t)s->max_batch * s->max_seq;
    int64_t chunk = s->max_seq > kPrefillChunkTokens ? s->max_seq : kPrefillChunkTokens;
    if (chunk > all) chunk = all;
    int64_t rows = chunk > s->max_batch ? chunk : s->max_batch;
    p.rows = (int)rows;
    size_t d = s->hidden, qd = (size_t)s->n_heads * s->head_dim, kvd = (size_t)s->n_kv_heads * s->head_dim;
    size_t nqkv = qd + 2 * kvd, nmax = nqkv > d ? nqkv : d;
    // the QKV projection may be fed the stacked two-term rows [h; h_lo]: twice the rows, twice the partials
    size_t skinny_rows = 2 * rows < kSkinnyMaxM ? (size_t)(2 * rows) : (size_t)kSkinnyMaxM;
    size_t part_elems = (size_t)2 * rows * nqkv;
    if ((size_t)kMaxSplits * skinny_rows * nmax > part_elems) part_elems = (size_t)kMaxSplits * skinny_rows * nmax;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    p.x = take((size_t)rows * d * 4);
    p.h = take((size_t)2 * rows * d * 2);
    p.part = take(part_elems * 4);
    p.part_elems = part_elems;
    p.qf32 = take((size_t)s->max_batch * qd * 4);
    p.qbf = take((size_t)2 * rows * qd * 2);    // rotated q of a prefill, and its low term behind the rows in use
    p.attn = take((size_t)2 * rows * qd * 2);   // attention output, and its low term behind the rows in use
    p.act = take((size_t)2 * rows * s->ffn * 2);  // SwiGLU output, likewise
    p.attn_ws = take(decode_attention_ws_floats(s->max_batch, s->n_heads, s->head_dim, attn_splits(s)) * 4 + 16);
    p.logits = take((size_t)s->max_batch * s->vocab * 4);
    p.next = take((size_t)s->max_batch * 4);
    p.draws = take((size_t)s->max_batch * 4);  // uniform draws of the current step of rl_gen_generate
    p.rope = take((size_t)s->max_seq * s->head_dim * 4);
    p.state = take(((size_t)2 * s->max_batch + 16) * 4);  // per-sequence lengths, per-sequence end flags, a constant 0
    p.table = take((size_t)s->max_batch * ceil_div(s->max_seq, kMinPage) * 4);  // page lists of a paged cache
    p.kept = take((size_t)s->max_batch * 4);   // batch compaction: old row of every kept sequence
    p.total = off;
    return p;
}

struct GraphEntry {
    const void *tokens, *logits, *next;
    int B;
    hipStream_t stream;
    int calls;
    hipGraphExec_t exec;
};

struct ProfEvent {
    hipEvent_t a, b;
    int cls;
};

}  // namespace

struct rl_gen {
    rl_gen_shape s;
    std::vector<const bf16_t *> lw[9];
    const bf16_t *tok_emb, *final_norm, *lm_head;
    std::vector<void *> owned;
    // fragment-order copies of the projection matrices (decode path); empty until rl_gen_pack_weights
    std::vector<const f16_t *> pw[9];
    const f16_t *p_lm_head;
    bool packed;
    int packed_gu_layers;  // layers 0 .. n-1 have fragment-order copies of the gate/up pair too (pw[W_GATE], pw[W_UP])
    f16_t *kv;
    unsigned char *work;
    WorkPlan wp;
    int nsplit_attn;
    int prec;      // resolved precision level (1..3)
    bool kv_i16;   // cache rows are 16-bit block-scaled fixed point; their fp32 scales follow all rows in the arena
    int B, len;
    bool graph_on, prof_on, qkv_two_term;
    // paged cache (rl_gen_create_paged): the kv arena is a pool of n_pages pages of 1 << page_shift positions
    int page_shift;          // 0: contiguous slabs
    int n_pages, table_stride;
    bool table_set;
    std::vector<int32_t> cap;        // HOST: positions reserved per sequence (rl_gen_set_block_table)
    std::vector<int32_t> host_len;   // HOST: upper bound of each sequence's length
    std::vector<int32_t> host_done;  // HOST: end flags as last read back
    std::vector<int32_t> table_img;  // HOST: image of the device page lists
    std::vector<int32_t> kept_img;   // HOST: source of the last compaction's copy to the device
    int eos;                 // end token (rl_gen_set_eos), -1: none
    float temperature;       // > 0: the next token is sampled (rl_gen_set_sampling); else greedy
    const float *sample_u;   // DEVICE [max_batch] uniform draws, borrowed, refreshed by the caller between steps
    std::vector<GraphEntry> graphs;
    std::vector<ProfEvent> prof_events;
    std::vector<ProfEvent> prof_pool;
    int prof_launches[RL_GEN_N_KERNEL_CLASSES];
    float prof_ms[RL_GEN_N_KERNEL_CLASSES];
    char err[512];

    float *x() const { return reinterpret_cast<float *>(work + wp.x); }
    f16_t *h() const { return reinterpret_cast<f16_t *>(work + wp.h); }
    float *part() const { return reinterpret_cast<float *>(work + wp.part); }
    float *qf32() const { return reinterpret_cast<float *>(work + wp.qf32); }
    f16_t *qbf() const { return reinterpret_cast<f16_t *>(work + wp.qbf); }
    f16_t *attn() const { return reinterpret_cast<f16_t *>(work + wp.attn); }
    f16_t *act() const { return reinterpret_cast<f16_t *>(work + wp.act); }
    float *attn_ws() const { return reinterpret_cast<float *>(work + wp.attn_ws); }
    float *logits_ws() const { return reinterpret_cast<float *>(work + wp.logits); }
    int32_t *next_ws() const { return reinterpret_cast<int32_t *>(work + wp.next); }
    float *draws_ws() const { return reinterpret_cast<float *>(work + wp.draws); }
    float *rope() const { return reinterpret_cast<float *>(work + wp.rope); }
    // device-side sequence state: tokens held per sequence, whether it has produced the end token, and a constant 0
    int32_t *d_lens() const { return reinterpret_cast<int32_t *>(work + wp.state); }
    int32_t *d_done() const { return d_lens() + s.max_batch; }
    int32_t *d_zero() const { return d_lens() + 2 * s.max_batch; }
    int32_t *d_table() const { return reinterpret_cast<int32_t *>(work + wp.table); }
    int32_t *d_kept() const { return reinterpret_cast<int32_t *>(work + wp.kept); }
    size_t area_elems() const {  // one layer's K (or V) area
        return page_shift ? ((size_t)n_pages * s.n_kv_heads << page_shift) * s.head_dim
                          : (size_t)s.max_batch * s.n_kv_heads * s.max_seq * s.head_dim;
    }
    f16_t *kslab(int l) const { return kv + (size_t)(2 * l) * area_elems(); }
    f16_t *vslab(int l) const { return kv + (size_t)(2 * l + 1) * area_elems(); }
    float *scales() const { return reinterpret_cast<float *>(kv + (size_t)2 * s.n_layers * area_elems()); }
    KvMap kvmap(int l) const {  // how layer l's K and V areas are addressed
        KvMap m;
        if (page_shift) { m.table = d_table(); m.table_stride = table_stride; m.page_shift = page_shift; }
        if (kv_i16) {
            const size_t area_rows = area_elems() / s.head_dim;
            m.kscale = scales() + (size_t)(2 * l) * area_rows;
            m.vscale = scales() + (size_t)(2 * l + 1) * area_rows;
        }
        return m;
    }
};

namespace {

enum { W_ATTN_NORM = 0, W_Q, W_K, W_V, W_O, W_FFN_NORM, W_GATE, W_UP, W_DOWN };

void set_err(rl_gen *h, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(h ? h->err : g_create_error, 512, fmt, ap);
    va_end(ap);
}

// brackets one kernel launch with events when per-kernel timing is on
struct Scope {
    rl_gen *h;
    hipStream_t st;
    ProfEvent ev;
    bool on;
    Scope(rl_gen *h_, int cls, hipStream_t st_) : h(h_), st(st_), on(h_->prof_on) {
        if (!on) return;
        if (!h->prof_pool.empty()) {
            ev = h->prof_pool.back();
            h->prof_pool.pop_back();
        } else {
            (void)hipEventCreate(&ev.a);
            (void)hipEventCreate(&ev.b);
        }
        ev.cls = cls;
        (void)hipEventRecord(ev.a, st);
    }
    ~Scope() {
        if (!on) return;
        (void)hipEventRecord(ev.b, st);
        h->prof_events.push_back(ev);
    }
};

// Projection of M <= kSkinnyMaxM rows over fragment-order weights: fp32 split-K partials in h->part().
// A_lo (optional): second term of the activations, folded into the same accumulators.
int project_packed(rl_gen *h, int cls, const f16_t *A, const f16_t *A_lo, int64_t lda, int M, int K, const f16_t *P0, int r0,
                   const f16_t *P1, int r1, const f16_t *P2, int r2, hipStream_t st) {
    PackedGemmArgs a;
    a.A = A; a.A_lo = A_lo; a.lda = lda; a.M = M; a.K = K;
    a.P[0] = P0; a.P[1] = P1; a.P[2] = P2;
    a.rows[0] = r0; a.rows[1] = r1; a.rows[2] = r2;
    int N = r0 + r1 + r2;
    int splits;
    gemm_packed_plan(N, K, M, &a.nb, &a.rows_per_wg, &splits);
    a.depth = 2;
    if (splits > kMaxSplits) splits = kMaxSplits;
    a.out = h->part(); a.ldc = N; a.split_stride = (size_t)M * N; a.splits = splits; a.epilogue = EPI_F32;
    Scope sc(h, cls, st);
    launch_gemm_packed(a, st);
    return splits;
}

// One projection.  Returns the number of fp32 partials written to h->part() (0 when the result was
// accumulated straight into `acc_out`).
// P0..P2: the matrices' fragment-order copies where they exist (the large-M kernel then copies both operands straight
// into LDS; same results).
int project(rl_gen *h, int cls, const f16_t *A, const f16_t *A_lo, int64_t lda, int M, int K, const bf16_t *W0, int r0,
            const bf16_t *W1, int r1, const bf16_t *W2, int r2, float *acc_out, int64_t ld_acc, hipStream_t st,
            const f16_t *P0 = nullptr, const f16_t *P1 = nullptr, const f16_t *P2 = nullptr) {
    GemmArgs a;
    a.A = A; a.lda = lda; a.M = M; a.K = K;
    a.A_lo = M > kSkinnyMaxM ? A_lo : nullptr;  // second activation term: large-M kernel only
    a.W[0] = W0; a.W[1] = W1; a.W[2] = W2;
    a.P[0] = P0; a.P[1] = P1; a.P[2] = P2;
    a.rows[0] = r0; a.rows[1] = r1; a.rows[2] = r2;
    int N = r0 + r1 + r2;
    Scope sc(h, cls, st);
    if (M <= kSkinnyMaxM) {
        int splits = gemm_skinny_default_splits(M, N, K);
        if (splits > kMaxSplits) splits = kMaxSplits;
        a.out = h->part(); a.ldc = N; a.split_stride = (size_t)M * N; a.splits = splits; a.epilogue = EPI_F32;
        launch_gemm_skinny(a, st);
        return splits;
    }
    if (acc_out) {
        if (a.A_lo && P0 && !W1 && !W2) {
            // two activation terms from the fragment-order copy: 128-row workgroups of the decode kernel, two per compute
            // unit (they hide each other's barriers and epilogues), run 3-6 % ahead of the tile kernel (16384 rows, 7B shape:
            // O 1.06 against 1.09 ms, down 2.47 against 2.59); with one term the tile kernel is ahead
            PackedGemmArgs q;
            q.A = A; q.A_lo = A_lo; q.lda = lda; q.M = M; q.K = K;
            q.P[0] = P0; q.P[1] = nullptr; q.P[2] = nullptr;
            q.rows[0] = r0; q.rows[1] = 0; q.rows[2] = 0;
            q.out = acc_out; q.ldc = ld_acc; q.split_stride = 0; q.splits = 1; q.epilogue = EPI_F32_ACC;
            q.nb = 2; q.rows_per_wg = 128; q.depth = 2;
            launch_gemm_packed(q, st);
            return 0;
        }
        a.out = acc_out; a.ldc = ld_acc; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_F32_ACC;
        launch_gemm_tiled(a, st);
        return 0;
    }
    a.out = h->part(); a.ldc = N; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_F32;
    launch_gemm_tiled(a, st);
    return 1;
}

// Is the fragment-order kernel the faster one for the fused gate/up projection of M rows?  The row-major kernel runs
// F / 64 workgroups that each own a compute unit, 128 rows at a time.  Measured crossovers: beyond 256 workgroups it needs
// a second, partly empty round (34B shape at 64 rows: 192 against 137 us; 70B shape at 32 rows: 219 against 163 us);
// above 128 rows it streams the weights once per 128-row block (13B shape at 256 rows: 164 against 110 us; 7B shape at
// 192 rows: 102 against 68 us); at FFN 14336 and 128 rows it is 10 % behind (63 against 57.5 us); otherwise -- the 7B
// shape at up to 128 rows -- it is level or slightly ahead (48 against 52 us at 32 rows, 54 against 55 us at 128).
bool packed_swiglu_wins(int M, int ffn) { return M > 128 || ffn > 256 * 64 || (ffn >= 14336 && M > 64); }

// Fused gate/up projection + SwiGLU of M rows into h->act().  A_lo (optional): second half term of the input; honoured by
// the kernel that reads fragment-order copies, dropped otherwise.  out_lo (optional): where the second half term of the
// result goes.  Returns whether out_lo was written (the row-major kernel for few rows has no such output).
bool swiglu_project(rl_gen *h, const f16_t *A, const f16_t *A_lo, f16_t *out_lo, int M, int l, hipStream_t st) {
    const bool copies = h->packed && l < h->packed_gu_layers;
    // Up to 128 rows and FFN widths up to 16384: the kernel that puts the K halves of each chunk on separate wavefronts (the
    // row-major kernel's sums in its order, from the copies).  Measured against the other two at 128 / 64 rows: FFN 11008
    // 46.6 us (row-major 52.2, packed 61); FFN 14336 54.0 / 49.7 us (packed 61 / 54.6, row-major 63 / 55.7).  Wider
    // FFNs (K = 8192 shapes) and more rows stay with the packed kernel (34B shape at 64 rows: 137 against 160 us).
    if (copies && !A_lo && M <= 128 && h->s.ffn <= 256 * 64 && gemm_packed_swiglu_halves_supported(h->s.ffn, h->s.hidden)) {
        PackedGemmArgs q;
        q.A = A; q.A_lo = nullptr; q.lda = h->s.hidden; q.M = M; q.K = h->s.hidden;
        q.P[0] = h->pw[W_GATE][l]; q.P[1] = h->pw[W_UP][l]; q.P[2] = nullptr;
        q.rows[0] = h->s.ffn; q.rows[1] = h->s.ffn; q.rows[2] = 0;
        q.out = h->act(); q.out_lo = out_lo; q.ldc = h->s.ffn; q.split_stride = 0; q.splits = 1; q.epilogue = EPI_SWIGLU;
        q.nb = 2; q.rows_per_wg = 128; q.depth = 2;
        Scope sc(h, RL_GEN_K_GEMM_GATE_UP, st);
        launch_gemm_packed_swiglu_halves(q, st);
        return out_lo != nullptr;
    }
    if (copies && (A_lo || packed_swiglu_wins(M, h->s.ffn))) {
        PackedGemmArgs q;
        q.A = A; q.A_lo = A_lo; q.lda = h->s.hidden; q.M = M; q.K = h->s.hidden;
        q.P[0] = h->pw[W_GATE][l]; q.P[1] = h->pw[W_UP][l]; q.P[2] = nullptr;
        q.rows[0] = h->s.ffn; q.rows[1] = h->s.ffn; q.rows[2] = 0;
        q.out = h->act(); q.out_lo = out_lo; q.ldc = h->s.ffn; q.split_stride = 0; q.splits = 1; q.epilogue = EPI_SWIGLU;
        q.nb = 2; q.rows_per_wg = M > 128 ? 128 : 64; q.depth = 2;
        Scope sc(h, RL_GEN_K_GEMM_GATE_UP, st);
        launch_gemm_packed(q, st);
        return out_lo != nullptr;
    }
    GemmArgs a;
    a.A = A; a.lda = h->s.hidden; a.M = M; a.K = h->s.hidden;
    a.W[0] = h->lw[W_GATE][l]; a.W[1] = h->lw[W_UP][l]; a.W[2] = nullptr;
    if (copies) { a.P[0] = h->pw[W_GATE][l]; a.P[1] = h->pw[W_UP][l]; }
    a.rows[0] = h->s.ffn; a.rows[1] = h->s.ffn; a.rows[2] = 0;
    a.out = h->act(); a.ldc = h->s.ffn; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_SWIGLU;
    Scope sc(h, RL_GEN_K_GEMM_GATE_UP, st);
    // the row-major kernel for few rows takes one activation term and writes one output term: with a second input term
    // the tile kernel (both terms in one contraction) serves every row count
    if (M <= kSkinnyMaxM && !A_lo) { launch_gemm_skinny(a, st); return false; }
    a.A_lo = A_lo;
    a.out_lo = out_lo;
    launch_gemm_tiled(a, st);
    return out_lo != nullptr;
}

// x += (A + A_lo) W^T for the O and down projections (N = hidden columns): through fp32 partials that the following
// add_rmsnorm adds (few rows; returns their number) or accumulated by the kernel itself (many rows; returns 0).
int project_resid(rl_gen *h, int cls, const f16_t *A, const f16_t *A_lo, int M, int K, const bf16_t *W, const f16_t *P, hipStream_t st) {
    const int d = h->s.hidden;
    if (h->packed && M <= kSkinnyMaxM) return project_packed(h, cls, A, A_lo, K, M, K, P, d, nullptr, 0, nullptr, 0, st);
    if (M > kSkinnyMaxM) return project(h, cls, A, A_lo, K, M, K, W, d, nullptr, 0, nullptr, 0, h->x(), d, st, h->packed ? P : nullptr);
    // row-major kernel for few rows: the low term sits in the rows right behind the high term ([A; A_lo], 2 M rows) and the
    // consumer adds the two row blocks of every partial like two partials
    const int terms = A_lo ? 2 : 1;
    return terms * project(h, cls, A, nullptr, K, terms * M, K, W, d, nullptr, 0, nullptr, 0, nullptr, 0, st);
}

// All layers for M = nb*T rows (sequences b0 .. b0+nb-1, T new positions each starting at *d_pos0),
// then final norm; leaves the normalised rows in h->h().  decode == (T == 1 and attention over the cache).
// d_valid (prefill of ragged prompts): per-sequence count of rows that exist; later rows never reach the cache.
// Returns whether the rows behind the first M of h->h() hold the low term of the final-norm output.
bool run_layers(rl_gen *h, const int32_t *tokens, int nb, int T, int b0, bool decode, hipStream_t st,
                const int32_t *d_valid = nullptr) {
    const rl_gen_shape &s = h->s;
    const int M = nb * T, d = s.hidden, qd = s.n_heads * s.head_dim, kvd = s.n_kv_heads * s.head_dim;
    const int L = s.n_layers;
    {
        Scope sc(h, RL_GEN_K_EMBED, st);
        launch_embed(tokens, h->tok_emb, h->x(), M, d, s.vocab, st);
    }
    // Two-term activations.  What feeds a projection is stored as IEEE half; where the level asks for it the value is kept
    // as a two-term half sum hi + lo (lo = half(y - half(y)): about 22 significant bits), the low term in the rows right
    // behind the M rows in use, and the projection multiplies both terms with the same weights.  Level 1: the attention-norm
    // output (q, k and v errors are what the logits are most sensitive to: k and v stay in the cache for every later
    // token); level 2: also the attention output and the SwiGLU output; level 3: also the FFN-norm and final-norm outputs.
    // (What a second term costs is its matrix-core time: at 128 rows about 4 us for the O projection, 10 us for down and 14 us
    // for gate/up per layer of the 7B shape.  Measured on the 7B benchmark workload, 2048 greedy decisions: level 2 as it is,
    // rms logit error 2.7e-3 and 11 disagreements with the oracle; without the second term into the down projection 3.0e-3
    // and 16 -- 20 are allowed.)
    const int terms = h->qkv_two_term ? 2 : 1;
    const bool two_o = h->prec >= 2, two_f = h->prec >= 3;
    f16_t *h_lo = h->h() + (size_t)M * d;
    f16_t *attn_lo = two_o ? h->attn() + (size_t)M * qd : nullptr;
    f16_t *act_lo = two_o ? h->act() + (size_t)M * s.ffn : nullptr;
    // a prefill over block-scaled cache rows multiplies two-term keys with two-term queries
    f16_t *q_lo = !decode && h->kv_i16 ? h->qbf() + (size_t)M * qd : nullptr;
    {
        Scope sc(h, RL_GEN_K_ADD_RMSNORM, st);
        const bool lo = L > 0 ? terms == 2 : two_f;
        launch_add_rmsnorm(h->x(), nullptr, 0, 0, L > 0 ? h->lw[W_ATTN_NORM][0] : h->final_norm, s.rms_eps, h->h(),
                           lo ? h_lo : nullptr, M, d, st);
    }
    for (int l = 0; l < L; ++l) {
        const KvMap map = h->kvmap(l);
        const bool pk = h->packed && M <= kSkinnyMaxM;
        const f16_t *hq_lo = terms == 2 ? h_lo : nullptr;
        bool qkv_stored = false;  // q and the cache rows already written by the projection itself
        int ns;
        if (pk)  // both terms go through the same weight fragments into the same accumulators
            ns = project_packed(h, RL_GEN_K_GEMM_QKV, h->h(), hq_lo, d, M, d, h->pw[W_Q][l], qd, h->pw[W_K][l], kvd, h->pw[W_V][l],
                                kvd, st);
        else if (!decode && gemm_tiled_rope_supported(M, d, d, s.n_heads, s.n_kv_heads, s.head_dim, s.rope_style, T, hq_lo != nullptr) &&
                 (!hq_lo || (size_t)(hq_lo - h->h()) * 2 < 0x70000000ull)) {
            // prefill: the projection's epilogue rotates q and k and stores q and the cache rows itself
            RopeEpilogue rp;
            rp.rope_tab = h->rope(); rp.T = T; rp.b0 = b0; rp.Hq = s.n_heads; rp.Hkv = s.n_kv_heads; rp.S = s.max_seq;
            rp.q_f16 = h->qbf(); rp.q_f16_lo = q_lo; rp.kc = h->kslab(l); rp.vc = h->vslab(l); rp.map = map; rp.d_valid = d_valid;
            GemmArgs a;
            a.A = h->h(); a.A_lo = hq_lo; a.lda = d; a.M = M; a.K = d;
            a.W[0] = h->lw[W_Q][l]; a.W[1] = h->lw[W_K][l]; a.W[2] = h->lw[W_V][l];
            if (h->packed) { a.P[0] = h->pw[W_Q][l]; a.P[1] = h->pw[W_K][l]; a.P[2] = h->pw[W_V][l]; }
            a.rows[0] = qd; a.rows[1] = kvd; a.rows[2] = kvd;
            a.out = nullptr; a.ldc = 0; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_ROPE; a.rope = &rp;
            {
                Scope sc(h, RL_GEN_K_GEMM_QKV, st);
                launch_gemm_tiled(a, st);
            }
            qkv_stored = true;
            ns = 0;
        } else if (M > kSkinnyMaxM)  // large-M kernel: one contraction over [h | h_lo] x [W | W]
            ns = project(h, RL_GEN_K_GEMM_QKV, h->h(), hq_lo, d, M, d, h->lw[W_Q][l], qd, h->lw[W_K][l], kvd, h->lw[W_V][l], kvd,
                         nullptr, 0, st, h->packed ? h->pw[W_Q][l] : nullptr, h->packed ? h->pw[W_K][l] : nullptr,
                         h->packed ? h->pw[W_V][l] : nullptr);
        else  // row-major skinny kernel: stacked rows [h; h_lo], the consumer adds the two row blocks
            ns = terms * project(h, RL_GEN_K_GEMM_QKV, h->h(), nullptr, d, terms * M, d, h->lw[W_Q][l], qd, h->lw[W_K][l], kvd,
                                 h->lw[W_V][l], kvd, nullptr, 0, st);
        if (!qkv_stored) {
            Scope sc(h, RL_GEN_K_ROPE_APPEND, st);
            launch_rope_append(h->part(), ns, (size_t)M * (qd + 2 * kvd), M, T, b0, decode ? h->d_lens() : h->d_zero(),
                               decode ? 1 : 0, h->rope(), s.rope_style, s.n_heads, s.n_kv_heads, s.head_dim, s.max_seq,
                               decode ? h->qf32() : nullptr, decode ? nullptr : h->qbf(), h->kslab(l), h->vslab(l), st, map,
                               d_valid, decode && h->eos >= 0 ? h->d_done() : nullptr,  // without an end token no sequence ever ends
                               q_lo);
        }
        // (A single kernel that takes q, k, v from the partials, rotates, appends and attends exists --
        // launch_decode_attention_fused -- but measured no faster per step: what the separate kernel costs, the
        // attention wavefronts then spend before their first cache load.)
        if (decode) {
            Scope sc(h, RL_GEN_K_DECODE_ATTN, st);
            launch_decode_attention(h->qf32(), h->kslab(l), h->vslab(l), h->d_lens(), 1, h->attn(), h->attn_ws(), nb,
                                    s.n_heads, s.n_kv_heads, s.head_dim, s.max_seq, h->nsplit_attn, st, map,
                                    h->eos >= 0 ? h->d_done() : nullptr, attn_lo);  // ended sequences cost no cache traffic
        } else {
            Scope sc(h, RL_GEN_K_PREFILL_ATTN, st);
            launch_prefill_attention(h->qbf(), h->kslab(l), h->vslab(l), h->attn(), nb, b0, T, s.n_heads, s.n_kv_heads,
                                     s.head_dim, s.max_seq, st, map, d_valid, attn_lo, q_lo);
        }
        ns = project_resid(h, RL_GEN_K_GEMM_O, h->attn(), attn_lo, M, qd, h->lw[W_O][l], h->packed ? h->pw[W_O][l] : nullptr, st);
        {
            Scope sc(h, RL_GEN_K_ADD_RMSNORM, st);
            launch_add_rmsnorm(h->x(), h->part(), ns, (size_t)M * d, h->lw[W_FFN_NORM][l], s.rms_eps, h->h(), two_f ? h_lo : nullptr, M, d, st);
        }
        const bool have_act_lo = swiglu_project(h, h->h(), two_f ? h_lo : nullptr, act_lo, M, l, st);
        ns = project_resid(h, RL_GEN_K_GEMM_DOWN, h->act(), have_act_lo ? act_lo : nullptr, M, s.ffn, h->lw[W_DOWN][l],
                           h->packed ? h->pw[W_DOWN][l] : nullptr, st);
        {
            Scope sc(h, RL_GEN_K_ADD_RMSNORM, st);
            const bool lo = l + 1 < L ? terms == 2 : two_f;
            launch_add_rmsnorm(h->x(), h->part(), ns, (size_t)M * d, l + 1 < L ? h->lw[W_ATTN_NORM][l + 1] : h->final_norm,
                               s.rms_eps, h->h(), lo ? h_lo : nullptr, M, d, st);
        }
    }
    return two_f;
}

// logits[b0 + i, :] = lm_head * h[row i*T + T-1]  for i < nb
// (rows: optional compact [nb, hidden] rows to use instead -- the last valid position of ragged sequences)
// lo: the rows behind the nb*T rows of h->h() hold the low term of the normalised rows (level 3); the kernel that reads the
// fragment-order copy multiplies both terms, the row-major kernels use the high term alone.
// Fused greedy choice: the LM-head projection also leaves, per row and per pass of 128 vocabulary columns, its largest logit
// and that logit's column (candidates), and a one-wavefront-per-row kernel picks the token from them: the [B, V] logits are
// neither re-read nor, when the caller did not ask for them, written at all.  Applies when the projection runs from the
// fragment-order copy in one launch with at most kSkinnyMaxM rows (every decode step and prefill chunk of the benchmark
// shapes) and the token is chosen greedily; the candidates live in the internal logits area, which is idle exactly then
// (the caller's buffer takes the logits, or nobody wants them).
bool greedy_fusable(const rl_gen *h, int rows_per_call) {
    return h->temperature <= 0.f && h->packed && rows_per_call <= kSkinnyMaxM && gemm_packed_single_launch(h->s.vocab, h->s.hidden) &&
           (size_t)2 * ceil_div(h->s.vocab, 128) <= (size_t)h->s.vocab;
}
float *cand_val_of(const rl_gen *h) { return h->logits_ws(); }
int32_t *cand_idx_of(const rl_gen *h) {
    return reinterpret_cast<int32_t *>(h->logits_ws() + (size_t)h->s.max_batch * ceil_div(h->s.vocab, 128));
}

// fuse: 0 plain logits; 1 logits and candidates; 2 candidates only (the logits are not stored)
void lm_head(rl_gen *h, int nb, int T, int b0, float *logits, hipStream_t st, const f16_t *rows = nullptr, bool lo = false,
             int fuse = 0) {
    const rl_gen_shape &s = h->s;
    GemmArgs a;
    a.A = h->h() + (size_t)(T - 1) * s.hidden; a.lda = (int64_t)T * s.hidden; a.M = nb; a.K = s.hidden;
    if (rows) { a.A = rows; a.lda = s.hidden; }
    a.W[0] = h->lm_head; a.W[1] = nullptr; a.W[2] = nullptr;
    a.rows[0] = s.vocab; a.rows[1] = 0; a.rows[2] = 0;
    a.out = logits + (size_t)b0 * s.vocab; a.ldc = s.vocab; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_F32;
    // low term of the final-norm output: behind the nb * T rows of h, or behind the nb gathered rows
    const f16_t *A_lo = !lo ? nullptr : rows ? rows + (size_t)nb * s.hidden : a.A + (size_t)nb * T * s.hidden;
    Scope sc(h, RL_GEN_K_GEMM_LM_HEAD, st);
    if (h->packed && nb <= kSkinnyMaxM) {
        PackedGemmArgs q;
        q.A = a.A; q.A_lo = A_lo; q.lda = a.lda; q.M = nb; q.K = s.hidden;
        q.P[0] = h->p_lm_head; q.P[1] = nullptr; q.P[2] = nullptr;
        q.rows[0] = s.vocab; q.rows[1] = 0; q.rows[2] = 0;
        q.out = a.out; q.ldc = s.vocab; q.split_stride = 0; q.splits = 1; q.epilogue = EPI_F32; q.nb = 1; q.rows_per_wg = 128; q.depth = 2;
        if (fuse) {
            const size_t tiles = (size_t)ceil_div(s.vocab, 128);
            q.cand_val = cand_val_of(h) + (size_t)b0 * tiles;
            q.cand_idx = cand_idx_of(h) + (size_t)b0 * tiles;
            q.no_store = fuse == 2;
        }
        launch_gemm_packed(q, st);
    } else if (nb <= kSkinnyMaxM && !A_lo) launch_gemm_skinny(a, st);
    else { a.A_lo = A_lo; launch_gemm_tiled(a, st); }
}

// logits: where the step's logits go (the caller's buffer or the internal one); wanted: the caller asked for them
void enqueue_decode(rl_gen *h, const int32_t *tokens, float *logits, bool wanted, int32_t *next, hipStream_t st) {
    const bool lo = run_layers(h, tokens, h->B, 1, 0, true, st);
    const bool fused = greedy_fusable(h, h->B);
    lm_head(h, h->B, 1, 0, logits, st, nullptr, lo, fused ? (wanted ? 1 : 2) : 0);
    Scope sc(h, RL_GEN_K_ARGMAX, st);
    if (h->temperature > 0.f)
        launch_sample(logits, h->B, h->s.vocab, h->temperature, h->sample_u, next, h->d_lens(), h->d_done(), h->eos, st);
    else if (fused)
        launch_argmax_merge(cand_val_of(h), cand_idx_of(h), h->B, ceil_div(h->s.vocab, 128), next, h->d_lens(), h->d_done(), h->eos, st);
    else
        launch_argmax(logits, h->B, h->s.vocab, next, h->d_lens(), h->d_done(), h->eos, st);
}

int check_hip(rl_gen *h, const char *where) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_err(h, "%s: %s", where, hipGetErrorString(e));
        return RL_GEN_E_HIP;
    }
    return RL_GEN_OK;
}

// Retires every captured decode step.  Replays may still be queued on the stream they were launched on, and nothing
// promises that an executable graph outlives its destruction while in flight: wait for that stream first.
void drop_graphs(rl_gen *h) {
    for (auto &g : h->graphs)
        if (g.exec) {
            (void)hipStreamSynchronize(g.stream);
            (void)hipGraphExecDestroy(g.exec);
        }
    h->graphs.clear();
}

}  // namespace

extern "C" {

int rl_gen_validate_shape(const rl_gen_shape *shape) { return validate(shape); }

int64_t rl_gen_param_count(const rl_gen_shape *s) {
    if (!s) return RL_GEN_E_NULL;
    if (s->n_layers < 0 || s->hidden <= 0 || s->n_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0 || s->ffn <= 0 ||
        s->vocab <= 0)
        return RL_GEN_E_SHAPE;
    int64_t d = s->hidden, qd = (int64_t)s->n_heads * s->head_dim, kvd = (int64_t)s->n_kv_heads * s->head_dim;
    int64_t emb = 2 * (int64_t)s->vocab * d;                      // input and output embeddings, untied
    int64_t attn = qd * d + 2 * kvd * d + d * qd;                 // Wq, Wk, Wv, Wo
    int64_t ffn = 3 * d * (int64_t)s->ffn;                        // gate, up, down
    return emb + (int64_t)s->n_layers * (attn + ffn + 2 * d) + d;  // + two gains per layer + final gain
}

size_t rl_gen_kv_bytes(const rl_gen_shape *s) {
    if (validate(s) != RL_GEN_OK) return 0;
    return (size_t)2 * s->n_layers * s->max_batch * s->n_kv_heads * s->max_seq * kv_row_bytes(s);
}

int rl_gen_precision_level(const rl_gen_shape *s) { return validate(s) != RL_GEN_OK ? RL_GEN_E_SHAPE : prec_level(s); }
int rl_gen_kv_block_scaled(const rl_gen_shape *s) { return validate(s) != RL_GEN_OK ? RL_GEN_E_SHAPE : (kv_block_scaled(s) ? 1 : 0); }

size_t rl_gen_work_bytes(const rl_gen_shape *s) {
    if (validate(s) != RL_GEN_OK) return 0;
    return plan_work(s).total;
}

// packed arena: per layer Wq, Wk, Wv, Wo, down; then the LM head; then the gate/up pairs of the first gu_layers layers.
// Every matrix is 256-byte aligned.
constexpr int kPackedPerLayer = 5;
static size_t packed_pair_bytes(const rl_gen_shape *s) { return 2 * align_up(packed_weight_bytes(s->ffn, s->hidden)); }
static size_t packed_plan(const rl_gen_shape *s, std::vector<size_t> *offs, int gu_layers) {
    const int d = s->hidden, qd = s->n_heads * s->head_dim, kvd = s->n_kv_heads * s->head_dim;
    const int NK[kPackedPerLayer][2] = {{qd, d}, {kvd, d}, {kvd, d}, {d, qd}, {d, s->ffn}};
    size_t off = 0;
    for (int l = 0; l < s->n_layers; ++l)
        for (int m = 0; m < kPackedPerLayer; ++m) {
            if (offs) offs->push_back(off);
            off += align_up(packed_weight_bytes(NK[m][0], NK[m][1]));
        }
    if (offs) offs->push_back(off);
    off += align_up(packed_weight_bytes(s->vocab, d));
    for (int l = 0; l < gu_layers; ++l)
        for (int m = 0; m < 2; ++m) {
            if (offs) offs->push_back(off);
            off += align_up(packed_weight_bytes(s->ffn, d));
        }
    return off;
}

size_t rl_gen_packed_bytes(const rl_gen_shape *s) {
    if (validate(s) != RL_GEN_OK) return 0;
    return packed_plan(s, nullptr, 0);
}

size_t rl_gen_packed_bytes_full(const rl_gen_shape *s) {
    if (validate(s) != RL_GEN_OK) return 0;
    return packed_plan(s, nullptr, s->n_layers);
}

int rl_gen_prefers_packed_gate_up(const rl_gen_shape *s) {
    if (validate(s) != RL_GEN_OK) return RL_GEN_E_SHAPE;
    // The prefill projection (thousands of rows) is faster from the copies at every width measured (7B shape, 16384
    // rows: 2.88 against 3.09 ms per layer); steps of few rows use them where packed_swiglu_wins says so.
    return 1;
}

int rl_gen_pack_weights(rl_gen_t *h, void *packed_arena, size_t packed_bytes, void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    drop_graphs(h);  // captured decode steps hold the old weight pointers
    if (!packed_arena) {
        h->packed = false;
        h->packed_gu_layers = 0;
        return RL_GEN_OK;
    }
    const rl_gen_shape &s = h->s;
    const size_t base_bytes = packed_plan(&s, nullptr, 0);
    if (packed_bytes < base_bytes) { set_err(h, "rl_gen_pack_weights: arena too small (%zu < %zu)", packed_bytes, base_bytes); return RL_GEN_E_CAPACITY; }
    if ((uintptr_t)packed_arena % kAlign) { set_err(h, "rl_gen_pack_weights: arena not 256-byte aligned"); return RL_GEN_E_SHAPE; }
    // what the arena holds beyond the five matrices per layer and the LM head goes to gate/up pairs, layer by layer
    const size_t pair = packed_pair_bytes(&s);
    int gu_layers = pair ? (int)((packed_bytes - base_bytes) / pair < (size_t)s.n_layers ? (packed_bytes - base_bytes) / pair : (size_t)s.n_layers) : 0;
    std::vector<size_t> offs;
    packed_plan(&s, &offs, gu_layers);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int d = s.hidden, qd = s.n_heads * s.head_dim, kvd = s.n_kv_heads * s.head_dim;
    const int which[kPackedPerLayer] = {W_Q, W_K, W_V, W_O, W_DOWN};
    const int NK[kPackedPerLayer][2] = {{qd, d}, {kvd, d}, {kvd, d}, {d, qd}, {d, s.ffn}};
    unsigned char *base = reinterpret_cast<unsigned char *>(packed_arena);
    for (int m = 0; m < kPackedPerLayer; ++m) h->pw[which[m]].assign(s.n_layers, nullptr);
    h->pw[W_GATE].assign(s.n_layers, nullptr);
    h->pw[W_UP].assign(s.n_layers, nullptr);
    size_t i = 0;
    for (int l = 0; l < s.n_layers; ++l)
        for (int m = 0; m < kPackedPerLayer; ++m, ++i) {
            f16_t *dst = reinterpret_cast<f16_t *>(base + offs[i]);
            launch_pack_weights(h->lw[which[m]][l], dst, NK[m][0], NK[m][1], st);
            h->pw[which[m]][l] = dst;
        }
    f16_t *dst = reinterpret_cast<f16_t *>(base + offs[i++]);
    launch_pack_weights(h->lm_head, dst, s.vocab, d, st);
    h->p_lm_head = dst;
    for (int l = 0; l < gu_layers; ++l)
        for (int m = 0; m < 2; ++m, ++i) {
            const int w = m == 0 ? W_GATE : W_UP;
            f16_t *dst2 = reinterpret_cast<f16_t *>(base + offs[i]);
            launch_pack_weights(h->lw[w][l], dst2, s.ffn, d, st);
            h->pw[w][l] = dst2;
        }
    int rc = check_hip(h, "rl_gen_pack_weights");
    if (rc != RL_GEN_OK) return rc;
    h->packed = true;
    h->packed_gu_layers = gu_layers;
    return RL_GEN_OK;
}

int rl_gen_packed_gate_up_layers(const rl_gen_t *h) { return h ? h->packed_gu_layers : RL_GEN_E_NULL; }

size_t rl_gen_page_bytes(const rl_gen_shape *s, int32_t page_size) {
    if (validate(s) != RL_GEN_OK || !page_shift_of(page_size)) return 0;
    return (size_t)2 * s->n_layers * s->n_kv_heads * page_size * kv_row_bytes(s);
}

int32_t rl_gen_plan_pages(const int32_t *capacity, int32_t B, int32_t page_size, int32_t n_pages, int32_t pages_per_seq,
                          int32_t *table) {
    if (!capacity || !table) return RL_GEN_E_NULL;
    if (B < 0 || !page_shift_of(page_size) || n_pages < 0 || pages_per_seq < 0) return RL_GEN_E_SHAPE;
    int64_t used = 0;
    for (int b = 0; b < B; ++b) {
        if (capacity[b] < 0) return RL_GEN_E_SHAPE;
        int64_t need = ((int64_t)capacity[b] + page_size - 1) / page_size;
        if (need > pages_per_seq || used + need > n_pages) return RL_GEN_E_CAPACITY;
        for (int i = 0; i < pages_per_seq; ++i) table[(size_t)b * pages_per_seq + i] = i < need ? (int32_t)(used + i) : -1;
        used += need;
    }
    return (int32_t)used;
}

static int create_impl(const rl_gen_shape *shape, const rl_gen_weights *w, void *kv_arena, size_t kv_bytes, void *work_arena,
                       size_t work_bytes, int page_size, rl_gen_t **out) {
    if (!shape || !w || !out) { set_err(nullptr, "rl_gen_create: NULL argument"); return RL_GEN_E_NULL; }
    *out = nullptr;
    int rc = validate(shape);
    if (rc != RL_GEN_OK) { set_err(nullptr, "rl_gen_create: unsupported shape"); return rc; }
    const int L = shape->n_layers;
    const void *const *arrs[9] = {w->attn_norm, w->wq, w->wk, w->wv, w->wo, w->ffn_norm, w->w_gate, w->w_up, w->w_down};
    if (!w->tok_emb || !w->final_norm || !w->lm_head) { set_err(nullptr, "rl_gen_create: NULL weight"); return RL_GEN_E_NULL; }
    for (int a = 0; a < 9; ++a) {
        if (L > 0 && !arrs[a]) { set_err(nullptr, "rl_gen_create: NULL weight array"); return RL_GEN_E_NULL; }
        for (int l = 0; l < L; ++l)
            if (!arrs[a][l]) { set_err(nullptr, "rl_gen_create: NULL layer weight"); return RL_GEN_E_NULL; }
    }
    const int page_shift = page_size ? page_shift_of(page_size) : 0;
    if (page_size && !page_shift) {
        set_err(nullptr, "rl_gen_create_paged: page size must be a power of two in [%d, %d]", kMinPage, kMaxPage);
        return RL_GEN_E_SHAPE;
    }
    // paged: any whole number of pages (at least one) makes a pool
    size_t need_kv = page_shift ? rl_gen_page_bytes(shape, page_size) : rl_gen_kv_bytes(shape);
    WorkPlan wp = plan_work(shape);
    if ((need_kv > 0 && !kv_arena) || !work_arena) { set_err(nullptr, "rl_gen_create: NULL arena"); return RL_GEN_E_NULL; }
    if (kv_bytes < need_kv || work_bytes < wp.total) {
        set_err(nullptr, "rl_gen_create: arena too small (kv %zu < %zu or work %zu < %zu)", kv_bytes, need_kv, work_bytes, wp.total);
        return RL_GEN_E_CAPACITY;
    }
    if (((uintptr_t)kv_arena | (uintptr_t)work_arena) % kAlign) { set_err(nullptr, "rl_gen_create: arena not 256-byte aligned"); return RL_GEN_E_SHAPE; }

    rl_gen *h = new rl_gen();
    h->s = *shape;
    h->kv = reinterpret_cast<f16_t *>(kv_arena);
    h->work = reinterpret_cast<unsigned char *>(work_arena);
    h->wp = wp;
    h->nsplit_attn = attn_splits(shape);
    h->prec = prec_level(shape);
    h->kv_i16 = kv_block_scaled(shape);
    h->B = 0; h->len = 0;
    h->graph_on = true; h->prof_on = false; h->qkv_two_term = true;
    h->packed = false; h->packed_gu_layers = 0; h->p_lm_head = nullptr;
    h->temperature = 0.f; h->sample_u = nullptr; h->eos = -1;
    h->page_shift = page_shift; h->n_pages = 0; h->table_stride = 0; h->table_set = false;
    if (page_shift) {
        h->table_stride = ceil_div(shape->max_seq, page_size);
        // a model without layers has no cache: any page number up to what the lists can name is accepted
        int64_t n = need_kv ? (int64_t)(kv_bytes / need_kv) : (int64_t)shape->max_batch * h->table_stride;
        h->n_pages = (int)(n < 0x7fffffff ? n : 0x7fffffff);
    }
    h->err[0] = 0;
    memset(h->prof_launches, 0, sizeof h->prof_launches);
    memset(h->prof_ms, 0, sizeof h->prof_ms);

    // weights: borrow bf16, convert fp32 once
    const size_t d = shape->hidden, qd = (size_t)shape->n_heads * shape->head_dim, kvd = (size_t)shape->n_kv_heads * shape->head_dim;
    const size_t elems[9] = {d, qd * d, kvd * d, kvd * d, d * qd, d, (size_t)shape->ffn * d, (size_t)shape->ffn * d, d * (size_t)shape->ffn};
    bool fail = false;
    auto adopt = [&](const void *p, size_t n) -> const bf16_t * {
        if (shape->weight_dtype == 1) return reinterpret_cast<const bf16_t *>(p);
        void *dst = nullptr;
        if (hipMalloc(&dst, n * sizeof(bf16_t)) != hipSuccess) { fail = true; return nullptr; }
        h->owned.push_back(dst);
        launch_f32_to_bf16(reinterpret_cast<const float *>(p), reinterpret_cast<bf16_t *>(dst), n, nullptr);
        return reinterpret_cast<const bf16_t *>(dst);
    };
    h->tok_emb = adopt(w->tok_emb, (size_t)shape->vocab * d);
    h->final_norm = adopt(w->final_norm, d);
    h->lm_head = adopt(w->lm_head, (size_t)shape->vocab * d);
    for (int a = 0; a < 9 && !fail; ++a) {
        h->lw[a].resize(L);
        for (int l = 0; l < L && !fail; ++l) h->lw[a][l] = adopt(arrs[a][l], elems[a]);
    }
    // rotary table (fp64 on the host) and the device-side state words
    if (!fail) {
        std::vector<float> tab((size_t)shape->max_seq * shape->head_dim);
        int half = shape->head_dim / 2;
        for (int pos = 0; pos < shape->max_seq; ++pos)
            for (int r = 0; r < half; ++r) {
                double ang = (double)pos * pow((double)shape->rope_base, -2.0 * r / (double)shape->head_dim);
                tab[((size_t)pos * half + r) * 2] = (float)cos(ang);
                tab[((size_t)pos * half + r) * 2 + 1] = (float)sin(ang);
            }
        if (hipMemcpy(h->rope(), tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemset(h->d_lens(), 0, ((size_t)2 * shape->max_batch + 16) * 4) != hipSuccess ||
            hipMemset(h->d_table(), 0, (size_t)shape->max_batch * ceil_div(shape->max_seq, kMinPage) * 4) != hipSuccess)
            fail = true;
    }
    if (!fail && hipDeviceSynchronize() != hipSuccess) fail = true;
    if (fail || hipGetLastError() != hipSuccess) {
        set_err(nullptr, "rl_gen_create: HIP failure while preparing weights/tables");
        for (void *p : h->owned) (void)hipFree(p);
        delete h;
        return RL_GEN_E_HIP;
    }
    *out = h;
    return RL_GEN_OK;
}

int rl_gen_create(const rl_gen_shape *shape, const rl_gen_weights *w, void *kv_arena, size_t kv_bytes, void *work_arena,
                  size_t work_bytes, rl_gen_t **out) {
    return create_impl(shape, w, kv_arena, kv_bytes, work_arena, work_bytes, 0, out);
}

int rl_gen_create_paged(const rl_gen_shape *shape, const rl_gen_weights *w, void *kv_arena, size_t kv_bytes, void *work_arena,
                        size_t work_bytes, int32_t page_size, rl_gen_t **out) {
    if (page_size == 0) { set_err(nullptr, "rl_gen_create_paged: page size 0"); return RL_GEN_E_SHAPE; }
    return create_impl(shape, w, kv_arena, kv_bytes, work_arena, work_bytes, page_size, out);
}

int rl_gen_pool_pages(const rl_gen_t *h) { return h ? h->n_pages : RL_GEN_E_NULL; }

int rl_gen_set_block_table(rl_gen_t *h, const int32_t *table, const int32_t *capacity, int32_t B, int32_t pages_per_seq,
                           void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    if (!h->page_shift) { set_err(h, "rl_gen_set_block_table: the cache of this generator is not paged"); return RL_GEN_E_STATE; }
    if (!table || !capacity) { set_err(h, "rl_gen_set_block_table: NULL argument"); return RL_GEN_E_NULL; }
    if (B <= 0 || B > h->s.max_batch || pages_per_seq <= 0) {
        set_err(h, "rl_gen_set_block_table: B=%d (max %d), pages_per_seq=%d", B, h->s.max_batch, pages_per_seq);
        return RL_GEN_E_SHAPE;
    }
    const int page = 1 << h->page_shift;
    std::vector<int32_t> img((size_t)h->s.max_batch * h->table_stride, 0);
    std::vector<unsigned char> taken((size_t)h->n_pages, 0);
    for (int b = 0; b < B; ++b) {
        if (capacity[b] < 0 || capacity[b] > h->s.max_seq) {
            set_err(h, "rl_gen_set_block_table: capacity[%d]=%d outside [0, %d]", b, capacity[b], h->s.max_seq);
            return RL_GEN_E_CAPACITY;
        }
        const int need = ceil_div(capacity[b], page);
        if (need > pages_per_seq) {
            set_err(h, "rl_gen_set_block_table: sequence %d needs %d pages, the table has %d per sequence", b, need, pages_per_seq);
            return RL_GEN_E_SHAPE;
        }
        for (int i = 0; i < need; ++i) {
            const int32_t pg = table[(size_t)b * pages_per_seq + i];
            if (pg < 0 || pg >= h->n_pages) {
                set_err(h, "rl_gen_set_block_table: page %d of sequence %d is %d, the pool has %d pages", i, b, pg, h->n_pages);
                return RL_GEN_E_CAPACITY;
            }
            if (taken[pg]) {
                set_err(h, "rl_gen_set_block_table: pool page %d is named twice", pg);
                return RL_GEN_E_SHAPE;
            }
            taken[pg] = 1;
            img[(size_t)b * h->table_stride + i] = pg;
        }
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    h->table_img.swap(img);  // the copy source must outlive the copy
    if (hipMemcpyAsync(h->d_table(), h->table_img.data(), h->table_img.size() * 4, hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        set_err(h, "rl_gen_set_block_table: copy failed");
        h->table_set = false;
        return RL_GEN_E_HIP;
    }
    h->cap.assign(capacity, capacity + B);
    h->table_set = true;
    return RL_GEN_OK;
}

// Paged cache: every one of the B sequences must have `need` positions reserved.
static int check_reserved(rl_gen_t *h, const char *who, int B, int need) {
    if (!h->page_shift) return RL_GEN_OK;
    if (!h->table_set || (int)h->cap.size() < B) {
        set_err(h, "%s: the page lists cover %d sequences, %d needed (rl_gen_set_block_table)", who,
                h->table_set ? (int)h->cap.size() : 0, B);
        return RL_GEN_E_STATE;
    }
    for (int b = 0; b < B; ++b)
        if (h->cap[b] < need) {
            set_err(h, "%s: sequence %d has %d positions reserved, %d needed", who, b, h->cap[b], need);
            return RL_GEN_E_CAPACITY;
        }
    return RL_GEN_OK;
}

static int prefill_impl(rl_gen_t *h, const char *who, const int32_t *tokens, const int32_t *lens, int32_t B, int32_t T,
                        float *logits, int32_t *next, void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    if (!tokens) { set_err(h, "%s: NULL tokens", who); return RL_GEN_E_NULL; }
    if (B <= 0 || T <= 0) { set_err(h, "%s: B and T must be positive", who); return RL_GEN_E_SHAPE; }
    if (B > h->s.max_batch || T > h->s.max_seq) {
        set_err(h, "%s: B=%d T=%d exceed capacity %d x %d", who, B, T, h->s.max_batch, h->s.max_seq);
        return RL_GEN_E_CAPACITY;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (h->page_shift) {
        // the host has to know how long each sequence is: it checks every later step against the reserved pages
        std::vector<int32_t> hl((size_t)B, T);
        if (lens) {
            if (hipMemcpyAsync(hl.data(), lens, (size_t)B * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
                hipStreamSynchronize(st) != hipSuccess) { set_err(h, "%s: reading lens failed", who); return RL_GEN_E_HIP; }
            for (auto &n : hl) n = n < 1 ? 1 : (n > T ? T : n);
        }
        int rc = check_reserved(h, who, B, 0);
        if (rc != RL_GEN_OK) return rc;
        for (int b = 0; b < B; ++b)
            if (hl[b] > h->cap[b]) {
                set_err(h, "%s: sequence %d holds %d tokens, %d positions reserved", who, b, hl[b], h->cap[b]);
                return RL_GEN_E_CAPACITY;
            }
        h->host_len.swap(hl);
        h->host_done.assign((size_t)B, 0);
    }
    float *lg = logits ? logits : h->logits_ws();
    int32_t *nx = next ? next : h->next_ws();
    {
        Scope sc(h, RL_GEN_K_MISC, st);
        launch_init_state(h->d_lens(), h->d_done(), B, lens, T, st);
    }
    int per_chunk = h->wp.rows / T;  // whole sequences per pass through the layers
    if (per_chunk < 1) per_chunk = 1;
    const bool fused = greedy_fusable(h, B < per_chunk ? B : per_chunk);
    const int fuse = fused ? (logits ? 1 : 2) : 0;
    for (int b0 = 0; b0 < B; b0 += per_chunk) {
        int nb = B - b0 < per_chunk ? B - b0 : per_chunk;
        const bool lo = run_layers(h, tokens + (size_t)b0 * T, nb, T, b0, false, st, lens ? h->d_lens() : nullptr);
        if (lens) {
            // ragged prompts: the row that feeds the LM head is each sequence's own last position; the attention
            // output area is idle by now and takes the gathered rows
            {
                Scope sc(h, RL_GEN_K_MISC, st);
                launch_gather_last_rows(h->h(), h->d_lens(), b0, nb, T, h->s.hidden, h->attn(), st);
                if (lo)
                    launch_gather_last_rows(h->h() + (size_t)nb * T * h->s.hidden, h->d_lens(), b0, nb, T, h->s.hidden,
                                            h->attn() + (size_t)nb * h->s.hidden, st);
            }
            lm_head(h, nb, T, b0, lg, st, h->attn(), lo, fuse);
        } else {
            lm_head(h, nb, T, b0, lg, st, nullptr, lo, fuse);
        }
    }
    {
        Scope sc(h, RL_GEN_K_ARGMAX, st);
        // lengths were set by launch_init_state; here only the end flags follow from the first generated token
        if (h->temperature > 0.f) launch_sample(lg, B, h->s.vocab, h->temperature, h->sample_u, nx, nullptr, h->d_done(), h->eos, st);
        else if (fused) launch_argmax_merge(cand_val_of(h), cand_idx_of(h), B, ceil_div(h->s.vocab, 128), nx, nullptr, h->d_done(), h->eos, st);
        else launch_argmax(lg, B, h->s.vocab, nx, nullptr, h->d_done(), h->eos, st);
    }
    int rc = check_hip(h, who);
    if (rc != RL_GEN_OK) return rc;
    h->B = B; h->len = T;
    return RL_GEN_OK;
}

int rl_gen_prefill(rl_gen_t *h, const int32_t *tokens, int32_t B, int32_t T, float *logits, int32_t *next, void *hip_stream) {
    return prefill_impl(h, "rl_gen_prefill", tokens, nullptr, B, T, logits, next, hip_stream);
}

int rl_gen_prefill_ragged(rl_gen_t *h, const int32_t *tokens, const int32_t *lens, int32_t B, int32_t T, float *logits,
                          int32_t *next, void *hip_stream) {
    if (h && !lens) { set_err(h, "rl_gen_prefill_ragged: NULL lens"); return RL_GEN_E_NULL; }
    return prefill_impl(h, "rl_gen_prefill_ragged", tokens, lens, B, T, logits, next, hip_stream);
}

int rl_gen_set_eos(rl_gen_t *h, int32_t eos) {
    if (!h) return RL_GEN_E_NULL;
    if (eos >= h->s.vocab) { set_err(h, "rl_gen_set_eos: token %d outside the vocabulary", eos); return RL_GEN_E_SHAPE; }
    drop_graphs(h);  // the end token is a kernel argument of captured steps
    h->eos = eos < 0 ? -1 : eos;
    return RL_GEN_OK;
}

int rl_gen_read_state(rl_gen_t *h, int32_t *lens, int32_t *done, void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (h->B <= 0) return RL_GEN_OK;
    if (h->page_shift) {  // the host-side bounds become exact: ended sequences stop counting against their pages
        h->host_len.resize((size_t)h->B);
        h->host_done.resize((size_t)h->B);
        if (hipMemcpyAsync(h->host_len.data(), h->d_lens(), (size_t)h->B * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipMemcpyAsync(h->host_done.data(), h->d_done(), (size_t)h->B * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) { set_err(h, "rl_gen_read_state: stream error"); return RL_GEN_E_HIP; }
        if (lens) memcpy(lens, h->host_len.data(), (size_t)h->B * 4);
        if (done) memcpy(done, h->host_done.data(), (size_t)h->B * 4);
        return RL_GEN_OK;
    }
    if (lens && hipMemcpyAsync(lens, h->d_lens(), (size_t)h->B * 4, hipMemcpyDeviceToHost, st) != hipSuccess) return RL_GEN_E_HIP;
    if (done && hipMemcpyAsync(done, h->d_done(), (size_t)h->B * 4, hipMemcpyDeviceToHost, st) != hipSuccess) return RL_GEN_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) { set_err(h, "rl_gen_read_state: stream error"); return RL_GEN_E_HIP; }
    return RL_GEN_OK;
}

int rl_gen_compact(rl_gen_t *h, int32_t *tokens, int32_t *kept, int32_t *n_kept, void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    if (!kept || !n_kept) { set_err(h, "rl_gen_compact: NULL argument"); return RL_GEN_E_NULL; }
    if (h->B <= 0) { set_err(h, "rl_gen_compact: no sequences (prefill first)"); return RL_GEN_E_STATE; }
    if (h->B > compact_state_max_batch()) {
        set_err(h, "rl_gen_compact: batches of up to %d sequences are served, this one has %d", compact_state_max_batch(), h->B);
        return RL_GEN_E_CAPACITY;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int B = h->B;
    std::vector<int32_t> lens((size_t)B), done((size_t)B);
    if (hipMemcpyAsync(lens.data(), h->d_lens(), (size_t)B * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipMemcpyAsync(done.data(), h->d_done(), (size_t)B * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) { set_err(h, "rl_gen_compact: stream error"); return RL_GEN_E_HIP; }
    int n = 0;
    for (int b = 0; b < B; ++b)
        if (!done[b]) kept[n++] = b;
    *n_kept = n;
    if (n == B) {  // nobody has ended; the host-side bounds of a paged cache become exact on the way
        if (h->page_shift) { h->host_len = lens; h->host_done = done; }
        return RL_GEN_OK;
    }
    if (n == 0) {  // everybody has ended: an empty batch, as before the first prefill
        h->B = 0; h->len = 0;
        return RL_GEN_OK;
    }
    h->kept_img.assign(kept, kept + n);  // the copy source must outlive the copy
    bool ok = hipMemcpyAsync(h->d_kept(), h->kept_img.data(), (size_t)n * 4, hipMemcpyHostToDevice, st) == hipSuccess;
    if (h->page_shift) {
        // a paged cache moves no rows: the page lists of the kept sequences move up
        const size_t stride = (size_t)h->table_stride;
        std::vector<int32_t> img(h->table_img.size(), 0), cap((size_t)n), hl((size_t)n);
        for (int i = 0; i < n; ++i) {
            memcpy(&img[(size_t)i * stride], &h->table_img[(size_t)kept[i] * stride], stride * 4);
            cap[(size_t)i] = h->cap[(size_t)kept[i]];
            hl[(size_t)i] = lens[(size_t)kept[i]];
        }
        h->table_img.swap(img);
        h->cap.swap(cap);
        h->host_len.swap(hl);
        h->host_done.assign((size_t)n, 0);
        ok = ok && hipMemcpyAsync(h->d_table(), h->table_img.data(), h->table_img.size() * 4, hipMemcpyHostToDevice, st) == hipSuccess;
    } else {
        // contiguous cache: the rows of sequence kept[i] move to slot i, in ascending i (kept[i] >= i and ascending, so a
        // slot is never overwritten before it has been read); launches on one stream run in order
        for (int i = 0; i < n; ++i)
            launch_kv_move(h->kv, h->kv_i16 ? h->scales() : nullptr, h->area_elems(), 2 * h->s.n_layers, h->s.n_kv_heads, h->s.max_seq,
                           h->s.head_dim, kept[i], i, lens[(size_t)kept[i]], st);
    }
    launch_compact_state(h->d_lens(), h->d_done(), tokens, h->d_kept(), n, st);
    if (!ok || hipStreamSynchronize(st) != hipSuccess) { set_err(h, "rl_gen_compact: stream error"); return RL_GEN_E_HIP; }
    int rc = check_hip(h, "rl_gen_compact");
    if (rc != RL_GEN_OK) return rc;
    h->B = n;
    return RL_GEN_OK;
}

int rl_gen_logprobs(rl_gen_t *h, const int32_t *tokens, int32_t B, int32_t T, float *logp, void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    if (!tokens || !logp) { set_err(h, "rl_gen_logprobs: NULL argument"); return RL_GEN_E_NULL; }
    if (B <= 0 || T <= 0) { set_err(h, "rl_gen_logprobs: B and T must be positive"); return RL_GEN_E_SHAPE; }
    if (B > h->s.max_batch || T > h->s.max_seq) {
        set_err(h, "rl_gen_logprobs: B=%d T=%d exceed capacity %d x %d", B, T, h->s.max_batch, h->s.max_seq);
        return RL_GEN_E_CAPACITY;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const rl_gen_shape &s = h->s;
    if (int rcp = check_reserved(h, "rl_gen_logprobs", B, T)) return rcp;
    int per_chunk = h->wp.rows / T;
    if (per_chunk < 1) per_chunk = 1;
    // logits of a block of rows live in the split-K partial area, which is idle once the layers are done
    int64_t rows_fit = (int64_t)(h->wp.part_elems / (size_t)s.vocab);
    if (rows_fit >= 256) rows_fit = rows_fit / 256 * 256;
    if (rows_fit < 1) { set_err(h, "rl_gen_logprobs: workspace holds no logit row"); return RL_GEN_E_CAPACITY; }
    for (int b0 = 0; b0 < B; b0 += per_chunk) {
        int nb = B - b0 < per_chunk ? B - b0 : per_chunk;
        const bool lo = run_layers(h, tokens + (size_t)b0 * T, nb, T, b0, false, st);
        const int M = nb * T;
        for (int m0 = 0; m0 < M; m0 += (int)rows_fit) {
            int mm = M - m0 < rows_fit ? M - m0 : (int)rows_fit;
            GemmArgs a;
            a.A = h->h() + (size_t)m0 * s.hidden; a.lda = s.hidden; a.M = mm; a.K = s.hidden;
            a.W[0] = h->lm_head; a.W[1] = nullptr; a.W[2] = nullptr;
            a.rows[0] = s.vocab; a.rows[1] = 0; a.rows[2] = 0;
            a.out = h->part(); a.ldc = s.vocab; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_F32;
            {
                Scope sc(h, RL_GEN_K_GEMM_LM_HEAD, st);
                if (lo) a.A_lo = a.A + (size_t)M * s.hidden;
                if (mm <= kSkinnyMaxM && !lo) launch_gemm_skinny(a, st);
                else launch_gemm_tiled(a, st);
            }
            Scope sc(h, RL_GEN_K_MISC, st);
            launch_logprob_gather(h->part(), s.vocab, mm, s.vocab, tokens, T, (int64_t)b0 * T + m0, logp, st);
        }
    }
    {
        Scope sc(h, RL_GEN_K_MISC, st);
        launch_init_state(h->d_lens(), h->d_done(), B, nullptr, T, st);
    }
    int rc = check_hip(h, "rl_gen_logprobs");
    if (rc != RL_GEN_OK) return rc;
    h->B = B; h->len = T;
    if (h->page_shift) { h->host_len.assign((size_t)B, T); h->host_done.assign((size_t)B, 0); }
    return RL_GEN_OK;
}

int rl_gen_values(rl_gen_t *h, const int32_t *tokens, int32_t B, int32_t T, const void *head, float *values, void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    if (!tokens || !head || !values) { set_err(h, "rl_gen_values: NULL argument"); return RL_GEN_E_NULL; }
    if (B <= 0 || T <= 0) { set_err(h, "rl_gen_values: B and T must be positive"); return RL_GEN_E_SHAPE; }
    if (B > h->s.max_batch || T > h->s.max_seq) {
        set_err(h, "rl_gen_values: B=%d T=%d exceed capacity %d x %d", B, T, h->s.max_batch, h->s.max_seq);
        return RL_GEN_E_CAPACITY;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (int rcp = check_reserved(h, "rl_gen_values", B, T)) return rcp;
    int per_chunk = h->wp.rows / T;
    if (per_chunk < 1) per_chunk = 1;
    for (int b0 = 0; b0 < B; b0 += per_chunk) {
        int nb = B - b0 < per_chunk ? B - b0 : per_chunk;
        const bool lo = run_layers(h, tokens + (size_t)b0 * T, nb, T, b0, false, st);
        Scope sc(h, RL_GEN_K_MISC, st);
        launch_rowdot(h->h(), lo ? h->h() + (size_t)nb * T * h->s.hidden : nullptr, head, h->s.weight_dtype == 0, nb * T, h->s.hidden,
                      values + (size_t)b0 * T, st);
    }
    {
        Scope sc(h, RL_GEN_K_MISC, st);
        launch_init_state(h->d_lens(), h->d_done(), B, nullptr, T, st);
    }
    int rc = check_hip(h, "rl_gen_values");
    if (rc != RL_GEN_OK) return rc;
    h->B = B; h->len = T;
    if (h->page_shift) { h->host_len.assign((size_t)B, T); h->host_done.assign((size_t)B, 0); }
    return RL_GEN_OK;
}

int rl_gen_decode_step(rl_gen_t *h, const int32_t *tokens, float *logits, int32_t *next, void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    if (!tokens) { set_err(h, "rl_gen_decode_step: NULL tokens"); return RL_GEN_E_NULL; }
    if (h->B <= 0) { set_err(h, "rl_gen_decode_step: no prefill yet"); return RL_GEN_E_STATE; }
    if (h->len + 1 > h->s.max_seq) { set_err(h, "rl_gen_decode_step: sequence capacity %d reached", h->s.max_seq); return RL_GEN_E_CAPACITY; }
    if (h->page_shift) {
        // a sequence that has not (to the host's knowledge) ended stores one more row: its pages must hold it
        for (int b = 0; b < h->B; ++b)
            if (!h->host_done[b] && h->host_len[b] + 1 > h->cap[b]) {
                set_err(h, "rl_gen_decode_step: sequence %d may hold %d tokens, %d positions reserved", b, h->host_len[b],
                        h->cap[b]);
                return RL_GEN_E_CAPACITY;
            }
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    float *lg = logits ? logits : h->logits_ws();
    int32_t *nx = next ? next : h->next_ws();
    bool use_graph = h->graph_on && !h->prof_on;
    if (!use_graph) {
        enqueue_decode(h, tokens, lg, logits != nullptr, nx, st);
    } else {
        GraphEntry *g = nullptr;
        for (auto &e : h->graphs)
            if (e.tokens == tokens && e.logits == lg && e.next == nx && e.B == h->B && e.stream == st) g = &e;
        if (!g) {
            if (h->graphs.size() >= 8) drop_graphs(h);
            h->graphs.push_back(GraphEntry{tokens, lg, nx, h->B, st, 0, nullptr});
            g = &h->graphs.back();
        }
        g->calls++;
        if (g->exec) {
            if (hipGraphLaunch(g->exec, st) != hipSuccess) { set_err(h, "rl_gen_decode_step: hipGraphLaunch failed"); return RL_GEN_E_HIP; }
        } else if (g->calls == 1) {
            enqueue_decode(h, tokens, lg, logits != nullptr, nx, st);  // first use: plain launches (also warms up lazy kernel attributes)
        } else {
            hipGraph_t graph = nullptr;
            if (hipStreamBeginCapture(st, hipStreamCaptureModeRelaxed) != hipSuccess) {
                (void)hipGetLastError();
                enqueue_decode(h, tokens, lg, logits != nullptr, nx, st);
            } else {
                enqueue_decode(h, tokens, lg, logits != nullptr, nx, st);
                hipError_t e = hipStreamEndCapture(st, &graph);
                if (e != hipSuccess || !graph) { set_err(h, "rl_gen_decode_step: stream capture failed: %s", hipGetErrorString(e)); return RL_GEN_E_HIP; }
                e = hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0);
                (void)hipGraphDestroy(graph);
                if (e != hipSuccess) { g->exec = nullptr; set_err(h, "rl_gen_decode_step: hipGraphInstantiate failed: %s", hipGetErrorString(e)); return RL_GEN_E_HIP; }
                if (hipGraphLaunch(g->exec, st) != hipSuccess) { set_err(h, "rl_gen_decode_step: hipGraphLaunch failed"); return RL_GEN_E_HIP; }
            }
        }
    }
    int rc = check_hip(h, "rl_gen_decode_step");
    if (rc != RL_GEN_OK) return rc;
    h->len += 1;
    if (h->page_shift)
        for (int b = 0; b < h->B; ++b)
            if (!h->host_done[b]) h->host_len[b] += 1;
    return RL_GEN_OK;
}

int rl_gen_generate(rl_gen_t *h, const int32_t *prompts, int32_t B, int32_t P, int32_t G, const float *u, int32_t *out,
                    void *hip_stream) {
    if (!h) return RL_GEN_E_NULL;
    if (!prompts || !out) { set_err(h, "rl_gen_generate: NULL argument"); return RL_GEN_E_NULL; }
    if (B <= 0 || P <= 0 || G <= 0) { set_err(h, "rl_gen_generate: B, P and G must be positive"); return RL_GEN_E_SHAPE; }
    if ((int64_t)P + G - 1 > h->s.max_seq) {
        set_err(h, "rl_gen_generate: P + G - 1 = %lld positions exceed capacity %d", (long long)P + G - 1, h->s.max_seq);
        return RL_GEN_E_CAPACITY;
    }
    const bool sampling = h->temperature > 0.f;
    if (sampling && !u) { set_err(h, "rl_gen_generate: sampling is on and no draws were given"); return RL_GEN_E_NULL; }
    const int portion = h->s.max_batch;
    if (int rcp = check_reserved(h, "rl_gen_generate", B < portion ? B : portion, P + G - 1)) return rcp;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    // the token-choice kernel of every step reads its draws from one fixed place, so captured steps stay valid
    const float *caller_u = h->sample_u;
    if (sampling && caller_u != h->draws_ws()) { drop_graphs(h); h->sample_u = h->draws_ws(); }
    int rc = RL_GEN_OK;
    for (int b0 = 0; b0 < B && rc == RL_GEN_OK; b0 += portion) {
        const int nb = B - b0 < portion ? B - b0 : portion;
        for (int g = 0; g < G && rc == RL_GEN_OK; ++g) {
            if (sampling) launch_copy_strided(u + (size_t)g * B + b0, 1, h->draws_ws(), 1, nb, st);
            if (g == 0) rc = prefill_impl(h, "rl_gen_generate", prompts + (size_t)b0 * P, nullptr, nb, P, nullptr, h->next_ws(), hip_stream);
            else rc = rl_gen_decode_step(h, h->next_ws(), nullptr, h->next_ws(), hip_stream);
            if (rc == RL_GEN_OK) launch_copy_strided(h->next_ws(), 1, out + (size_t)b0 * G + g, G, nb, st);
        }
    }
    if (sampling && caller_u != h->draws_ws()) { drop_graphs(h); h->sample_u = caller_u; }
    if (rc != RL_GEN_OK) return rc;
    return check_hip(h, "rl_gen_generate");
}

int rl_gen_set_graph(rl_gen_t *h, int32_t enabled) {
    if (!h) return RL_GEN_E_NULL;
    h->graph_on = enabled != 0;
    return RL_GEN_OK;
}

int rl_gen_set_sampling(rl_gen_t *h, float temperature, const float *u) {
    if (!h) return RL_GEN_E_NULL;
    if (temperature > 0.f && !u) { set_err(h, "rl_gen_set_sampling: NULL draws"); return RL_GEN_E_NULL; }
    if (temperature != temperature) { set_err(h, "rl_gen_set_sampling: temperature is NaN"); return RL_GEN_E_SHAPE; }
    drop_graphs(h);  // captured steps end in the other kernel
    h->temperature = temperature > 0.f ? temperature : 0.f;
    h->sample_u = temperature > 0.f ? u : nullptr;
    return RL_GEN_OK;
}

int rl_gen_set_qkv_terms(rl_gen_t *h, int32_t terms) {
    if (!h) return RL_GEN_E_NULL;
    if (terms != 1 && terms != 2) { set_err(h, "rl_gen_set_qkv_terms: terms must be 1 or 2"); return RL_GEN_E_SHAPE; }
    if ((terms == 2) != h->qkv_two_term) drop_graphs(h);
    h->qkv_two_term = terms == 2;
    return RL_GEN_OK;
}

int rl_gen_reset(rl_gen_t *h) {
    if (!h) return RL_GEN_E_NULL;
    h->B = 0; h->len = 0;
    return RL_GEN_OK;
}

int rl_gen_state(const rl_gen_t *h, int32_t *batch, int32_t *length) {
    if (!h) return RL_GEN_E_NULL;
    if (batch) *batch = h->B;
    if (length) *length = h->len;
    return RL_GEN_OK;
}

void rl_gen_destroy(rl_gen_t *h) {
    if (!h) return;
    (void)hipDeviceSynchronize();
    drop_graphs(h);
    for (auto &e : h->prof_events) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    for (auto &e : h->prof_pool) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    for (void *p : h->owned) (void)hipFree(p);
    delete h;
}

const char *rl_gen_last_error(const rl_gen_t *h) { return h ? h->err : g_create_error; }

int rl_gen_profile(rl_gen_t *h, int32_t enabled) {
    if (!h) return RL_GEN_E_NULL;
    h->prof_on = enabled != 0;
    return RL_GEN_OK;
}

int rl_gen_profile_read(rl_gen_t *h, int32_t *launches, float *milliseconds, void *hip_stream) {
    if (!h || !launches || !milliseconds) return RL_GEN_E_NULL;
    if (hipStreamSynchronize(reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess) { set_err(h, "rl_gen_profile_read: sync failed"); return RL_GEN_E_HIP; }
    for (auto &e : h->prof_events) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e.a, e.b) == hipSuccess) {
            h->prof_launches[e.cls] += 1;
            h->prof_ms[e.cls] += ms;
        }
        h->prof_pool.push_back(e);
    }
    h->prof_events.clear();
    for (int i = 0; i < RL_GEN_N_KERNEL_CLASSES; ++i) {
        launches[i] = h->prof_launches[i];
        milliseconds[i] = h->prof_ms[i];
        h->prof_launches[i] = 0;
        h->prof_ms[i] = 0.f;
    }
    (void)hipGetLastError();
    return RL_GEN_OK;
}

const char *rl_gen_kernel_class_name(int32_t id) {
    static const char *names[RL_GEN_N_KERNEL_CLASSES] = {"embed", "add_rmsnorm", "gemm_qkv", "rope_append", "decode_attention",
                                                         "attention_merge", "prefill_attention", "gemm_o", "gemm_gate_up",
                                                         "gemm_down", "gemm_lm_head", "argmax", "misc"};
    return id >= 0 && id < RL_GEN_N_KERNEL_CLASSES ? names[id] : "?";
}

// ------------------------------------------------------------------ single-kernel entry points

#define RL_OP_RETURN()                                         \
    do {                                                       \
        return hipGetLastError() == hipSuccess ? RL_GEN_OK : RL_GEN_E_HIP; \
    } while (0)

int rl_op_embed(const int32_t *tokens, const uint16_t *emb, float *x, int32_t M, int32_t d, int32_t vocab, void *st) {
    if (!tokens || !emb || !x) return RL_GEN_E_NULL;
    if (M < 0 || d <= 0 || d % 8 || vocab <= 0) return RL_GEN_E_SHAPE;
    launch_embed(tokens, emb, x, M, d, vocab, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_add_rmsnorm(float *x, const float *part, int32_t nsplit, size_t part_stride, const uint16_t *gain, float eps,
                      uint16_t *h, uint16_t *h_lo, int32_t M, int32_t d, void *st) {
    if (!x || !gain || !h || (nsplit > 0 && !part)) return RL_GEN_E_NULL;
    if (M < 0 || d <= 0 || d % 4 || d > 8192 || nsplit < 0) return RL_GEN_E_SHAPE;
    launch_add_rmsnorm(x, part, nsplit, part_stride, gain, eps, h, h_lo, M, d, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_gemm(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *W0, const uint16_t *W1, const uint16_t *W2,
               int32_t rows0, int32_t rows1, int32_t rows2, int32_t M, int32_t K, void *out, int64_t ldc, size_t split_stride,
               int32_t splits, int32_t epilogue, int32_t kernel, uint16_t *out_lo, void *st) {
    if (!A || !W0 || !out) return RL_GEN_E_NULL;
    if (out_lo && (epilogue != EPI_SWIGLU || kernel != 2)) return RL_GEN_E_SHAPE;
    if (A_lo && (kernel != 2 || epilogue == EPI_SWIGLU || A_lo <= A)) return RL_GEN_E_SHAPE;
    if (M < 0 || K <= 0 || K % 8 || lda % 8 || lda < K || rows0 <= 0 || rows1 < 0 || rows2 < 0) return RL_GEN_E_SHAPE;
    if (epilogue < 0 || epilogue > 2 || kernel < 0 || kernel > 2 || splits < 1) return RL_GEN_E_SHAPE;
    if (epilogue == EPI_SWIGLU && (!W1 || rows1 != rows0 || W2)) return RL_GEN_E_SHAPE;
    if (epilogue != EPI_F32 && splits != 1) return RL_GEN_E_SHAPE;
    if (kernel == 1 && M > kSkinnyMaxM) return RL_GEN_E_SHAPE;
    if (kernel == 2 && splits != 1) return RL_GEN_E_SHAPE;
    if ((uint64_t)rows0 * K * 2 > 0xffffffffull || (uint64_t)rows1 * K * 2 > 0xffffffffull || (uint64_t)rows2 * K * 2 > 0xffffffffull)
        return RL_GEN_E_SHAPE;
    GemmArgs a;
    a.A = A; a.A_lo = A_lo; a.lda = lda; a.M = M; a.K = K;
    a.W[0] = W0; a.W[1] = rows1 > 0 ? W1 : nullptr; a.W[2] = rows2 > 0 ? W2 : nullptr;
    a.rows[0] = rows0; a.rows[1] = rows1; a.rows[2] = rows2;
    a.out = out; a.ldc = ldc; a.split_stride = split_stride; a.splits = splits; a.epilogue = epilogue; a.out_lo = out_lo;
    bool skinny = kernel == 1 || (kernel == 0 && M <= kSkinnyMaxM);
    if (skinny) launch_gemm_skinny(a, reinterpret_cast<hipStream_t>(st));
    else launch_gemm_tiled(a, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_gemm_tiled_packed(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *W0, const uint16_t *W1,
                            const uint16_t *W2, const uint16_t *P0, const uint16_t *P1, const uint16_t *P2, int32_t rows0, int32_t rows1,
                            int32_t rows2, int32_t M, int32_t K, void *out, int64_t ldc, int32_t epilogue, void *st) {
    if (!A || !W0 || !P0 || !out) return RL_GEN_E_NULL;
    if (A_lo && (epilogue == EPI_SWIGLU || A_lo <= A)) return RL_GEN_E_SHAPE;
    if (M < 0 || K <= 0 || K % 8 || lda % 8 || lda < K || rows0 <= 0 || rows1 < 0 || rows2 < 0) return RL_GEN_E_SHAPE;
    if (epilogue < 0 || epilogue > 2) return RL_GEN_E_SHAPE;
    if ((rows1 > 0 && (!W1 || !P1)) || (rows2 > 0 && (!W2 || !P2))) return RL_GEN_E_NULL;
    if (epilogue == EPI_SWIGLU && (rows1 != rows0 || rows2 != 0)) return RL_GEN_E_SHAPE;
    if ((uint64_t)rows0 * K * 2 > 0xffffffffull || (uint64_t)rows1 * K * 2 > 0xffffffffull || (uint64_t)rows2 * K * 2 > 0xffffffffull)
        return RL_GEN_E_SHAPE;
    GemmArgs a;
    a.A = A; a.A_lo = A_lo; a.lda = lda; a.M = M; a.K = K;
    a.W[0] = W0; a.W[1] = rows1 > 0 ? W1 : nullptr; a.W[2] = rows2 > 0 ? W2 : nullptr;
    a.P[0] = P0; a.P[1] = rows1 > 0 ? P1 : nullptr; a.P[2] = rows2 > 0 ? P2 : nullptr;
    a.rows[0] = rows0; a.rows[1] = rows1; a.rows[2] = rows2;
    a.out = out; a.ldc = ldc; a.split_stride = 0; a.splits = 1; a.epilogue = epilogue;
    launch_gemm_tiled(a, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_gemm_rope(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *Wq, const uint16_t *Wk, const uint16_t *Wv,
                    const uint16_t *Pq, const uint16_t *Pk, const uint16_t *Pv,
                    int32_t Hq, int32_t Hkv, int32_t hd, int32_t M, int32_t K, int32_t T, int32_t b0, const float *rope_tab,
                    int32_t rope_style, int32_t S, uint16_t *q_f16, uint16_t *kc, uint16_t *vc, float *kscale, float *vscale,
                    uint16_t *q_f16_lo, void *st) {
    if (!A || !Wq || !Wk || !Wv || !rope_tab || !q_f16 || !kc || !vc) return RL_GEN_E_NULL;
    if ((kscale == nullptr) != (vscale == nullptr)) return RL_GEN_E_NULL;
    if (M <= 0 || K <= 0 || K % 8 || lda % 8 || lda < K || Hq <= 0 || Hkv <= 0 || T <= 0 || b0 < 0 || S < T) return RL_GEN_E_SHAPE;
    if (A_lo && A_lo <= A) return RL_GEN_E_SHAPE;
    if (!gemm_tiled_rope_supported(M, K, lda, Hq, Hkv, hd, rope_style, T, A_lo != nullptr)) return RL_GEN_E_SHAPE;
    if (A_lo && (size_t)(A_lo - A) * 2 >= 0x70000000ull) return RL_GEN_E_SHAPE;
    RopeEpilogue rp;
    rp.rope_tab = rope_tab; rp.T = T; rp.b0 = b0; rp.Hq = Hq; rp.Hkv = Hkv; rp.S = S;
    rp.q_f16 = q_f16; rp.kc = kc; rp.vc = vc; rp.map = KvMap(); rp.d_valid = nullptr;
    rp.map.kscale = kscale; rp.map.vscale = vscale; rp.q_f16_lo = q_f16_lo;
    GemmArgs a;
    a.A = A; a.A_lo = A_lo; a.lda = lda; a.M = M; a.K = K;
    a.W[0] = Wq; a.W[1] = Wk; a.W[2] = Wv;
    a.rows[0] = Hq * hd; a.rows[1] = Hkv * hd; a.rows[2] = Hkv * hd;
    a.out = nullptr; a.ldc = 0; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_ROPE; a.rope = &rp;
    if (Pq && Pk && Pv) { a.P[0] = Pq; a.P[1] = Pk; a.P[2] = Pv; }
    launch_gemm_tiled(a, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

size_t rl_op_packed_weight_bytes(int32_t N, int32_t K) {
    if (N <= 0 || K <= 0) return 0;
    return packed_weight_bytes(N, K);
}

int rl_op_pack_weights(const uint16_t *W, uint16_t *P, int32_t N, int32_t K, void *st) {
    if (!W || !P) return RL_GEN_E_NULL;
    if (N <= 0 || K <= 0 || K % 8) return RL_GEN_E_SHAPE;
    launch_pack_weights(W, P, N, K, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_gemm_packed(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *P0, const uint16_t *P1,
                      const uint16_t *P2, int32_t rows0, int32_t rows1, int32_t rows2, int32_t M, int32_t K, void *out,
                      int64_t ldc, size_t split_stride, int32_t splits, int32_t epilogue, int32_t nb, int32_t rows_per_wg, int32_t depth,
                      uint16_t *out_lo, void *st) {
    if (!A || !P0 || !out) return RL_GEN_E_NULL;
    if (out_lo && epilogue != EPI_SWIGLU) return RL_GEN_E_SHAPE;
    if (M < 0 || K <= 0 || K % 8 || lda % 8 || lda < K || rows0 <= 0 || rows1 < 0 || rows2 < 0) return RL_GEN_E_SHAPE;
    if (epilogue < 0 || epilogue > 2 || splits < 1 || nb < 0 || nb > 2) return RL_GEN_E_SHAPE;
    if (rows_per_wg != 0 && rows_per_wg != 32 && rows_per_wg != 64 && rows_per_wg != 128) return RL_GEN_E_SHAPE;
    if (depth != 0 && depth != 2 && depth != 4) return RL_GEN_E_SHAPE;
    if (epilogue == EPI_SWIGLU && (!P1 || rows1 != rows0 || P2)) return RL_GEN_E_SHAPE;
    if (epilogue != EPI_F32 && splits != 1) return RL_GEN_E_SHAPE;
    if (((uint64_t)M * (uint64_t)lda + (uint64_t)K) * 2 > 0xf0000000ull) return RL_GEN_E_SHAPE;
    PackedGemmArgs a;
    a.A = A; a.A_lo = A_lo; a.lda = lda; a.M = M; a.K = K;
    a.P[0] = P0; a.P[1] = rows1 > 0 ? P1 : nullptr; a.P[2] = rows2 > 0 ? P2 : nullptr;
    a.rows[0] = rows0; a.rows[1] = rows1; a.rows[2] = rows2;
    a.out = out; a.ldc = ldc; a.split_stride = split_stride; a.splits = splits; a.epilogue = epilogue; a.out_lo = out_lo;
    int pnb, prows, psplits;
    gemm_packed_plan(rows0 + rows1 + rows2, K, M, &pnb, &prows, &psplits);
    a.nb = nb == 0 ? pnb : nb;
    a.rows_per_wg = rows_per_wg;
    a.depth = depth;
    launch_gemm_packed(a, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

size_t rl_op_lm_head_argmax_ws_floats(int32_t M, int32_t V) {
    return M > 0 && V > 0 ? (size_t)2 * M * ceil_div(V, 128) : 0;
}

int rl_op_lm_head_argmax(const uint16_t *A, const uint16_t *A_lo, int64_t lda, const uint16_t *P, int32_t V, int32_t M, int32_t K,
                         float *logits, int64_t ldc, float *ws, int32_t *next, void *st) {
    if (!A || !P || !ws || !next) return RL_GEN_E_NULL;
    if (M < 0 || K <= 0 || K % 8 || lda % 8 || lda < K || V <= 0 || (logits && ldc < V)) return RL_GEN_E_SHAPE;
    if (((uint64_t)M * (uint64_t)lda + (uint64_t)K) * 2 > 0xf0000000ull || !gemm_packed_single_launch(V, K)) return RL_GEN_E_SHAPE;
    const int tiles = ceil_div(V, 128);
    PackedGemmArgs a;
    a.A = A; a.A_lo = A_lo; a.lda = lda; a.M = M; a.K = K;
    a.P[0] = P; a.P[1] = nullptr; a.P[2] = nullptr;
    a.rows[0] = V; a.rows[1] = 0; a.rows[2] = 0;
    a.out = logits; a.ldc = logits ? ldc : V; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_F32;
    a.nb = 1; a.rows_per_wg = 128; a.depth = 2;
    a.cand_val = ws;
    a.cand_idx = reinterpret_cast<int32_t *>(ws + (size_t)M * tiles);
    a.no_store = logits == nullptr;
    launch_gemm_packed(a, reinterpret_cast<hipStream_t>(st));
    launch_argmax_merge(a.cand_val, a.cand_idx, M, tiles, next, nullptr, nullptr, -1, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_gemm_packed_swiglu_halves(const uint16_t *A, int64_t lda, const uint16_t *Pg, const uint16_t *Pu, int32_t F, int32_t M,
                                    int32_t K, uint16_t *out, int64_t ldc, int32_t depth, uint16_t *out_lo, void *st) {
    if (!A || !Pg || !Pu || !out) return RL_GEN_E_NULL;
    if (M < 0 || K <= 0 || K % 8 || lda % 8 || lda < K || F <= 0 || ldc < F) return RL_GEN_E_SHAPE;
    if (depth != 0 && depth != 2 && depth != 4) return RL_GEN_E_SHAPE;
    if (((uint64_t)M * (uint64_t)lda + (uint64_t)K) * 2 > 0xf0000000ull) return RL_GEN_E_SHAPE;
    if (!gemm_packed_swiglu_halves_supported(F, K)) return RL_GEN_E_SHAPE;
    PackedGemmArgs a;
    a.A = A; a.A_lo = nullptr; a.lda = lda; a.M = M; a.K = K;
    a.P[0] = Pg; a.P[1] = Pu; a.P[2] = nullptr;
    a.rows[0] = F; a.rows[1] = F; a.rows[2] = 0;
    a.out = out; a.ldc = ldc; a.split_stride = 0; a.splits = 1; a.epilogue = EPI_SWIGLU; a.out_lo = out_lo;
    a.nb = 2; a.rows_per_wg = 128; a.depth = depth;
    launch_gemm_packed_swiglu_halves(a, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_build_rope_table(float *tab, int32_t max_seq, int32_t head_dim, float base) {
    if (!tab) return RL_GEN_E_NULL;
    if (max_seq <= 0 || head_dim <= 0 || head_dim % 2 || !(base > 0.f)) return RL_GEN_E_SHAPE;
    std::vector<float> t((size_t)max_seq * head_dim);
    int half = head_dim / 2;
    for (int pos = 0; pos < max_seq; ++pos)
        for (int r = 0; r < half; ++r) {
            double ang = (double)pos * pow((double)base, -2.0 * r / (double)head_dim);
            t[((size_t)pos * half + r) * 2] = (float)cos(ang);
            t[((size_t)pos * half + r) * 2 + 1] = (float)sin(ang);
        }
    return hipMemcpy(tab, t.data(), t.size() * sizeof(float), hipMemcpyHostToDevice) == hipSuccess ? RL_GEN_OK : RL_GEN_E_HIP;
}

int rl_op_rope_append(const float *qkv, int32_t nsplit, size_t split_stride, int32_t M, int32_t T, int32_t b0,
                      const int32_t *d_pos0, int32_t pos_stride, const float *rope_tab, int32_t rope_style, int32_t Hq, int32_t Hkv, int32_t hd,
                      int32_t S, float *q_f32, uint16_t *q_f16, uint16_t *kc, uint16_t *vc, float *kscale, float *vscale,
                      uint16_t *q_f16_lo, void *st) {
    if (!qkv || !d_pos0 || !rope_tab || !kc || !vc) return RL_GEN_E_NULL;
    if ((kscale == nullptr) != (vscale == nullptr)) return RL_GEN_E_NULL;
    if (kscale && hd != 64 && hd != 128) return RL_GEN_E_SHAPE;
    if (q_f16_lo && !q_f16) return RL_GEN_E_NULL;
    if (nsplit < 1 || M < 0 || T <= 0 || b0 < 0 || Hq <= 0 || Hkv <= 0 || hd <= 0 || hd % 2 || S <= 0 || (rope_style != 0 && rope_style != 1))
        return RL_GEN_E_SHAPE;
    if (pos_stride != 0 && pos_stride != 1) return RL_GEN_E_SHAPE;
    KvMap map;
    map.kscale = kscale; map.vscale = vscale;
    launch_rope_append(qkv, nsplit, split_stride, M, T, b0, d_pos0, pos_stride, rope_tab, rope_style, Hq, Hkv, hd, S, q_f32, q_f16, kc, vc,
                       reinterpret_cast<hipStream_t>(st), map, nullptr, nullptr, q_f16_lo);
    RL_OP_RETURN();
}

size_t rl_op_decode_attention_ws_floats(int32_t B, int32_t Hq, int32_t hd, int32_t nsplit) {
    return decode_attention_ws_floats(B, Hq, hd, nsplit);
}

int rl_op_decode_attention(const float *q, const uint16_t *kc, const uint16_t *vc, const int32_t *d_len, int32_t len_stride,
                           uint16_t *out, float *ws,
                           int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit, const int32_t *d_done,
                           const float *kscale, const float *vscale, uint16_t *out_lo, void *st) {
    if (!q || !kc || !vc || !d_len || !out || (nsplit > 1 && !ws)) return RL_GEN_E_NULL;
    if ((kscale == nullptr) != (vscale == nullptr)) return RL_GEN_E_NULL;
    if (B < 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || (hd != 64 && hd != 128) || S <= 0 || nsplit < 1) return RL_GEN_E_SHAPE;
    if (len_stride != 0 && len_stride != 1) return RL_GEN_E_SHAPE;
    KvMap map;
    map.kscale = const_cast<float *>(kscale); map.vscale = const_cast<float *>(vscale);
    launch_decode_attention(q, kc, vc, d_len, len_stride, out, ws, B, Hq, Hkv, hd, S, nsplit, reinterpret_cast<hipStream_t>(st), map,
                            d_done, out_lo);
    RL_OP_RETURN();
}

int rl_op_decode_attention_noalloc(const float *q, const uint16_t *kc, const uint16_t *vc, const int32_t *d_len, int32_t len_stride,
                                   uint16_t *out, int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit,
                                   const int32_t *d_done, const float *kscale, const float *vscale, uint16_t *out_lo, void *st) {
    if (!q || !kc || !vc || !d_len || !out) return RL_GEN_E_NULL;
    if ((kscale == nullptr) != (vscale == nullptr)) return RL_GEN_E_NULL;
    if (B < 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || (hd != 64 && hd != 128) || S <= 0 || nsplit < 1) return RL_GEN_E_SHAPE;
    if (len_stride != 0 && len_stride != 1) return RL_GEN_E_SHAPE;
    const size_t need = decode_attention_ws_floats(B, Hq, hd, nsplit) * sizeof(float);
    if (need > (size_t)RL_OP_NOALLOC_SCRATCH_BYTES) {
        set_err(nullptr, "rl_op_decode_attention_noalloc: the split partials need %zu bytes, the built-in scratch holds %zu", need,
                (size_t)RL_OP_NOALLOC_SCRATCH_BYTES);
        return RL_GEN_E_CAPACITY;
    }
    void *ws = nullptr;
    if (int rc = scratch_of_current_device(&ws)) {
        set_err(nullptr, "rl_op_decode_attention_noalloc: hipGetSymbolAddress(scratch) failed");
        return rc;
    }
    // every partial a merge reads is written by this call's attention kernel first: nothing to clear
    KvMap map;
    map.kscale = const_cast<float *>(kscale); map.vscale = const_cast<float *>(vscale);
    launch_decode_attention(q, kc, vc, d_len, len_stride, out, reinterpret_cast<float *>(ws), B, Hq, Hkv, hd, S, nsplit,
                            reinterpret_cast<hipStream_t>(st), map, d_done, out_lo);
    RL_OP_RETURN();
}

int rl_op_decode_attention_paged(const float *q, const uint16_t *k_pool, const uint16_t *v_pool, const int32_t *table,
                                 int32_t table_stride, int32_t page_size, const int32_t *d_len, int32_t len_stride, uint16_t *out,
                                 float *ws, int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit,
                                 const float *kscale, const float *vscale, void *st) {
    if (!q || !k_pool || !v_pool || !table || !d_len || !out || (nsplit > 1 && !ws)) return RL_GEN_E_NULL;
    if ((kscale == nullptr) != (vscale == nullptr)) return RL_GEN_E_NULL;
    if (B < 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || (hd != 64 && hd != 128) || S <= 0 || nsplit < 1) return RL_GEN_E_SHAPE;
    if (len_stride != 0 && len_stride != 1) return RL_GEN_E_SHAPE;
    const int shift = page_shift_of(page_size);
    if (!shift || (int64_t)table_stride * page_size < S) return RL_GEN_E_SHAPE;
    KvMap map;
    map.table = table; map.table_stride = table_stride; map.page_shift = shift;
    map.kscale = const_cast<float *>(kscale); map.vscale = const_cast<float *>(vscale);
    launch_decode_attention(q, k_pool, v_pool, d_len, len_stride, out, ws, B, Hq, Hkv, hd, S, nsplit, reinterpret_cast<hipStream_t>(st),
                            map);
    RL_OP_RETURN();
}

int rl_op_decode_attention_fused(const float *qkv, int32_t nsplit_qkv, size_t split_stride, const float *rope_tab,
                                 int32_t rope_style, uint16_t *kc, uint16_t *vc, const int32_t *d_len, int32_t len_stride,
                                 uint16_t *out, float *ws,
                                 int32_t B, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, int32_t nsplit, void *st) {
    if (!qkv || !rope_tab || !kc || !vc || !d_len || !out || (nsplit > 1 && !ws)) return RL_GEN_E_NULL;
    if (B < 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || (hd != 64 && hd != 128) || S <= 0 || nsplit < 1 || nsplit_qkv < 1 ||
        (rope_style != 0 && rope_style != 1) || split_stride % 4)
        return RL_GEN_E_SHAPE;
    if (len_stride != 0 && len_stride != 1) return RL_GEN_E_SHAPE;
    launch_decode_attention_fused(qkv, nsplit_qkv, split_stride, rope_tab, rope_style, kc, vc, d_len, len_stride, out, ws, B, Hq, Hkv, hd, S,
                                  nsplit, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_prefill_attention(const uint16_t *q, const uint16_t *kc, const uint16_t *vc, uint16_t *out, int32_t nb, int32_t b0,
                            int32_t T, int32_t Hq, int32_t Hkv, int32_t hd, int32_t S, const float *kscale, const float *vscale,
                            uint16_t *out_lo, const uint16_t *q_lo, void *st) {
    if (!q || !kc || !vc || !out) return RL_GEN_E_NULL;
    if ((kscale == nullptr) != (vscale == nullptr)) return RL_GEN_E_NULL;
    if (q_lo && !kscale) return RL_GEN_E_SHAPE;
    if (nb < 0 || b0 < 0 || T <= 0 || T > S || Hq <= 0 || Hkv <= 0 || Hq % Hkv || (hd != 64 && hd != 128) || nb > 65535)
        return RL_GEN_E_SHAPE;
    KvMap map;
    map.kscale = const_cast<float *>(kscale); map.vscale = const_cast<float *>(vscale);
    launch_prefill_attention(q, kc, vc, out, nb, b0, T, Hq, Hkv, hd, S, reinterpret_cast<hipStream_t>(st), map, nullptr, out_lo, q_lo);
    RL_OP_RETURN();
}

int rl_op_sample(const float *logits, int32_t B, int32_t V, float temperature, const float *u, int32_t *next, void *st) {
    if (!logits || !u || !next) return RL_GEN_E_NULL;
    if (B < 0 || V <= 0 || !(temperature > 0.f)) return RL_GEN_E_SHAPE;
    launch_sample(logits, B, V, temperature, u, next, nullptr, nullptr, -1, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_logprob_gather(const float *logits, int64_t ld, int32_t M, int32_t V, const int32_t *tokens, int32_t T, int64_t m_first,
                         float *out, void *st) {
    if (!logits || !tokens || !out) return RL_GEN_E_NULL;
    if (M < 0 || V <= 0 || ld < V || T <= 0 || m_first < 0) return RL_GEN_E_SHAPE;
    launch_logprob_gather(logits, ld, M, V, tokens, T, m_first, out, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_copy(const void *src, void *dst, size_t bytes, void *st) {
    if (!src || !dst) return RL_GEN_E_NULL;
    if (bytes % 16 || ((uintptr_t)src | (uintptr_t)dst) % 16) return RL_GEN_E_SHAPE;
    launch_copy(src, dst, bytes, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

int rl_op_argmax(const float *logits, int32_t B, int32_t V, int32_t *next, void *st) {
    if (!logits || !next) return RL_GEN_E_NULL;
    if (B < 0 || V <= 0) return RL_GEN_E_SHAPE;
    launch_argmax(logits, B, V, next, nullptr, nullptr, -1, reinterpret_cast<hipStream_t>(st));
    RL_OP_RETURN();
}

}  // extern "C"
