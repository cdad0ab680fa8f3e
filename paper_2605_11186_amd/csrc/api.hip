// Host side of the C ABI: argument validation, scratch ownership and the order
// in which one verify step's kernels are enqueued (paper Algorithm 1, Stage 3
// through the commit step).
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>

#include "common.hpp"

constexpr int CATS_PROF_MAX = 1024;  // GEMM launches that can be timed between two reads

struct cats_ctx {
    cats_model_desc d;
    int device;
    int n_cus;   // compute units of that device
    // uploaded tree (device) and its host copy
    int32_t *token, *parent, *depth;
    u32x4* anc;  // [max_tree] ancestor-or-self masks of the uploaded tree
    int32_t h_parent[CATS_MAX_TREE], h_depth[CATS_MAX_TREE];
    int T;  // 0 = no tree set
    // the call being enqueued (set by every entry point before its helpers run): the row
    // kernels and GEMMs work on `rows` rows, which are nodes n0 .. n0 + rows - 1 of the tree
    int n0 = 0;
    int rows = 0;
    // acceptance criterion of cats_verify_tree[_streamed]: 0 greedy, 1 typical
    int accept_mode = 0;
    float typ_epsilon = 0.09f, typ_delta = 0.3f, typ_inv_temp = 1.f;
    // scratch
    float* x;        // [max_tree][H] residual stream
    // activations that feed a GEMM or the attention products: high and low bf16 parts
    bf16_t *xn, *xn_lo;      // [max_tree][H] rows times gain (norm factor applied downstream)
    float* ss;               // [max_tree][SS_STRIDE] sums of squares per column block
    bf16_t *q, *q_lo;        // [max_tree][H] rotated queries
    bf16_t *attn, *attn_lo;  // [max_tree][H] attention output
    bf16_t *hact, *hact_lo;  // [max_tree][F] SwiGLU output
    float* part;     // split-K partial sums
    size_t part_elems;
    // Single-row calls (rows == 1) run on cats_gemv_row, which folds the residual / norm and SwiGLU
    // steps into the product behind them.  Between two products the row is therefore (x, pend):
    // the residual row as of its last update and the partial sums of the last product, still to be
    // added.  Products alternate between two partial-sum buffers (a product reads the one before
    // while it writes its own) and residual updates between two rows.  At the start of the draft
    // loop's steps the row is (embed, token) instead: an embedding row that no kernel has copied yet.
    struct {
        float* x;               // the residual row as of its last update
        const bf16_t* embed;    // not null: the row is embed[*token] and x does not hold it yet
        const int32_t* token;   // device
        const float* pend;      // [pieces][hidden] partial sums still to be added to it; null: none
        GemmPlan pend_plan;
        const void* next_gain;  // gain of the norm that follows the pending update (LM head)
    } row = {nullptr, nullptr, nullptr, nullptr, {}, nullptr};
    float* x_row;     // [hidden] second residual row
    float* part_row;  // second partial-sum buffer, one row
    float2* rope_cs;  // [max_tree][d/2]
    float* attn_po;
    float* attn_pml;
    int* attn_arrivals;        // [n_heads][query groups] chunk arrival counters (zero between launches)
    bf16_t *k_lo, *vt_lo;      // low parts of the K/V rows that the running call appends (see AttnArgs)
    int attn_max_chunks;
    int32_t* amax;   // [max_tree]
    float *am_best, *am_second;   // [max_tree][ARGMAX_SLICES] slice results of the argmax
    int *am_idx, *am_arrivals;    // [max_tree][ARGMAX_SLICES] indices, [max_tree] arrival counters (zero between launches)
    float* am_wg_best;            // [compute units] per-workgroup results of the greedy token inside the
    int* am_wg_idx;               // single-row LM head product (see GemvArgs::amax)
    // typical acceptance: per node log-sum-exp, entropy, per-slice triples behind them; per node
    // probability of its token at its parent, the threshold there, and the decision
    float *typ_lse = nullptr, *typ_entropy = nullptr, *typ_slice = nullptr, *typ_prob = nullptr, *typ_thr = nullptr;
    uint8_t* typ_edge = nullptr;
    char* flat;      // the single allocation behind all of the above
    // offload regime: copy stream and the events that order it against the compute stream
    hipStream_t copy_stream;
    hipEvent_t ev_copied[2], ev_consumed[2];
    // optional timing of the weight-streaming GEMM launches (measurement aid)
    bool prof_on;
    int prof_n;
    hipEvent_t prof_ev[2 * CATS_PROF_MAX];
};

namespace {

thread_local hipError_t g_last_hip = hipSuccess;

inline int hip_fail(hipError_t e) {
    g_last_hip = e;
    return CATS_EHIP;
}
#define HIP_TRY(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return hip_fail(e_);     \
    } while (0)

inline size_t align256(size_t n) { return (n + 255) & ~static_cast<size_t>(255); }

// Workgroups per GEMM launch: one per compute unit of the context's device (the GEMM kernel's
// register footprint lets one 512-thread workgroup live on a CU); cats_create reads the count.
int target_wgs(const cats_ctx* c) { return c->n_cus; }

// Key chunks per (head, query group): the launch has heads * query groups * chunks workgroups,
// about one per compute unit (the kernel's register footprint allows one four-wave workgroup
// per unit); more chunks than that only add hand-over traffic between workgroups.
int attn_chunks(int rows, int n_heads, int max_chunks, int n_cus, int n_keys) {
    const int n_blocks = (n_keys + ATTN_KB - 1) / ATTN_KB;
    const int groups = (rows + ATTN_QN - 1) / ATTN_QN;
    const int chunks = std::max(1, n_cus / std::max(1, n_heads * groups));
    return std::min(chunks, std::min(n_blocks, max_chunks));
}

hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

NormScale norm_scale(const cats_ctx* c) {
    return NormScale{c->ss, (c->d.hidden + SS_COLS - 1) / SS_COLS, c->d.hidden, c->d.rms_eps};
}

// Common checks of the entry points that work on the tree; on success the call's row range
// defaults to the whole tree (cats_verify_nodes narrows it afterwards).
int check_ctx_len(cats_ctx* c, int32_t ctx_len) {
    if (!c) return CATS_EINVAL;
    if (c->T < 1) return CATS_ESTATE;
    if (ctx_len < 0) return CATS_EINVAL;
    if (static_cast<int64_t>(ctx_len) + c->T > c->d.max_ctx) return CATS_ECAPACITY;
    c->n0 = 0;
    c->rows = c->T;
    c->row.pend = nullptr;
    c->row.embed = nullptr;
    return CATS_OK;
}

// A full decoder layer, or an attention-only block (the adapters: norm, attention, residual):
// then the three feed-forward matrices and g_ffn are all NULL.
bool has_ffn(const cats_layer_weights* w) { return w->w_gate != nullptr; }
bool layer_ok(const cats_layer_weights* w) {
    if (!w || !w->wq || !w->wk || !w->wv || !w->wo || !w->g_attn) return false;
    if (w->w_gate || w->w_up || w->w_down || w->g_ffn) return w->w_gate && w->w_up && w->w_down && w->g_ffn;
    return true;
}

int seg_pad_of(const cats_ctx* c, int seg_rows) {
    return c->d.packed_weights ? (seg_rows + PACK_ROWS - 1) / PACK_ROWS * PACK_ROWS : seg_rows;
}

// The single-row product (rows == 1); g carries the mode and its operands.  It writes into the
// partial-sum buffer that its own input does not come from.
GemmPlan enqueue_gemv(cats_ctx* c, GemvArgs& g, const void* w0, const void* w1, const void* w2, int n_seg,
                      int seg_rows, int K, hipStream_t st) {
    g.w[0] = static_cast<const bf16_t*>(w0);
    g.w[1] = static_cast<const bf16_t*>(w1 ? w1 : w0);
    g.w[2] = static_cast<const bf16_t*>(w2 ? w2 : w0);
    g.n_seg = n_seg;
    g.seg_rows = seg_rows;
    g.seg_pad = seg_pad_of(c, seg_rows);
    g.packed = c->d.packed_weights;
    g.N = n_seg * g.seg_pad;
    g.K = K;
    g.plan = make_gemm_plan(g.N, K, target_wgs(c), 1);
    g.part = (g.mode != GEMV_PLAIN && g.pend == c->part) ? c->part_row : c->part;
    const bool timed = c->prof_on && c->prof_n < CATS_PROF_MAX;
    if (timed) {
        launch_gemv(g, st, c->prof_ev[2 * c->prof_n], c->prof_ev[2 * c->prof_n + 1]);
        ++c->prof_n;
    } else {
        launch_gemv(g, st);
    }
    return g.plan;
}
GemvArgs gemv_plain(const bf16_t* x_hi, const bf16_t* x_lo) {
    GemvArgs g{};
    g.mode = GEMV_PLAIN;
    g.x_hi = x_hi;
    g.x_lo = x_lo;
    return g;
}
// The pending residual update, the norm input for `gain`, and the row's sums of squares; the
// updated row goes to x_out (null: to the residual row that is not the current one).
GemvArgs gemv_norm(cats_ctx* c, const void* gain, float* x_out) {
    GemvArgs g{};
    g.mode = GEMV_NORM;
    g.x_in = c->row.x;
    g.embed = c->row.embed;
    g.token = c->row.token;
    g.x_out = x_out ? x_out : (c->row.x == c->x_row ? c->x : c->x_row);
    g.gain = static_cast<const bf16_t*>(gain);
    g.ss_out = c->ss;
    g.pend = c->row.pend;
    g.pend_plan = c->row.pend_plan;
    g.pend_ld = c->d.hidden;
    c->row.x = g.x_out;
    c->row.embed = nullptr;
    c->row.pend = nullptr;
    return g;
}
// The attention output as cats_decode_attention left it: one partial result per key chunk.
GemvArgs gemv_attn(const cats_ctx* c, int n_chunks) {
    GemvArgs g{};
    g.mode = GEMV_ATTN;
    g.po = c->attn_po;
    g.pml = c->attn_pml;
    g.n_chunks = n_chunks;
    g.head_dim = c->d.head_dim;
    return g;
}

// One weight-streaming product over n_seg row segments of seg_rows rows each.
GemmPlan enqueue_gemm(cats_ctx* c, const bf16_t* x, const bf16_t* x_lo, const void* w0, const void* w1,
                      const void* w2, int n_seg, int seg_rows, int K, hipStream_t st) {
    if (c->rows == 1) {
        GemvArgs gv = gemv_plain(x, x_lo);
        return enqueue_gemv(c, gv, w0, w1, w2, n_seg, seg_rows, K, st);
    }
    GemmArgs g;
    g.x = x;
    g.x_lo = x_lo;
    g.w[0] = static_cast<const bf16_t*>(w0);
    g.w[1] = static_cast<const bf16_t*>(w1 ? w1 : w0);
    g.w[2] = static_cast<const bf16_t*>(w2 ? w2 : w0);
    g.n_seg = n_seg;
    g.seg_rows = seg_rows;
    g.seg_pad = seg_pad_of(c, seg_rows);
    g.packed = c->d.packed_weights;
    g.N = n_seg * g.seg_pad;
    g.K = K;
    g.T = c->rows;
    g.plan = make_gemm_plan(g.N, K, target_wgs(c), g.T);
    g.part = c->part;
    const bool timed = c->prof_on && c->prof_n < CATS_PROF_MAX;
    if (timed) {
        launch_gemm(g, st, c->prof_ev[2 * c->prof_n], c->prof_ev[2 * c->prof_n + 1]);
        ++c->prof_n;
    } else {
        launch_gemm(g, st);
    }
    return g.plan;
}

// with_lo: the call's own rows (nodes n0 .. n0 + rows - 1) have their low parts in the window
void enqueue_attention(cats_ctx* c, const bf16_t* q, const bf16_t* q_lo, const cats_kv_layer* kv,
                       int ctx_len, bf16_t* out, bf16_t* out_lo, bool with_lo, hipStream_t st) {
    AttnArgs a;
    a.q = q;
    a.q_lo = q_lo;
    a.out_lo = out_lo;
    a.k_lo = with_lo ? c->k_lo : nullptr;
    a.vt_lo = with_lo ? c->vt_lo : nullptr;
    a.lo_begin = ctx_len + c->n0;
    a.lo_end = with_lo ? ctx_len + c->n0 + c->rows : a.lo_begin;
    a.arrivals = c->attn_arrivals;
    a.kc = static_cast<const bf16_t*>(kv->k);
    a.vt = static_cast<const bf16_t*>(kv->v);
    a.anc = c->anc;
    a.T = c->n0 + c->rows;   // keys: the tree rows up to the call's last node (later rows may not exist yet)
    a.Tq = c->rows;
    a.q0 = c->n0;
    a.H = c->d.hidden;
    a.nh = c->d.n_heads;
    a.d = c->d.head_dim;
    a.max_ctx = c->d.max_ctx;
    a.ctx_len = ctx_len;
    const int n_keys = ctx_len + c->T;
    a.n_chunks = attn_chunks(c->rows, c->d.n_heads, c->attn_max_chunks, c->n_cus, n_keys);
    a.t_pad = (a.Tq + 31) / 32 * 32;
    a.po = c->attn_po;
    a.pml = c->attn_pml;
    a.out = out;
    launch_attention(a, st);
}

// The attention block of a single-row call: q|k|v from the product's partial sums, cache append
// and attention over the context and the node's own path in one kernel.  Key chunks of at least
// four 32-key blocks, as many as the context's scratch holds at most.  Returns the number of
// chunks: the product that follows merges their results (gemv_attn).
int enqueue_row_attention(cats_ctx* c, const float* part, const GemmPlan& plan, const cats_kv_layer* kv,
                           int ctx_len, hipStream_t st) {
    DecodeAttnArgs a;
    a.part = part;
    a.plan = plan;
    a.ns = norm_scale(c);
    a.cs = c->rope_cs + static_cast<size_t>(c->n0) * (c->d.head_dim / 2);
    a.kc = static_cast<bf16_t*>(kv->k);
    a.vt = static_cast<bf16_t*>(kv->v);
    a.anc = c->anc;
    a.node = c->n0;
    a.H = c->d.hidden;
    a.nh = c->d.n_heads;
    a.d = c->d.head_dim;
    a.max_ctx = c->d.max_ctx;
    a.ctx_len = ctx_len;
    const int n_blocks = (ctx_len + c->n0 + 1 + ATTN_KB - 1) / ATTN_KB;
    const int per_chunk = std::max(DEC_TILE / ATTN_KB, (n_blocks + DEC_MAX_CHUNKS - 1) / DEC_MAX_CHUNKS);
    a.n_chunks = (n_blocks + per_chunk - 1) / per_chunk;
    a.span = per_chunk * ATTN_KB;
    a.po = c->attn_po;
    a.pml = c->attn_pml;
    launch_decode_attention(a, st);
    return a.n_chunks;
}

// One decoder layer.  On entry c->xn holds rmsnorm(x)*g_attn of this layer; on
// exit x is updated and, if next_gain is given, c->xn holds rmsnorm(x)*next_gain.
void enqueue_layer(cats_ctx* c, const cats_layer_weights* w, float* x, const cats_kv_layer* kv,
                   int ctx_len, const void* next_gain, hipStream_t st) {
    const int H = c->d.hidden, F = c->d.ffn, T = c->rows;   // nodes n0 .. n0 + rows - 1
    // attention block
    GemmPlan plan = enqueue_gemm(c, c->xn, c->xn_lo, w->wq, w->wk, w->wv, 3, H, H, st);
    QkvRopeArgs qa;
    qa.part = c->part;
    qa.plan = plan;
    qa.ns = norm_scale(c);
    qa.cs = c->rope_cs + static_cast<size_t>(c->n0) * (c->d.head_dim / 2);
    qa.q = c->q;
    qa.q_lo = c->q_lo;
    qa.kc = static_cast<bf16_t*>(kv->k);
    qa.vt = static_cast<bf16_t*>(kv->v);
    qa.T = T;
    qa.H = H;
    qa.nh = c->d.n_heads;
    qa.d = c->d.head_dim;
    qa.max_ctx = c->d.max_ctx;
    qa.row0 = ctx_len + c->n0;
    qa.k_lo = c->k_lo;
    qa.vt_lo = c->vt_lo;
    qa.win0 = ctx_len % ATTN_KB + c->n0;
    if (T > 1) {
        launch_qkv_rope(qa, st);
        enqueue_attention(c, c->q, c->q_lo, kv, ctx_len, c->attn, c->attn_lo, true, st);
        plan = enqueue_gemm(c, c->attn, c->attn_lo, w->wo, nullptr, nullptr, 1, H, H, st);
    } else {
        GemvArgs g = gemv_attn(c, enqueue_row_attention(c, c->part, plan, kv, ctx_len, st));
        plan = enqueue_gemv(c, g, w->wo, nullptr, nullptr, 1, H, H, st);
    }
    ResidualNormArgs rn;
    rn.x = x;
    rn.x_in = nullptr;
    rn.embed = nullptr;
    rn.token = nullptr;
    rn.part = c->part;
    rn.plan = plan;
    rn.gain = static_cast<const bf16_t*>(has_ffn(w) ? w->g_ffn : next_gain);
    rn.xn = c->xn;
    rn.xn_lo = c->xn_lo;
    rn.ss = c->ss;
    rn.T = T;
    rn.H = H;
    rn.eps = c->d.rms_eps;
    launch_residual_norm(rn, st);
    if (!has_ffn(w)) return;   // attention-only block
    // feed-forward block
    plan = enqueue_gemm(c, c->xn, c->xn_lo, w->w_gate, w->w_up, nullptr, 2, F, H, st);
    SwigluArgs sa;
    sa.part = c->part;
    sa.plan = plan;
    sa.ns = norm_scale(c);
    sa.h = c->hact;
    sa.h_lo = c->hact_lo;
    sa.T = T;
    sa.F = F;
    sa.f_pad = seg_pad_of(c, F);
    launch_swiglu(sa, st);
    plan = enqueue_gemm(c, c->hact, c->hact_lo, w->w_down, nullptr, nullptr, 1, H, F, st);
    rn.plan = plan;
    rn.gain = static_cast<const bf16_t*>(next_gain);
    launch_residual_norm(rn, st);
}

// The same layer for a single-row call, from and to the (x, pend) form described at cats_ctx::row.
// On entry either a residual update is pending or the row is still an embedding row (the first
// product then works out its own input), or c->xn holds the row times this layer's g_attn (a row
// kernel has just written it).  first_x_out: where the first residual update of the layer
// leaves the row (null: the spare residual row).
void enqueue_layer_row(cats_ctx* c, const cats_layer_weights* w, const cats_kv_layer* kv, int ctx_len,
                       float* first_x_out, hipStream_t st) {
    const int H = c->d.hidden, F = c->d.ffn;
    GemvArgs g = (c->row.pend || c->row.embed) ? gemv_norm(c, w->g_attn, first_x_out) : gemv_plain(c->xn, c->xn_lo);
    GemmPlan plan = enqueue_gemv(c, g, w->wq, w->wk, w->wv, 3, H, H, st);
    g = gemv_attn(c, enqueue_row_attention(c, g.part, plan, kv, ctx_len, st));
    c->row.pend_plan = enqueue_gemv(c, g, w->wo, nullptr, nullptr, 1, H, H, st);
    c->row.pend = g.part;
    if (!has_ffn(w)) return;   // attention-only block
    g = gemv_norm(c, w->g_ffn, nullptr);
    plan = enqueue_gemv(c, g, w->w_gate, w->w_up, nullptr, 2, F, H, st);
    GemvArgs gd{};
    gd.mode = GEMV_SWIGLU;
    gd.pend = g.part;
    gd.pend_plan = plan;
    gd.pend_ld = 2 * seg_pad_of(c, F);
    gd.f_pad = seg_pad_of(c, F);
    gd.ns = norm_scale(c);
    c->row.pend_plan = enqueue_gemv(c, gd, w->w_down, nullptr, nullptr, 1, H, F, st);
    c->row.pend = gd.part;
}

// Brings a single-row call's row into dst (pending update added), with the next norm's input if a
// gain is given.
void finish_row(cats_ctx* c, float* dst, const void* gain, hipStream_t st) {
    if (!c->row.pend && c->row.x == dst && !gain) return;
    ResidualNormArgs rn;
    rn.x = dst;
    rn.x_in = c->row.x == dst ? nullptr : c->row.x;
    rn.embed = nullptr;
    rn.token = nullptr;
    rn.part = c->row.pend;
    rn.plan = c->row.pend ? c->row.pend_plan : GemmPlan{1, GEMM_KC, 1, 1, 1};
    rn.gain = static_cast<const bf16_t*>(gain);
    rn.xn = c->xn;
    rn.xn_lo = c->xn_lo;
    rn.ss = c->ss;
    rn.T = 1;
    rn.H = c->d.hidden;
    rn.eps = c->d.rms_eps;
    launch_residual_norm(rn, st);
    c->row.x = dst;
    c->row.pend = nullptr;
}

void enqueue_rope_table(cats_ctx* c, int ctx_len, hipStream_t st) {
    RopeTableArgs r;
    r.depth = c->depth;
    r.cs = c->rope_cs;
    r.T = c->T;
    r.d = c->d.head_dim;
    r.ctx_len = ctx_len;
    r.base = c->d.rope_base;
    launch_rope_table(r, st);
}

// typical: also the per-node log-sum-exp / entropy and, per node, whether its token passes the
// typical criterion at its parent (needs the whole tree as rows)
void enqueue_lm_head(cats_ctx* c, const void* w_lm, float* logits_out, int32_t* argmax_out,
                     float* margin_out, hipStream_t st, bool typical = false) {
    GemmPlan plan;
    const float* part = c->part;
    if (c->rows == 1) {
        // with a residual update pending, it and the final norm ride in the product
        GemvArgs g = c->row.pend ? gemv_norm(c, c->row.next_gain, nullptr) : gemv_plain(c->xn, c->xn_lo);
        // Only the greedy token wanted, and every workgroup of the product ends up with complete
        // sums (true of the 7B and 13B shapes on 256 compute units): the product picks it itself.
        if (!logits_out && !margin_out && !typical &&
            plan_whole_tiles(make_gemm_plan(seg_pad_of(c, c->d.vocab), c->d.hidden, target_wgs(c), 1))) {
            g.amax = argmax_out;
            g.am_best = c->am_wg_best;
            g.am_idx = c->am_wg_idx;
            g.am_arrivals = c->am_arrivals;
            enqueue_gemv(c, g, w_lm, nullptr, nullptr, 1, c->d.vocab, c->d.hidden, st);
            return;
        }
        plan = enqueue_gemv(c, g, w_lm, nullptr, nullptr, 1, c->d.vocab, c->d.hidden, st);
        part = g.part;
    } else {
        plan = enqueue_gemm(c, c->xn, c->xn_lo, w_lm, nullptr, nullptr, 1, c->d.vocab, c->d.hidden, st);
    }
    ArgmaxArgs am;
    am.part = part;
    am.plan = plan;
    am.ns = norm_scale(c);
    am.T = c->rows;
    am.V = c->d.vocab;
    am.ld = seg_pad_of(c, c->d.vocab);
    am.logits = logits_out;
    am.amax = argmax_out;
    am.slice_best = c->am_best;
    am.slice_second = c->am_second;
    am.slice_idx = c->am_idx;
    am.arrivals = c->am_arrivals;
    am.margin = margin_out;
    am.inv_temp = c->typ_inv_temp;
    am.lse = typical ? c->typ_lse : nullptr;
    am.entropy = c->typ_entropy;
    am.slice_stat = c->typ_slice;
    launch_argmax(am, st);
    if (typical) {
        TypicalArgs ta;
        ta.token = c->token;
        ta.parent = c->parent;
        ta.part = part;
        ta.plan = plan;
        ta.ns = am.ns;
        ta.T = c->T;
        ta.ld = am.ld;
        ta.lse = c->typ_lse;
        ta.entropy = c->typ_entropy;
        ta.inv_temp = c->typ_inv_temp;
        ta.epsilon = c->typ_epsilon;
        ta.delta = c->typ_delta;
        ta.edge_ok = c->typ_edge;
        ta.prob = c->typ_prob;
        ta.thr = c->typ_thr;
        launch_typical_edges(ta, st);
    }
}

void enqueue_compact(cats_ctx* c, const cats_kv_layer* kv, int layer_begin, int layer_end, int ctx_len,
                     const cats_accept_result* res_dev, hipStream_t st) {
    if (layer_end <= layer_begin) return;
    CompactArgs ca;
    ca.n_layers = layer_end - layer_begin;
    for (int l = layer_begin; l < layer_end; ++l) {
        ca.k[l - layer_begin] = static_cast<bf16_t*>(kv[l].k);
        ca.v[l - layer_begin] = static_cast<bf16_t*>(kv[l].v);
    }
    ca.nh = c->d.n_heads;
    ca.d = c->d.head_dim;
    ca.max_ctx = c->d.max_ctx;
    ca.ctx_len = ctx_len;
    ca.res = res_dev;
    launch_compact(ca, st);
}

int enqueue_accept_compact(cats_ctx* c, const int32_t* amax, const cats_kv_layer* kv, int layer_begin,
                           int layer_end, int ctx_len, cats_accept_result* out_dev,
                           cats_accept_result* out_host, hipStream_t st, bool typical = false) {
    launch_accept(c->token, c->parent, c->depth, amax, typical ? c->typ_edge : nullptr, c->T, ctx_len, out_dev,
                  st);
    enqueue_compact(c, kv, layer_begin, layer_end, ctx_len, out_dev, st);
    HIP_TRY(hipGetLastError());
    if (out_host) {
        HIP_TRY(hipMemcpyAsync(out_host, out_dev, sizeof(cats_accept_result), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
    }
    return CATS_OK;
}

bool kv_ok(const cats_kv_layer* kv, int lb, int le) {
    if (!kv) return false;
    for (int l = lb; l < le; ++l)
        if (!kv[l].k || !kv[l].v) return false;
    return true;
}

}  // namespace

extern "C" {

int cats_create(const cats_model_desc* desc, cats_ctx** out) {
    if (!desc || !out) return CATS_EINVAL;
    const cats_model_desc& d = *desc;
    if (d.n_layers < 1 || d.n_layers > CATS_MAX_LAYERS || d.hidden < 64 || d.hidden % 64 != 0 ||
        d.hidden > 8192 || d.n_heads < 1 || (d.head_dim != 64 && d.head_dim != 128) ||
        d.n_heads * d.head_dim != d.hidden || d.ffn < 16 || d.ffn % 16 != 0 || d.vocab < 2 ||
        d.max_ctx < 64 || d.max_ctx % 64 != 0 || d.max_tree < 1 || d.max_tree > CATS_MAX_TREE ||
        !(d.rms_eps > 0.f) || !(d.rope_base > 1.f) || (d.packed_weights != 0 && d.packed_weights != 1))
        return CATS_EINVAL;
    cats_ctx* c = new (std::nothrow) cats_ctx();
    if (!c) return CATS_EHIP;
    c->d = d;
    c->T = 0;
    c->copy_stream = nullptr;
    for (int i = 0; i < 2; ++i) c->ev_copied[i] = c->ev_consumed[i] = nullptr;
    c->prof_on = false;
    c->prof_n = 0;
    for (auto& e : c->prof_ev) e = nullptr;
    if (hipGetDevice(&c->device) != hipSuccess ||
        hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess ||
        c->n_cus < 1) {
        delete c;
        return hip_fail(hipGetLastError());
    }
    const size_t Tm = d.max_tree, H = d.hidden, F = d.ffn;
    // split-K partials: the largest splits*N over the five GEMM shapes
    size_t part_cols = 0;
    const auto pad32 = [&](int n) { return d.packed_weights ? (n + 31) / 32 * 32 : n; };
    const int shapes[5][2] = {{3 * d.hidden, d.hidden}, {d.hidden, d.hidden}, {2 * pad32(d.ffn), d.hidden},
                              {d.hidden, d.ffn}, {pad32(d.vocab), d.hidden}};
    for (auto& s : shapes)
        for (int rows : {1, 33, 97})   // one row count per tile shape / pairing of the plan
            part_cols = std::max(part_cols, static_cast<size_t>(gemm_plan_max_pieces(
                                                make_gemm_plan(s[0], s[1], target_wgs(c), rows))) * s[0]);
    c->part_elems = part_cols * Tm;
    c->attn_max_chunks = 32;
    const size_t t_pad = (Tm + 31) / 32 * 32;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += align256(bytes);
        return o;
    };
    const size_t o_tok = take(Tm * 4), o_par = take(Tm * 4), o_dep = take(Tm * 4);
    const size_t o_anc = take(Tm * sizeof(u32x4));
    const size_t o_x = take(Tm * H * 4), o_xn = take(Tm * H * 2), o_q = take(Tm * H * 2);
    const size_t o_attn = take(Tm * H * 2), o_h = take(Tm * F * 2);
    const size_t o_xn_lo = take(Tm * H * 2), o_q_lo = take(Tm * H * 2), o_attn_lo = take(Tm * H * 2);
    const size_t o_h_lo = take(Tm * F * 2);
    const size_t o_ss = take(Tm * SS_STRIDE * 4);
    const size_t o_part = take(c->part_elems * 4);
    const size_t o_xrow = take(H * 4), o_partrow = take(part_cols * 4);
    const size_t o_cs = take(Tm * (d.head_dim / 2) * sizeof(float2));
    const size_t o_po = take(static_cast<size_t>(d.n_heads) * c->attn_max_chunks * t_pad * d.head_dim * 4);
    const size_t o_pml = take(static_cast<size_t>(d.n_heads) * c->attn_max_chunks * t_pad * 2 * 4);
    const size_t o_aarr = take(static_cast<size_t>(d.n_heads) * ATTN_MAX_QGROUPS * 4);   // zero from the memset below
    const size_t o_klo = take(static_cast<size_t>(d.n_heads) * TREE_WIN * d.head_dim * 2);
    const size_t o_vlo = take(static_cast<size_t>(d.n_heads) * TREE_WIN * d.head_dim * 2);
    const size_t o_amax = take(Tm * 4);
    const size_t o_sb = take(Tm * ARGMAX_SLICES * 4), o_s2 = take(Tm * ARGMAX_SLICES * 4);
    const size_t o_si = take(Tm * ARGMAX_SLICES * 4), o_arr = take(Tm * 4);   // zero from the memset below
    const size_t o_wb = take(static_cast<size_t>(c->n_cus) * 4), o_wi = take(static_cast<size_t>(c->n_cus) * 4);
    const size_t o_tl = take(Tm * 4), o_te = take(Tm * 4), o_ts = take(Tm * ARGMAX_SLICES * 3 * 4);
    const size_t o_tp = take(Tm * 4), o_tt = take(Tm * 4), o_tg = take(Tm);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->flat), off);
    if (e != hipSuccess) {
        delete c;
        return hip_fail(e);
    }
    // The zeros (arrival counters, unused sum-of-squares slots) must be in place before a first
    // call on any stream, also one that does not synchronise with the null stream: wait here once.
    e = hipMemset(c->flat, 0, off);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) {
        (void)hipFree(c->flat);
        delete c;
        return hip_fail(e);
    }
    char* b = c->flat;
    c->token = reinterpret_cast<int32_t*>(b + o_tok);
    c->parent = reinterpret_cast<int32_t*>(b + o_par);
    c->depth = reinterpret_cast<int32_t*>(b + o_dep);
    c->anc = reinterpret_cast<u32x4*>(b + o_anc);
    c->x = reinterpret_cast<float*>(b + o_x);
    c->xn = reinterpret_cast<bf16_t*>(b + o_xn);
    c->q = reinterpret_cast<bf16_t*>(b + o_q);
    c->attn = reinterpret_cast<bf16_t*>(b + o_attn);
    c->hact = reinterpret_cast<bf16_t*>(b + o_h);
    c->xn_lo = reinterpret_cast<bf16_t*>(b + o_xn_lo);
    c->q_lo = reinterpret_cast<bf16_t*>(b + o_q_lo);
    c->attn_lo = reinterpret_cast<bf16_t*>(b + o_attn_lo);
    c->hact_lo = reinterpret_cast<bf16_t*>(b + o_h_lo);
    c->ss = reinterpret_cast<float*>(b + o_ss);
    c->part = reinterpret_cast<float*>(b + o_part);
    c->x_row = reinterpret_cast<float*>(b + o_xrow);
    c->part_row = reinterpret_cast<float*>(b + o_partrow);
    c->rope_cs = reinterpret_cast<float2*>(b + o_cs);
    c->attn_po = reinterpret_cast<float*>(b + o_po);
    c->attn_pml = reinterpret_cast<float*>(b + o_pml);
    c->attn_arrivals = reinterpret_cast<int*>(b + o_aarr);
    c->k_lo = reinterpret_cast<bf16_t*>(b + o_klo);
    c->vt_lo = reinterpret_cast<bf16_t*>(b + o_vlo);
    c->amax = reinterpret_cast<int32_t*>(b + o_amax);
    c->am_best = reinterpret_cast<float*>(b + o_sb);
    c->am_second = reinterpret_cast<float*>(b + o_s2);
    c->am_idx = reinterpret_cast<int*>(b + o_si);
    c->am_arrivals = reinterpret_cast<int*>(b + o_arr);
    c->am_wg_best = reinterpret_cast<float*>(b + o_wb);
    c->am_wg_idx = reinterpret_cast<int*>(b + o_wi);
    c->typ_lse = reinterpret_cast<float*>(b + o_tl);
    c->typ_entropy = reinterpret_cast<float*>(b + o_te);
    c->typ_slice = reinterpret_cast<float*>(b + o_ts);
    c->typ_prob = reinterpret_cast<float*>(b + o_tp);
    c->typ_thr = reinterpret_cast<float*>(b + o_tt);
    c->typ_edge = reinterpret_cast<uint8_t*>(b + o_tg);
    *out = c;
    return CATS_OK;
}

int cats_destroy(cats_ctx* ctx) {
    if (!ctx) return CATS_EINVAL;
    for (auto& ev : ctx->prof_ev)
        if (ev) (void)hipEventDestroy(ev);
    for (int i = 0; i < 2; ++i) {
        if (ctx->ev_copied[i]) (void)hipEventDestroy(ctx->ev_copied[i]);
        if (ctx->ev_consumed[i]) (void)hipEventDestroy(ctx->ev_consumed[i]);
    }
    if (ctx->copy_stream) (void)hipStreamDestroy(ctx->copy_stream);
    hipError_t e = hipFree(ctx->flat);
    delete ctx;
    return e == hipSuccess ? CATS_OK : hip_fail(e);
}

int cats_set_tree(cats_ctx* ctx, const cats_tree* tree, void* stream) {
    if (!ctx || !tree || !tree->token || !tree->parent || !tree->depth) return CATS_EINVAL;
    const int n = tree->n;
    if (n < 1 || n > ctx->d.max_tree) return CATS_EINVAL;
    if (tree->parent[0] != -1 || tree->depth[0] != 0) return CATS_EINVAL;
    for (int i = 0; i < n; ++i) {
        if (tree->token[i] < 0 || tree->token[i] >= ctx->d.vocab) return CATS_EINVAL;
        if (i > 0) {
            const int p = tree->parent[i];
            if (p < 0 || p >= i) return CATS_EINVAL;
            if (tree->depth[i] != tree->depth[p] + 1 || tree->depth[i] > CATS_MAX_DEPTH) return CATS_EINVAL;
        }
    }
    TreeUploadArgs up;
    std::memset(&up, 0, sizeof up);
    std::memcpy(up.token, tree->token, sizeof(int32_t) * n);
    std::memcpy(up.parent, tree->parent, sizeof(int32_t) * n);
    std::memcpy(up.depth, tree->depth, sizeof(int32_t) * n);
    launch_tree_upload(up, n, ctx->token, ctx->parent, ctx->depth, as_stream(stream));
    launch_tree_masks(ctx->parent, n, ctx->anc, as_stream(stream));
    HIP_TRY(hipGetLastError());
    std::memcpy(ctx->h_parent, tree->parent, sizeof(int32_t) * n);
    std::memcpy(ctx->h_depth, tree->depth, sizeof(int32_t) * n);
    ctx->T = n;
    return CATS_OK;
}

int cats_verify_layer(cats_ctx* ctx, const cats_layer_weights* w, float* hidden, const cats_kv_layer* kv,
                      int32_t ctx_len, void* stream) {
    const int rc = check_ctx_len(ctx, ctx_len);
    if (rc != CATS_OK) return rc;
    if (!layer_ok(w) || !hidden || !kv_ok(kv, 0, 1)) return CATS_EINVAL;
    hipStream_t st = as_stream(stream);
    enqueue_rope_table(ctx, ctx_len, st);
    ResidualNormArgs rn;
    rn.x = hidden;
    rn.x_in = nullptr;
    rn.embed = nullptr;
    rn.token = nullptr;
    rn.part = nullptr;
    rn.plan = GemmPlan{1, GEMM_KC, 1, 1, 1};
    rn.gain = static_cast<const bf16_t*>(w->g_attn);
    rn.xn = ctx->xn;
    rn.xn_lo = ctx->xn_lo;
    rn.ss = ctx->ss;
    rn.T = ctx->T;
    rn.H = ctx->d.hidden;
    rn.eps = ctx->d.rms_eps;
    launch_residual_norm(rn, st);
    if (ctx->rows == 1) {
        ctx->row.x = hidden;
        enqueue_layer_row(ctx, w, kv, ctx_len, nullptr, st);
        finish_row(ctx, hidden, nullptr, st);
    } else {
        enqueue_layer(ctx, w, hidden, kv, ctx_len, nullptr, st);
    }
    HIP_TRY(hipGetLastError());
    return CATS_OK;
}

int cats_tree_attention(cats_ctx* ctx, const void* q, const cats_kv_layer* kv, int32_t ctx_len, void* out,
                        void* stream) {
    const int rc = check_ctx_len(ctx, ctx_len);
    if (rc != CATS_OK) return rc;
    if (!q || !out || !kv_ok(kv, 0, 1)) return CATS_EINVAL;
    enqueue_attention(ctx, static_cast<const bf16_t*>(q), nullptr, kv, ctx_len, static_cast<bf16_t*>(out),
                      nullptr, false, as_stream(stream));
    HIP_TRY(hipGetLastError());
    return CATS_OK;
}

int cats_accept_and_compact(cats_ctx* ctx, const int32_t* node_argmax, const cats_kv_layer* kv,
                            int32_t layer_begin, int32_t layer_end, int32_t ctx_len,
                            cats_accept_result* out_dev, cats_accept_result* out_host, void* stream) {
    const int rc = check_ctx_len(ctx, ctx_len);
    if (rc != CATS_OK) return rc;
    if (!node_argmax || !out_dev || layer_begin < 0 || layer_end < layer_begin ||
        layer_end > ctx->d.n_layers)
        return CATS_EINVAL;
    if (layer_end > layer_begin && !kv_ok(kv, layer_begin, layer_end)) return CATS_EINVAL;
    return enqueue_accept_compact(ctx, node_argmax, kv, layer_begin, layer_end, ctx_len, out_dev, out_host,
                                  as_stream(stream));
}

int cats_lm_head_argmax(cats_ctx* ctx, const float* hidden, int32_t n_rows, const void* g_final,
                        const void* w_lm, float* logits_out, int32_t* argmax_out, float* margin_out,
                        void* stream) {
    if (!ctx) return CATS_EINVAL;
    if (!hidden || !g_final || !w_lm || !argmax_out) return CATS_EINVAL;
    if (n_rows < 1 || n_rows > ctx->d.max_tree) return CATS_EINVAL;
    ctx->n0 = 0;
    ctx->rows = n_rows;
    ctx->row.pend = nullptr;
    ctx->row.embed = nullptr;
    hipStream_t st = as_stream(stream);
    ResidualNormArgs rn;
    rn.x = const_cast<float*>(hidden);  // read only: no source/partials given, so nothing is written back
    rn.x_in = nullptr;
    rn.embed = nullptr;
    rn.token = nullptr;
    rn.part = nullptr;
    rn.plan = GemmPlan{1, GEMM_KC, 1, 1, 1};
    rn.gain = static_cast<const bf16_t*>(g_final);
    rn.xn = ctx->xn;
    rn.xn_lo = ctx->xn_lo;
    rn.ss = ctx->ss;
    rn.T = ctx->rows;
    rn.H = ctx->d.hidden;
    rn.eps = ctx->d.rms_eps;
    launch_residual_norm(rn, st);
    enqueue_lm_head(ctx, w_lm, logits_out, argmax_out, margin_out, st);
    HIP_TRY(hipGetLastError());
    return CATS_OK;
}

// Rows n0..T-1 of the residual stream from the embedding table or from the caller's rows, plus
// the first layer's normalised input; then layers [layer_begin, layer_end).
static void enqueue_rows_and_layers(cats_ctx* ctx, const cats_layer_weights* layers, int layer_begin,
                                    int layer_end, const void* embed, const float* hidden_in,
                                    const void* last_gain, const cats_kv_layer* kv, int ctx_len,
                                    hipStream_t st) {
    enqueue_rope_table(ctx, ctx_len, st);
    ResidualNormArgs rn;
    rn.x = ctx->x;
    rn.x_in = hidden_in;
    rn.embed = static_cast<const bf16_t*>(embed);
    rn.token = ctx->token + ctx->n0;
    rn.part = nullptr;
    rn.plan = GemmPlan{1, GEMM_KC, 1, 1, 1};
    rn.gain = static_cast<const bf16_t*>(layer_end > layer_begin ? layers[layer_begin].g_attn : last_gain);
    rn.xn = ctx->xn;
    rn.xn_lo = ctx->xn_lo;
    rn.ss = ctx->ss;
    rn.T = ctx->rows;
    rn.H = ctx->d.hidden;
    rn.eps = ctx->d.rms_eps;
    launch_residual_norm(rn, st);
    if (ctx->rows == 1) {
        // single row: the last layer's residual update stays pending for the LM head's product
        // (which also leaves the final row in ctx->row.x), or is carried out here if none follows
        ctx->row.x = ctx->x;
        ctx->row.pend = nullptr;
        for (int l = layer_begin; l < layer_end; ++l) enqueue_layer_row(ctx, &layers[l], &kv[l], ctx_len, nullptr, st);
        if (last_gain)
            ctx->row.next_gain = last_gain;
        else
            finish_row(ctx, ctx->x, nullptr, st);
        return;
    }
    for (int l = layer_begin; l < layer_end; ++l) {
        const void* next_gain = (l + 1 < layer_end) ? layers[l + 1].g_attn : last_gain;
        enqueue_layer(ctx, &layers[l], ctx->x, &kv[l], ctx_len, next_gain, st);
    }
}

static int check_layer_range(const cats_ctx* ctx, const cats_layer_weights* layers, int layer_begin,
                             int layer_end, const cats_kv_layer* kv) {
    if (layer_begin < 0 || layer_end < layer_begin || layer_end > ctx->d.n_layers) return CATS_EINVAL;
    if (layer_end > layer_begin) {
        if (!layers || !kv_ok(kv, layer_begin, layer_end)) return CATS_EINVAL;
        for (int l = layer_begin; l < layer_end; ++l)
            if (!layer_ok(&layers[l])) return CATS_EINVAL;
    }
    return CATS_OK;
}

int cats_verify_tree(cats_ctx* ctx, const cats_layer_weights* layers, int32_t layer_begin, int32_t layer_end,
                     const void* embed, const float* hidden_in, const void* g_final, const void* w_lm,
                     const cats_kv_layer* kv, int32_t ctx_len, float* hidden_out, float* logits_out,
                     int32_t* argmax_out, float* margin_out, cats_accept_result* out_dev,
                     cats_accept_result* out_host, void* stream) {
    int rc = check_ctx_len(ctx, ctx_len);
    if (rc != CATS_OK) return rc;
    if ((rc = check_layer_range(ctx, layers, layer_begin, layer_end, kv)) != CATS_OK) return rc;
    if ((embed == nullptr) == (hidden_in == nullptr)) return CATS_EINVAL;  // exactly one input source
    if (!g_final || !w_lm || !out_dev) return CATS_EINVAL;
    hipStream_t st = as_stream(stream);
    const int T = ctx->T, H = ctx->d.hidden;
    enqueue_rows_and_layers(ctx, layers, layer_begin, layer_end, embed, hidden_in, g_final, kv, ctx_len, st);
    if (hidden_out && T > 1)
        HIP_TRY(hipMemcpyAsync(hidden_out, ctx->x, sizeof(float) * T * H, hipMemcpyDeviceToDevice, st));
    int32_t* amax = argmax_out ? argmax_out : ctx->amax;
    const bool typical = ctx->accept_mode == 1;
    enqueue_lm_head(ctx, w_lm, logits_out, amax, margin_out, st, typical);
    if (hidden_out && T == 1)   // a single row is final only once the LM head's product has updated it
        HIP_TRY(hipMemcpyAsync(hidden_out, ctx->row.x, sizeof(float) * H, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipGetLastError());
    return enqueue_accept_compact(ctx, amax, kv, layer_begin, layer_end, ctx_len, out_dev, out_host, st,
                                  typical);
}

int cats_set_acceptance(cats_ctx* ctx, int32_t mode, float epsilon, float delta, float temperature) {
    if (!ctx || (mode != 0 && mode != 1)) return CATS_EINVAL;
    if (mode == 1 && !(epsilon >= 0.f && delta >= 0.f && temperature > 0.f)) return CATS_EINVAL;
    ctx->accept_mode = mode;
    if (mode == 1) {
        ctx->typ_epsilon = epsilon;
        ctx->typ_delta = delta;
        ctx->typ_inv_temp = 1.f / temperature;
    }
    return CATS_OK;
}

int cats_typical_stats(cats_ctx* ctx, float* lse_out, float* entropy_out, float* prob_out, float* threshold_out,
                       void* stream) {
    if (!ctx) return CATS_EINVAL;
    if (ctx->T < 1) return CATS_ESTATE;
    hipStream_t st = as_stream(stream);
    const size_t bytes = sizeof(float) * ctx->T;
    const float* src[4] = {ctx->typ_lse, ctx->typ_entropy, ctx->typ_prob, ctx->typ_thr};
    float* dst[4] = {lse_out, entropy_out, prob_out, threshold_out};
    for (int i = 0; i < 4; ++i)
        if (dst[i]) HIP_TRY(hipMemcpyAsync(dst[i], src[i], bytes, hipMemcpyDeviceToDevice, st));
    return CATS_OK;
}

int cats_compact_along(cats_ctx* ctx, const cats_accept_result* result_dev, const cats_kv_layer* kv,
                       int32_t layer_begin, int32_t layer_end, int32_t ctx_len, void* stream) {
    const int rc = check_ctx_len(ctx, ctx_len);
    if (rc != CATS_OK) return rc;
    if (!result_dev || layer_begin < 0 || layer_end < layer_begin || layer_end > ctx->d.n_layers)
        return CATS_EINVAL;
    if (layer_end > layer_begin && !kv_ok(kv, layer_begin, layer_end)) return CATS_EINVAL;
    enqueue_compact(ctx, kv, layer_begin, layer_end, ctx_len, result_dev, as_stream(stream));
    HIP_TRY(hipGetLastError());
    return CATS_OK;
}

int cats_verify_nodes(cats_ctx* ctx, const cats_layer_weights* layers, int32_t layer_begin, int32_t layer_end,
                      const void* embed, const float* hidden_in, const cats_kv_layer* kv, int32_t ctx_len,
                      int32_t node_begin, float* hidden_out, void* stream) {
    int rc = check_ctx_len(ctx, ctx_len);
    if (rc != CATS_OK) return rc;
    if ((rc = check_layer_range(ctx, layers, layer_begin, layer_end, kv)) != CATS_OK) return rc;
    if ((embed == nullptr) == (hidden_in == nullptr)) return CATS_EINVAL;
    if (node_begin < 0 || node_begin >= ctx->T || !hidden_out) return CATS_EINVAL;
    hipStream_t st = as_stream(stream);
    ctx->n0 = node_begin;   // read by the enqueue helpers
    ctx->rows = ctx->T - node_begin;
    enqueue_rows_and_layers(ctx, layers, layer_begin, layer_end, embed, hidden_in, nullptr, kv, ctx_len, st);
    const size_t bytes = sizeof(float) * static_cast<size_t>(ctx->T - node_begin) * ctx->d.hidden;
    HIP_TRY(hipMemcpyAsync(hidden_out, ctx->x, bytes, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipGetLastError());
    return CATS_OK;
}

int cats_draft_chain(cats_ctx* ctx, const cats_layer_weights* layers, int32_t layer_begin, int32_t layer_end,
                     const cats_layer_weights* adapter, const void* g_adapter_out, const void* w_lm,
                     const void* embed, const cats_kv_layer* kv, const cats_kv_layer* kv_adapter, int32_t ctx_len,
                     int32_t root_token, int32_t gamma, int32_t* tokens_out, float* hidden_out, void* stream) {
    if (!ctx || !adapter || !g_adapter_out || !w_lm || !embed || !tokens_out) return CATS_EINVAL;
    if (gamma < 1 || gamma > CATS_MAX_DEPTH || gamma + 1 > ctx->d.max_tree) return CATS_EINVAL;
    if (root_token < 0 || root_token >= ctx->d.vocab || ctx_len < 0) return CATS_EINVAL;
    if (static_cast<int64_t>(ctx_len) + gamma + 1 > ctx->d.max_ctx) return CATS_ECAPACITY;
    int rc = check_layer_range(ctx, layers, layer_begin, layer_end, kv);
    if (rc != CATS_OK) return rc;
    if (layer_end <= layer_begin) return CATS_EINVAL;
    if (!layer_ok(adapter) || has_ffn(adapter) || !kv_ok(kv_adapter, 0, 1)) return CATS_EINVAL;
    hipStream_t st = as_stream(stream);
    // the chain root, d_1 .. d_gamma as the context's tree; the draft tokens are filled in on
    // the device as they are produced
    const int n = gamma + 1;
    TreeUploadArgs up;
    std::memset(&up, 0, sizeof up);
    up.token[0] = root_token;
    for (int i = 0; i < n; ++i) {
        up.parent[i] = i - 1;
        up.depth[i] = i;
        ctx->h_parent[i] = i - 1;
        ctx->h_depth[i] = i;
    }
    launch_tree_upload(up, n, ctx->token, ctx->parent, ctx->depth, st);
    launch_tree_masks(ctx->parent, n, ctx->anc, st);
    ctx->T = n;
    enqueue_rope_table(ctx, ctx_len, st);
    const size_t H = ctx->d.hidden;
    for (int k = 0; k <= gamma; ++k) {
        if (k == gamma && !hidden_out) break;   // the last draft only needs its hidden state
        ctx->n0 = k;
        ctx->rows = 1;
        // the row starts as the embedding of token k (written by the step before); the first
        // product reads it from the table
        ctx->row.x = ctx->x;
        ctx->row.embed = static_cast<const bf16_t*>(embed);
        ctx->row.token = ctx->token + k;
        ctx->row.pend = nullptr;
        for (int l = layer_begin; l < layer_end; ++l) enqueue_layer_row(ctx, &layers[l], &kv[l], ctx_len, nullptr, st);
        // the row after the draft layers is written straight into hidden_out: by the adapter's first
        // product, which carries out the last layer's residual update, or by a row kernel at the end
        float* h_k = hidden_out ? hidden_out + k * H : nullptr;
        if (k == gamma) {
            finish_row(ctx, h_k, nullptr, st);
            break;
        }
        enqueue_layer_row(ctx, adapter, kv_adapter, ctx_len, h_k, st);
        ctx->row.next_gain = g_adapter_out;
        enqueue_lm_head(ctx, w_lm, nullptr, ctx->token + k + 1, nullptr, st);
    }
    HIP_TRY(hipMemcpyAsync(tokens_out, ctx->token, sizeof(int32_t) * n, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipGetLastError());
    ctx->n0 = 0;
    ctx->rows = n;
    return CATS_OK;
}

int cats_build_tree(int32_t root_token, const int32_t* main_tokens, int32_t gamma, const int32_t* corrections,
                    int32_t capacity, int32_t* token, int32_t* parent, int32_t* depth, int32_t* n_out,
                    int32_t* corr_node) {
    if (gamma < 0 || gamma > CATS_MAX_DEPTH || (gamma > 0 && !main_tokens) || !token || !parent || !depth || !n_out)
        return CATS_EINVAL;
    int n_corr = 0;
    for (int i = 0; i < gamma; ++i)
        if (corrections && corrections[i] >= 0 && corrections[i] != main_tokens[i]) ++n_corr;
    const int n = 1 + gamma + n_corr;
    if (n > capacity || n > CATS_MAX_TREE) return CATS_ECAPACITY;
    token[0] = root_token;
    parent[0] = -1;
    depth[0] = 0;
    for (int i = 0; i < gamma; ++i) {   // draft position i is node i+1, child of node i
        token[i + 1] = main_tokens[i];
        parent[i + 1] = i;
        depth[i + 1] = i + 1;
    }
    int next = gamma + 1;
    for (int i = 0; i < gamma; ++i) {   // a correction at position i is a sibling of draft position i
        const bool has = corrections && corrections[i] >= 0 && corrections[i] != main_tokens[i];
        if (has) {
            token[next] = corrections[i];
            parent[next] = i;
            depth[next] = i + 1;
        }
        if (corr_node) corr_node[i] = has ? next : -1;
        if (has) ++next;
    }
    *n_out = n;
    return CATS_OK;
}

int cats_profile_gemm(cats_ctx* ctx, int enable) {
    if (!ctx) return CATS_EINVAL;
    if (enable && !ctx->prof_ev[0])
        for (auto& ev : ctx->prof_ev) HIP_TRY(hipEventCreate(&ev));
    ctx->prof_on = enable != 0;
    ctx->prof_n = 0;
    return CATS_OK;
}

int cats_profile_gemm_read(cats_ctx* ctx, float* total_ms, int32_t* launches) {
    if (!ctx || !total_ms || !launches) return CATS_EINVAL;
    float sum = 0.f;
    for (int i = 0; i < ctx->prof_n; ++i) {
        HIP_TRY(hipEventSynchronize(ctx->prof_ev[2 * i + 1]));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
        sum += ms;
    }
    *total_ms = sum;
    *launches = ctx->prof_n;
    ctx->prof_n = 0;
    return CATS_OK;
}

// bf16 elements of the nine arrays of one layer, in staging order
static void layer_array_elems(const cats_model_desc& d, size_t out[9]) {
    const int H = d.hidden, F = d.ffn;
    const int shp[7][2] = {{H, H}, {H, H}, {H, H}, {H, H}, {F, H}, {F, H}, {H, F}};
    for (int i = 0; i < 7; ++i)
        out[i] = d.packed_weights ? packed_matrix_elems(shp[i][0], shp[i][1])
                                  : static_cast<size_t>(shp[i][0]) * shp[i][1];
    out[7] = out[8] = H;
}

size_t cats_layer_weight_bytes(const cats_model_desc* desc) {
    if (!desc) return 0;
    size_t e[9], tot = 0;
    layer_array_elems(*desc, e);
    for (size_t v : e) tot += v;
    return tot * sizeof(bf16_t);
}

size_t cats_packed_matrix_bytes(int32_t rows, int32_t cols) {
    if (rows < 1 || cols < 1) return 0;
    return packed_matrix_elems(rows, cols) * sizeof(bf16_t);
}

int cats_pack_matrix(const void* src, void* dst, int32_t rows, int32_t cols, void* stream) {
    if (!src || !dst || rows < 1 || cols < 16 || cols % 16 != 0) return CATS_EINVAL;
    launch_pack_matrix(static_cast<const bf16_t*>(src), static_cast<bf16_t*>(dst), rows, cols, as_stream(stream));
    HIP_TRY(hipGetLastError());
    return CATS_OK;
}

int cats_verify_tree_streamed(cats_ctx* ctx, const cats_layer_weights* host_layers, int32_t layer_begin,
                              int32_t layer_end, void* const staging[2], const void* embed,
                              const float* hidden_in, const void* g_final, const void* w_lm,
                              const cats_kv_layer* kv, int32_t ctx_len, float* hidden_out, float* logits_out,
                              int32_t* argmax_out, float* margin_out, cats_accept_result* out_dev,
                              cats_accept_result* out_host, void* stream) {
    const int rc = check_ctx_len(ctx, ctx_len);
    if (rc != CATS_OK) return rc;
    if (layer_begin < 0 || layer_end <= layer_begin || layer_end > ctx->d.n_layers) return CATS_EINVAL;
    if ((embed == nullptr) == (hidden_in == nullptr)) return CATS_EINVAL;
    if (!g_final || !w_lm || !out_dev || !host_layers || !staging || !staging[0] || !staging[1] ||
        !kv_ok(kv, layer_begin, layer_end))
        return CATS_EINVAL;
    for (int l = layer_begin; l < layer_end; ++l)
        if (!layer_ok(&host_layers[l]) || !has_ffn(&host_layers[l])) return CATS_EINVAL;
    if (!ctx->copy_stream) {  // created on first use, at the default priority
        HIP_TRY(hipStreamCreateWithFlags(&ctx->copy_stream, hipStreamNonBlocking));
        for (int i = 0; i < 2; ++i) {
            HIP_TRY(hipEventCreateWithFlags(&ctx->ev_copied[i], hipEventDisableTiming));
            HIP_TRY(hipEventCreateWithFlags(&ctx->ev_consumed[i], hipEventDisableTiming));
        }
    }
    hipStream_t st = as_stream(stream), cs = ctx->copy_stream;
    const size_t H = ctx->d.hidden;
    const int T = ctx->T;
    // layout of one staged layer: wq | wk | wv | wo | w_gate | w_up | w_down | g_attn | g_ffn
    size_t sizes[9];
    layer_array_elems(ctx->d, sizes);
    auto staged = [&](int b) {
        cats_layer_weights w;
        const void** fields[9] = {&w.wq, &w.wk, &w.wv, &w.wo, &w.w_gate, &w.w_up, &w.w_down, &w.g_attn, &w.g_ffn};
        char* p = static_cast<char*>(staging[b]);
        for (int i = 0; i < 9; ++i) {
            *fields[i] = p;
            p += sizes[i] * sizeof(bf16_t);
        }
        return w;
    };
    auto enqueue_copy = [&](int l, bool wait_consumed) -> int {
        const int b = (l - layer_begin) & 1;
        if (wait_consumed) HIP_TRY(hipStreamWaitEvent(cs, ctx->ev_consumed[b], 0));
        const cats_layer_weights& hw = host_layers[l];
        const void* src[9] = {hw.wq, hw.wk, hw.wv, hw.wo, hw.w_gate, hw.w_up, hw.w_down, hw.g_attn, hw.g_ffn};
        char* p = static_cast<char*>(staging[b]);
        for (int i = 0; i < 9; ++i) {
            HIP_TRY(hipMemcpyAsync(p, src[i], sizes[i] * sizeof(bf16_t), hipMemcpyHostToDevice, cs));
            p += sizes[i] * sizeof(bf16_t);
        }
        HIP_TRY(hipEventRecord(ctx->ev_copied[b], cs));
        return CATS_OK;
    };

    // the copy stream must not overtake work already queued on the compute stream that may
    // still read the staging buffers (a previous call): order it behind that work once
    HIP_TRY(hipEventRecord(ctx->ev_consumed[0], st));
    HIP_TRY(hipStreamWaitEvent(cs, ctx->ev_consumed[0], 0));
    int erc = enqueue_copy(layer_begin, false);
    if (erc != CATS_OK) return erc;

    enqueue_rope_table(ctx, ctx_len, st);
    ResidualNormArgs rn;
    rn.x = ctx->x;
    rn.x_in = hidden_in;
    rn.embed = static_cast<const bf16_t*>(embed);
    rn.token = ctx->token;
    rn.part = nullptr;
    rn.plan = GemmPlan{1, GEMM_KC, 1, 1, 1};
    rn.gain = nullptr;  // input rows only; each layer's first norm is launched once its gains have arrived
    rn.xn = ctx->xn;
    rn.xn_lo = ctx->xn_lo;
    rn.ss = ctx->ss;
    rn.T = T;
    rn.H = ctx->d.hidden;
    rn.eps = ctx->d.rms_eps;
    launch_residual_norm(rn, st);
    rn.x_in = nullptr;
    rn.embed = nullptr;
    for (int l = layer_begin; l < layer_end; ++l) {
        const int b = (l - layer_begin) & 1;
        if (l + 1 < layer_end) {
            erc = enqueue_copy(l + 1, l + 1 - layer_begin >= 2);
            if (erc != CATS_OK) return erc;
        }
        HIP_TRY(hipStreamWaitEvent(st, ctx->ev_copied[b], 0));
        const cats_layer_weights w = staged(b);
        rn.gain = static_cast<const bf16_t*>(w.g_attn);
        launch_residual_norm(rn, st);
        enqueue_layer(ctx, &w, ctx->x, &kv[l], ctx_len, nullptr, st);
        HIP_TRY(hipEventRecord(ctx->ev_consumed[b], st));
    }
    rn.gain = static_cast<const bf16_t*>(g_final);
    launch_residual_norm(rn, st);
    if (hidden_out)
        HIP_TRY(hipMemcpyAsync(hidden_out, ctx->x, sizeof(float) * T * H, hipMemcpyDeviceToDevice, st));
    int32_t* amax = argmax_out ? argmax_out : ctx->amax;
    const bool typical = ctx->accept_mode == 1;
    enqueue_lm_head(ctx, w_lm, logits_out, amax, margin_out, st, typical);
    HIP_TRY(hipGetLastError());
    return enqueue_accept_compact(ctx, amax, kv, layer_begin, layer_end, ctx_len, out_dev, out_host, st,
                                  typical);
}

// ---------------------------------------------------------------- no-allocation entry point
// Scratch of cats_tree_attention_noalloc: a fixed array in the code object, one copy per GPU,
// held until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress; kernels and copies get the device address it returns.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[CATS_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int NOALLOC_MAX_DEVICES = 64;
struct NoallocDevice {
    unsigned char* ptr = nullptr;   // device address of this GPU's copy of `scratch`
    int n_cus = 0;
};
NoallocDevice g_noalloc[NOALLOC_MAX_DEVICES];
std::mutex g_noalloc_mutex;

// Address of the current device's scratch array, looked up once per device.
int noalloc_device(NoallocDevice** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return CATS_ECAPACITY;
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    NoallocDevice& d = g_noalloc[dev];
    if (!d.ptr) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return hip_fail(hipErrorInvalidSymbol);
        int n_cus = 0;
        HIP_TRY(hipDeviceGetAttribute(&n_cus, hipDeviceAttributeMultiprocessorCount, dev));
        if (n_cus < 1) return hip_fail(hipErrorInvalidDevice);
        d.n_cus = n_cus;
        d.ptr = static_cast<unsigned char*>(p);
    }
    *out = &d;
    return CATS_OK;
}
}  // namespace

int cats_tree_attention_noalloc(const void* q, const cats_kv_layer* kv, const int32_t* parent, int32_t n_nodes,
                                int32_t n_heads, int32_t head_dim, int32_t max_ctx, int32_t ctx_len, void* out,
                                void* stream) {
    if (!q || !out || !parent || !kv_ok(kv, 0, 1)) return CATS_EINVAL;
    if (n_nodes < 1 || n_heads < 1 || (head_dim != 64 && head_dim != 128) || max_ctx < 64 || max_ctx % 64 != 0 ||
        ctx_len < 0)
        return CATS_EINVAL;
    if (n_nodes > CATS_MAX_TREE) return CATS_ECAPACITY;
    if (static_cast<int64_t>(ctx_len) + n_nodes > max_ctx) return CATS_ECAPACITY;
    TreeUploadArgs up;
    std::memset(&up, 0, sizeof up);
    if (parent[0] != -1) return CATS_EINVAL;
    up.parent[0] = -1;
    for (int i = 1; i < n_nodes; ++i) {
        const int p = parent[i];
        if (p < 0 || p >= i) return CATS_EINVAL;
        up.parent[i] = p;
        up.depth[i] = up.depth[p] + 1;
        if (up.depth[i] > CATS_MAX_DEPTH) return CATS_EINVAL;
    }
    NoallocDevice* dev = nullptr;
    const int rc = noalloc_device(&dev);
    if (rc != CATS_OK) return rc;

    AttnArgs a;
    a.q = static_cast<const bf16_t*>(q);
    a.q_lo = nullptr;
    a.out = static_cast<bf16_t*>(out);
    a.out_lo = nullptr;
    a.k_lo = a.vt_lo = nullptr;
    a.lo_begin = a.lo_end = ctx_len;
    a.kc = static_cast<const bf16_t*>(kv->k);
    a.vt = static_cast<const bf16_t*>(kv->v);
    a.T = a.Tq = n_nodes;
    a.q0 = 0;
    a.H = n_heads * head_dim;
    a.nh = n_heads;
    a.d = head_dim;
    a.max_ctx = max_ctx;
    a.ctx_len = ctx_len;
    const int n_keys = ctx_len + n_nodes;
    const int n_blocks = (n_keys + ATTN_KB - 1) / ATTN_KB;
    a.n_chunks = attn_chunks(n_nodes, n_heads, 32, dev->n_cus, n_keys);
    a.t_pad = (n_nodes + 31) / 32 * 32;
    // layout of the scratch array: tree arrays, ancestor masks, then the chunk partials
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += align256(bytes);
        return o;
    };
    const size_t o_tok = take(CATS_MAX_TREE * 4), o_par = take(CATS_MAX_TREE * 4), o_dep = take(CATS_MAX_TREE * 4);
    const size_t o_anc = take(CATS_MAX_TREE * sizeof(u32x4));
    const int n_counters = n_heads * ((n_nodes + ATTN_QN - 1) / ATTN_QN);
    const size_t o_arr = take(static_cast<size_t>(n_counters) * sizeof(int));
    const size_t slots = static_cast<size_t>(n_heads) * a.n_chunks * a.t_pad;
    const size_t o_pml = take(slots * 2 * sizeof(float));
    const size_t o_po = take(slots * head_dim * sizeof(float));
    if (off > CATS_NOALLOC_SCRATCH_BYTES) return CATS_ECAPACITY;
    unsigned char* b = dev->ptr;
    int32_t* d_parent = reinterpret_cast<int32_t*>(b + o_par);
    a.anc = reinterpret_cast<u32x4*>(b + o_anc);
    a.pml = reinterpret_cast<float*>(b + o_pml);
    a.po = reinterpret_cast<float*>(b + o_po);
    a.arrivals = reinterpret_cast<int*>(b + o_arr);
    hipStream_t st = as_stream(stream);
    // the array keeps whatever the last call left: the arrival counters must start at zero
    launch_zero_i32(a.arrivals, n_counters, st);
    launch_tree_upload(up, n_nodes, reinterpret_cast<int32_t*>(b + o_tok), d_parent,
                       reinterpret_cast<int32_t*>(b + o_dep), st);
    launch_tree_masks(d_parent, n_nodes, reinterpret_cast<u32x4*>(b + o_anc), st);
    launch_attention(a, st);
    HIP_TRY(hipGetLastError());
    return CATS_OK;
}

const char* cats_gemm_kernel_name(void) { return "cats_gemm_skinny_bf16"; }

const char* cats_strerror(int status) {
    switch (status) {
        case CATS_OK: return "ok";
        case CATS_EINVAL: return "invalid argument (null pointer, bad shape, malformed tree or token out of range)";
        case CATS_ECAPACITY:
            return "capacity exceeded (ctx_len + tree size > max_ctx, more nodes than the arrays hold, or a shape too "
                   "large for the fixed scratch of the no-allocation entry point)";
        case CATS_ESTATE: return "no tree has been set on this context";
        case CATS_EHIP: return hipGetErrorString(g_last_hip);
        default: return "unknown status";
    }
}

}  // extern "C"
