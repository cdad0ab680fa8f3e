// CPU oracle for draft-tree verification (the target verification pass of
// the cascaded speculative decoding method: Sec. "Cascaded verification
// design", paragraph "Target verification pass", and Algorithm 1, Stage 3 and
// the walk / bonus / commit steps that follow it).
//
// THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, definition-level
// implementation used only to check the GPU library and to be timed beside it.
// It shares no code, header, table or helper with the GPU path and must never
// be called from it.
//
// Precision: `real` is float by default and double with -DCATS_ORACLE_F64.
// Weights arrive as bf16 bit patterns and are widened exactly.
//
// Layer shape (the paper names LLaMA-family targets without spelling the layer
// out; the benchmark configurations fix it): pre-norm RMSNorm, multi-head
// attention with rotary position embedding (half-split pairing: dimension j
// pairs with j + d/2, angle pos * base^(-2j/d)), SwiGLU feed-forward, no
// biases, untied LM head.
//
// Two independent routes to the same numbers live here:
//   oracle_causal_decode : ordinary token-at-a-time decoding with a KV cache
//                          (no tree concept at all) - the definition that
//                          lossless speculative decoding must reproduce;
//   oracle_tree_forward  : the batched pass over all tree nodes under the tree
//                          attention mask (Fig. 4 right, Algorithm 1 Stage 3).
// Tests pin the second against the first on every small tree.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifdef CATS_ORACLE_F64
typedef double real;
#else
typedef float real;
#endif

namespace {

inline real widen(uint16_t b) {
    uint32_t u = static_cast<uint32_t>(b) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<real>(f);
}

// y[n] = sum_k x[k] * W[n][k], W stored [N][K] (output-major) as bf16 bits.
void matvec(const real* x, const uint16_t* W, int K, int N, real* y) {
#pragma omp parallel
    {
        std::vector<real> row(K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            const uint16_t* w = W + static_cast<size_t>(n) * K;
            for (int k = 0; k < K; ++k) row[k] = widen(w[k]);
            real acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += x[k] * row[k];
            y[n] = acc;
        }
    }
}

// Y[t][n] = sum_k X[t][k] * W[n][k] for t < T: the same product for every row.
void linear(const real* X, const uint16_t* W, int T, int K, int N, real* Y) {
#pragma omp parallel
    {
        std::vector<real> row(K);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            const uint16_t* w = W + static_cast<size_t>(n) * K;
            for (int k = 0; k < K; ++k) row[k] = widen(w[k]);
            for (int t = 0; t < T; ++t) {
                const real* x = X + static_cast<size_t>(t) * K;
                real acc = 0;
#pragma omp simd reduction(+ : acc)
                for (int k = 0; k < K; ++k) acc += x[k] * row[k];
                Y[static_cast<size_t>(t) * N + n] = acc;
            }
        }
    }
}

// out = x / sqrt(mean(x^2) + eps) * g
void rmsnorm(const real* x, const uint16_t* g, int H, float eps, real* out) {
    real ss = 0;
    for (int j = 0; j < H; ++j) ss += x[j] * x[j];
    const real scale = real(1) / std::sqrt(ss / real(H) + real(eps));
    for (int j = 0; j < H; ++j) out[j] = x[j] * scale * widen(g[j]);
}

// Rotary embedding at position pos, applied head by head, in place.
void rope(real* v, int n_heads, int d, int pos, float base) {
    const int half = d / 2;
    for (int h = 0; h < n_heads; ++h) {
        real* p = v + static_cast<size_t>(h) * d;
        for (int j = 0; j < half; ++j) {
            const double inv_freq = std::pow(static_cast<double>(base), -2.0 * j / d);
            const double ang = static_cast<double>(pos) * inv_freq;
            const real c = static_cast<real>(std::cos(ang));
            const real s = static_cast<real>(std::sin(ang));
            const real a = p[j], b = p[j + half];
            p[j] = a * c - b * s;
            p[j + half] = a * s + b * c;
        }
    }
}

// Softmax attention of one query vector q[H] over the listed cache rows.
// Kc, Vc are [rows][H]; head h uses columns h*d .. h*d+d-1.
void attend(const real* q, const real* Kc, const real* Vc, const int32_t* rows, int n_rows,
            int n_heads, int d, real* out) {
    const int H = n_heads * d;
    const real inv_sqrt_d = real(1) / std::sqrt(static_cast<real>(d));
#pragma omp parallel for schedule(static)
    for (int h = 0; h < n_heads; ++h) {
        std::vector<real> s(n_rows);
        real mx = -INFINITY;
        for (int r = 0; r < n_rows; ++r) {
            const real* k = Kc + static_cast<size_t>(rows[r]) * H + h * d;
            real acc = 0;
            for (int j = 0; j < d; ++j) acc += q[h * d + j] * k[j];
            s[r] = acc * inv_sqrt_d;
            mx = std::max(mx, s[r]);
        }
        real denom = 0;
        for (int r = 0; r < n_rows; ++r) {
            s[r] = std::exp(s[r] - mx);
            denom += s[r];
        }
        real* o = out + h * d;
        for (int j = 0; j < d; ++j) o[j] = 0;
        for (int r = 0; r < n_rows; ++r) {
            const real p = s[r] / denom;
            const real* v = Vc + static_cast<size_t>(rows[r]) * H + h * d;
            for (int j = 0; j < d; ++j) o[j] += p * v[j];
        }
    }
}

inline real silu(real z) { return z / (real(1) + std::exp(-z)); }

}  // namespace

extern "C" {

struct oracle_dims {
    int32_t n_layers, hidden, n_heads, head_dim, ffn, vocab;
    float rms_eps, rope_base;
};

// One decoder layer's weights, bf16 bits, matrices stored [out][in].
struct oracle_layer {
    const uint16_t *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down, *g_attn, *g_ffn;
};

// Outcome of the greedy walk (Algorithm 1, walk + bonus + commit).
struct oracle_accept {
    int32_t n_accepted;   // accepted draft tokens, = depth of the last accepted node
    int32_t path[32];     // node indices root .. last accepted node (n_accepted + 1 entries)
    int32_t tokens[32];   // their token ids
    int32_t bonus_token;  // target's own next token after the last accepted node
    int32_t new_ctx_len;  // ctx_len + n_accepted + 1
};

int oracle_real_bytes(void) { return static_cast<int>(sizeof(real)); }

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// ---- single operations, exported so that tests can pin each one -----------

void oracle_rmsnorm(const real* x, const uint16_t* g, int H, float eps, real* out) {
    rmsnorm(x, g, H, eps, out);
}

void oracle_linear(const real* X, const uint16_t* W, int T, int K, int N, real* Y) {
    linear(X, W, T, K, N, Y);
}

void oracle_rope(real* v, int n_heads, int d, int pos, float base) { rope(v, n_heads, d, pos, base); }

void oracle_attend(const real* q, const real* Kc, const real* Vc, const int32_t* rows, int n_rows,
                   int n_heads, int d, real* out) {
    attend(q, Kc, Vc, rows, n_rows, n_heads, d, out);
}

// ---- ordinary causal decoding: the definition ------------------------------
//
// Feeds n inputs one at a time at positions ctx_len, ctx_len+1, ...  Each
// input is embed[tokens[i]] when embed is given, else hidden_in[i].  Layers
// [layer_begin, layer_end) are applied.  K/V caches are real arrays
// [n_layers][max_ctx][hidden] holding post-rotation keys; rows
// ctx_len .. ctx_len+n-1 of the layers used are written.  hidden_out[i] is the
// residual stream after the last applied layer.  Returns 0, or -1 on overflow.
int oracle_causal_decode(const oracle_dims* dm, const oracle_layer* layers, int layer_begin,
                         int layer_end, const uint16_t* embed, const real* hidden_in,
                         const int32_t* tokens, int n, real* kcache, real* vcache, int max_ctx,
                         int ctx_len, real* hidden_out) {
    const int H = dm->hidden, F = dm->ffn;
    if (ctx_len + n > max_ctx) return -1;
    std::vector<real> x(H), xn(H), q(H), k(H), v(H), o(H), t(H), g(F), u(F);
    std::vector<int32_t> rows;
    for (int i = 0; i < n; ++i) {
        const int pos = ctx_len + i;
        for (int j = 0; j < H; ++j)
            x[j] = embed ? widen(embed[static_cast<size_t>(tokens[i]) * H + j])
                         : hidden_in[static_cast<size_t>(i) * H + j];
        for (int l = layer_begin; l < layer_end; ++l) {
            const oracle_layer& w = layers[l];
            real* Kc = kcache + static_cast<size_t>(l) * max_ctx * H;
            real* Vc = vcache + static_cast<size_t>(l) * max_ctx * H;
            rmsnorm(x.data(), w.g_attn, H, dm->rms_eps, xn.data());
            matvec(xn.data(), w.wq, H, H, q.data());
            matvec(xn.data(), w.wk, H, H, k.data());
            matvec(xn.data(), w.wv, H, H, v.data());
            rope(q.data(), dm->n_heads, dm->head_dim, pos, dm->rope_base);
            rope(k.data(), dm->n_heads, dm->head_dim, pos, dm->rope_base);
            std::copy(k.begin(), k.end(), Kc + static_cast<size_t>(pos) * H);
            std::copy(v.begin(), v.end(), Vc + static_cast<size_t>(pos) * H);
            rows.resize(pos + 1);
            for (int r = 0; r <= pos; ++r) rows[r] = r;  // everything so far, itself included
            attend(q.data(), Kc, Vc, rows.data(), pos + 1, dm->n_heads, dm->head_dim, o.data());
            matvec(o.data(), w.wo, H, H, t.data());
            for (int j = 0; j < H; ++j) x[j] += t[j];
            rmsnorm(x.data(), w.g_ffn, H, dm->rms_eps, xn.data());
            matvec(xn.data(), w.w_gate, H, F, g.data());
            matvec(xn.data(), w.w_up, H, F, u.data());
            for (int j = 0; j < F; ++j) g[j] = silu(g[j]) * u[j];
            matvec(g.data(), w.w_down, F, H, t.data());
            for (int j = 0; j < H; ++j) x[j] += t[j];
        }
        std::copy(x.begin(), x.end(), hidden_out + static_cast<size_t>(i) * H);
    }
    return 0;
}

// ---- the batched tree pass --------------------------------------------------
//
// All T tree nodes go through layers [layer_begin, layer_end) together.  Node i
// sits at position ctx_len + depth[i]; its key and value are stored in cache
// row ctx_len + i; it attends to the ctx_len committed rows and to the rows of
// its ancestors and itself (the tree attention mask).  x is [T][hidden]: the
// inputs on entry (filled from embed[token] when embed is given) and the
// residual stream after the last applied layer on return.
int oracle_tree_forward(const oracle_dims* dm, const oracle_layer* layers, int layer_begin,
                        int layer_end, const uint16_t* embed, const int32_t* token,
                        const int32_t* parent, const int32_t* depth, int T, real* kcache,
                        real* vcache, int max_ctx, int ctx_len, real* x) {
    const int H = dm->hidden, F = dm->ffn;
    if (ctx_len + T > max_ctx) return -1;
    if (embed)
        for (int i = 0; i < T; ++i)
            for (int j = 0; j < H; ++j)
                x[static_cast<size_t>(i) * H + j] = widen(embed[static_cast<size_t>(token[i]) * H + j]);
    const size_t TH = static_cast<size_t>(T) * H, TF = static_cast<size_t>(T) * F;
    std::vector<real> xn(TH), q(TH), k(TH), v(TH), o(TH), t(TH), g(TF), u(TF);
    std::vector<int32_t> rows;
    for (int l = layer_begin; l < layer_end; ++l) {
        const oracle_layer& w = layers[l];
        real* Kc = kcache + static_cast<size_t>(l) * max_ctx * H;
        real* Vc = vcache + static_cast<size_t>(l) * max_ctx * H;
        for (int i = 0; i < T; ++i)
            rmsnorm(x + static_cast<size_t>(i) * H, w.g_attn, H, dm->rms_eps, xn.data() + static_cast<size_t>(i) * H);
        linear(xn.data(), w.wq, T, H, H, q.data());
        linear(xn.data(), w.wk, T, H, H, k.data());
        linear(xn.data(), w.wv, T, H, H, v.data());
        for (int i = 0; i < T; ++i) {
            const int pos = ctx_len + depth[i];
            rope(q.data() + static_cast<size_t>(i) * H, dm->n_heads, dm->head_dim, pos, dm->rope_base);
            rope(k.data() + static_cast<size_t>(i) * H, dm->n_heads, dm->head_dim, pos, dm->rope_base);
            std::copy(k.begin() + static_cast<size_t>(i) * H, k.begin() + static_cast<size_t>(i + 1) * H,
                      Kc + static_cast<size_t>(ctx_len + i) * H);
            std::copy(v.begin() + static_cast<size_t>(i) * H, v.begin() + static_cast<size_t>(i + 1) * H,
                      Vc + static_cast<size_t>(ctx_len + i) * H);
        }
        for (int i = 0; i < T; ++i) {
            rows.clear();
            for (int r = 0; r < ctx_len; ++r) rows.push_back(r);
            std::vector<int32_t> chain;  // i, parent(i), ... , root
            for (int a = i; a >= 0; a = parent[a]) chain.push_back(a);
            for (auto it = chain.rbegin(); it != chain.rend(); ++it) rows.push_back(ctx_len + *it);
            attend(q.data() + static_cast<size_t>(i) * H, Kc, Vc, rows.data(), static_cast<int>(rows.size()),
                   dm->n_heads, dm->head_dim, o.data() + static_cast<size_t>(i) * H);
        }
        linear(o.data(), w.wo, T, H, H, t.data());
        for (size_t j = 0; j < TH; ++j) x[j] += t[j];
        for (int i = 0; i < T; ++i)
            rmsnorm(x + static_cast<size_t>(i) * H, w.g_ffn, H, dm->rms_eps, xn.data() + static_cast<size_t>(i) * H);
        linear(xn.data(), w.w_gate, T, H, F, g.data());
        linear(xn.data(), w.w_up, T, H, F, u.data());
        for (size_t j = 0; j < TF; ++j) g[j] = silu(g[j]) * u[j];
        linear(g.data(), w.w_down, T, F, H, t.data());
        for (size_t j = 0; j < TH; ++j) x[j] += t[j];
    }
    return 0;
}

// logits[i][v] = rmsnorm(x[i], g_final) . w_lm[v]   (Algorithm 1: LM head on every node)
void oracle_lm_head(const oracle_dims* dm, const uint16_t* g_final, const uint16_t* w_lm,
                    const real* x, int T, real* logits) {
    const int H = dm->hidden;
    std::vector<real> xn(static_cast<size_t>(T) * H);
    for (int i = 0; i < T; ++i)
        rmsnorm(x + static_cast<size_t>(i) * H, g_final, H, dm->rms_eps, xn.data() + static_cast<size_t>(i) * H);
    linear(xn.data(), w_lm, T, H, dm->vocab, logits);
}

// argmax per row (lowest index on ties) and the gap between the two largest.
void oracle_argmax_margin(const real* logits, int T, int V, int32_t* amax, real* margin) {
    for (int i = 0; i < T; ++i) {
        const real* row = logits + static_cast<size_t>(i) * V;
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (row[v] > row[best]) best = v;
        real second = -INFINITY;
        for (int v = 0; v < V; ++v)
            if (v != best) second = std::max(second, row[v]);
        amax[i] = best;
        margin[i] = row[best] - second;
    }
}

// Greedy acceptance on a general tree.  A node is accepted when its parent is
// accepted and its token equals the target's argmax at the parent (the draft or
// correction candidate is judged by the distribution at the position before
// it); the root is accepted by definition.  The committed path ends at the
// deepest accepted node (lowest index among equally deep ones) and the bonus
// token is the target's argmax at that node.  Returns 0, or -1 if the path is
// deeper than the result arrays hold.
int oracle_accept(const int32_t* token, const int32_t* parent, const int32_t* depth,
                  const int32_t* amax, int T, int ctx_len, oracle_accept* out) {
    std::vector<char> ok(T, 0);
    ok[0] = 1;
    int best = 0;
    for (int j = 1; j < T; ++j) {
        ok[j] = ok[parent[j]] && token[j] == amax[parent[j]];
        if (ok[j] && depth[j] > depth[best]) best = j;
    }
    const int n = depth[best];
    if (n + 1 > 32) return -1;
    out->n_accepted = n;
    int node = best;
    for (int k = n; k >= 0; --k) {
        out->path[k] = node;
        out->tokens[k] = token[node];
        node = parent[node];
    }
    for (int k = n + 1; k < 32; ++k) out->path[k] = out->tokens[k] = -1;
    out->bonus_token = amax[best];
    out->new_ctx_len = ctx_len + n + 1;
    return 0;
}

// KV roll-back along the accepted path: the row of path[k] moves to row
// ctx_len + k, for every layer, keys and values alike.  Rows from
// ctx_len + n_path on are left as they are (don't-care).
void oracle_compact(real* kcache, real* vcache, int n_layers, int max_ctx, int H, int ctx_len,
                    const int32_t* path, int n_path) {
    for (int l = 0; l < n_layers; ++l)
        for (int which = 0; which < 2; ++which) {
            real* c = (which ? vcache : kcache) + static_cast<size_t>(l) * max_ctx * H;
            for (int k = 0; k < n_path; ++k) {  // ascending k: a source row is never overwritten early
                if (path[k] == k) continue;
                std::memmove(c + static_cast<size_t>(ctx_len + k) * H,
                             c + static_cast<size_t>(ctx_len + path[k]) * H, sizeof(real) * H);
            }
        }
}

}  // extern "C"
