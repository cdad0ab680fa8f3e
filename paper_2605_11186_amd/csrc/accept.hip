// Greedy acceptance, bonus token and KV roll-back (paper Algorithm 1: the walk
// for the longest accepted prefix, the bonus token from the target's own
// prediction, and the roll-back of the KV cache along the accepted path).  All
// integer work; results are exact.
#include "common.hpp"

namespace {

__global__ void cats_tree_upload(TreeUploadArgs a, int n, int32_t* token, int32_t* parent, int32_t* depth) {
    const int i = threadIdx.x;
    if (i < n) {
        token[i] = a.token[i];
        parent[i] = a.parent[i];
        depth[i] = a.depth[i];
    }
}

// A node is accepted when every node on its path (root excluded) carries the
// token the target predicts at that node's parent.  The committed path ends at
// the deepest accepted node, lowest index first among equals.  One workgroup of
// CATS_MAX_TREE threads.
// edge_ok (optional): per node, 1 when the node's token passes the acceptance criterion at its
// parent; absent = greedy, the token must equal the parent's argmax.
__global__ __launch_bounds__(CATS_MAX_TREE) void cats_accept(const int32_t* token, const int32_t* parent,
                                                           const int32_t* depth, const int32_t* amax,
                                                           const uint8_t* edge_ok, int T, int ctx_len,
                                                           cats_accept_result* out) {
    __shared__ int32_t s_tok[CATS_MAX_TREE], s_par[CATS_MAX_TREE], s_dep[CATS_MAX_TREE], s_amax[CATS_MAX_TREE];
    __shared__ int s_key[CATS_MAX_TREE];
    const int i = threadIdx.x;
    if (i < T) {
        s_tok[i] = token[i];
        s_par[i] = parent[i];
        s_dep[i] = depth[i];
        s_amax[i] = amax[i];
    }
    __syncthreads();
    int key = -1;  // depth * MAX_TREE + (MAX_TREE-1 - index): larger = deeper, then lower index
    if (i < T) {
        bool ok = true;
        int node = i;
        for (int step = 0; step < CATS_MAX_DEPTH && node > 0; ++step) {
            const int p = s_par[node];
            ok = ok && (edge_ok ? edge_ok[node] != 0 : s_tok[node] == s_amax[p]);
            node = p;
        }
        if (ok) key = s_dep[i] * CATS_MAX_TREE + (CATS_MAX_TREE - 1 - i);
    }
    s_key[i] = key;
    __syncthreads();
    if (i == 0) {
        int best_key = -1;
        for (int j = 0; j < T; ++j) best_key = max(best_key, s_key[j]);
        const int best = CATS_MAX_TREE - 1 - (best_key % CATS_MAX_TREE);
        const int n = s_dep[best];
        out->n_accepted = n;
        int node = best;
        for (int k = CATS_MAX_DEPTH; k >= 0; --k) {
            if (k > n) {
                out->path[k] = -1;
                out->tokens[k] = -1;
            } else {
                out->path[k] = node;
                out->tokens[k] = s_tok[node];
                node = s_par[node];
            }
        }
        out->bonus_token = s_amax[best];
        out->new_ctx_len = ctx_len + n + 1;
    }
}

// Typical acceptance (the criterion the paper cites for Acc = typical): node j passes when the
// probability of its token under its parent's distribution p = softmax(logits / temperature)
// exceeds min(epsilon, delta * exp(-H(p))).  The parent's log-sum-exp and entropy come from the
// LM-head epilogue; the one logit needed per node is added up from the GEMM's partial tiles.
__global__ __launch_bounds__(CATS_MAX_TREE) void cats_typical_edges(TypicalArgs a) {
    const int j = threadIdx.x;
    if (j >= a.T) return;
    if (j == 0) {
        a.edge_ok[0] = 1;
        a.prob[0] = 1.f;
        a.thr[0] = 0.f;
        return;
    }
    const int p = a.parent[j];
    const float logit = row_scale(a.ns, p) * sum_pieces(a.part, a.plan, a.T, a.ld, p, a.token[j]);
    const float prob = expf(logit * a.inv_temp - a.lse[p]);
    const float thr = fminf(a.epsilon, a.delta * expf(-a.entropy[p]));
    a.prob[j] = prob;
    a.thr[j] = thr;
    a.edge_ok[j] = prob > thr ? 1 : 0;
}

// Row ctx_len + path[k] -> row ctx_len + k for k = 0..n_accepted.  grid
// (layers, heads, 2): z = 0 keys ([row][dim]), z = 1 values ([dim][row]); thread
// dd owns one head dimension, reads all its source elements first and only then
// writes, so overlapping source/destination rows cannot clobber each other.
__global__ void cats_kv_compact(CompactArgs a) {
    const int l = blockIdx.x, h = blockIdx.y, which = blockIdx.z, dd = threadIdx.x;
    const int n = a.res->n_accepted + 1;
    int path[CATS_MAX_DEPTH + 1];
    bf16_t val[CATS_MAX_DEPTH + 1];
#pragma unroll
    for (int k = 0; k <= CATS_MAX_DEPTH; ++k) path[k] = k < n ? a.res->path[k] : k;
    if (which == 0) {
        bf16_t* base = a.k[l] + (static_cast<size_t>(h) * a.max_ctx + a.ctx_len) * a.d + dd;
#pragma unroll
        for (int k = 0; k <= CATS_MAX_DEPTH; ++k)
            if (k < n) val[k] = base[static_cast<size_t>(path[k]) * a.d];
#pragma unroll
        for (int k = 0; k <= CATS_MAX_DEPTH; ++k)
            if (k < n && path[k] != k) base[static_cast<size_t>(k) * a.d] = val[k];
    } else {
        bf16_t* base = a.v[l] + (static_cast<size_t>(h) * a.d + dd) * a.max_ctx + a.ctx_len;
#pragma unroll
        for (int k = 0; k <= CATS_MAX_DEPTH; ++k)
            if (k < n) val[k] = base[path[k]];
#pragma unroll
        for (int k = 0; k <= CATS_MAX_DEPTH; ++k)
            if (k < n && path[k] != k) base[k] = val[k];
    }
}

}  // namespace

void launch_tree_upload(const TreeUploadArgs& a, int n, int32_t* token, int32_t* parent,
                        int32_t* depth, hipStream_t st) {
    hipLaunchKernelGGL(cats_tree_upload, dim3(1), dim3(CATS_MAX_TREE), 0, st, a, n, token, parent, depth);
}

void launch_accept(const int32_t* token, const int32_t* parent, const int32_t* depth,
                   const int32_t* amax, const uint8_t* edge_ok, int T, int ctx_len, cats_accept_result* out,
                   hipStream_t st) {
    hipLaunchKernelGGL(cats_accept, dim3(1), dim3(CATS_MAX_TREE), 0, st, token, parent, depth, amax, edge_ok, T,
                       ctx_len, out);
}

void launch_typical_edges(const TypicalArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(cats_typical_edges, dim3(1), dim3(CATS_MAX_TREE), 0, st, a);
}

void launch_compact(const CompactArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(cats_kv_compact, dim3(a.n_layers, a.nh, 2), dim3(a.d), 0, st, a);
}
