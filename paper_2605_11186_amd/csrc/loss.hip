// Reduced KL loss (paper Section 3.3, Eq. 2; Appendix B steps 1-3) and its gradient with
// respect to the draft logits.
//
// Per position t: T_K = the K tokens of highest target probability (= highest target logit;
// equal values go to the lower index), p~ = target probabilities renormalised over T_K (the
// full-vocabulary normaliser cancels: p~_v = e^{a_v - a_max} / sum_{u in T_K} e^{a_u - a_max}),
// loss_t = -sum_{v in T_K} p~_v log q_v with log q_v = z_v - logsumexp(z).  The loss is the mean
// of loss_t over the unmasked positions; d loss / d z_v = (q_v - p~_v) / |M|.
//
// One workgroup of 512 threads per position, two workgroups per compute unit; each logit row is
// read from HBM exactly once and only one row is held (in registers, vocab / 512 values per
// thread) at a time: first the draft row (log-sum-exp, then the dense part q / |M| of the
// gradient row goes out), then the target row (selection, loss, and the K entries of the
// gradient that also carry -p~ / |M|).  Selection without sorting the row: the K-th largest of
// the maxima of 128 thread groups is a lower bound L of the K-th largest value (K groups have a
// value at or above it); the few elements >= L are gathered in LDS and ranked exactly (value
// descending, index ascending).  Rows with very many values >= L (e.g. all equal) take a slow
// exact path that ranks against the whole row in memory.  Every sum has a fixed order: results
// do not change from run to run.  The two per-element exponentials (log-sum-exp, q in the
// gradient) use the hardware exp2 (relative error about |x| * 1e-7 for an argument x <= 0);
// the K selected terms use the accurate expf.
#include "common.hpp"

#include <cmath>

namespace {

constexpr int LOSS_NT = 512;     // threads per workgroup
constexpr int LOSS_CAP = 1024;   // candidates ranked on the fast path
constexpr int LOSS_WAVES = LOSS_NT / 64;
constexpr int LOSS_GROUPS = LOSS_NT / 4;   // thread groups whose maxima bound the selection
constexpr int LOSS_MAXI_TOP = CATS_LOSS_MAX_VOCAB / 4 / LOSS_NT;   // most 16-byte pieces per thread and row
static_assert(LOSS_MAXI_TOP * 4 * LOSS_NT == CATS_LOSS_MAX_VOCAB, "vocab limit must fill the threads evenly");
static_assert(CATS_LOSS_MAX_K <= 64 && CATS_LOSS_MAX_K <= LOSS_GROUPS, "one wave handles the K terms");

struct LossArgs {
    const float* target;   // [P][V]
    const float* draft;    // [P][V]
    const uint8_t* mask;   // [P] or null
    int P, V, K;
    float* per_pos;        // [P]
    int32_t* topk;         // [P][K] or null
    float* grad;           // [P][V] or null
};

// true when (value b, index ib) comes before (value a, index ia) in the selection order
__device__ __forceinline__ bool before(float b, int ib, float a, int ia) {
    return b > a || (b == a && ib < ia);
}

// LOSS_MAXI: 16-byte pieces per thread the registers are laid out for (>= vocab / 2048); piece j
// of a thread is 16-byte piece tid + j * 512 of the row.  (The second launch bound is waves per
// SIMD: four, so that two workgroups share a compute unit and one's arithmetic hides behind the
// other's memory traffic.)
template <int LOSS_MAXI>
__global__ __launch_bounds__(LOSS_NT, 4) void cats_reduced_kl_positions(LossArgs a) {
    __shared__ __align__(16) float s_gmax[LOSS_GROUPS];
    __shared__ float s_cval[LOSS_CAP];
    __shared__ int s_cidx[LOSS_CAP];
    __shared__ float s_sval[CATS_LOSS_MAX_K];
    __shared__ int s_sidx[CATS_LOSS_MAX_K];
    __shared__ float s_m[LOSS_WAVES], s_s[LOSS_WAVES], s_L;
    __shared__ int s_cnt[LOSS_WAVES], s_ncand;

    const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.V, K = a.K, V4 = V / 4;
    const size_t row = static_cast<size_t>(t) * V;
    const bool masked = a.mask && a.mask[t] == 0;
    if (masked) {   // uniform over the workgroup
        if (tid == 0) a.per_pos[t] = 0.f;
        if (a.topk && tid < K) a.topk[static_cast<size_t>(t) * K + tid] = -1;
        if (a.grad)
            for (int i = tid; i < V4; i += LOSS_NT)
                reinterpret_cast<f32x4*>(a.grad + row)[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        return;
    }
    // (uniform row base + 32-bit byte offset: one address register per load)
    const char* tg_bytes = reinterpret_cast<const char*>(a.target + row);
    const char* dr_bytes = reinterpret_cast<const char*>(a.draft + row);
    f32x4 rv[LOSS_MAXI];   // the row in hand: first the draft row, then the target row

    // ================= draft row: log-sum-exp, dense part of the gradient =================
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const unsigned off = 16u * static_cast<unsigned>(min(tid + j * LOSS_NT, V4 - 1));
        rv[j] = *reinterpret_cast<const f32x4*>(dr_bytes + off);
    }
    int n_unmasked = 0;
    if (a.mask && a.grad)
        for (int i = tid; i < a.P; i += LOSS_NT) n_unmasked += a.mask[i] != 0;
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        if (tid + j * LOSS_NT < V4) m = fmaxf(fmaxf(fmaxf(m, rv[j][0]), fmaxf(rv[j][1], rv[j][2])), rv[j][3]);
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        m = fmaxf(m, __shfl_xor(m, off));
        n_unmasked += __shfl_xor(n_unmasked, off);
    }
    if (lane == 0) {
        s_m[wave] = m;
        s_cnt[wave] = n_unmasked;
    }
    if (tid == 0) s_ncand = 0;
    __syncthreads();
    float z_max = s_m[0];
    n_unmasked = s_cnt[0];
    for (int w = 1; w < LOSS_WAVES; ++w) {
        z_max = fmaxf(z_max, s_m[w]);
        n_unmasked += s_cnt[w];
    }
    if (!a.mask) n_unmasked = a.P;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        if (tid + j * LOSS_NT < V4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) s += __expf(rv[j][e] - z_max);
        }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) s += __shfl_xor(s, off);
    if (lane == 0) s_s[wave] = s;
    __syncthreads();
    float lse;
    {
        float S = 0.f;
        for (int w = 0; w < LOSS_WAVES; ++w) S += s_s[w];
        lse = z_max + logf(S);
    }
    const float inv_n = 1.f / static_cast<float>(n_unmasked);
    if (a.grad) {   // q / |M| everywhere; the K selected entries get their -p~ / |M| at the end
        char* gr_bytes = reinterpret_cast<char*>(a.grad + row);
#pragma unroll
        for (int j = 0; j < LOSS_MAXI; ++j) {
            const int i = tid + j * LOSS_NT;
            if (i < V4) {
                f32x4 g;
#pragma unroll
                for (int e = 0; e < 4; ++e) g[e] = __expf(rv[j][e] - lse) * inv_n;
                *reinterpret_cast<f32x4*>(gr_bytes + 16u * static_cast<unsigned>(i)) = g;
            }
        }
    }

    // ================= target row: selection, loss =================
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const unsigned off = 16u * static_cast<unsigned>(min(tid + j * LOSS_NT, V4 - 1));
        rv[j] = *reinterpret_cast<const f32x4*>(tg_bytes + off);
    }
    float a_max = -INFINITY;
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        if (tid + j * LOSS_NT < V4)
            a_max = fmaxf(fmaxf(fmaxf(a_max, rv[j][0]), fmaxf(rv[j][1], rv[j][2])), rv[j][3]);
    }
    float gmax = fmaxf(a_max, __shfl_xor(a_max, 1));
    gmax = fmaxf(gmax, __shfl_xor(gmax, 2));
    if ((tid & 3) == 0) s_gmax[tid >> 2] = gmax;
    __syncthreads();

    // ---- lower bound L of the K-th largest value: the K-th largest group maximum.  The four
    //      threads of a group each compare against a quarter of the groups.
    {
        const int g = tid >> 2, q = tid & 3;
        int rank = 0;
#pragma unroll 2
        for (int j = q * (LOSS_GROUPS / 4); j < (q + 1) * (LOSS_GROUPS / 4); j += 4) {
            const f32x4 o = *reinterpret_cast<const f32x4*>(s_gmax + j);
#pragma unroll
            for (int e = 0; e < 4; ++e) rank += before(o[e], j + e, gmax, g);
        }
        rank += __shfl_xor(rank, 1);
        rank += __shfl_xor(rank, 2);
        if (rank == K - 1 && q == 0) s_L = gmax;
    }
    __syncthreads();
    const float L = s_L;

    // ---- gather the elements >= L
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const int i = tid + j * LOSS_NT;
        if (i < V4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (rv[j][e] >= L) {
                    const int slot = atomicAdd(&s_ncand, 1);
                    if (slot < LOSS_CAP) {
                        s_cval[slot] = rv[j][e];
                        s_cidx[slot] = 4 * i + e;
                    }
                }
            }
        }
    }
    __syncthreads();
    const int n_cand = s_ncand;

    // ---- exact ranks (value descending, index ascending); ranks below K are the selection
    if (n_cand <= LOSS_CAP) {
        for (int c = tid; c < n_cand; c += LOSS_NT) {
            const float val = s_cval[c];
            const int idx = s_cidx[c];
            int rank = 0;
            for (int u = 0; u < n_cand; ++u) rank += before(s_cval[u], s_cidx[u], val, idx);
            if (rank < K) {
                s_sval[rank] = val;
                s_sidx[rank] = idx;
            }
        }
    } else {   // slow exact path: rank every element >= L against the whole row in memory
        const f32x4* tg = reinterpret_cast<const f32x4*>(tg_bytes);
        for (int i = tid; i < V4; i += LOSS_NT) {
            const f32x4 mine = tg[i];
            for (int e = 0; e < 4; ++e) {
                const float val = e == 0 ? mine[0] : (e == 1 ? mine[1] : (e == 2 ? mine[2] : mine[3]));
                if (val >= L) {
                    const int idx = 4 * i + e;
                    int rank = 0;
                    for (int u = 0; u < V4 && rank < K; ++u) {
                        const f32x4 o = tg[u];
#pragma unroll
                        for (int f = 0; f < 4; ++f) rank += before(o[f], 4 * u + f, val, idx);
                    }
                    if (rank < K) {
                        s_sval[rank] = val;
                        s_sidx[rank] = idx;
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- the K terms of the loss and of the gradient (one wave; lane = rank).  The dense
    //      gradient stores of every wave were complete before the barriers above.
    if (wave == 0) {
        float w = 0.f, num = 0.f;
        int idx = 0;
        if (lane < K) {
            idx = s_sidx[lane];
            w = expf(s_sval[lane] - s_sval[0]);
            num = w * a.draft[row + idx];
            if (a.topk) a.topk[static_cast<size_t>(t) * K + lane] = idx;
        }
        float den = w;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            num += __shfl_xor(num, off);
            den += __shfl_xor(den, off);
        }
        if (lane == 0) a.per_pos[t] = lse - num / den;
        if (a.grad && lane < K) a.grad[row + idx] -= (w / den) * inv_n;
    }
}

// loss = sum of the per-position terms / number of unmasked positions (0 when there is none);
// one workgroup, fixed summation order.
__global__ __launch_bounds__(1024) void cats_reduced_kl_mean(const float* per_pos, const uint8_t* mask, int P,
                                                             float* loss) {
    __shared__ float s_sum[16];
    __shared__ int s_cnt[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float sum = 0.f;
    int cnt = 0;
    for (int i = tid; i < P; i += 1024) {
        const bool on = !mask || mask[i] != 0;
        sum += on ? per_pos[i] : 0.f;
        cnt += on;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        sum += __shfl_xor(sum, off);
        cnt += __shfl_xor(cnt, off);
    }
    if (lane == 0) {
        s_sum[wave] = sum;
        s_cnt[wave] = cnt;
    }
    __syncthreads();
    if (tid == 0) {
        float total = 0.f;
        int n = 0;
        for (int w = 0; w < 16; ++w) {
            total += s_sum[w];
            n += s_cnt[w];
        }
        loss[0] = n ? total / static_cast<float>(n) : 0.f;
    }
}

}  // namespace

extern "C" int cats_reduced_kl_loss(const float* target_logits, const float* draft_logits, const uint8_t* mask,
                                    int32_t n_pos, int32_t vocab, int32_t top_k, float* loss_out,
                                    float* per_pos_out, int32_t* topk_idx_out, float* grad_out, void* stream) {
    if (!target_logits || !draft_logits || !loss_out || !per_pos_out) return CATS_EINVAL;
    if (n_pos < 1 || vocab < 4 || vocab % 4 != 0 || top_k < 1 || top_k > CATS_LOSS_MAX_K || top_k > vocab)
        return CATS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(target_logits) | reinterpret_cast<uintptr_t>(draft_logits) |
         reinterpret_cast<uintptr_t>(grad_out)) & 15)
        return CATS_EINVAL;
    if (vocab > CATS_LOSS_MAX_VOCAB) return CATS_ECAPACITY;
    hipStream_t st = static_cast<hipStream_t>(stream);
    LossArgs a{target_logits, draft_logits, mask, n_pos, vocab, top_k, per_pos_out, topk_idx_out, grad_out};
    const int pieces = (vocab / 4 + LOSS_NT - 1) / LOSS_NT;
    if (pieces <= 4)
        hipLaunchKernelGGL(cats_reduced_kl_positions<4>, dim3(n_pos), dim3(LOSS_NT), 0, st, a);
    else if (pieces <= 16)
        hipLaunchKernelGGL(cats_reduced_kl_positions<16>, dim3(n_pos), dim3(LOSS_NT), 0, st, a);
    else
        hipLaunchKernelGGL(cats_reduced_kl_positions<LOSS_MAXI_TOP>, dim3(n_pos), dim3(LOSS_NT), 0, st, a);
    hipLaunchKernelGGL(cats_reduced_kl_mean, dim3(1), dim3(1024), 0, st, per_pos_out, mask, n_pos, loss_out);
    return hipGetLastError() == hipSuccess ? CATS_OK : CATS_EHIP;
}
