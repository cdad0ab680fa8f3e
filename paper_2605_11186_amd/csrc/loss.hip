// Reduced KL loss (paper Section 3.3, Eq. 2; Appendix B steps 1-3) and its gradient with
// respect to the draft logits.
//
// Per position t: T_K = the K tokens of highest target probability (= highest target logit;
// equal values go to the lower index), p~ = target probabilities renormalised over T_K (the
// full-vocabulary normaliser cancels: p~_v = e^{a_v - a_max} / sum_{u in T_K} e^{a_u - a_max}),
// loss_t = -sum_{v in T_K} p~_v log q_v with log q_v = z_v - logsumexp(z).  The loss is the mean
// of loss_t over the unmasked positions; d loss / d z_v = (q_v - p~_v) / |M|.
//
// One workgroup of 1024 threads per position; both logit rows are read from HBM exactly once:
// the target row goes to LDS (the selection looks at it again), the draft row stays in
// registers (vocab / 1024 values per thread), so the gradient row is written without a second
// read.  Selection without sorting the row: the K-th largest of the
// maxima of 256 thread groups is a lower bound L of the K-th largest value (K groups have a
// value at or above it); the few elements >= L are gathered in LDS and ranked exactly (value
// descending, index ascending).  Rows with very many values >= L (e.g. all equal) take a slow
// exact path that ranks against the whole row.  Every sum has a fixed order: results
// do not change from run to run.  The two per-element exponentials (log-sum-exp, q in the
// gradient) use the hardware exp2 (relative error about |x| * 1e-7 for an argument x <= 0);
// the K selected terms use the accurate expf.
#include "common.hpp"

#include <cmath>

namespace {

constexpr int LOSS_NT = 1024;    // threads per workgroup
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

// LOSS_MAXI: 16-byte pieces per thread and row the registers are laid out for (>= vocab / 4096).
template <int LOSS_MAXI>
__global__ __launch_bounds__(LOSS_NT) void cats_reduced_kl_positions(LossArgs a) {
    extern __shared__ __align__(16) float s_row[];   // the target row, V floats
    __shared__ __align__(16) float s_gmax[LOSS_GROUPS];
    __shared__ float s_cval[LOSS_CAP];
    __shared__ int s_cidx[LOSS_CAP];
    __shared__ float s_sval[CATS_LOSS_MAX_K];
    __shared__ int s_sidx[CATS_LOSS_MAX_K];
    __shared__ float s_pt[CATS_LOSS_MAX_K];
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

    // ---- both rows into registers: piece j of this thread is 16-byte piece tid + j * 1024
    const f32x4* tg = reinterpret_cast<const f32x4*>(a.target + row);
    const f32x4* dr = reinterpret_cast<const f32x4*>(a.draft + row);
    // (uniform row base + 32-bit byte offset: one address register per load)
    const char* tg_bytes = reinterpret_cast<const char*>(tg);
    const char* dr_bytes = reinterpret_cast<const char*>(dr);
    f32x4 av[LOSS_MAXI], zv[LOSS_MAXI];
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const unsigned off = 16u * static_cast<unsigned>(min(tid + j * LOSS_NT, V4 - 1));
        av[j] = *reinterpret_cast<const f32x4*>(tg_bytes + off);
    }
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const unsigned off = 16u * static_cast<unsigned>(min(tid + j * LOSS_NT, V4 - 1));
        zv[j] = *reinterpret_cast<const f32x4*>(dr_bytes + off);
    }
    float a_max = -INFINITY;
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const int i = tid + j * LOSS_NT;
        if (i < V4) {
            reinterpret_cast<f32x4*>(s_row)[i] = av[j];
            a_max = fmaxf(fmaxf(fmaxf(a_max, av[j][0]), fmaxf(av[j][1], av[j][2])), av[j][3]);
        }
    }
    int n_unmasked = 0;
    if (a.mask)
        for (int i = tid; i < a.P; i += LOSS_NT) n_unmasked += a.mask[i] != 0;

    // ---- own maxima; log-sum-exp of the draft row (thread, wave, workgroup: fixed order)
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        if (tid + j * LOSS_NT < V4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) m = fmaxf(m, zv[j][e]);
        }
    }
    float gmax = fmaxf(a_max, __shfl_xor(a_max, 1));
    gmax = fmaxf(gmax, __shfl_xor(gmax, 2));
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        m = fmaxf(m, __shfl_xor(m, off));
        n_unmasked += __shfl_xor(n_unmasked, off);
    }
    if ((tid & 3) == 0) s_gmax[tid >> 2] = gmax;
    if (lane == 0) {
        s_m[wave] = m;
        s_cnt[wave] = n_unmasked;
    }
    if (tid == 0) s_ncand = 0;
    __syncthreads();
    float z_max = s_m[0];
    {
        int n = s_cnt[0];
        for (int w = 1; w < LOSS_WAVES; ++w) {
            z_max = fmaxf(z_max, s_m[w]);
            n += s_cnt[w];
        }
        n_unmasked = a.mask ? n : a.P;
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        if (tid + j * LOSS_NT < V4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) s += __expf(zv[j][e] - z_max);
        }
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) s += __shfl_xor(s, off);
    if (lane == 0) s_s[wave] = s;

    // ---- lower bound L of the K-th largest value: the K-th largest group maximum.  The four
    //      threads of a group each compare against a quarter of the groups.
    {
        const int g = tid >> 2, q = tid & 3;
        int rank = 0;
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
    float lse;
    {
        float S = 0.f;
        for (int w = 0; w < LOSS_WAVES; ++w) S += s_s[w];
        lse = z_max + logf(S);
    }

    // ---- gather the elements >= L; from here on one bit per own element stands for the target row
    uint64_t cand_bits = 0;
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const int i = tid + j * LOSS_NT;
        if (i < V4) {
            const f32x4 mine = reinterpret_cast<const f32x4*>(s_row)[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (mine[e] >= L) {
                    cand_bits |= 1ull << (4 * j + e);
                    const int slot = atomicAdd(&s_ncand, 1);
                    if (slot < LOSS_CAP) {
                        s_cval[slot] = mine[e];
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
    } else {   // slow exact path: rank every element >= L against the whole row
        for (int i = tid; i < V4; i += LOSS_NT) {
            const f32x4 mine = reinterpret_cast<const f32x4*>(s_row)[i];
            for (int e = 0; e < 4; ++e) {
                const float val = e == 0 ? mine[0] : (e == 1 ? mine[1] : (e == 2 ? mine[2] : mine[3]));
                if (val >= L) {
                    const int idx = 4 * i + e;
                    int rank = 0;
                    for (int u = 0; u < V4 && rank < K; ++u) {
                        const f32x4 o = reinterpret_cast<const f32x4*>(s_row)[u];
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

    // ---- the K terms of the loss (one wave; lane = rank)
    if (wave == 0) {
        float w = 0.f, num = 0.f;
        if (lane < K) {
            w = expf(s_sval[lane] - s_sval[0]);
            num = w * a.draft[row + s_sidx[lane]];
            if (a.topk) a.topk[static_cast<size_t>(t) * K + lane] = s_sidx[lane];
        }
        float den = w;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            num += __shfl_xor(num, off);
            den += __shfl_xor(den, off);
        }
        if (lane == 0) a.per_pos[t] = lse - num / den;
        if (lane < K) s_pt[lane] = w / den;   // p~ of the selected tokens
    }
    if (!a.grad) return;
    __syncthreads();

    // ---- gradient row: (q - p~) / |M|.  q for every element first; the few elements flagged as
    //      candidates then look themselves up among the K selected tokens (same thread, same
    //      address: program order holds).
    const float inv_n = 1.f / static_cast<float>(n_unmasked);
    char* gr_bytes = reinterpret_cast<char*>(a.grad + row);
#pragma unroll
    for (int j = 0; j < LOSS_MAXI; ++j) {
        const int i = tid + j * LOSS_NT;
        if (i < V4) {
            f32x4 g;
#pragma unroll
            for (int e = 0; e < 4; ++e) g[e] = __expf(zv[j][e] - lse) * inv_n;
            *reinterpret_cast<f32x4*>(gr_bytes + 16u * static_cast<unsigned>(i)) = g;
        }
    }
    while (cand_bits) {
        const int b = __builtin_ctzll(cand_bits);
        cand_bits &= cand_bits - 1;
        const int idx = 4 * (tid + (b >> 2) * LOSS_NT) + (b & 3);
        for (int r = 0; r < K; ++r)
            if (s_sidx[r] == idx) a.grad[row + idx] -= s_pt[r] * inv_n;
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

// The target row needs more dynamic LDS than the default limit: raised once per kernel variant.
template <int MAXI>
int launch_positions(const LossArgs& a, size_t lds, hipStream_t st) {
    static bool limit_raised = false;
    if (!limit_raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(cats_reduced_kl_positions<MAXI>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                static_cast<int>(sizeof(float) * CATS_LOSS_MAX_VOCAB)) != hipSuccess) {
            (void)hipGetLastError();
            return CATS_EHIP;
        }
        limit_raised = true;
    }
    hipLaunchKernelGGL(cats_reduced_kl_positions<MAXI>, dim3(a.P), dim3(LOSS_NT), lds, st, a);
    return CATS_OK;
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
    const size_t lds = sizeof(float) * static_cast<size_t>(vocab);
    int rc;
    if (pieces <= 2)
        rc = launch_positions<2>(a, lds, st);
    else if (pieces <= 8)
        rc = launch_positions<8>(a, lds, st);
    else
        rc = launch_positions<LOSS_MAXI_TOP>(a, lds, st);
    if (rc != CATS_OK) return rc;
    hipLaunchKernelGGL(cats_reduced_kl_mean, dim3(1), dim3(1024), 0, st, per_pos_out, mask, n_pos, loss_out);
    return hipGetLastError() == hipSuccess ? CATS_OK : CATS_EHIP;
}
