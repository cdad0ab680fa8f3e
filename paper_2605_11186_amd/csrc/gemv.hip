// The weight-streaming product for a single row (T = 1): the stage-1 draft loop of
// paper Algorithm 1 (one token at a time through the draft layers, the adapter and the
// shared LM head) and plain decoding.
//
// With one row, a layer is a chain of dependent launches that each stream a few tens of
// megabytes; the row kernels between the products (residual update + RMSNorm input,
// SwiGLU) move a few kilobytes and cost a launch each.  Here they are folded into the
// product that follows them: a workgroup builds the input columns of its own work items
// from the partial sums of the product before (a few KB per item, read while its first
// weight fragments are on their way), keeps them in LDS for the whole launch, and the
// workgroups that own the items of row tile 0 (together they cover every column once)
// also write the updated residual row and its sums of squares.
//
// The multiply itself needs no matrix core: one row times 32 weight rows per wave is 64
// fused multiply-adds per lane and item, against about 7000 cycles of streaming time.
// Weight fragments arrive exactly as in the GEMM (same plan, same layouts, same register
// ring of 128-bit non-temporal loads): lane l holds weight row l % 32, k = 16 j + 8 (l / 32)
// .. + 7 of fragment j; the wave's two half-sums meet through a lane exchange, the two k
// groups through LDS, and one float per weight row leaves as the partial tile.
#include <hip/hip_ext.h>

#include "common.hpp"

namespace {

constexpr int GEMV_KC = 2 * GEMM_KC;   // k values per work item (the plan's kc)
constexpr int GEMV_XI = 32;            // work items whose input columns are held in LDS at a time
static_assert(GEMV_KC == SS_COLS, "an item's columns are one sum-of-squares block");

__device__ __forceinline__ void lds_barrier() {   // orders LDS traffic only: the weight ring stays in flight
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Input columns of NE of the round's items, by one wave: local item indices it0 and, for NE = 2,
// it0 + 8 (global index first + local index).  All loads are requested, then hook() runs (the
// kernel issues its first weight loads there: they queue behind these small loads instead of in
// front of them), then the loads are used.  Nothing is requested that is not needed: a compute
// unit passes 64 bytes per cycle to and from its cache, and a launch's first microsecond goes
// into requesting the first two items' 128 KB of weights as it is.
template <int MODE, int NE, class Hook>
__device__ __forceinline__ void stage_x(const GemvArgs& a, float (*xrow)[GEMV_KC], int first, int C, int it0, Hook hook) {
    const int lane = threadIdx.x & 63;
    int it[NE], k[NE], kk[NE], chunk[NE];
    bool in_k[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        it[e] = it0 + 8 * e;
        const unsigned gi = static_cast<unsigned>(first + it[e]);
        chunk[e] = static_cast<int>(gi % static_cast<unsigned>(C));
        k[e] = chunk[e] * GEMV_KC + 4 * lane;
        in_k[e] = k[e] < a.K;
        kk[e] = min(k[e], a.K - 4);   // clamped address: K is a multiple of 4
    }
    f32x4 xv[NE];
    if (MODE == GEMV_PLAIN) {
        uint2 hi[NE], lo[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            hi[e] = *reinterpret_cast<const uint2*>(a.x_hi + kk[e]);
            lo[e] = *reinterpret_cast<const uint2*>(a.x_lo + kk[e]);
        }
        __builtin_amdgcn_sched_barrier(0);
        hook();
#pragma unroll
        for (int e = 0; e < NE; ++e) xv[e] = join_bf4(hi[e], lo[e]);
    } else if (MODE == GEMV_NORM) {
        f32x4 xin[NE], sum[NE];
        uint2 gb[NE];
        if (a.embed) {   // the row is still its embedding: bf16 -> float32 is exact
            const bf16_t* row = a.embed + static_cast<size_t>(a.token[0]) * a.K;
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const uint2 eb = *reinterpret_cast<const uint2*>(row + kk[e]);
                xin[e] = f32x4{__uint_as_float(eb.x << 16), __uint_as_float(eb.x & 0xFFFF0000u),
                               __uint_as_float(eb.y << 16), __uint_as_float(eb.y & 0xFFFF0000u)};
            }
        } else {
#pragma unroll
            for (int e = 0; e < NE; ++e) xin[e] = *reinterpret_cast<const f32x4*>(a.x_in + kk[e]);
        }
#pragma unroll
        for (int e = 0; e < NE; ++e) gb[e] = *reinterpret_cast<const uint2*>(a.gain + kk[e]);
        if (a.pend) {
            const float* pp[NE];
            int np[NE];
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                pp[e] = a.pend + kk[e];
                np[e] = plan_pieces(a.pend_plan, kk[e] / a.pend_plan.bn);
            }
            sum_pieces4_multi_hook<NE, 10>(pp, static_cast<size_t>(a.pend_ld), np, sum, hook);
        } else {
            __builtin_amdgcn_sched_barrier(0);
            hook();
#pragma unroll
            for (int e = 0; e < NE; ++e) sum[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const f32x4 val = xin[e] + sum[e];
            const float ss = wave_sum64(in_k[e] ? sum_squares4(val) : 0.f);
            if (first + it[e] < C) {   // this item lies in row tile 0: its owner writes the row
                if (in_k[e] && a.x_out) *reinterpret_cast<f32x4*>(a.x_out + k[e]) = val;
                if (lane == 0) a.ss_out[chunk[e]] = ss;
            }
            uint2 hi, lo;
            gain_split4(val, gb[e], hi, lo);
            xv[e] = join_bf4(hi, lo);
        }
    } else if (MODE == GEMV_ATTN) {
        // columns k .. k+3 belong to head k / head_dim; its chunks are merged in index order, MG
        // chunks' loads in flight at a time, rescaled to the running maximum between groups
        constexpr int MG = 8;
        const float* po[NE];
        const float* ml[NE];
        f32x4 num[NE];
        float den[NE], Mg[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const int h = kk[e] / a.head_dim;
            po[e] = a.po + static_cast<size_t>(h) * a.n_chunks * a.head_dim + (kk[e] - h * a.head_dim);
            ml[e] = a.pml + static_cast<size_t>(h) * a.n_chunks * 2;
            num[e] = f32x4{0.f, 0.f, 0.f, 0.f};
            den[e] = 0.f;
            Mg[e] = -1e30f;
        }
        for (int c0 = 0; c0 < a.n_chunks; c0 += MG) {
            f32x4 v[NE][MG];
            float mc[NE][MG], lc[NE][MG];
#pragma unroll
            for (int e = 0; e < NE; ++e)
#pragma unroll
                for (int j = 0; j < MG; ++j) {
                    const int c = min(c0 + j, a.n_chunks - 1);
                    mc[e][j] = ml[e][2 * c];
                    lc[e][j] = ml[e][2 * c + 1];
                    v[e][j] = *reinterpret_cast<const f32x4*>(po[e] + static_cast<size_t>(c) * a.head_dim);
                }
            if (c0 == 0) {
                __builtin_amdgcn_sched_barrier(0);
                hook();
            }
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                float Mn = Mg[e];
#pragma unroll
                for (int j = 0; j < MG; ++j) Mn = fmaxf(Mn, mc[e][j]);   // clamped repeats do not change the maximum
                const float resc = __builtin_amdgcn_exp2f(Mg[e] - Mn);
                den[e] *= resc;
                num[e] *= resc;
                Mg[e] = Mn;
#pragma unroll
                for (int j = 0; j < MG; ++j)
                    if (c0 + j < a.n_chunks) {
                        const float wc = __builtin_amdgcn_exp2f(mc[e][j] - Mn);
                        den[e] += wc * lc[e][j];
                        num[e] += wc * v[e][j];
                    }
            }
        }
#pragma unroll
        for (int e = 0; e < NE; ++e) xv[e] = num[e] * (1.0f / den[e]);
    } else {
        const RowSquares sq = row_squares_load(a.ns, 0);
        const float* pp[2 * NE];
        int np[2 * NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            pp[2 * e] = a.pend + kk[e];
            pp[2 * e + 1] = a.pend + a.f_pad + kk[e];
            np[2 * e] = plan_pieces(a.pend_plan, kk[e] / a.pend_plan.bn);
            np[2 * e + 1] = plan_pieces(a.pend_plan, (a.f_pad + kk[e]) / a.pend_plan.bn);
        }
        f32x4 gu[2 * NE];
        sum_pieces4_multi_hook<2 * NE, 3>(pp, static_cast<size_t>(a.pend_ld), np, gu, hook);
        const float rs = row_scale(a.ns, sq);
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            uint2 hi, lo;
            swiglu_split4(gu[2 * e], gu[2 * e + 1], rs, hi, lo);
            xv[e] = join_bf4(hi, lo);
        }
    }
#pragma unroll
    for (int e = 0; e < NE; ++e)
        *reinterpret_cast<f32x4*>(&xrow[it[e]][4 * lane]) = in_k[e] ? xv[e] : f32x4{0.f, 0.f, 0.f, 0.f};
}

// 512 threads: four waves along the 128 weight rows of a tile, times two k groups that take one
// 128-wide half of every 256-wide item each.
template <bool PACKED, int MODE>
__global__ __launch_bounds__(512) void cats_gemv_row(GemvArgs a) {
    __shared__ float xrow[GEMV_XI][GEMV_KC];
    __shared__ float red[4][32];
    __shared__ float s_am_best[4];
    __shared__ int s_am_idx[4];
    __shared__ int s_am_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = (tid >> 6) & 3, kg = tid >> 8;
    const int col = lane & 31, g = lane >> 5;
    const int wg = blockIdx.x;
    const int C = a.plan.chunks;
    const int C128 = (a.K + GEMM_KC - 1) / GEMM_KC;
    (void)C128;
    const int item_lo = plan_item_begin(a.plan, wg);
    const int n_items = plan_item_begin(a.plan, wg + 1) - item_lo;
    const int k_last_w = a.K - 16;
    const int rb_per_seg = a.seg_pad / PACK_ROWS, n_rb_total = a.n_seg * rb_per_seg;   // packed only
    (void)rb_per_seg;
    (void)n_rb_total;
    (void)k_last_w;

    u32x4 wst[2][8];
    float acc0 = 0.f, acc1 = 0.f;
    float am_best = -INFINITY;   // greedy token among this lane's columns (a.amax given)
    int am_idx = 0x7fffffff;

    for (int base = 0; base < n_items; base += GEMV_XI) {   // one round unless the range is longer than GEMV_XI items
        const int n_round = min(GEMV_XI, n_items - base);
        const int first = item_lo + base;
        if (base) lds_barrier();   // every wave is done with the columns of the round before

#define CATS_ITEM(i, tile_, k0_)                                                                        \
    const int gi_ = first + (i);                                                                        \
    const int tile_ = static_cast<int>(static_cast<unsigned>(gi_) / static_cast<unsigned>(C));          \
    const int k0_ = (gi_ - tile_ * C) * GEMV_KC;

        // Unconditional loads at clamped addresses, as in the GEMM: columns past K meet zeros in xrow.
#define CATS_LOAD_W(slot, i)                                                                            \
    {                                                                                                   \
        CATS_ITEM(i, lt_, lk_)                                                                          \
        const bf16_t* lw_;                                                                              \
        if (PACKED) {                                                                                   \
            const int lrb_ = min((lt_ * 128 + wave * 32) / PACK_ROWS, n_rb_total - 1);                  \
            const int lseg_ = lrb_ / rb_per_seg;                                                        \
            lw_ = (lseg_ == 0 ? a.w[0] : (lseg_ == 1 ? a.w[1] : a.w[2])) +                              \
                  (static_cast<size_t>(lrb_ - lseg_ * rb_per_seg) * C128 + min(lk_ / GEMM_KC + kg, C128 - 1)) * \
                      (8 * PACK_FRAG) + lane * 8;                                                       \
        } else {                                                                                        \
            const int lv_ = min(lt_ * 128 + wave * 32 + col, a.N - 1);                                  \
            const int lseg_ = lv_ / a.seg_pad;                                                          \
            lw_ = (lseg_ == 0 ? a.w[0] : (lseg_ == 1 ? a.w[1] : a.w[2])) +                              \
                  static_cast<size_t>(min(lv_ - lseg_ * a.seg_pad, a.seg_rows - 1)) * a.K + 8 * g;      \
        }                                                                                               \
        _Pragma("unroll") for (int j = 0; j < 8; ++j)                                                   \
            wst[slot][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(                   \
                PACKED ? lw_ + j * PACK_FRAG : lw_ + min(lk_ + GEMM_KC * kg + 16 * j, k_last_w)));      \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }

        // One item: refill the other ring slot with the next item, multiply this one, and hand the
        // partial tile over when the tile (or this workgroup's range) ends.
#define CATS_STEP(s, i, REFILL)                                                                         \
    {                                                                                                   \
        CATS_ITEM(i, tile, k0)                                                                          \
        if (REFILL) CATS_LOAD_W(1 - (s), min((i) + 1, n_round - 1))                                     \
        const float* xp = &xrow[i][GEMM_KC * kg + 8 * g];                                               \
        _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                                 \
            const f32x4 xa = *reinterpret_cast<const f32x4*>(xp + 16 * j);                              \
            const f32x4 xb = *reinterpret_cast<const f32x4*>(xp + 16 * j + 4);                          \
            const u32x4 w = wst[s][j];                                                                  \
            float t_ = (j & 1) ? acc1 : acc0;                                                           \
            t_ = fmaf(__uint_as_float(w[0] << 16), xa[0], t_);                                          \
            t_ = fmaf(__uint_as_float(w[0] & 0xFFFF0000u), xa[1], t_);                                  \
            t_ = fmaf(__uint_as_float(w[1] << 16), xa[2], t_);                                          \
            t_ = fmaf(__uint_as_float(w[1] & 0xFFFF0000u), xa[3], t_);                                  \
            t_ = fmaf(__uint_as_float(w[2] << 16), xb[0], t_);                                          \
            t_ = fmaf(__uint_as_float(w[2] & 0xFFFF0000u), xb[1], t_);                                  \
            t_ = fmaf(__uint_as_float(w[3] << 16), xb[2], t_);                                          \
            t_ = fmaf(__uint_as_float(w[3] & 0xFFFF0000u), xb[3], t_);                                  \
            if (j & 1) acc1 = t_; else acc0 = t_;                                                       \
        }                                                                                               \
        if (k0 + GEMV_KC >= a.K || base + (i) == n_items - 1) {                                         \
            float v = acc0 + acc1;                                                                      \
            v += __shfl_xor(v, 32);      /* the lane pair that shares a weight row */                   \
            if (kg == 1 && g == 0) red[wave][col] = v;                                                  \
            lds_barrier();                                                                              \
            if (kg == 0 && g == 0) {                                                                    \
                v += red[wave][col];                                                                    \
                const int n = tile * 128 + wave * 32 + col;                                             \
                if (n < a.N && n % a.seg_pad < a.seg_rows) {                                            \
                    if (a.amax) {   /* columns ascend within a lane: strict > keeps the lowest */      \
                        if (v > am_best) {                                                              \
                            am_best = v;                                                                \
                            am_idx = n;                                                                 \
                        }                                                                               \
                    } else {                                                                            \
                        const int piece = wg - plan_first_wg(a.plan, tile);                             \
                        /* write-through, like the GEMM's partial tiles */                              \
                        __hip_atomic_store(a.part + static_cast<size_t>(piece) * a.N + n, v, __ATOMIC_RELAXED, \
                                           __HIP_MEMORY_SCOPE_AGENT);                                   \
                    }                                                                                   \
                }                                                                                       \
            }                                                                                           \
            lds_barrier();   /* red is free again before any wave reaches the next tile end */         \
            acc0 = 0.f;                                                                                 \
            acc1 = 0.f;                                                                                 \
        }                                                                                               \
    }

        // The round's input columns and its first two items' weights: the small loads go out first,
        // both ring slots behind them, so that the columns are ready by the time item 0 has arrived
        // and item 1 is already on its way.
        // (The barrier inside: no wave requests weights before every wave has requested its columns.)
        const int wv = tid >> 6;
        auto issue_w = [&]() {
            __builtin_amdgcn_s_barrier();
            CATS_LOAD_W(0, 0)
            CATS_LOAD_W(1, min(1, n_round - 1))
        };
        if (wv + 8 < n_round) {
            stage_x<MODE, 2>(a, xrow, first, C, wv, issue_w);
        } else if (wv < n_round) {
            stage_x<MODE, 1>(a, xrow, first, C, wv, issue_w);
        } else {
            issue_w();
        }
        for (int p0 = 16; p0 < n_round; p0 += 16) {
            if (p0 + wv + 8 < n_round) {
                stage_x<MODE, 2>(a, xrow, first, C, p0 + wv, []() {});
            } else if (p0 + wv < n_round) {
                stage_x<MODE, 1>(a, xrow, first, C, p0 + wv, []() {});
            }
        }
        lds_barrier();

        // Item 0 finds item 1 already requested; from item 1 on, every step requests the item after
        // it.  Pairs of items whose refills lie inside the round run without any condition (see the GEMM).
        CATS_STEP(0, 0, false)
        int c0 = 1;
        for (; c0 + 3 <= n_round; c0 += 2) {
            CATS_STEP(1, c0, true)
            CATS_STEP(0, c0 + 1, true)
        }
#define CATS_TAIL(j)                                  \
    if (c0 + (j) + 1 < n_round) {                     \
        CATS_STEP(((j) + 1) % 2, c0 + (j), true)      \
    } else {                                          \
        CATS_STEP(((j) + 1) % 2, c0 + (j), false)     \
    }
        if (c0 < n_round) {
            CATS_TAIL(0)
            if (c0 + 1 < n_round) {
                CATS_TAIL(1)
            }
        }
#undef CATS_TAIL
#undef CATS_STEP
#undef CATS_LOAD_W
#undef CATS_ITEM
    }
    if (!a.amax) return;

    // Greedy token: best of this workgroup's columns, then the best of all workgroups by the last
    // one to arrive (results move with device-scope atomics, acknowledged before the count is raised).
    auto better = [](float ob, int oi, float b, int bi) { return ob > b || (ob == b && oi < bi); };
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(am_best, o);
        const int oi = __shfl_xor(am_idx, o);
        if (better(ob, oi, am_best, am_idx)) {
            am_best = ob;
            am_idx = oi;
        }
    }
    if (kg == 0 && lane == 0) {
        s_am_best[wave] = am_best;
        s_am_idx[wave] = am_idx;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            if (better(s_am_best[w], s_am_idx[w], am_best, am_idx)) {
                am_best = s_am_best[w];
                am_idx = s_am_idx[w];
            }
        __hip_atomic_store(a.am_best + wg, am_best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.am_idx + wg, am_idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        s_am_last = __hip_atomic_fetch_add(a.am_arrivals, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                    static_cast<int>(gridDim.x) - 1;
    }
    __syncthreads();
    if (!s_am_last || tid >= 64) return;
    am_best = -INFINITY;
    am_idx = 0x7fffffff;
    for (int w = lane; w < static_cast<int>(gridDim.x); w += 64) {
        const float ob = __hip_atomic_load(a.am_best + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int oi = __hip_atomic_load(a.am_idx + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (better(ob, oi, am_best, am_idx)) {
            am_best = ob;
            am_idx = oi;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(am_best, o);
        const int oi = __shfl_xor(am_idx, o);
        if (better(ob, oi, am_best, am_idx)) {
            am_best = ob;
            am_idx = oi;
        }
    }
    if (lane == 0) {
        a.amax[0] = am_idx;
        __hip_atomic_store(a.am_arrivals, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
    }
}

}  // namespace

void launch_gemv(const GemvArgs& a, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
    const dim3 grid(a.plan.n_wgs), block(512);
#define CATS_LAUNCH_M(MODEV)                                                                              \
    if (a.packed)                                                                                         \
        hipExtLaunchKernelGGL((cats_gemv_row<true, MODEV>), grid, block, 0, st, ev_start, ev_stop, 0, a); \
    else                                                                                                  \
        hipExtLaunchKernelGGL((cats_gemv_row<false, MODEV>), grid, block, 0, st, ev_start, ev_stop, 0, a)
    if (a.mode == GEMV_NORM) {
        CATS_LAUNCH_M(GEMV_NORM);
    } else if (a.mode == GEMV_SWIGLU) {
        CATS_LAUNCH_M(GEMV_SWIGLU);
    } else if (a.mode == GEMV_ATTN) {
        CATS_LAUNCH_M(GEMV_ATTN);
    } else {
        CATS_LAUNCH_M(GEMV_PLAIN);
    }
#undef CATS_LAUNCH_M
}
