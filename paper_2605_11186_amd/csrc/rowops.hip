// Small per-row kernels around the weight-streaming GEMMs of one decoder layer
// (the layer internals are those of the LLaMA-family targets the paper
// evaluates: RMSNorm, rotary embedding, SwiGLU).  Each one also adds up the
// GEMM's split-K partial sums in a fixed order, so results do not depend on
// scheduling.
#include "common.hpp"

namespace {

// x[t] <- (x_in[t] | embed[token[t]] | x[t]) + sum of the GEMM pieces;  xn[t] = x[t] * gain as
// high + low bf16 parts;  ss[t][block] = sum of x^2 over the block's columns.  One wave per
// (row, block of 256 columns): nothing here needs a whole row, so the launch has T * H/256
// independent waves.
__global__ __launch_bounds__(64) void cats_residual_rmsnorm(ResidualNormArgs a) {
    const int t = blockIdx.x, blk = blockIdx.y;
    const int j = blk * SS_COLS + 4 * threadIdx.x;
    float ss = 0.f;
    if (j < a.H) {
        const size_t row = static_cast<size_t>(t) * a.H;
        f32x4 val;
        if (a.embed) {
            const uint2 e = *reinterpret_cast<const uint2*>(a.embed + static_cast<size_t>(a.token[t]) * a.H + j);
            val = f32x4{__uint_as_float(e.x << 16), __uint_as_float(e.x & 0xFFFF0000u),
                        __uint_as_float(e.y << 16), __uint_as_float(e.y & 0xFFFF0000u)};
        } else {
            val = *reinterpret_cast<const f32x4*>((a.x_in ? a.x_in : a.x) + row + j);
        }
        if (a.part) {
            val += sum_pieces4<16>(a.part + row + j, static_cast<size_t>(a.T) * a.H, plan_pieces(a.plan, j / a.plan.bn));
        }
        ss = sum_squares4(val);
        if (a.embed || a.x_in || a.part) *reinterpret_cast<f32x4*>(a.x + row + j) = val;
        if (a.gain) {
            uint2 hi, lo;
            gain_split4(val, *reinterpret_cast<const uint2*>(a.gain + j), hi, lo);
            *reinterpret_cast<uint2*>(a.xn + row + j) = hi;
            *reinterpret_cast<uint2*>(a.xn_lo + row + j) = lo;
        }
    }
    if (!a.gain) return;
    ss = wave_sum64(ss);
    if (threadIdx.x == 0) a.ss[t * SS_STRIDE + blk] = ss;
}

// cos/sin of pos * base^(-2j/d) for pos = ctx_len + depth[t]; computed in double so
// that the angle carries no float rounding of a four-digit position.
__global__ void cats_rope_table(RopeTableArgs a) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int half = a.d / 2;
    if (idx >= a.T * half) return;
    const int t = idx / half, j = idx - t * half;
    const double inv_freq = pow(static_cast<double>(a.base), -2.0 * j / a.d);
    const double ang = static_cast<double>(a.ctx_len + a.depth[t]) * inv_freq;
    a.cs[idx] = make_float2(static_cast<float>(cos(ang)), static_cast<float>(sin(ang)));
}

// Adds up q|k|v partials, scales by the row's norm factor, rotates q and k (pairs j, j+d/2),
// writes q (high and low bf16 parts) and appends the key row and the (transposed) value column
// of row t at cache row row0 + t (bf16), with their rounding remainders in the low-part window
// (see AttnArgs).  All piece loads are 16-byte loads issued in batches.
// Blocks [0, T * gy): q and k, one thread per (node, head, 4 consecutive pairs).
// Blocks after those: values, one block per (head, 32 dims): the sums go through LDS so that
// the stores into the transposed cache run along the node index (contiguous in memory).
constexpr int V_DIMS = 32;   // head dims per value block
__global__ __launch_bounds__(256) void cats_qkv_rope_append(QkvRopeArgs a) {
    __shared__ bf16_t s_v[2][V_DIMS][CATS_MAX_TREE + 2];   // [0] high parts, [1] low parts
    const int half = a.d / 2;
    const int N = 3 * a.H;
    const size_t stride = static_cast<size_t>(a.T) * N;
    const int threads_per_head = half / 4;
    const int heads_per_block = 256 / threads_per_head;
    const int gy = (a.nh + heads_per_block - 1) / heads_per_block;
    const int n_qk = a.T * gy;
    if (static_cast<int>(blockIdx.x) >= n_qk) {
        const int vb = blockIdx.x - n_qk, slices = a.d / V_DIMS;
        const int h = vb / slices, ds = (vb - h * slices) * V_DIMS;
        const int col = 2 * a.H + h * a.d + ds + 4 * (threadIdx.x & 7);
        const int pieces = plan_pieces(a.plan, col / a.plan.bn);
        for (int t0 = 0; t0 < a.T; t0 += 64) {   // two nodes per thread and pass
            const int ta = t0 + (threadIdx.x >> 3), tb = ta + 32;
            const int ca = min(ta, a.T - 1), cb = min(tb, a.T - 1);
            const RowSquares sqa = row_squares_load(a.ns, ca), sqb = row_squares_load(a.ns, cb);
            const float* const pv[2] = {a.part + static_cast<size_t>(ca) * N + col,
                                        a.part + static_cast<size_t>(cb) * N + col};
            const int npv[2] = {pieces, pieces};
            f32x4 sv[2];
            sum_pieces4_multi<2, 8>(pv, stride, npv, sv);
            f32x4 va = sv[0] * row_scale(a.ns, sqa);
            f32x4 vb4 = sv[1] * row_scale(a.ns, sqb);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bf16_t ha = f2bf(va[e]), hb = f2bf(vb4[e]);
                if (ta < a.T) {
                    s_v[0][4 * (threadIdx.x & 7) + e][ta] = ha;
                    s_v[1][4 * (threadIdx.x & 7) + e][ta] = f2bf(va[e] - bf2f(ha));
                }
                if (tb < a.T) {
                    s_v[0][4 * (threadIdx.x & 7) + e][tb] = hb;
                    s_v[1][4 * (threadIdx.x & 7) + e][tb] = f2bf(vb4[e] - bf2f(hb));
                }
            }
        }
        __syncthreads();
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        bf16_t* vt = a.vt + (static_cast<size_t>(h) * a.d + ds) * a.max_ctx + a.row0;
        bf16_t* vl = a.vt_lo + (static_cast<size_t>(h) * a.d + ds) * TREE_WIN + a.win0;
        for (int dd = wave; dd < V_DIMS; dd += 4)
            for (int t = lane; t < a.T; t += 64) {
                vt[static_cast<size_t>(dd) * a.max_ctx + t] = s_v[0][dd][t];
                vl[dd * TREE_WIN + t] = s_v[1][dd][t];
            }
        return;
    }
    const int t = blockIdx.x / gy, h = (blockIdx.x - t * gy) * heads_per_block + threadIdx.x / threads_per_head;
    const int j = 4 * (threadIdx.x % threads_per_head);
    if (h >= a.nh) return;
    f32x4 v4[4];
    const int c0 = h * a.d + j;
    // the column groups of one head lie in different row tiles; within a head all columns
    // share a tile (head_dim divides the tile height)
    const RowSquares sq = row_squares_load(a.ns, t);
    {
        const float* pq = a.part + static_cast<size_t>(t) * N + c0;
        const float* const pp[4] = {pq, pq + half, pq + a.H, pq + a.H + half};
        const int nq = plan_pieces(a.plan, c0 / a.plan.bn), nk = plan_pieces(a.plan, (a.H + c0) / a.plan.bn);
        const int np[4] = {nq, nq, nk, nk};
        sum_pieces4_multi<4, 8>(pp, stride, np, v4);
    }
    const float rs = row_scale(a.ns, sq);
#pragma unroll
    for (int m = 0; m < 4; ++m) v4[m] *= rs;
    const size_t qo = static_cast<size_t>(t) * a.H + c0;
    bf16_t* k = a.kc + (static_cast<size_t>(h) * a.max_ctx + a.row0 + t) * a.d + j;
    bf16_t* kl = a.k_lo + (static_cast<size_t>(h) * TREE_WIN + a.win0 + t) * a.d + j;
    float q0[4], q1[4], k0[4], k1[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float2 cs = a.cs[t * half + j + e];
        q0[e] = v4[0][e] * cs.x - v4[1][e] * cs.y;
        q1[e] = v4[0][e] * cs.y + v4[1][e] * cs.x;
        k0[e] = v4[2][e] * cs.x - v4[3][e] * cs.y;
        k1[e] = v4[2][e] * cs.y + v4[3][e] * cs.x;
    }
    uint2 qh0, ql0, qh1, ql1, kh0, kl0, kh1, kl1;
    split_bf2(q0[0], q0[1], qh0.x, ql0.x);
    split_bf2(q0[2], q0[3], qh0.y, ql0.y);
    split_bf2(q1[0], q1[1], qh1.x, ql1.x);
    split_bf2(q1[2], q1[3], qh1.y, ql1.y);
    split_bf2(k0[0], k0[1], kh0.x, kl0.x);
    split_bf2(k0[2], k0[3], kh0.y, kl0.y);
    split_bf2(k1[0], k1[1], kh1.x, kl1.x);
    split_bf2(k1[2], k1[3], kh1.y, kl1.y);
    *reinterpret_cast<uint2*>(a.q + qo) = qh0;
    *reinterpret_cast<uint2*>(a.q_lo + qo) = ql0;
    *reinterpret_cast<uint2*>(a.q + qo + half) = qh1;
    *reinterpret_cast<uint2*>(a.q_lo + qo + half) = ql1;
    *reinterpret_cast<uint2*>(k) = kh0;
    *reinterpret_cast<uint2*>(k + half) = kh1;
    *reinterpret_cast<uint2*>(kl) = kl0;
    *reinterpret_cast<uint2*>(kl + half) = kl1;
}

// h[t][n] = silu(gate[t][n]) * up[t][n] after scaling both by the row's norm factor; four
// columns per thread (16-byte piece loads in batches), high and low bf16 parts out.
__global__ void cats_swiglu(SwigluArgs a) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int quarter_f = a.F / 4;
    if (idx >= a.T * quarter_f) return;
    const int t = idx / quarter_f, n = 4 * (idx - t * quarter_f);
    const int N = 2 * a.f_pad;
    const size_t stride = static_cast<size_t>(a.T) * N;
    const float* p = a.part + static_cast<size_t>(t) * N + n;
    // n % 4 == 0 and the tile height is a multiple of 4: the four columns share a tile
    const RowSquares sq = row_squares_load(a.ns, t);
    const float* const pp[2] = {p, p + a.f_pad};
    const int np[2] = {plan_pieces(a.plan, n / a.plan.bn), plan_pieces(a.plan, (a.f_pad + n) / a.plan.bn)};
    f32x4 gu[2];
    sum_pieces4_multi<2, 4>(pp, stride, np, gu);
    uint2 hi, lo;
    swiglu_split4(gu[0], gu[1], row_scale(a.ns, sq), hi, lo);
    const size_t o = static_cast<size_t>(t) * a.F + n;
    *reinterpret_cast<uint2*>(a.h + o) = hi;
    *reinterpret_cast<uint2*>(a.h_lo + o) = lo;
}

// Per node: add up the logits partials, optionally store them, find the largest (lowest index
// on ties) and the runner-up value.  grid (T, AM_SLICES): every workgroup takes one slice of the
// vocabulary (16-byte piece loads in batches when the row pitch allows, else one column at a
// time), leaves its (best, index, runner-up) in scratch and the last workgroup of a node to
// arrive merges the slices in slice order and resets the node's arrival counter.
constexpr int AM_THREADS = 256;
constexpr int AM_SLICES = ARGMAX_SLICES;

__device__ __forceinline__ void top2_merge(float& b, int& bi, float& s2, float ob, int oi, float os) {
    if (ob > b || (ob == b && oi < bi)) {
        s2 = fmaxf(fmaxf(s2, os), b);
        b = ob;
        bi = oi;
    } else {
        s2 = fmaxf(s2, ob);
    }
}

__global__ __launch_bounds__(AM_THREADS) void cats_argmax(ArgmaxArgs a) {
    __shared__ float s_best[AM_THREADS / 64], s_second[AM_THREADS / 64];
    __shared__ int s_idx[AM_THREADS / 64];
    __shared__ float s_stat[AM_THREADS / 64][3];
    const int t = blockIdx.x, slice = blockIdx.y, tid = threadIdx.x;
    float best = -INFINITY, second = -INFINITY;
    int bidx = 0x7fffffff;
    const float rs = row_scale(a.ns, t);
    // running (max, sum exp, sum exp * z) of z = logit * inv_temp for the log-sum-exp and the entropy
    const bool stats = a.lse != nullptr;
    float zm = -INFINITY, zs = 0.f, zw = 0.f;
    auto take = [&](float val, int v) {   // indices ascend within a thread: strict > keeps the lowest
        if (val > best) {
            second = best;
            best = val;
            bidx = v;
        } else if (val > second) {
            second = val;
        }
        if (stats) {
            const float z = val * a.inv_temp;
            if (z > zm) {
                const float c = __expf(zm - z);   // 0 on the first element (zm = -inf)
                zs = zs * c + 1.f;
                zw = zw * c + z;
                zm = z;
            } else {
                const float e = __expf(z - zm);
                zs += e;
                zw += e * z;
            }
        }
    };
    auto stat_merge = [](float& m, float& s1, float& w, float om, float os, float ow) {
        const float mn = fmaxf(m, om);
        const float ca = m == mn ? 1.f : __expf(m - mn), cb = om == mn ? 1.f : __expf(om - mn);
        s1 = s1 * ca + os * cb;
        w = w * ca + ow * cb;
        m = mn;
    };
    if (a.ld % 4 == 0) {
        const int groups = (a.V + 3) / 4;
        const int g_begin = static_cast<int>(static_cast<int64_t>(groups) * slice / AM_SLICES);
        const int g_end = static_cast<int>(static_cast<int64_t>(groups) * (slice + 1) / AM_SLICES);
        const size_t stride = static_cast<size_t>(a.T) * a.ld;
        for (int g = g_begin + tid; g < g_end; g += AM_THREADS) {
            const int v = 4 * g;   // the four columns share a tile (tile heights are multiples of 4)
            f32x4 val = sum_pieces4(a.part + static_cast<size_t>(t) * a.ld + v, stride, plan_pieces(a.plan, v / a.plan.bn));
            val *= rs;
            if (a.logits) {
                if (a.V % 4 == 0) {
                    *reinterpret_cast<f32x4*>(a.logits + static_cast<size_t>(t) * a.V + v) = val;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (v + e < a.V) a.logits[static_cast<size_t>(t) * a.V + v + e] = val[e];
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (v + e < a.V) take(val[e], v + e);
        }
    } else {
        const int v_begin = static_cast<int>(static_cast<int64_t>(a.V) * slice / AM_SLICES);
        const int v_end = static_cast<int>(static_cast<int64_t>(a.V) * (slice + 1) / AM_SLICES);
        for (int v = v_begin + tid; v < v_end; v += AM_THREADS) {
            const float val = rs * sum_pieces(a.part, a.plan, a.T, a.ld, t, v);
            if (a.logits) a.logits[static_cast<size_t>(t) * a.V + v] = val;
            take(val, v);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o), os = __shfl_xor(second, o);
        const int oi = __shfl_xor(bidx, o);
        top2_merge(best, bidx, second, ob, oi, os);
        if (stats) stat_merge(zm, zs, zw, __shfl_xor(zm, o), __shfl_xor(zs, o), __shfl_xor(zw, o));
    }
    if ((tid & 63) == 0) {
        s_best[tid >> 6] = best;
        s_second[tid >> 6] = second;
        s_idx[tid >> 6] = bidx;
        s_stat[tid >> 6][0] = zm;
        s_stat[tid >> 6][1] = zs;
        s_stat[tid >> 6][2] = zw;
    }
    __syncthreads();
    if (tid != 0) return;
    for (int w = 1; w < AM_THREADS / 64; ++w) {
        top2_merge(best, bidx, second, s_best[w], s_idx[w], s_second[w]);
        if (stats) stat_merge(zm, zs, zw, s_stat[w][0], s_stat[w][1], s_stat[w][2]);
    }
    // publish this slice; the last arriver of the node merges.  The slice results move with
    // device-coherent (relaxed, device-scope) atomic stores and loads, which bypass the
    // per-XCD caches; waiting for the stores' acknowledgement before the arrival count is
    // raised orders them without a cache write-back / invalidate, which costs microseconds here.
    float* pb = a.slice_best + static_cast<size_t>(t) * AM_SLICES;
    float* ps = a.slice_second + static_cast<size_t>(t) * AM_SLICES;
    int* pi = a.slice_idx + static_cast<size_t>(t) * AM_SLICES;
    __hip_atomic_store(pb + slice, best, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(ps + slice, second, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(pi + slice, bidx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    float* pst = a.slice_stat + (static_cast<size_t>(t) * AM_SLICES + slice) * 3;
    if (stats) {
        __hip_atomic_store(pst, zm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(pst + 1, zs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(pst + 2, zw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const int arrived = __hip_atomic_fetch_add(a.arrivals + t, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("" ::: "memory");
    if (arrived != AM_SLICES - 1) return;
    best = -INFINITY;
    second = -INFINITY;
    bidx = 0x7fffffff;
    for (int sl = 0; sl < AM_SLICES; ++sl)
        top2_merge(best, bidx, second, __hip_atomic_load(pb + sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                   __hip_atomic_load(pi + sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                   __hip_atomic_load(ps + sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    a.amax[t] = bidx;
    if (a.margin) a.margin[t] = best - second;
    if (stats) {
        const float* ps0 = a.slice_stat + static_cast<size_t>(t) * AM_SLICES * 3;
        zm = -INFINITY;
        zs = 0.f;
        zw = 0.f;
        for (int sl = 0; sl < AM_SLICES; ++sl)
            stat_merge(zm, zs, zw, __hip_atomic_load(ps0 + 3 * sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                       __hip_atomic_load(ps0 + 3 * sl + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                       __hip_atomic_load(ps0 + 3 * sl + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        const float lse = zm + logf(zs);
        a.lse[t] = lse;
        a.entropy[t] = lse - zw / zs;   // H = -sum p log p = lse - sum p z
    }
    __hip_atomic_store(a.arrivals + t, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
}

}  // namespace

void launch_residual_norm(const ResidualNormArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(cats_residual_rmsnorm, dim3(a.T, (a.H + SS_COLS - 1) / SS_COLS), dim3(64), 0, st, a);
}

void launch_rope_table(const RopeTableArgs& a, hipStream_t st) {
    const int n = a.T * (a.d / 2);
    hipLaunchKernelGGL(cats_rope_table, dim3((n + 255) / 256), dim3(256), 0, st, a);
}

void launch_qkv_rope(const QkvRopeArgs& a, hipStream_t st) {
    const int heads_per_block = 256 / (a.d / 8);
    const int gy = (a.nh + heads_per_block - 1) / heads_per_block;
    hipLaunchKernelGGL(cats_qkv_rope_append, dim3(a.T * gy + a.nh * (a.d / V_DIMS)), dim3(256), 0, st, a);
}

void launch_swiglu(const SwigluArgs& a, hipStream_t st) {
    const int n = a.T * (a.F / 4);
    hipLaunchKernelGGL(cats_swiglu, dim3((n + 255) / 256), dim3(256), 0, st, a);
}

void launch_argmax(const ArgmaxArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(cats_argmax, dim3(a.T, AM_SLICES), dim3(AM_THREADS), 0, st, a);
}
