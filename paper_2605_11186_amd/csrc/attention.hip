// Tree-masked attention over the KV cache plus the tree nodes (paper Fig. 4,
// right-lower: the tree attention mask; Sec. 3.2 "Target verification pass").
//
// Node i attends to cache rows [0, ctx_len) and to rows ctx_len + a for every a
// on its root-to-node path.  The ancestor sets are 128-bit masks, built from parent[] in
// LDS by cats_tree_masks when the tree is uploaded and read here one mask per query.
//
// Work split: one workgroup of ATTN_WAVES waves per (head, chunk of key blocks, group of
// 32 queries); wave w takes the chunk's blocks w, w + ATTN_WAVES, ... and the waves'
// partial results are merged through LDS.  With more than one chunk the workgroup then
// publishes its chunk's result, and the last workgroup of a (head, query group) to arrive adds
// up all chunks in chunk order with the usual log-sum-exp rescaling and writes the output:
// one kernel, no separate merge launch.
// Scores are computed transposed, S^T = K Q^T, with the 16x16x32 bf16 MFMA, so a
// lane owns ONE query column and 8 keys of every 32-key block: the running
// max / sum of the online softmax are per-lane scalars shared by four lanes and
// reduced with two wave shuffles, and the probabilities are already laid out as
// the B operand of the second product O^T = V^T P^T.  Queries and probabilities are
// fed as high + low bf16 parts.  V is cached transposed ([head][dim][row]) so that its A
// operand is a plain 128-bit load as well; no LDS round trip for K, V or P.
// The key blocks that hold rows appended by the running call (the tree's own rows) also take
// those rows' low parts from the window beside the cache (see AttnArgs): one more product per
// fragment there, so that tree nodes see each other at about 16 mantissa bits while context
// rows are what the bf16 cache holds.
#include <type_traits>

#include "common.hpp"

namespace {

// zero the 16-bit elements of an 8-key vector whose key index key0 + e lies outside [lo, hi)
__device__ __forceinline__ u32x4 keep_keys(u32x4 v, int key0, int lo, int hi) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int ka = key0 + 2 * e, kb = ka + 1;
        if (ka < lo || ka >= hi) v[e] &= 0xFFFF0000u;
        if (kb < lo || kb >= hi) v[e] &= 0x0000FFFFu;
    }
    return v;
}

// 16-byte device-coherent accesses (they bypass the per-XCD caches).  The compiler does not see
// the load behind the asm: every value must pass through wait_coherent before its first use.
__device__ __forceinline__ void store_coherent16(float* p, f32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ f32x4 load_coherent16(const float* p) {
    f32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    return v;
}
__device__ __forceinline__ void wait_coherent(f32x4& v) { asm volatile("s_waitcnt vmcnt(0)" : "+v"(v)::"memory"); }

// MFMA 16x16x32 bf16 (wave64): lane l supplies, for A, row l%16 and
// k = 8*(l/16)..+7; for B, column l%16 and the same k; its 4 results are
// D[4*(l/16) + r][l%16].
template <int D>
__global__ __launch_bounds__(64 * ATTN_WAVES) void cats_tree_attention_kernel(AttnArgs a) {
    constexpr int KS = D / 32;  // k-steps of the score product
    constexpr int DB = D / 16;  // 16-row blocks of O^T
    __shared__ float s_o[ATTN_WAVES][32][D + 4];
    __shared__ float s_ml[ATTN_WAVES][32][2];
    __shared__ int s_last;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, q4 = lane >> 4;
    const int chunk = blockIdx.x, h = blockIdx.y, qbase = blockIdx.z * 32;
    const int S = a.ctx_len, T = a.T, Tq = a.Tq;   // T tree nodes are keys; Tq of them (from q0) are queries
    const int n_keys = S + T;

    // ancestor-or-self masks of this lane's two queries
    u32x4 anc[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int t = qbase + 16 * qb + m;
        anc[qb] = t < Tq ? a.anc[a.q0 + t] : u32x4{0u, 0u, 0u, 0u};
    }

    // Q^T fragments (B operand of the score product): column = query, k = dim; queries come
    // as high + low bf16 parts (the low part may be absent)
    bf16x8 qf[2][KS], qfl[2][KS];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int t = qbase + 16 * qb + m;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            u32x4 v = u32x4{0u, 0u, 0u, 0u}, vl = u32x4{0u, 0u, 0u, 0u};
            const size_t off = static_cast<size_t>(min(t, Tq - 1)) * a.H + h * D + 32 * s + 8 * q4;
            if (t < Tq) {
                v = *reinterpret_cast<const u32x4*>(a.q + off);
                if (a.q_lo) vl = *reinterpret_cast<const u32x4*>(a.q_lo + off);
            }
            qf[qb][s] = as_bf16x8(v);
            qfl[qb][s] = as_bf16x8(vl);
        }
    }

    f32x4 o[2][DB];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db) o[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun[2] = {-1e30f, -1e30f};
    float lrun[2] = {0.f, 0.f};  // this lane's share of the row sum

    const float scale = rsqrtf(static_cast<float>(D));
    const bf16_t* kbase = a.kc + static_cast<size_t>(h) * a.max_ctx * D;
    const bf16_t* vbase = a.vt + static_cast<size_t>(h) * D * a.max_ctx;

    const int n_blocks = (n_keys + ATTN_KB - 1) / ATTN_KB;
    const int blk_begin = chunk * a.blocks_per_chunk;
    const int blk_end = min(n_blocks, blk_begin + a.blocks_per_chunk);

    // The K / V fragments of one 32-key block.  Score-block rows are permuted so that a lane
    // ends up with 8 consecutive keys: sub-block b, MFMA row mm <-> key j0 + 8*(mm/4) + 4*b + mm%4.
    // V^T fragments: row = dim, k = 8 consecutive keys starting at j0 + 8*q4.
    auto load_block = [&](bf16x8 (&kf)[2][KS], bf16x8 (&vf)[DB], int blk) {
        const int j0 = blk * ATTN_KB;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int key = j0 + 8 * (m >> 2) + 4 * b + (m & 3);
#pragma unroll
            for (int s = 0; s < KS; ++s)
                kf[b][s] = as_bf16x8(*reinterpret_cast<const u32x4*>(
                    kbase + static_cast<size_t>(key) * D + 32 * s + 8 * q4));
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
            vf[db] = as_bf16x8(*reinterpret_cast<const u32x4*>(
                vbase + static_cast<size_t>(16 * db + m) * a.max_ctx + j0 + 8 * q4));
        __builtin_amdgcn_sched_barrier(0);
    };
    // The low parts of the same fragments from the window; rows outside [lo_begin, lo_end) are
    // stale there and come out as zeros.  Addresses are clamped into the window (what a clamp
    // moves is masked anyway: the window covers every row of the range).
    const int win_base = S & ~(ATTN_KB - 1);
    auto load_block_lo = [&](bf16x8 (&kf)[2][KS], bf16x8 (&vf)[DB], int blk) {
        const int j0 = blk * ATTN_KB;
        const bf16_t* kl = a.k_lo + static_cast<size_t>(h) * TREE_WIN * D;
        const bf16_t* vl = a.vt_lo + static_cast<size_t>(h) * D * TREE_WIN;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int key = j0 + 8 * (m >> 2) + 4 * b + (m & 3);
            const bool ok = key >= a.lo_begin && key < a.lo_end;
            const int w = min(key - win_base, TREE_WIN - 1);
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(kl + static_cast<size_t>(w) * D + 32 * s + 8 * q4);
                kf[b][s] = as_bf16x8(ok ? v : u32x4{0u, 0u, 0u, 0u});
            }
        }
        const int key0 = j0 + 8 * q4;
        const int w0 = min(key0 - win_base, TREE_WIN - 8);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(vl + static_cast<size_t>(16 * db + m) * TREE_WIN + w0);
            vf[db] = as_bf16x8(keep_keys(v, key0, a.lo_begin, a.lo_end));
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // LO: the block also has low parts of keys (kfl) and values (vfl)
    auto compute_block = [&](const bf16x8 (&kf)[2][KS], const bf16x8 (&vf_in)[DB], const bf16x8 (&kfl)[2][KS],
                             const bf16x8 (&vfl)[DB], int blk, auto lo_tag) {
        constexpr bool LO = decltype(lo_tag)::value;
        const int j0 = blk * ATTN_KB;
        const int key0 = j0 + 8 * q4;
        bf16x8 vf[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            u32x4 v = __builtin_bit_cast(u32x4, vf_in[db]);
            if (key0 + 8 > n_keys) v = keep_keys(v, key0, 0, n_keys);  // rows past the tree may hold anything
            vf[db] = as_bf16x8(v);
        }
        const bool all_ctx = j0 + ATTN_KB <= S;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            f32x4 st[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                st[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    st[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[b][s], qf[qb][s], st[b], 0, 0, 0);
                    st[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[b][s], qfl[qb][s], st[b], 0, 0, 0);
                    if constexpr (LO)
                        st[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfl[b][s], qf[qb][s], st[b], 0, 0, 0);
                }
            }
            // this lane: query column m of group qb, keys key0 + 4*b + r
            float sc[8];
            bool vis[8];
            float bmax = -1e30f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int key = key0 + i;
                bool v = true;
                if (!all_ctx) {
                    const int rel = key - S;
                    v = rel < 0;
                    if (rel >= 0 && rel < T) {
                        const int w = rel >> 5;
                        const u32x4 am = anc[qb];
                        const uint32_t word = w == 0 ? am[0] : (w == 1 ? am[1] : (w == 2 ? am[2] : am[3]));
                        v = (word >> (rel & 31)) & 1u;
                    }
                }
                vis[i] = v;
                sc[i] = v ? st[i >> 2][i & 3] * scale : -1e30f;
                bmax = fmaxf(bmax, sc[i]);
            }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
            const float mnew = fmaxf(mrun[qb], bmax);
            const float alpha = __expf(mrun[qb] - mnew);
            mrun[qb] = mnew;
            float p[8];
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = vis[i] ? __expf(sc[i] - mnew) : 0.f;
                psum += p[i];
            }
            lrun[qb] = lrun[qb] * alpha + psum;
            // probabilities as high + low bf16 parts: the second product sees them to ~16 bits
            u32x4 pv, pvl;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t hi, lo;
                split_bf2(p[2 * e], p[2 * e + 1], hi, lo);
                pv[e] = hi;
                pvl[e] = lo;
            }
            const bf16x8 pf = as_bf16x8(pv), pfl = as_bf16x8(pvl);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                o[qb][db] *= alpha;
                o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pf, o[qb][db], 0, 0, 0);
                o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pfl, o[qb][db], 0, 0, 0);
                if constexpr (LO)
                    o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vfl[db], pf, o[qb][db], 0, 0, 0);
            }
        }
    };

    // Two register sets.  Blocks without low parts: the fragments of block b+1 are requested
    // before block b is multiplied, so the cache latency of one block hides behind the
    // arithmetic of the other.  Blocks with low parts (the last ones, at most five per head):
    // set A holds the high parts, set B the low parts.
    bf16x8 kfA[2][KS], kfB[2][KS], vfA[DB], vfB[DB];
    const bool have_lo = a.k_lo != nullptr && a.lo_end > a.lo_begin;
    const int plain_end = have_lo ? min(blk_end, a.lo_begin / ATTN_KB) : blk_end;
    const int my_begin = blk_begin + wave;
    if (my_begin < plain_end) {
        const int last = my_begin + (plain_end - 1 - my_begin) / ATTN_WAVES * ATTN_WAVES;  // this wave's last plain block
        load_block(kfA, vfA, my_begin);
        for (int blk = my_begin; blk < plain_end; blk += 2 * ATTN_WAVES) {
            load_block(kfB, vfB, min(blk + ATTN_WAVES, last));
            compute_block(kfA, vfA, kfB, vfB, blk, std::false_type{});
            if (blk + ATTN_WAVES < plain_end) {
                load_block(kfA, vfA, min(blk + 2 * ATTN_WAVES, last));
                compute_block(kfB, vfB, kfA, vfA, blk + ATTN_WAVES, std::false_type{});
            }
        }
    }
    if (have_lo) {
        // this wave's first block at or after plain_end
        const int skipped = max(plain_end - my_begin, 0);
        for (int blk = my_begin + (skipped + ATTN_WAVES - 1) / ATTN_WAVES * ATTN_WAVES; blk < blk_end;
             blk += ATTN_WAVES) {
            load_block(kfA, vfA, blk);
            load_block_lo(kfB, vfB, blk);
            compute_block(kfA, vfA, kfB, vfB, blk, std::true_type{});
        }
    }

    // every wave parks its running max, row sum and unnormalised output in LDS ...
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l = lrun[qb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int ql = 16 * qb + m;
#pragma unroll
        for (int db = 0; db < DB; ++db)
            *reinterpret_cast<f32x4*>(&s_o[wave][ql][16 * db + 4 * q4]) = o[qb][db];
        if (q4 == 0) {
            s_ml[wave][ql][0] = mrun[qb];
            s_ml[wave][ql][1] = l;
        }
    }
    __syncthreads();
    // ... and the workgroup merges them (fixed wave order) into the chunk's result.
    // thread -> (query ql, dims 32 i + 4 c .. + 3 for i < D/32): the eight threads of a query
    // cover 32 consecutive dims per i, so every 16-byte access of a wave falls into whole
    // 128-byte lines
    constexpr int NI = D / 32;
    const int ql = threadIdx.x >> 3, c4 = 4 * (threadIdx.x & 7);
    float M = -1e30f;
#pragma unroll
    for (int w = 0; w < ATTN_WAVES; ++w) M = fmaxf(M, s_ml[w][ql][0]);
    float wgt[ATTN_WAVES], l = 0.f;
#pragma unroll
    for (int w = 0; w < ATTN_WAVES; ++w) {
        wgt[w] = __expf(s_ml[w][ql][0] - M);
        l += wgt[w] * s_ml[w][ql][1];
    }
    f32x4 acc[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < ATTN_WAVES; ++w) acc[i] += wgt[w] * *reinterpret_cast<const f32x4*>(&s_o[w][ql][32 * i + c4]);
    }

    // out[t][h*D + dims] = num / den as high (+ low) bf16 parts
    auto write_out = [&](const f32x4 (&num)[NI], float den) {
        const int t = qbase + ql;
        if (t >= Tq) return;
        const float inv = 1.0f / den;
        const size_t o_off = static_cast<size_t>(t) * a.H + h * D + c4;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            uint2 hi, lo;
            split_bf2(num[i][0] * inv, num[i][1] * inv, hi.x, lo.x);
            split_bf2(num[i][2] * inv, num[i][3] * inv, hi.y, lo.y);
            *reinterpret_cast<uint2*>(a.out + o_off + 32 * i) = hi;
            if (a.out_lo) *reinterpret_cast<uint2*>(a.out_lo + o_off + 32 * i) = lo;
        }
    };
    if (a.n_chunks == 1) {
        write_out(acc, l);
        return;
    }

    // Publish this chunk.  The values move with device-coherent stores and loads (sc1: they
    // bypass the per-XCD caches) in whole 128-byte lines; waiting for the stores' acknowledgement
    // before the arrival count is raised orders them without a cache write-back / invalidate.
    const size_t slot = (static_cast<size_t>(h) * a.n_chunks + chunk) * a.t_pad + qbase + ql;
    {
        float* po = a.po + slot * D + c4;
#pragma unroll
        for (int i = 0; i < NI; ++i) store_coherent16(po + 32 * i, acc[i]);
        if ((threadIdx.x & 7) == 0) {
            __hip_atomic_store(a.pml + slot * 2, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.pml + slot * 2 + 1, l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();   // every thread's stores have been acknowledged
    int* counter = a.arrivals + h * (a.t_pad / 32) + blockIdx.z;
    if (threadIdx.x == 0)
        s_last = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.n_chunks - 1;
    __syncthreads();
    if (!s_last) return;
    // last workgroup of this (head, query group): out = sum_c exp(m_c - M) O_c / sum_c exp(m_c - M) l_c,
    // chunks in index order, four chunks' loads in flight at a time
    float Mg = -1e30f;
    for (int c = 0; c < a.n_chunks; ++c) {
        const size_t sl = (static_cast<size_t>(h) * a.n_chunks + c) * a.t_pad + qbase + ql;
        Mg = fmaxf(Mg, __hip_atomic_load(a.pml + sl * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    f32x4 num[NI];
    float den = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) num[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < a.n_chunks; c0 += 4) {
        f32x4 v[4][NI];
        float mc[4], lc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = min(c0 + j, a.n_chunks - 1);
            const size_t sl = (static_cast<size_t>(h) * a.n_chunks + c) * a.t_pad + qbase + ql;
            mc[j] = __hip_atomic_load(a.pml + sl * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            lc[j] = __hip_atomic_load(a.pml + sl * 2 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float* po = a.po + sl * D + c4;
#pragma unroll
            for (int i = 0; i < NI; ++i) v[j][i] = load_coherent16(po + 32 * i);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < NI; ++i) wait_coherent(v[j][i]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (c0 + j < a.n_chunks) {
                const float wc = __expf(mc[j] - Mg);
                den += wc * lc[j];
#pragma unroll
                for (int i = 0; i < NI; ++i) num[i] += wc * v[j][i];
            }
        }
    }
    write_out(num, den);
    if (threadIdx.x == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
}

// Ancestor-or-self set of every node as a 128-bit mask (bit a of anc[i] set when a is on the
// path root..i): the tree attention mask in compact form.  One workgroup, parent[] in LDS.
__global__ __launch_bounds__(CATS_MAX_TREE) void cats_tree_masks(const int32_t* parent, int T, u32x4* anc) {
    __shared__ int32_t s_parent[CATS_MAX_TREE];
    const int i = threadIdx.x;
    if (i < T) s_parent[i] = parent[i];
    __syncthreads();
    if (i >= T) return;
    u32x4 mask = u32x4{0u, 0u, 0u, 0u};
    int node = i;
    for (int step = 0; step <= CATS_MAX_DEPTH && node >= 0; ++step) {
        const uint32_t bit = 1u << (node & 31);
        const int w = node >> 5;
        mask |= u32x4{w == 0 ? bit : 0u, w == 1 ? bit : 0u, w == 2 ? bit : 0u, w == 3 ? bit : 0u};
        node = s_parent[node];
    }
    anc[i] = mask;
}

__global__ void cats_zero_i32(int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace

void launch_zero_i32(int* p, int n, hipStream_t st) {
    hipLaunchKernelGGL(cats_zero_i32, dim3((n + 255) / 256), dim3(256), 0, st, p, n);
}

void launch_tree_masks(const int32_t* parent, int T, u32x4* anc, hipStream_t st) {
    hipLaunchKernelGGL(cats_tree_masks, dim3(1), dim3(CATS_MAX_TREE), 0, st, parent, T, anc);
}

void launch_attention(const AttnArgs& a, hipStream_t st) {
    dim3 grid(a.n_chunks, a.nh, a.t_pad / 32);
    if (a.d == 128)
        hipLaunchKernelGGL(cats_tree_attention_kernel<128>, grid, dim3(64 * ATTN_WAVES), 0, st, a);
    else
        hipLaunchKernelGGL(cats_tree_attention_kernel<64>, grid, dim3(64 * ATTN_WAVES), 0, st, a);
}
