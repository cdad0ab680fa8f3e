// Tree-masked attention over the KV cache plus the tree nodes (paper Fig. 4,
// right-lower: the tree attention mask; Sec. 3.2 "Target verification pass").
//
// Node i attends to cache rows [0, ctx_len) and to rows ctx_len + a for every a
// on its root-to-node path.  The ancestor sets are 128-bit masks, built from parent[] in
// LDS by cats_tree_masks when the tree is uploaded and read here one mask per query.
//
// Work split: one workgroup of ATTN_WAVES waves per (head, chunk of key blocks, group of
// ATTN_QN queries); wave w takes the chunk's blocks w, w + ATTN_WAVES, ... and the waves'
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
// QB: 16-query groups per wave (a workgroup covers QN = 16 * QB queries); W: waves per workgroup.
template <int D, int QB, int W>
__global__ __launch_bounds__(64 * W) void cats_tree_attention_kernel(AttnArgs a) {
    constexpr int QN = 16 * QB;
    constexpr int KS = D / 32;  // k-steps of the score product
    constexpr int DB = D / 16;  // 16-row blocks of O^T
    __shared__ float s_o[W][QN][D + 4];
    __shared__ float s_ml[W][QN][2];
    __shared__ int s_last;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, q4 = lane >> 4;
    const int chunk = blockIdx.x, h = blockIdx.y, qbase = blockIdx.z * QN;
    const int S = a.ctx_len, T = a.T, Tq = a.Tq;   // T tree nodes are keys; Tq of them (from q0) are queries
    const int n_keys = S + T;

    // ancestor-or-self masks of this lane's queries
    u32x4 anc[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int t = qbase + 16 * qb + m;
        anc[qb] = t < Tq ? a.anc[a.q0 + t] : u32x4{0u, 0u, 0u, 0u};
    }

    // Q^T fragments (B operand of the score product): column = query, k = dim; queries come
    // as high + low bf16 parts (the low part may be absent)
    bf16x8 qf[QB][KS], qfl[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
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

    f32x4 o[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db) o[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun[QB], lrun[QB];   // running maximum (base 2), this lane's share of the row sum
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        mrun[qb] = -1e30f;
        lrun[qb] = 0.f;
    }
    bool fresh = true;           // nothing accumulated yet (wave-uniform)

    const float scale = rsqrtf(static_cast<float>(D)) * 1.44269504088896340736f;   // 1/sqrt(d) * log2(e)
    const bf16_t* kbase = a.kc + static_cast<size_t>(h) * a.max_ctx * D;
    const bf16_t* vbase = a.vt + static_cast<size_t>(h) * D * a.max_ctx;

    const int n_blocks = (n_keys + ATTN_KB - 1) / ATTN_KB;
    // Chunks are contiguous runs of key blocks (neighbouring blocks share cache lines of the
    // transposed values) of equal cost: a block that holds tree rows counts twice (masks, low
    // parts, no prefetch), so the chunk that ends with them gets fewer blocks.  Cost units: block b
    // starts at unit b below the first tree block tb, at tb + 2 (b - tb) from there on; chunk c
    // owns the blocks whose first unit lies in [c U / n, (c + 1) U / n).
    const int tree_blk = min(n_blocks, S / ATTN_KB);
    const int units = tree_blk + 2 * (n_blocks - tree_blk);
    auto first_block_at = [&](int u) {   // first block whose first unit is >= u
        return u <= tree_blk ? u : tree_blk + (u - tree_blk + 1) / 2;
    };
    const int blk_begin = first_block_at((chunk * units + a.n_chunks - 1) / a.n_chunks);
    const int blk_end = chunk + 1 == a.n_chunks ? n_blocks
                                                : first_block_at(((chunk + 1) * units + a.n_chunks - 1) / a.n_chunks);
    constexpr int blk_stride = W;

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

    // MODE 0: every key of the block is a context row (no mask, no tail: straight-line code);
    // MODE 1: the block may hold tree rows and rows past the tree; MODE 2: as 1, and the block
    // also has low parts of keys (kfl) and values (vfl).  Scores and running maxima are kept in
    // the base-2 domain (the scale carries log2 e), so that every exponential is one v_exp_f32.
    auto compute_block = [&](const bf16x8 (&kf)[2][KS], const bf16x8 (&vf_in)[DB], const bf16x8 (&kfl)[2][KS],
                             const bf16x8 (&vfl)[DB], int blk, auto mode_tag) {
        constexpr int MODE = decltype(mode_tag)::value;
        constexpr bool LO = MODE == 2;
        const int j0 = blk * ATTN_KB;
        const int key0 = j0 + 8 * q4;
        bf16x8 vf[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            u32x4 v = __builtin_bit_cast(u32x4, vf_in[db]);
            if constexpr (MODE != 0) v = keep_keys(v, key0, 0, n_keys);  // rows past the tree may hold anything
            vf[db] = as_bf16x8(v);
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
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
                bool v = true;
                if constexpr (MODE != 0) {
                    // branch-free: the ancestor word is picked with selects, a key outside the
                    // tree's rows reads bit 0 of a zero word
                    const int rel = key0 + i - S;
                    const bool in_tree = rel >= 0 && rel < T;
                    const int w = rel >> 5;
                    const u32x4 am = anc[qb];
                    uint32_t word = w == 0 ? am[0] : (w == 1 ? am[1] : (w == 2 ? am[2] : am[3]));
                    word = in_tree ? word : 0u;
                    v = rel < 0 || ((word >> (rel & 31)) & 1u);
                }
                vis[i] = v;
                sc[i] = v ? st[i >> 2][i & 3] * scale : -1e30f;
                bmax = fmaxf(bmax, sc[i]);
            }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
            // The running maximum may lag behind the true one by up to 8 (base 2): the
            // probabilities then reach 2^8 at most, and the accumulated output is rescaled only
            // when some lane of the wave needs it (wave-uniform branch; rare after the first
            // block), which saves the pass over the accumulators in the common case.
            if (__builtin_amdgcn_ballot_w64(bmax > mrun[qb] + 8.f) != 0) {
                const float mnew = fmaxf(mrun[qb], bmax);
                const float alpha = __builtin_amdgcn_exp2f(mrun[qb] - mnew);
                mrun[qb] = mnew;
                lrun[qb] *= alpha;
                if (!fresh) {
#pragma unroll
                    for (int db = 0; db < DB; ++db) o[qb][db] *= alpha;
                }
            }
            const float mref = mrun[qb];
            float p[8];
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float e = __builtin_amdgcn_exp2f(sc[i] - mref);
                p[i] = (MODE == 0 || vis[i]) ? e : 0.f;
                psum += p[i];
            }
            lrun[qb] += psum;
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
                o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pf, o[qb][db], 0, 0, 0);
                o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[db], pfl, o[qb][db], 0, 0, 0);
                if constexpr (LO)
                    o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vfl[db], pf, o[qb][db], 0, 0, 0);
            }
        }
        fresh = false;
    };

    // Two register sets.  This wave's blocks come in three runs.  Context-only blocks (all of
    // them but the last few): the fragments of block b+1 are requested before block b is
    // multiplied, so the cache latency of one block hides behind the arithmetic of the other.
    // Then the blocks that hold tree rows without low parts (rows an earlier call appended, or a
    // caller's own rows), one at a time; then the blocks with low parts, set A holding the high
    // parts and set B the low parts.  The last two runs are at most five blocks per head.
    bf16x8 kfA[2][KS], kfB[2][KS], vfA[DB], vfB[DB];
    const bool have_lo = a.k_lo != nullptr && a.lo_end > a.lo_begin;
    const int lo_blk = have_lo ? min(blk_end, a.lo_begin / ATTN_KB) : blk_end;   // first block with low parts
    const int ctx_end = min(lo_blk, tree_blk);                                // blocks below hold context rows only
    const int my_begin = blk_begin + wave;
    // this wave's first block at or after `from`
    auto my_first = [&](int from) {
        return my_begin + (max(from - my_begin, 0) + blk_stride - 1) / blk_stride * blk_stride;
    };
    // the costlier blocks first: their loads go out with the kernel's first requests
    if (have_lo) {
        for (int blk = my_first(lo_blk); blk < blk_end; blk += blk_stride) {
            load_block(kfA, vfA, blk);
            load_block_lo(kfB, vfB, blk);
            compute_block(kfA, vfA, kfB, vfB, blk, std::integral_constant<int, 2>{});
        }
    }
    for (int blk = my_first(ctx_end); blk < lo_blk; blk += blk_stride) {
        load_block(kfA, vfA, blk);
        compute_block(kfA, vfA, kfB, vfB, blk, std::integral_constant<int, 1>{});
    }
    if (my_begin < ctx_end) {
        const int last = my_begin + (ctx_end - 1 - my_begin) / blk_stride * blk_stride;  // this wave's last such block
        load_block(kfA, vfA, my_begin);
        for (int blk = my_begin; blk < ctx_end; blk += 2 * blk_stride) {
            load_block(kfB, vfB, min(blk + blk_stride, last));
            compute_block(kfA, vfA, kfB, vfB, blk, std::integral_constant<int, 0>{});
            if (blk + blk_stride < ctx_end) {
                load_block(kfA, vfA, min(blk + 2 * blk_stride, last));
                compute_block(kfB, vfB, kfA, vfA, blk + blk_stride, std::integral_constant<int, 0>{});
            }
        }
    }

    // every wave parks its running max, row sum and unnormalised output in LDS ...
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
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
    // thread -> (query ql, dims 4 (i TPQ + c) .. + 3 for i < NI): the TPQ threads of a query cover
    // 4 TPQ consecutive dims per i, so every 16-byte access of a wave falls into whole 128-byte lines
    constexpr int TPQ = 64 * W / QN;      // threads per query
    constexpr int NI = D / (4 * TPQ);
    static_assert(NI >= 1 && NI * 4 * TPQ == D, "merge mapping");
    const int ql = threadIdx.x / TPQ, c4 = 4 * (threadIdx.x % TPQ);
    float M = -1e30f;
#pragma unroll
    for (int w = 0; w < W; ++w) M = fmaxf(M, s_ml[w][ql][0]);
    float wgt[W], l = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) {
        wgt[w] = __builtin_amdgcn_exp2f(s_ml[w][ql][0] - M);
        l += wgt[w] * s_ml[w][ql][1];
    }
    f32x4 acc[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < W; ++w) acc[i] += wgt[w] * *reinterpret_cast<const f32x4*>(&s_o[w][ql][4 * TPQ * i + c4]);
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
            *reinterpret_cast<uint2*>(a.out + o_off + 4 * TPQ * i) = hi;
            if (a.out_lo) *reinterpret_cast<uint2*>(a.out_lo + o_off + 4 * TPQ * i) = lo;
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
        for (int i = 0; i < NI; ++i) store_coherent16(po + 4 * TPQ * i, acc[i]);
        if (threadIdx.x % TPQ == 0) {
            __hip_atomic_store(a.pml + slot * 2, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(a.pml + slot * 2 + 1, l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();   // every thread's stores have been acknowledged
    int* counter = a.arrivals + h * gridDim.z + blockIdx.z;
    if (threadIdx.x == 0)
        s_last = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.n_chunks - 1;
    __syncthreads();
    if (!s_last) return;
    // last workgroup of this (head, query group): out = sum_c exp2(m_c - M) O_c / sum_c exp2(m_c - M) l_c,
    // chunks in index order, eight chunks' loads in flight at a time (one memory round trip for
    // up to eight chunks), rescaled to the running maximum between groups
    constexpr int MG = 8;
    float Mg = -1e30f;
    f32x4 num[NI];
    float den = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) num[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < a.n_chunks; c0 += MG) {
        f32x4 v[MG][NI];
        float mc[MG], lc[MG];
#pragma unroll
        for (int j = 0; j < MG; ++j) {
            const int c = min(c0 + j, a.n_chunks - 1);
            const size_t sl = (static_cast<size_t>(h) * a.n_chunks + c) * a.t_pad + qbase + ql;
            mc[j] = __hip_atomic_load(a.pml + sl * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            lc[j] = __hip_atomic_load(a.pml + sl * 2 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float* po = a.po + sl * D + c4;
#pragma unroll
            for (int i = 0; i < NI; ++i) v[j][i] = load_coherent16(po + 4 * TPQ * i);
        }
#pragma unroll
        for (int j = 0; j < MG; ++j)
#pragma unroll
            for (int i = 0; i < NI; ++i) wait_coherent(v[j][i]);
        float Mn = Mg;
#pragma unroll
        for (int j = 0; j < MG; ++j) Mn = fmaxf(Mn, mc[j]);   // clamped repeats do not change the maximum
        const float resc = __builtin_amdgcn_exp2f(Mg - Mn);
        den *= resc;
#pragma unroll
        for (int i = 0; i < NI; ++i) num[i] *= resc;
        Mg = Mn;
#pragma unroll
        for (int j = 0; j < MG; ++j) {
            if (c0 + j < a.n_chunks) {
                const float wc = __builtin_amdgcn_exp2f(mc[j] - Mg);
                den += wc * lc[j];
#pragma unroll
                for (int i = 0; i < NI; ++i) num[i] += wc * v[j][i];
            }
        }
    }
    write_out(num, den);
    if (threadIdx.x == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
}

// ---------------------------------------------------------------- single query
// One query node against rows [0, ctx_len) and its own path (see DecodeAttnArgs).  grid (chunks,
// heads), 256 threads; a workgroup takes its chunk in passes of DEC_TILE keys (normally one).
// Nothing here is a matrix product worth a matrix core: a pass is 64 KB of keys and values, and
// the launch is one memory round trip (partial sums, keys and values are all requested before the
// first of them is used), a few hundred fused multiply-adds per thread, and the store of the
// chunk's result (see DecodeAttnArgs: the following product merges the chunks).
//   scores: a key row is D/8 16-byte pieces, one per lane, summed over those lanes;
//   values: the cache is transposed, a dim's 128 keys are 16 16-byte pieces, one per lane.
// Rows that must stay invisible (later siblings, rows past the tree, the node's own row, which is
// being written meanwhile) are excluded by selects, never by a multiplication with zero.
__device__ __forceinline__ bool mask_bit(const u32x4& m, int i) {
    const uint32_t w = i < 64 ? (i < 32 ? m[0] : m[1]) : (i < 96 ? m[2] : m[3]);
    return (w >> (i & 31)) & 1u;
}

template <int D>
__global__ __launch_bounds__(256) void cats_decode_attention(DecodeAttnArgs a) {
    constexpr int LPK = D / 8;           // lanes per key row
    constexpr int KPP = 256 / LPK;       // keys per score pass
    constexpr int KP = DEC_TILE / KPP;   // score passes per tile
    constexpr int VP = D / 16;           // value passes per tile (16 dims each)
    constexpr int HALF = D / 2;
    constexpr int PB = 8;                // partial sums requested at once per column
    __shared__ float s_q[D], s_kn[D], s_vn[D];
    __shared__ float s_sc[DEC_TILE];
    __shared__ __align__(16) float s_o[D];
    __shared__ float s_new;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x, h = blockIdx.y;
    const int S = a.ctx_len, node = a.node;
    const int n_keys = S + node + 1, own = S + node;
    const int key_begin = chunk * a.span, key_end = min(key_begin + a.span, n_keys);
    const bool owner = own >= key_begin && own < key_end;
    const u32x4 anc = a.anc[node];
    bf16_t* kbase = a.kc + static_cast<size_t>(h) * a.max_ctx * D;
    bf16_t* vbase = a.vt + static_cast<size_t>(h) * D * a.max_ctx;
    const float scale = rsqrtf(static_cast<float>(D)) * 1.44269504088896340736f;   // 1/sqrt(d) * log2(e)
    auto visible = [&](int j) { return j < key_end && j != own && (j < S || mask_bit(anc, j - S)); };

    // requests: this wave's two columns of q, k or v (waves 0..2; k and v only where the node's
    // own row lives), then the first tile's keys and values
    const int role = wave;
    const bool builds = lane < HALF && (role == 0 || (owner && role <= 2));
    const int N = 3 * a.H;
    const int col = min(role, 2) * a.H + h * D + min(lane, HALF - 1);
    const int pieces = plan_pieces(a.plan, col / a.plan.bn);   // both columns lie in the same tile
    float pa[PB], pb[PB];
    RowSquares sq;
    float2 cs = make_float2(1.f, 0.f);
    if (builds) {
        sq = row_squares_load(a.ns, 0);
        if (role < 2) cs = a.cs[lane];
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const float* p = a.part + static_cast<size_t>(min(i, pieces - 1)) * N + col;
            pa[i] = p[0];
            pb[i] = p[HALF];
        }
    }
    u32x4 kf[KP], vf[VP];
    auto load_tile = [&](int t0) {
#pragma unroll
        for (int p = 0; p < KP; ++p) {
            const int key = min(t0 + KPP * p + tid / LPK, a.max_ctx - 1);
            kf[p] = *reinterpret_cast<const u32x4*>(kbase + static_cast<size_t>(key) * D + 8 * (tid % LPK));
        }
#pragma unroll
        for (int p = 0; p < VP; ++p) {
            const int j0 = min(t0 + 8 * (tid % 16), a.max_ctx - 8);
            vf[p] = *reinterpret_cast<const u32x4*>(vbase + static_cast<size_t>(16 * p + tid / 16) * a.max_ctx + j0);
        }
    };
    load_tile(key_begin);

    // q (every workgroup), k and v of the node's own row (its owner): sum, scale, rotate
    if (builds) {
        float va = 0.f, vb = 0.f;
#pragma unroll
        for (int i = 0; i < PB; ++i)
            if (i < pieces) {
                va += pa[i];
                vb += pb[i];
            }
        for (int i = PB; i < pieces; ++i) {
            const float* p = a.part + static_cast<size_t>(i) * N + col;
            va += p[0];
            vb += p[HALF];
        }
        const float rs = row_scale(a.ns, sq);
        va *= rs;
        vb *= rs;
        const float r0 = role < 2 ? va * cs.x - vb * cs.y : va;
        const float r1 = role < 2 ? va * cs.y + vb * cs.x : vb;
        if (role == 0) {
            s_q[lane] = r0;
            s_q[lane + HALF] = r1;
        } else {
            const bf16_t h0 = f2bf(r0), h1 = f2bf(r1);
            float* dst = role == 1 ? s_kn : s_vn;
            dst[lane] = bf2f(h0) + bf2f(f2bf(r0 - bf2f(h0)));   // the row as later products of this call see it:
            dst[lane + HALF] = bf2f(h1) + bf2f(f2bf(r1 - bf2f(h1)));   // high + low part
            if (role == 1) {
                kbase[static_cast<size_t>(own) * D + lane] = h0;
                kbase[static_cast<size_t>(own) * D + lane + HALF] = h1;
            } else {
                vbase[static_cast<size_t>(lane) * a.max_ctx + own] = h0;
                vbase[static_cast<size_t>(lane + HALF) * a.max_ctx + own] = h1;
            }
        }
    }
    __syncthreads();
    float qs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) qs[e] = s_q[8 * (tid % LPK) + e];
    if (wave == 3 && owner) {   // the node's own key
        float acc = 0.f;
        for (int d = lane; d < D; d += 64) acc += s_q[d] * s_kn[d];
        acc = wave_sum64(acc);
        if (lane == 0) s_new = acc * scale;
    }

    float m_run = -1e30f, l_run = 0.f, o_run[VP];
#pragma unroll
    for (int p = 0; p < VP; ++p) o_run[p] = 0.f;
    for (int t0 = key_begin;;) {
        // scores of the tile's keys
#pragma unroll
        for (int p = 0; p < KP; ++p) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dot = fmaf(__uint_as_float(kf[p][e] << 16), qs[2 * e], dot);
                dot = fmaf(__uint_as_float(kf[p][e] & 0xFFFF0000u), qs[2 * e + 1], dot);
            }
#pragma unroll
            for (int o = LPK / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
            const int kl = KPP * p + tid / LPK;
            if (tid % LPK == 0) s_sc[kl] = visible(t0 + kl) ? dot * scale : -INFINITY;
        }
        __syncthreads();
        const bool own_here = owner && own >= t0 && own < t0 + DEC_TILE;
        // tile maximum (every wave works it out for itself), this thread's 8 keys' weights, tile sum
        float m_t = fmaxf(s_sc[lane], s_sc[lane + 64]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m_t = fmaxf(m_t, __shfl_xor(m_t, o));
        if (own_here) m_t = fmaxf(m_t, s_new);
        m_t = fmaxf(m_t, -1e30f);
        float pw[8], l_t = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            pw[e] = __builtin_amdgcn_exp2f(s_sc[8 * (tid % 16) + e] - m_t);
            l_t += pw[e];
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) l_t += __shfl_xor(l_t, o);
        const float p_new = own_here ? __builtin_amdgcn_exp2f(s_new - m_t) : 0.f;
        l_t += p_new;
        // weighted values: 16 dims per pass, a dim's keys over 16 lanes
        const float m_new = fmaxf(m_run, m_t);
        const float c_run = __builtin_amdgcn_exp2f(m_run - m_new), c_t = __builtin_amdgcn_exp2f(m_t - m_new);
#pragma unroll
        for (int p = 0; p < VP; ++p) {
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v0 = __uint_as_float(vf[p][e] << 16), v1 = __uint_as_float(vf[p][e] & 0xFFFF0000u);
                acc += pw[2 * e] != 0.f ? pw[2 * e] * v0 : 0.f;
                acc += pw[2 * e + 1] != 0.f ? pw[2 * e + 1] * v1 : 0.f;
            }
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
            if (own_here) acc += p_new * s_vn[16 * p + tid / 16];
            o_run[p] = o_run[p] * c_run + acc * c_t;
        }
        l_run = l_run * c_run + l_t * c_t;
        m_run = m_new;
        t0 += DEC_TILE;
        if (t0 >= key_end) break;
        __syncthreads();   // the scores are overwritten by the next tile
        load_tile(t0);
    }
    if (tid % 16 == 0) {
#pragma unroll
        for (int p = 0; p < VP; ++p) s_o[16 * p + tid / 16] = o_run[p];
    }
    __syncthreads();

    // The chunk's result: unnormalised sums, running maximum and row sum.  The output projection
    // merges a head's chunks while it builds its input columns, so nothing is handed over between
    // workgroups here and the launch ends with these stores.
    const size_t slot = static_cast<size_t>(h) * a.n_chunks + chunk;
    if (tid < D / 4)
        *reinterpret_cast<f32x4*>(a.po + slot * D + 4 * tid) = *reinterpret_cast<const f32x4*>(&s_o[4 * tid]);
    if (tid == 0) {
        a.pml[slot * 2] = m_run;
        a.pml[slot * 2 + 1] = l_run;
    }
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

void launch_decode_attention(const DecodeAttnArgs& a, hipStream_t st) {
    const dim3 grid(a.n_chunks, a.nh);
    if (a.d == 128)
        hipLaunchKernelGGL((cats_decode_attention<128>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((cats_decode_attention<64>), grid, dim3(256), 0, st, a);
}

void launch_attention(const AttnArgs& a, hipStream_t st) {
    dim3 grid(a.n_chunks, a.nh, (a.Tq + ATTN_QN - 1) / ATTN_QN);
    if (a.d == 128)
        hipLaunchKernelGGL((cats_tree_attention_kernel<128, ATTN_QN / 16, ATTN_WAVES>), grid, dim3(64 * ATTN_WAVES), 0, st, a);
    else
        hipLaunchKernelGGL((cats_tree_attention_kernel<64, ATTN_QN / 16, ATTN_WAVES>), grid, dim3(64 * ATTN_WAVES), 0, st, a);
}
