// Tree-masked attention over the KV cache plus the tree nodes (paper Fig. 4,
// right-lower: the tree attention mask; Sec. 3.2 "Target verification pass").
//
// Node i attends to cache rows [0, ctx_len) and to rows ctx_len + a for every a
// on its root-to-node path.  The ancestor sets are 128-bit masks, built from parent[] in
// LDS by cats_tree_masks when the tree is uploaded and read here one mask per query.
//
// Work split: one workgroup of ATTN_WAVES waves per (head, chunk of key blocks, group of
// 32 queries); wave w takes the chunk's blocks w, w + ATTN_WAVES, ... and the waves'
// partial results are merged through LDS before the chunk's result is written.
// Scores are computed transposed, S^T = K Q^T, with the 16x16x32 bf16 MFMA, so a
// lane owns ONE query column and 8 keys of every 32-key block: the running
// max / sum of the online softmax are per-lane scalars shared by four lanes and
// reduced with two wave shuffles, and the probabilities are already laid out as
// the B operand of the second product O^T = V^T P^T.  Queries and probabilities are
// fed as high + low bf16 parts so that only the cache's own bf16 format limits accuracy.  V is cached transposed
// ([head][dim][row]) so that its A operand is a plain 128-bit load as well; no
// LDS round trip for K, V or P.  Chunks are merged afterwards with the usual
// log-sum-exp rescaling.
#include "common.hpp"

namespace {

// MFMA 16x16x32 bf16 (wave64): lane l supplies, for A, row l%16 and
// k = 8*(l/16)..+7; for B, column l%16 and the same k; its 4 results are
// D[4*(l/16) + r][l%16].
template <int D>
__global__ __launch_bounds__(64 * ATTN_WAVES) void cats_tree_attention_partial(AttnArgs a) {
    constexpr int KS = D / 32;  // k-steps of the score product
    constexpr int DB = D / 16;  // 16-row blocks of O^T
    __shared__ float s_o[ATTN_WAVES][32][D + 4];
    __shared__ float s_ml[ATTN_WAVES][32][2];

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

    auto compute_block = [&](const bf16x8 (&kf)[2][KS], const bf16x8 (&vf_in)[DB], int blk) {
        const int j0 = blk * ATTN_KB;
        const int key0 = j0 + 8 * q4;
        bf16x8 vf[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            u32x4 v = __builtin_bit_cast(u32x4, vf_in[db]);
            if (key0 + 8 > n_keys) {  // rows past the tree may hold anything: zero them
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (key0 + 2 * e >= n_keys) v[e] &= 0xFFFF0000u;
                    if (key0 + 2 * e + 1 >= n_keys) v[e] &= 0x0000FFFFu;
                }
            }
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
            }
        }
    };

    // Two register sets: the fragments of block b+1 are requested before block b is
    // multiplied, so the cache latency of one block hides behind the arithmetic of the other.
    bf16x8 kfA[2][KS], kfB[2][KS], vfA[DB], vfB[DB];
    const int my_begin = blk_begin + wave;
    if (my_begin < blk_end) {
        const int last = my_begin + (blk_end - 1 - my_begin) / ATTN_WAVES * ATTN_WAVES;  // this wave's last block
        load_block(kfA, vfA, my_begin);
        for (int blk = my_begin; blk < blk_end; blk += 2 * ATTN_WAVES) {
            load_block(kfB, vfB, min(blk + ATTN_WAVES, last));
            compute_block(kfA, vfA, blk);
            if (blk + ATTN_WAVES < blk_end) {
                load_block(kfA, vfA, min(blk + 2 * ATTN_WAVES, last));
                compute_block(kfB, vfB, blk + ATTN_WAVES);
            }
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
    // ... and the workgroup merges them (fixed wave order) into the chunk's partial result:
    // thread -> (query ql, D/8 consecutive dims)
    {
        const int ql = threadIdx.x >> 3, d0 = (threadIdx.x & 7) * (D / 8);
        float M = -1e30f;
#pragma unroll
        for (int w = 0; w < ATTN_WAVES; ++w) M = fmaxf(M, s_ml[w][ql][0]);
        float wgt[ATTN_WAVES], l = 0.f;
#pragma unroll
        for (int w = 0; w < ATTN_WAVES; ++w) {
            wgt[w] = __expf(s_ml[w][ql][0] - M);
            l += wgt[w] * s_ml[w][ql][1];
        }
        const size_t slot = (static_cast<size_t>(h) * a.n_chunks + chunk) * a.t_pad + qbase + ql;
        float* po = a.po + slot * D + d0;
#pragma unroll
        for (int e = 0; e < D / 8; e += 4) {
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < ATTN_WAVES; ++w)
                acc += wgt[w] * *reinterpret_cast<const f32x4*>(&s_o[w][ql][d0 + e]);
            *reinterpret_cast<f32x4*>(po + e) = acc;
        }
        if ((threadIdx.x & 7) == 0) {
            a.pml[slot * 2] = M;
            a.pml[slot * 2 + 1] = l;
        }
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

// out[t][h*D + dd] = sum_c exp(m_c - M) O_c[dd] / sum_c exp(m_c - M) l_c
template <int D>
__global__ void cats_tree_attention_merge(AttnArgs a) {
    const int t = blockIdx.x, h = blockIdx.y, dd = threadIdx.x;
    float M = -1e30f;
    for (int c = 0; c < a.n_chunks; ++c) {
        const size_t slot = (static_cast<size_t>(h) * a.n_chunks + c) * a.t_pad + t;
        M = fmaxf(M, a.pml[slot * 2]);
    }
    float num = 0.f, den = 0.f;
    for (int c = 0; c < a.n_chunks; ++c) {
        const size_t slot = (static_cast<size_t>(h) * a.n_chunks + c) * a.t_pad + t;
        const float wgt = __expf(a.pml[slot * 2] - M);
        num += wgt * a.po[slot * D + dd];
        den += wgt * a.pml[slot * 2 + 1];
    }
    const float r = num / den;
    const bf16_t hi = f2bf(r);
    const size_t o = static_cast<size_t>(t) * a.H + h * D + dd;
    a.out[o] = hi;
    if (a.out_lo) a.out_lo[o] = f2bf(r - bf2f(hi));
}

}  // namespace

void launch_tree_masks(const int32_t* parent, int T, u32x4* anc, hipStream_t st) {
    hipLaunchKernelGGL(cats_tree_masks, dim3(1), dim3(CATS_MAX_TREE), 0, st, parent, T, anc);
}

void launch_attention(const AttnArgs& a, hipStream_t st) {
    dim3 grid(a.n_chunks, a.nh, a.t_pad / 32);
    if (a.d == 128) {
        hipLaunchKernelGGL(cats_tree_attention_partial<128>, grid, dim3(64 * ATTN_WAVES), 0, st, a);
        hipLaunchKernelGGL(cats_tree_attention_merge<128>, dim3(a.Tq, a.nh), dim3(128), 0, st, a);
    } else {
        hipLaunchKernelGGL(cats_tree_attention_partial<64>, grid, dim3(64 * ATTN_WAVES), 0, st, a);
        hipLaunchKernelGGL(cats_tree_attention_merge<64>, dim3(a.Tq, a.nh), dim3(64), 0, st, a);
    }
}
