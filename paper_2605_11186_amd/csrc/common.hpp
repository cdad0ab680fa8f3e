// Shared device helpers and kernel argument blocks of the gfx950 verify library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cats.h"

typedef uint16_t bf16_t;  // raw bf16 bits
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 128-bit load

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// float32 -> bf16, round-to-nearest-even, two values per instruction (v_cvt_pk_bf16_f32 on
// gfx950); inputs here are always finite
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

__device__ __forceinline__ bf16_t f2bf(float f) { return static_cast<bf16_t>(pack_bf2(f, 0.f) & 0xFFFFu); }

// x ~= hi + lo with hi = bf16(x), lo = bf16(x - hi)
__device__ __forceinline__ void split_bf2(float a, float b, uint32_t& hi, uint32_t& lo) {
    hi = pack_bf2(a, b);
    lo = pack_bf2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// ---------------------------------------------------------------- GEMM
// Y[t][n] = sum_k X[t][k] * W[n][k] for t < T.  The work is the list of
// (row tile, K chunk) items in tile-major order, cut into n_wgs equal contiguous
// ranges, one per workgroup, so every CU streams the same number of weight bytes
// whatever the shape.  A tile whose chunks are spread over several workgroups gets one
// float32 partial result ("piece") from each of them: part[piece][t][n], piece =
// workgroup - first workgroup of that tile.  Consumers add the pieces in index order.
struct GemmPlan {
    int bn;      // weight rows per tile
    int kc;      // k values per work item (128 or 256)
    int chunks;  // work items (K chunks of kc values) per tile
    int n_wgs;   // ranges of work items (one partial tile per range and tile it touches)
    int items;   // tiles * chunks
    int ts = 1;  // workgroups per range: each takes its own block of X rows (see the GEMM kernel)
};
// 32-bit unsigned arithmetic (a 64-bit division costs a few hundred scalar instructions on the
// device, at the head of every launch): make_gemm_plan guarantees items * n_wgs < 2^31.
__host__ __device__ inline int plan_owner(const GemmPlan& p, int item) {
    return static_cast<int>((static_cast<unsigned>(item + 1) * static_cast<unsigned>(p.n_wgs) - 1u) /
                            static_cast<unsigned>(p.items));
}
__host__ __device__ inline int plan_item_begin(const GemmPlan& p, int wg) {
    return static_cast<int>(static_cast<unsigned>(wg) * static_cast<unsigned>(p.items) / static_cast<unsigned>(p.n_wgs));
}
__host__ __device__ inline int plan_first_wg(const GemmPlan& p, int tile) { return plan_owner(p, tile * p.chunks); }
__host__ __device__ inline int plan_pieces(const GemmPlan& p, int tile) {
    return plan_owner(p, tile * p.chunks + p.chunks - 1) - plan_owner(p, tile * p.chunks) + 1;
}
// W may be given as up to three row segments of seg_rows rows each (q|k|v, gate|up).
// Activations are carried as a pair of bf16 arrays (hi, lo) with x = hi + lo to about 16
// mantissa bits: bf16 weights times (hi + lo) on the bf16 MFMA keeps the products close to
// fp32 accuracy, which the exact-acceptance requirement needs (a single bf16 rounding of
// every GEMM input moves 7B-scale logits by several 1e-2).
// Output column v of the product belongs to weight segment v / seg_pad, row v % seg_pad of
// it; seg_pad is seg_rows for row-major weights and seg_rows rounded up to 32 for packed ones
// (columns whose row index is >= seg_rows do not exist and are never written).
struct GemmArgs {
    const bf16_t* x;     // [T][K] high parts
    const bf16_t* x_lo;  // [T][K] low parts
    const bf16_t* w[3];
    int n_seg, seg_rows, seg_pad;
    int packed;  // weights are cats_pack_matrix outputs
    int N, K, T;  // N = n_seg * seg_pad
    GemmPlan plan;
    float* part;  // [pieces][T][N]
};
constexpr int PACK_ROWS = 32;   // rows per packed row block
constexpr int PACK_FRAG = 512;  // bf16 elements per packed 1 KB fragment
void launch_pack_matrix(const bf16_t* src, bf16_t* dst, int rows, int cols, hipStream_t st);
size_t packed_matrix_elems(int rows, int cols);
constexpr int GEMM_KC = 128;             // k elements per pipeline stage
constexpr int GEMM_ST = 2;               // register ring depth
GemmPlan make_gemm_plan(int N, int K, int target_wgs, int rows);   // rows of X decide the tile shape (see gemm.hip)
int gemm_plan_max_pieces(const GemmPlan& p);
void launch_gemm(const GemmArgs& a, hipStream_t st, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// Sums of the pieces of G 16-byte groups at once: acc[g] = sum over s < pieces[g] of
// p[g][s * stride], each in index order (deterministic).  The loads of all G groups go out
// together in batches of B pieces (indices past a group's end are clamped and masked), so a
// reader waits for one memory round trip per batch, not one per piece or per group.
template <int G, int B>
__device__ __forceinline__ void sum_pieces4_multi(const float* const (&p)[G], size_t stride, const int (&pieces)[G],
                                                  f32x4 (&acc)[G]) {
    int most = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
        most = max(most, pieces[g]);
    }
    for (int s0 = 0; s0 < most; s0 += B) {
        f32x4 v[G][B];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < B; ++i)
                v[g][i] = *reinterpret_cast<const f32x4*>(p[g] + static_cast<size_t>(min(s0 + i, pieces[g] - 1)) * stride);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < B; ++i)
                if (s0 + i < pieces[g]) acc[g] += v[g][i];
    }
}

// The same sums with a hook that runs between the requests of the first batch and their first use:
// loads that the caller issues there queue behind this batch and do not hold up its arrival.
template <int G, int B, class Hook>
__device__ __forceinline__ void sum_pieces4_multi_hook(const float* const (&p)[G], size_t stride, const int (&pieces)[G],
                                                       f32x4 (&acc)[G], Hook hook) {
    int most = 0;
    f32x4 v[G][B];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
        most = max(most, pieces[g]);
#pragma unroll
        for (int i = 0; i < B; ++i)
            v[g][i] = *reinterpret_cast<const f32x4*>(p[g] + static_cast<size_t>(min(i, pieces[g] - 1)) * stride);
    }
    __builtin_amdgcn_sched_barrier(0);
    hook();
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < B; ++i)
            if (i < pieces[g]) acc[g] += v[g][i];
    for (int s0 = B; s0 < most; s0 += B) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < B; ++i)
                v[g][i] = *reinterpret_cast<const f32x4*>(p[g] + static_cast<size_t>(min(s0 + i, pieces[g] - 1)) * stride);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < B; ++i)
                if (s0 + i < pieces[g]) acc[g] += v[g][i];
    }
}

// Sum of `pieces` 16-byte groups p[s * stride] (fixed order), B loads in flight.
template <int B = 8>
__device__ __forceinline__ f32x4 sum_pieces4(const float* p, size_t stride, int pieces) {
    const float* const pp[1] = {p};
    const int np[1] = {pieces};
    f32x4 acc[1];
    sum_pieces4_multi<1, B>(pp, stride, np, acc);
    return acc[0];
}

// Sum of the pieces of column n of row t (fixed order).
__device__ __forceinline__ float sum_pieces(const float* part, const GemmPlan& p, int T, int N, int t, int n) {
    const int pieces = plan_pieces(p, n / p.bn);
    float v = 0.f;
    for (int s = 0; s < pieces; ++s) v += part[(static_cast<size_t>(s) * T + t) * N + n];
    return v;
}

// ---------------------------------------------------------------- row kernels
// RMSNorm is applied in two halves so that no kernel needs a whole row at once: the kernel
// that updates the residual stream writes x*gain (not yet scaled) as the next GEMM's input
// and, per block of 256 columns, the sum of squares of x; the kernel that consumes that
// GEMM's output multiplies by 1/sqrt(mean(x^2)+eps), which commutes with the product.
constexpr int SS_COLS = 256;   // columns per sum-of-squares block
constexpr int SS_STRIDE = 32;  // blocks per row kept in scratch (hidden <= 8192)
struct NormScale {
    const float* ss;  // [T][SS_STRIDE]
    int n_ss;         // blocks in use
    int H;
    float eps;
};
// Entries past n_ss are never written and stay zero, so the whole row of SS_STRIDE floats is
// added up with eight independent 16-byte loads (fixed order: deterministic).  In two halves, so
// that a kernel can request the row before its partial-sum loads and use it after them: one
// memory round trip instead of two.
struct RowSquares {
    f32x4 v[SS_STRIDE / 4];
};
__device__ __forceinline__ RowSquares row_squares_load(const NormScale& ns, int t) {
    const f32x4* p = reinterpret_cast<const f32x4*>(ns.ss + t * SS_STRIDE);
    RowSquares r;
#pragma unroll
    for (int b = 0; b < SS_STRIDE / 4; ++b) r.v[b] = p[b];
    __builtin_amdgcn_sched_barrier(0);   // keep the requests ahead of what follows
    return r;
}
__device__ __forceinline__ float row_scale(const NormScale& ns, const RowSquares& r) {
    f32x4 acc = r.v[0];
#pragma unroll
    for (int b = 1; b < SS_STRIDE / 4; ++b) acc += r.v[b];
    const float tot = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    return 1.0f / sqrtf(tot / static_cast<float>(ns.H) + ns.eps);
}
__device__ __forceinline__ float row_scale(const NormScale& ns, int t) { return row_scale(ns, row_squares_load(ns, t)); }

__device__ __forceinline__ float wave_sum64(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// The arithmetic of the row kernels, shared with the single-row product that applies the same
// steps to its own input columns (cats_gemv_row): both must give the same bits, so the
// multiply-add contraction is switched off here instead of being left to each call site.
__device__ __forceinline__ float sum_squares4(f32x4 v) {
#pragma clang fp contract(off)
    return ((v[0] * v[0] + v[1] * v[1]) + v[2] * v[2]) + v[3] * v[3];
}
// (val * gain) as high and low bf16 parts; gbits: four bf16 gains
__device__ __forceinline__ void gain_split4(f32x4 val, uint2 gbits, uint2& hi, uint2& lo) {
#pragma clang fp contract(off)
    const float p0 = val[0] * __uint_as_float(gbits.x << 16), p1 = val[1] * __uint_as_float(gbits.x & 0xFFFF0000u);
    const float p2 = val[2] * __uint_as_float(gbits.y << 16), p3 = val[3] * __uint_as_float(gbits.y & 0xFFFF0000u);
    split_bf2(p0, p1, hi.x, lo.x);
    split_bf2(p2, p3, hi.y, lo.y);
}
// silu(gate * rs) * (up * rs) as high and low bf16 parts
__device__ __forceinline__ void swiglu_split4(f32x4 gt, f32x4 up, float rs, uint2& hi, uint2& lo) {
#pragma clang fp contract(off)
    float hv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float g = gt[e] * rs, u = up[e] * rs;
        hv[e] = g / (1.0f + __expf(-g)) * u;
    }
    split_bf2(hv[0], hv[1], hi.x, lo.x);
    split_bf2(hv[2], hv[3], hi.y, lo.y);
}
// four values from their high and low bf16 parts
__device__ __forceinline__ f32x4 join_bf4(uint2 hi, uint2 lo) {
#pragma clang fp contract(off)
    return f32x4{__uint_as_float(hi.x << 16) + __uint_as_float(lo.x << 16),
                 __uint_as_float(hi.x & 0xFFFF0000u) + __uint_as_float(lo.x & 0xFFFF0000u),
                 __uint_as_float(hi.y << 16) + __uint_as_float(lo.y << 16),
                 __uint_as_float(hi.y & 0xFFFF0000u) + __uint_as_float(lo.y & 0xFFFF0000u)};
}

struct ResidualNormArgs {
    float* x;               // [T][H] residual stream, in/out
    const float* x_in;      // optional [T][H]: start from this instead of x
    const bf16_t* embed;    // optional [V][H]: start from embed[token[t]]
    const int32_t* token;   // device [T]
    const float* part;      // optional [pieces][T][H] partial sums to add
    GemmPlan plan;
    const bf16_t* gain;     // optional [H]: if given, xn = x * gain (unscaled) and ss are written
    bf16_t* xn;             // [T][H] high parts of x * gain
    bf16_t* xn_lo;          // [T][H] low parts
    float* ss;              // [T][SS_STRIDE] sums of squares of x per block of SS_COLS columns
    int T, H;
    float eps;
};
void launch_residual_norm(const ResidualNormArgs& a, hipStream_t st);

struct RopeTableArgs {
    const int32_t* depth;  // device [T]
    float2* cs;            // [T][d/2] (cos, sin)
    int T, d, ctx_len;
    float base;
};
void launch_rope_table(const RopeTableArgs& a, hipStream_t st);

struct QkvRopeArgs {
    const float* part;  // [pieces][T][3H]: q | k | v, still to be scaled by the row's norm factor
    GemmPlan plan;
    NormScale ns;
    const float2* cs;   // [T][d/2]
    bf16_t* q;          // [T][H] high parts of the rotated queries
    bf16_t* q_lo;       // [T][H] low parts
    bf16_t* kc;         // [nh][max_ctx][d]
    bf16_t* vt;         // [nh][d][max_ctx]
    bf16_t* k_lo;       // [nh][TREE_WIN][d]   low parts of the key rows written here (see AttnArgs)
    bf16_t* vt_lo;      // [nh][d][TREE_WIN]   low parts of the value columns
    int T, H, nh, d, max_ctx;
    int row0;           // cache row of the first of the T rows (ctx_len + index of its node)
    int win0;           // window index of that row: row0 - (ctx_len rounded down to a multiple of 32)
};
void launch_qkv_rope(const QkvRopeArgs& a, hipStream_t st);

struct SwigluArgs {
    const float* part;  // [pieces][T][2F]: gate | up, still to be scaled by the row's norm factor
    GemmPlan plan;
    NormScale ns;
    bf16_t* h;          // [T][F] high parts
    bf16_t* h_lo;       // [T][F] low parts
    int T, F;
    int f_pad;          // column offset of the up half inside a row of part (row length 2*f_pad)
};
void launch_swiglu(const SwigluArgs& a, hipStream_t st);

struct ArgmaxArgs {
    const float* part;  // [pieces][T][V], still to be scaled by the row's norm factor
    GemmPlan plan;
    NormScale ns;
    int T, V;
    int ld;             // row length of part (V rounded up for packed weights)
    float* logits;      // optional [T][V]
    int32_t* amax;      // [T]
    float* margin;      // optional [T]
    // scratch of the slice merge: [T][ARGMAX_SLICES] each, and [T] arrival counters that are zero
    // between launches
    float* slice_best;
    float* slice_second;
    int* slice_idx;
    int* arrivals;
    // optional (typical acceptance): log-sum-exp and entropy of softmax(logits * inv_temp) per
    // node, from per-slice (max, sum of exponentials, exponential-weighted sum) triples
    float inv_temp;
    float* lse;             // [T] or null
    float* entropy;         // [T]
    float* slice_stat;      // [T][ARGMAX_SLICES][3]
};
constexpr int ARGMAX_SLICES = 16;
void launch_argmax(const ArgmaxArgs& a, hipStream_t st);

// ---------------------------------------------------------------- single-row product
// The same product for a single row (T = 1: the stage-1 draft loop and plain decoding), with the
// row kernel that would run in front of it folded into the way each workgroup builds the input
// columns of its own work items.  Same plan (128-row tiles, 256-wide items), weight layouts and
// partial-tile layout ([piece][N]) as the GEMM above, so the consumers are the same kernels.
//   GEMV_PLAIN   X = x_hi + x_lo (a row that a row kernel or the attention kernel has written)
//   GEMV_NORM    x_out = x_in (or the embedding row of *token) + sum of the pieces of the product
//                before, if any (residual update); X = x_out * gain (as high + low bf16 parts, like
//                the row kernel); the workgroup that owns item (tile 0, chunk c) also writes x_out
//                and ss_out[c] for chunk c's columns
//   GEMV_SWIGLU  X = silu(g) * u, g | u = norm factor * sums of the pieces of the gate|up product
//   GEMV_ATTN    X = the attention output of the single query: the key chunks' partial results that
//                cats_decode_attention left (unnormalised sums, running maximum and row sum per
//                chunk), merged in chunk order with the usual log-sum-exp rescaling
// x_in and x_out must not overlap; pend must not be the buffer `part` points into.
enum { GEMV_PLAIN = 0, GEMV_NORM = 1, GEMV_SWIGLU = 2, GEMV_ATTN = 3 };
struct GemvArgs {
    const bf16_t* w[3];
    int n_seg, seg_rows, seg_pad;
    int packed;
    int N, K;
    GemmPlan plan;       // bn 128, kc 256
    float* part;         // [pieces][N]
    int mode;
    const bf16_t *x_hi, *x_lo;   // PLAIN: [K]
    const float* x_in;           // NORM: [K] (unused when embed is given)
    const bf16_t* embed;         // NORM, optional: [V][K] table; the row starts as embed[*token]
    const int32_t* token;        // device, one entry
    float* x_out;                // NORM: [K] or null
    const bf16_t* gain;          // NORM: [K]
    float* ss_out;               // NORM: [SS_STRIDE]
    const float* pend;           // NORM, SWIGLU: [pieces][pend_ld] partial sums of the product before
    GemmPlan pend_plan;
    int pend_ld;
    NormScale ns;                // SWIGLU: the norm factor of the row (row 0 of ns.ss)
    int f_pad;                   // SWIGLU: column offset of the up half
    const float* po;             // ATTN: [K / head_dim][n_chunks][head_dim] unnormalised chunk sums
    const float* pml;            // ATTN: [K / head_dim][n_chunks][2] running maximum (base 2), row sum
    int n_chunks, head_dim;      // ATTN
    // Optional, any mode: the product is the LM head and only the greedy token is wanted.  Every
    // range of the plan must consist of whole tiles (plan_whole_tiles), so that each workgroup holds
    // complete sums; it then keeps the best of its columns (lowest index among equals; the row's
    // positive norm factor does not change the order), no partial tile is written, and the last
    // workgroup to arrive picks the best of all and writes it to amax[0].
    int32_t* amax;               // null: off
    float* am_best;              // [n_wgs] scratch
    int* am_idx;                 // [n_wgs] scratch
    int* am_arrivals;            // one counter, zero between launches
};
// every workgroup's range is a whole number of tiles
inline bool plan_whole_tiles(const GemmPlan& p) {
    return p.items % p.n_wgs == 0 && (p.items / p.n_wgs) % p.chunks == 0;
}
void launch_gemv(const GemvArgs& a, hipStream_t st, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// ---------------------------------------------------------------- attention
// The cache holds bf16 rows.  The rows that the running call itself appends (the tree nodes it
// forwards) also keep their rounding remainders (k - bf16(k), as bf16) in a small window beside
// the cache, so that within the call tree nodes see one another's keys and values to about 16
// mantissa bits; once committed, a row is its bf16 cache entry.  Window index of cache row r:
// r - (ctx_len & ~31), i.e. the window starts at the 32-key block that holds row ctx_len, which
// keeps 8-key vector loads 16-byte aligned.  Entries outside [lo_begin, lo_end) are stale.
constexpr int TREE_WIN = 32 + CATS_MAX_TREE;   // rows of the window
struct AttnArgs {
    const bf16_t* q;        // [Tq][H]
    const bf16_t* q_lo;     // optional [Tq][H] low parts of q
    const bf16_t* kc;       // [nh][max_ctx][d]
    const bf16_t* vt;       // [nh][d][max_ctx]
    const bf16_t* k_lo;     // optional [nh][TREE_WIN][d] low parts of key rows lo_begin .. lo_end - 1
    const bf16_t* vt_lo;    // optional [nh][d][TREE_WIN]
    int lo_begin, lo_end;   // cache rows that have low parts (empty range: none)
    const u32x4* anc;       // device [T] ancestor-or-self masks (cats_tree_masks)
    int T, H, nh, d, max_ctx, ctx_len;   // T: tree nodes whose K/V rows ctx_len.. take part as keys
    int Tq, q0;             // the queries are nodes q0 .. q0+Tq-1 (rows 0..Tq-1 of q / out)
    int n_chunks, t_pad;    // key chunks per (head, query group); rows per (head, chunk) in po / pml
    float* po;              // [nh][n_chunks][t_pad][d]
    float* pml;             // [nh][n_chunks][t_pad][2]
    int* arrivals;          // [nh][query groups] chunk arrival counters, zero between launches
    bf16_t* out;            // [Tq][H]
    bf16_t* out_lo;         // optional [Tq][H] low parts of the output
};
constexpr int ATTN_KB = 32;    // keys per block
// An attention workgroup: ATTN_WAVES waves, each taking every ATTN_WAVES-th key block of the
// workgroup's chunk for all ATTN_QN queries of the workgroup (two 16-query groups per wave).
// Measured on the 7B shape (T = 63, S = 1024): eight waves of 16 queries with two chunks take the
// same 19 us per layer; a single chunk with eight waves 24 us (every wave then walks five blocks
// one memory round trip after the other).
constexpr int ATTN_WAVES = 4;
constexpr int ATTN_QN = 32;
constexpr int ATTN_MAX_QGROUPS = CATS_MAX_TREE / ATTN_QN;   // query groups per head at most
// Attention of a single-row call (one query node, T = 1 per step: the stage-1 draft loop, plain
// decoding) with the q|k|v step folded in: every workgroup adds up the query columns of its head
// from the q|k|v product's partial sums, scales and rotates them; the workgroup whose key chunk
// holds the node's own cache row does the same for the key and value columns, appends them to the
// cache (bf16) and uses them (high + low part) without reading them back.  The kernel ends with
// one partial result per (head, key chunk); the output projection that follows merges them while
// it builds its input columns (GEMV_ATTN), so no workgroup waits for another.
constexpr int DEC_TILE = 128;       // keys per pass of a workgroup
constexpr int DEC_MAX_CHUNKS = 32;  // key chunks per head at most (the context's scratch holds that many)
struct DecodeAttnArgs {
    const float* part;   // [pieces][3H] partial sums of q | k | v, still to be scaled by the row's norm factor
    GemmPlan plan;
    NormScale ns;        // row 0
    const float2* cs;    // [d/2] (cos, sin) at the node's position
    bf16_t* kc;          // [nh][max_ctx][d]; row ctx_len + node is written
    bf16_t* vt;          // [nh][d][max_ctx]
    const u32x4* anc;    // ancestor-or-self masks of the uploaded tree
    int node;            // the query node; keys: rows [0, ctx_len) and ctx_len + j for j <= node on its path
    int H, nh, d, max_ctx, ctx_len;
    int n_chunks, span;  // chunk c owns keys [c * span, (c + 1) * span); span is a multiple of 32
    float* po;           // [nh][n_chunks][d]  unnormalised weighted value sums of the chunk
    float* pml;          // [nh][n_chunks][2]  running maximum (base 2) and row sum of the chunk
};
void launch_decode_attention(const DecodeAttnArgs& a, hipStream_t st);
void launch_tree_masks(const int32_t* parent, int T, u32x4* anc, hipStream_t st);
void launch_attention(const AttnArgs& a, hipStream_t st);
void launch_zero_i32(int* p, int n, hipStream_t st);   // fill kernel (a memset node must not enter a captured graph)

// ---------------------------------------------------------------- accept / compact
struct TreeUploadArgs {
    int32_t token[CATS_MAX_TREE], parent[CATS_MAX_TREE], depth[CATS_MAX_TREE];
};
void launch_tree_upload(const TreeUploadArgs& a, int n, int32_t* token, int32_t* parent,
                        int32_t* depth, hipStream_t st);

void launch_accept(const int32_t* token, const int32_t* parent, const int32_t* depth,
                   const int32_t* amax, const uint8_t* edge_ok, int T, int ctx_len,
                   cats_accept_result* out, hipStream_t st);

struct TypicalArgs {
    const int32_t* token;
    const int32_t* parent;
    const float* part;      // LM-head partial tiles [pieces][T][ld]
    GemmPlan plan;
    NormScale ns;
    int T, ld;
    const float* lse;       // [T] log-sum-exp of logits / temperature
    const float* entropy;   // [T] entropy of softmax(logits / temperature)
    float inv_temp, epsilon, delta;
    uint8_t* edge_ok;       // [T]
    float* prob;            // [T] probability of the node's token under its parent
    float* thr;             // [T] threshold at its parent
};
void launch_typical_edges(const TypicalArgs& a, hipStream_t st);

struct CompactArgs {
    bf16_t* k[CATS_MAX_LAYERS];
    bf16_t* v[CATS_MAX_LAYERS];
    int n_layers;  // entries used
    int nh, d, max_ctx, ctx_len;
    const cats_accept_result* res;
};
void launch_compact(const CompactArgs& a, hipStream_t st);
