// Skinny bf16 GEMM on MFMA: the weight stream of the verification pass
// (paper Sec. 3.2, "Target verification pass": the layer weights are brought in
// once and applied to every tree token in a single batched forward).
//
// Y[t][n] = sum_k X[t][k] W[n][k], T <= 128 rows, N and K large.  Every weight
// element is loaded from HBM exactly once, straight into the MFMA B-operand
// registers by 128-bit loads; the T activations of the current K chunk (a high and a
// low bf16 part each, see GemmArgs) are staged in LDS and shared by all waves.  Each wave owns 32
// weight rows.  The kernel is bound by HBM latency x bandwidth, so each wave keeps
// a ring of ST-1 future K chunks (8 KB of weights each) in flight in registers.
// Work is balanced over the CUs: the (row tile, K chunk) items, in tile-major order,
// are cut into one equal contiguous range per workgroup; a workgroup streams through
// its range without a break (the ring keeps prefetching across tile boundaries) and
// writes one float32 partial tile ("piece") for every tile it touches.  The following
// epilogue kernel adds a tile's pieces in a fixed order.
#include <hip/hip_ext.h>

#include <algorithm>

#include "common.hpp"

namespace {


// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait
// for every outstanding global load (vmcnt(0)), i.e. drain the prefetch ring.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// MFMA 32x32x16 bf16 operand layout (wave64): lane l supplies, for A, row l%32
// and k = 8*(l/32)..+7; for B, column l%32 and the same k; the 16 results of a
// lane are D[8*(r/4) + 4*(l/32) + r%4][l%32].
//
// TB: 32-row blocks of X one wave accumulates (T <= 32 * TB).  NWR: waves along the weight
// rows (a tile has 32 * NWR rows).  KG: groups of such waves along k: an item then spans KG
// chunks of 128 k-values, group kg multiplies chunk kg of it for the same weight rows, and the
// groups' sums are added through LDS when a tile (or the workgroup's range) ends, so that a
// partial tile is 32 * NWR rows high whatever the number of waves.  ST: ring depth.  PACKED:
// weights come in the packed fragment order (contiguous 1 KB per wave load).
// TS: workgroups per range of work items.  With TS = 2 the launch has two workgroups per range,
// on the same XCD (workgroup b of a launch runs on XCD b % 8, so the pair is b and b + 8): both
// stream the range's weights, one for the first 32 * TB rows of X and one for the rows behind them.
// The pair's loads of a weight line meet in the XCD's L2 (the line leaves memory once), and a
// range is twice as long as with one workgroup each, i.e. half as many partial tiles.  Used for
// more than 96 rows, where one workgroup per range would need four accumulator blocks per wave
// (248 registers, 139 KB of staged X): measured at 128 rows 35.7 against 38.7 us per launch
// (6.24 against 6.84 ms per 7B step); at 80 and 96 rows the pairs are 3 % slower than three
// accumulator blocks, at 63 rows 7 % slower than two.
template <int TB, int NWR, int KG, int ST, bool PACKED, int TS = 1>
__global__ __launch_bounds__(64 * NWR * KG) void cats_gemm_skinny_bf16(GemmArgs a) {
    constexpr int THREADS = 64 * NWR * KG;
    constexpr int BN = 32 * NWR;
    constexpr int KC = GEMM_KC * KG;               // k elements per item
    constexpr int XCOLS = KC / 8;                  // 16-byte columns of a staged row
    constexpr int XS_ROW = XCOLS + 1;              // u32x4 per staged row: data + 16 B pad
    constexpr int XPT = TB * 32 * XCOLS / THREADS;      // u32x4 of the X tile per thread
    constexpr int XROWS_PER_PASS = THREADS / XCOLS;     // tile rows covered by one pass of the block
    constexpr int NBUF = (ST % 2 == 0) ? 2 : ST;  // LDS buffers; the index is static under unrolling
    static_assert(ST >= 2 && ST <= 3, "ring depth");
    __shared__ u32x4 xs[NBUF][2][TB * 32][XS_ROW];  // [.][0] high parts, [.][1] low parts

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = (tid >> 6) % NWR, kg = (tid >> 6) / NWR;
    const int col = lane & 31, g = lane >> 5;
    // pairs: with a multiple of eight ranges, blocks b and b + 8 of every group of 16 share a range
    // (same XCD); otherwise (small products) neighbouring blocks do
    const int pg = (TS > 1 && (a.plan.n_wgs & 7) == 0) ? 8 : 1;
    const int wg = TS == 1 ? static_cast<int>(blockIdx.x)
                           : static_cast<int>(blockIdx.x / (2 * pg) * pg + blockIdx.x % pg);
    const int t_base = TS == 1 ? 0 : static_cast<int>(blockIdx.x / pg % 2) * 32 * TB;   // first row of X of this workgroup
    const int T_loc = min(a.T - t_base, 32 * TB);                                           // its rows
    if (TS > 1 && T_loc <= 0) return;   // (whole workgroup; does not happen with the plans make_gemm_plan hands out)
    const int C = a.plan.chunks;
    const int C128 = (a.K + GEMM_KC - 1) / GEMM_KC;
    (void)C128;
    const int item_lo = plan_item_begin(a.plan, wg);
    const int n_items = plan_item_begin(a.plan, wg + 1) - item_lo;

    // staging assignment: thread -> (row, 16-byte column) of the X tile
    const int xr = tid / XCOLS, xc = tid % XCOLS;

    u32x4 wst[ST][8];
    u32x4 xst[2 * XPT];  // X of the next item only: it comes from L2, one step ahead is enough
    const u32x4 zero4 = u32x4{0u, 0u, 0u, 0u};

    // Loads are unconditional (clamped addresses) so that the pipeline is straight-line code:
    // a predicated load would put every load in its own basic block and the compiler would
    // then wait for ALL outstanding loads at each use.  Out-of-range X entries are zeroed by
    // a select at use; the matching W values are finite and get multiplied by those zeros.
    // The scheduling barriers keep the chunks' loads in issue order.
    bool x_row_ok[XPT];
    size_t x_off[XPT];
#pragma unroll
    for (int p = 0; p < XPT; ++p) {
        const int r = xr + XROWS_PER_PASS * p;
        x_row_ok[p] = r < T_loc;
        x_off[p] = static_cast<size_t>(t_base + min(r, T_loc - 1)) * a.K;
    }
    const int k_last_x = a.K - 8, k_last_w = a.K - 16;
    const int rb_per_seg = a.seg_pad / PACK_ROWS, n_rb_total = a.n_seg * rb_per_seg;  // packed only
    (void)rb_per_seg;
    (void)n_rb_total;
    (void)k_last_w;

    // item (local index i) -> tile and first k of its chunk
#define CATS_ITEM(i, tile_, k0_)                  \
    const int gi_ = item_lo + (i);                \
    const int tile_ = static_cast<int>(static_cast<unsigned>(gi_) / static_cast<unsigned>(C)); \
    const int k0_ = (gi_ - tile_ * C) * KC;

#define CATS_LOAD_X(i)                                                                              \
    {                                                                                               \
        CATS_ITEM(i, xt_, xk_)                                                                      \
        (void)xt_;                                                                                  \
        const int kx = xk_ + 8 * xc;                                                                \
        _Pragma("unroll") for (int p = 0; p < XPT; ++p) {                                           \
            const size_t xo_ = x_off[p] + min(kx, k_last_x);                                        \
            xst[2 * p] = *reinterpret_cast<const u32x4*>(a.x + xo_);                                \
            xst[2 * p + 1] = *reinterpret_cast<const u32x4*>(a.x_lo + xo_);                         \
        }                                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                          \
    }
    // (Weight fragments are read once per launch: non-temporal loads keep them from displacing
    // the X rows and partial tiles that are re-read from the caches; measured -3 % per launch.)
    // Weight address of this lane for item i.  Row-major: row v of the product, 8 k-values
    // from column 16 j + 8 g of the chunk (clamped inside the row).  Packed: the wave's 32-row
    // block is one contiguous run of 1 KB fragments, 8 per chunk, lane l owning bytes 16 l.
#define CATS_LOAD_W(slot, i)                                                                        \
    {                                                                                               \
        CATS_ITEM(i, lt_, lk_)                                                                      \
        const bf16_t* lw_;                                                                          \
        if (PACKED) {                                                                               \
            const int lrb_ = min((lt_ * BN + wave * 32) / PACK_ROWS, n_rb_total - 1);               \
            const int lseg_ = lrb_ / rb_per_seg;                                                    \
            lw_ = (lseg_ == 0 ? a.w[0] : (lseg_ == 1 ? a.w[1] : a.w[2])) +                          \
                  (static_cast<size_t>(lrb_ - lseg_ * rb_per_seg) * C128 + min(lk_ / GEMM_KC + kg, C128 - 1)) * \
                      (8 * PACK_FRAG) + lane * 8;                                                   \
        } else {                                                                                    \
            const int lv_ = min(lt_ * BN + wave * 32 + col, a.N - 1);                               \
            const int lseg_ = lv_ / a.seg_pad;                                                      \
            lw_ = (lseg_ == 0 ? a.w[0] : (lseg_ == 1 ? a.w[1] : a.w[2])) +                          \
                  static_cast<size_t>(min(lv_ - lseg_ * a.seg_pad, a.seg_rows - 1)) * a.K + 8 * g;  \
        }                                                                                           \
        _Pragma("unroll") for (int j = 0; j < 8; ++j)                                               \
            wst[slot][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(               \
                PACKED ? lw_ + j * PACK_FRAG : lw_ + min(lk_ + GEMM_KC * kg + 16 * j, k_last_w)));  \
        __builtin_amdgcn_sched_barrier(0);                                                          \
    }

    f32x16 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tb][r] = 0.f;

    // One pipeline step: stage X of item i in LDS, fetch X of item i+1, optionally refill the
    // W ring slot freed by the previous step with item i+ST-1, multiply W (ring slot s), and hand the partial tile over
    // when the tile (or this workgroup's range) ends.
#define CATS_STEP(s, i, REFILL)                                                                     \
    {                                                                                               \
        constexpr int buf = (s) % NBUF;                                                             \
        CATS_ITEM(i, tile, k0)                                                                      \
        _Pragma("unroll") for (int p = 0; p < XPT; ++p) { /* zero what lies outside the tile */     \
            const bool ok_ = x_row_ok[p] && k0 + 8 * xc < a.K;                                      \
            xs[buf][0][xr + XROWS_PER_PASS * p][xc] = ok_ ? xst[2 * p] : zero4;                     \
            xs[buf][1][xr + XROWS_PER_PASS * p][xc] = ok_ ? xst[2 * p + 1] : zero4;                 \
        }                                                                                           \
        lds_barrier();                                                                              \
        CATS_LOAD_X(min((i) + 1, n_items - 1))                                                      \
        if (REFILL) CATS_LOAD_W(((s) + ST - 1) % ST, min((i) + ST - 1, n_items - 1))                \
        _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                             \
            const bf16x8 b = as_bf16x8(wst[s][j]);                                                  \
            _Pragma("unroll") for (int tb = 0; tb < TB; ++tb) {                                     \
                const bf16x8 ah = as_bf16x8(xs[buf][0][tb * 32 + col][16 * kg + 2 * j + g]); \
                const bf16x8 al = as_bf16x8(xs[buf][1][tb * 32 + col][16 * kg + 2 * j + g]); \
                acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b, acc[tb], 0, 0, 0);         \
                acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b, acc[tb], 0, 0, 0);         \
            }                                                                                       \
        }                                                                                           \
        if (k0 + KC >= a.K || (i) == n_items - 1) {                                                 \
            if (KG > 1) { /* add the k groups: the other LDS buffer is idle at this point */        \
                float* red = reinterpret_cast<float*>(&xs[(buf + 1) % NBUF][0][0][0]);              \
                if (kg > 0) {                                                                       \
                    _Pragma("unroll") for (int tb = 0; tb < TB; ++tb)                               \
                        _Pragma("unroll") for (int r = 0; r < 16; ++r)                              \
                            red[((wave * TB + tb) * 16 + r) * 64 + lane] = acc[tb][r];              \
                }                                                                                   \
                lds_barrier();                                                                      \
                if (kg == 0) {                                                                      \
                    _Pragma("unroll") for (int tb = 0; tb < TB; ++tb)                               \
                        _Pragma("unroll") for (int r = 0; r < 16; ++r)                              \
                            acc[tb][r] += red[((wave * TB + tb) * 16 + r) * 64 + lane];             \
                }                                                                                   \
                lds_barrier(); /* the buffer is staged again in the next step */                   \
            }                                                                                       \
            const int n = tile * BN + wave * 32 + col;                                              \
            if (kg == 0 && n < a.N && n % a.seg_pad < a.seg_rows) {                                 \
                const int piece = wg - plan_first_wg(a.plan, tile);                                 \
                /* The row offsets below are loop-invariant; computed ahead of the loop they     */ \
                /* would occupy two registers per store for the whole kernel.  Passing the lane  */ \
                /* term through an empty asm ties them to this block.                            */ \
                int g_here = g;                                                                     \
                asm volatile("" : "+v"(g_here));                                                    \
                float* out = a.part + (static_cast<size_t>(piece) * a.T + t_base) * a.N + n;        \
                _Pragma("unroll") for (int tb = 0; tb < TB; ++tb)                                   \
                    _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                \
                    const int t = tb * 32 + 8 * (r >> 2) + 4 * g_here + (r & 3);            \
                    /* write-through store: the partial tile goes on to memory at once instead   */ \
                    /* of waiting, dirty, in the XCD's L2 for the write-back at the kernel's end */ \
                    if (t < T_loc)                                                                  \
                        __hip_atomic_store(out + static_cast<size_t>(t) * a.N, acc[tb][r], __ATOMIC_RELAXED, \
                                           __HIP_MEMORY_SCOPE_AGENT);                               \
                }                                                                                   \
            }                                                                                       \
            _Pragma("unroll") for (int tb = 0; tb < TB; ++tb)                                       \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[tb][r] = 0.f;                    \
        }                                                                                           \
    }

    // prologue: items 0 .. ST-2 in flight (indices past the range are clamped: harmless reloads)
    CATS_LOAD_X(0)
#pragma unroll
    for (int s = 0; s < ST - 1; ++s) CATS_LOAD_W(s, min(s, n_items - 1))

    // Full groups of ST items whose refills all lie inside the range run without any
    // condition: a conditional step inside the loop would give the compiler a (never taken)
    // path on which ring loads stay unconsumed, and it would drain all loads at the loop head.
    int c0 = 0;
    for (; c0 + 2 * ST - 1 <= n_items; c0 += ST) {
        CATS_STEP(0, c0, true)
        CATS_STEP(1, c0 + 1, true)
        if constexpr (ST > 2) CATS_STEP(2, c0 + 2, true)
    }
    // tail: at most 2*ST-2 items left; item c0+j sits in ring slot j % ST and is refilled
    // from only while the refill index stays inside the range
#define CATS_TAIL(j)                                                 \
    if (c0 + (j) + ST - 1 < n_items) {                               \
        CATS_STEP((j) % ST, c0 + (j), true)                          \
    } else {                                                         \
        CATS_STEP((j) % ST, c0 + (j), false)                         \
    }
    if (c0 < n_items) {
        CATS_TAIL(0)
        if (c0 + 1 < n_items) {
            CATS_TAIL(1)
            if constexpr (ST > 2) {
                if (c0 + 2 < n_items) {
                    CATS_TAIL(2)
                    if (c0 + 3 < n_items) {
                        CATS_TAIL(3)
                    }
                }
            }
        }
    }
#undef CATS_TAIL
#undef CATS_STEP
#undef CATS_LOAD_X
#undef CATS_LOAD_W
#undef CATS_ITEM
}

// One thread per 16 bytes of the packed matrix: fragment f = (rb * C + c) * 8 + j, lane l.
__global__ void cats_pack_matrix_kernel(const bf16_t* src, bf16_t* dst, int rows, int cols, int C, size_t n_vec) {
    const size_t idx = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n_vec) return;
    const int l = static_cast<int>(idx & 63);
    const size_t f = idx >> 6;
    const int j = static_cast<int>(f & 7);
    const size_t rc = f >> 3;
    const int c = static_cast<int>(rc % C);
    const int rb = static_cast<int>(rc / C);
    const int row = rb * PACK_ROWS + (l & 31);
    const int k = c * GEMM_KC + 16 * j + 8 * (l >> 5);
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (row < rows && k < cols) v = *reinterpret_cast<const u32x4*>(src + static_cast<size_t>(row) * cols + k);
    reinterpret_cast<u32x4*>(dst)[idx] = v;
}

}  // namespace

size_t packed_matrix_elems(int rows, int cols) {
    const size_t rb = (rows + PACK_ROWS - 1) / PACK_ROWS, C = (cols + GEMM_KC - 1) / GEMM_KC;
    return rb * C * 8 * PACK_FRAG;
}

void launch_pack_matrix(const bf16_t* src, bf16_t* dst, int rows, int cols, hipStream_t st) {
    const size_t n_vec = packed_matrix_elems(rows, cols) / 8;
    const int C = (cols + GEMM_KC - 1) / GEMM_KC;
    hipLaunchKernelGGL(cats_pack_matrix_kernel, dim3(static_cast<unsigned>((n_vec + 255) / 256)), dim3(256), 0, st,
                       src, dst, rows, cols, C, n_vec);
}

// Tile shape and workgroups per range by the number of rows of X.
// Up to 32 rows, two groups of four waves share a 128-row tile, each multiplying one 128-wide half
// of a 256-wide item, and add their sums through LDS when the tile ends: the same bytes in flight
// as with eight waves on 256 rows, but half the bytes of partial sums to write here and to read
// back in the consumer, paid for with twice the X bytes staged per weight byte.  Measured on one
// device (7B shapes, per step): T = 1 -2.7 %, T = 8 -3.7 %, T = 16 / 24 -4.3 %, T = 32 -5.2 %; with
// two accumulator blocks per wave (T = 48, 63) the staging costs more than the partial sums save
// (+0.7 %).  Larger trees run on 256-row tiles, one 32-row accumulator block per wave for every 32
// rows of T up to 96 (256-row tiles halve the re-reads of X, 128-row tiles halve the number of
// partial tiles; at T = 63, 128 rows for every product 5.10 ms per step against 5.09 ms), and beyond
// 96 rows as pairs of workgroups with two blocks each (see TS at the kernel).
static int plan_kc(int rows) { return rows <= 32 ? 2 * GEMM_KC : GEMM_KC; }
static int plan_bn(int rows) { return rows <= 32 ? 128 : 256; }
static int plan_ts(int rows) { return rows > 96 ? 2 : 1; }

// The work items are cut into n equal contiguous ranges, one per workgroup (or pair), and the
// launch lasts as long as the longest range: ceil(items / n) item times.  The product is bound by
// memory bandwidth, so what counts is how much of n * ceil(items / n) is real work, not how many
// compute units are busy (measured: 224 instead of 256 busy units cost 2 %).  n is therefore
// the count in [3/4 target, target] with the fewest item slots, idle units priced in.  7B down
// projection: 1376 items, 256 workgroups would run 6 items each with 10 % of the slots empty;
// 230 workgroups run 5.98.  With pairs, target is half the workgroups and n a multiple of eight
// (the kernel then finds a pair's range from the block index in groups of 16, one pair per XCD).
GemmPlan make_gemm_plan(int N, int K, int target_wgs, int rows) {
    GemmPlan p;
    p.bn = plan_bn(rows);
    p.kc = plan_kc(rows);
    p.ts = 1;
    p.chunks = (K + p.kc - 1) / p.kc;
    const int tiles = (N + p.bn - 1) / p.bn;
    p.items = tiles * p.chunks;
    // the device-side plan arithmetic is 32-bit: items * workgroups stays far below 2^31 for every
    // supported shape (at most 128 Ki rows x 8 Ki columns per product)
    if (static_cast<long long>(p.items) * target_wgs >= (1ll << 31)) target_wgs = static_cast<int>((1ll << 31) / p.items) - 1;
    const int ts = plan_ts(rows);
    p.ts = ts;
    const int step = (ts > 1 && target_wgs / ts >= 8) ? 8 : 1;
    const int target = std::max(1, target_wgs / ts / step * step);
    if (target >= p.items) {
        p.n_wgs = p.items;
        return p;
    }
    // cost = item slots, weighted by the measured price of idle compute units (0.07 % each)
    auto cost = [&](int n) {
        return static_cast<double>((p.items + n - 1) / n) * n * (1.0 + 0.0007 * ts * (target - n));
    };
    int best = target;
    double best_cost = cost(target);
    for (int n = target - step; n >= target - target / 4 && n >= step; n -= step) {
        const double c = cost(n);
        if (c < best_cost) {
            best_cost = c;
            best = n;
        }
    }
    p.n_wgs = best;
    return p;
}

int gemm_plan_max_pieces(const GemmPlan& p) {
    const int tiles = p.items / p.chunks;
    int m = 1;
    for (int t = 0; t < tiles; ++t) {
        const int k = plan_pieces(p, t);
        m = k > m ? k : m;
    }
    return m;
}

// With events given, they are attached to the dispatch itself (kernel begin / end
// timestamps), so the elapsed time is the kernel's execution time without launch latency.
void launch_gemm(const GemmArgs& a, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
    // one 32-row block of X per 32 rows of T; 8 waves: on 256-row tiles, or as two k groups on
    // 128-row tiles (the plan says which); 4 waves on 128-row tiles are kept for experiments
    const int tb = (a.T + 32 * a.plan.ts - 1) / (32 * a.plan.ts);
    const int nwr = a.plan.bn / 32, kgs = a.plan.kc / GEMM_KC;
    const dim3 grid(a.plan.n_wgs * a.plan.ts), block(64 * nwr * kgs);
#define CATS_LAUNCH_V(TBV, NWRV, KGV)                                                                   \
    if (a.packed)                                                                                       \
        hipExtLaunchKernelGGL((cats_gemm_skinny_bf16<TBV, NWRV, KGV, GEMM_ST, true>), grid, block, 0, st,    \
                              ev_start, ev_stop, 0, a);                                                 \
    else                                                                                                \
        hipExtLaunchKernelGGL((cats_gemm_skinny_bf16<TBV, NWRV, KGV, GEMM_ST, false>), grid, block, 0, st,   \
                              ev_start, ev_stop, 0, a)
#define CATS_LAUNCH_TS(TBV)                                                                             \
    if (a.packed)                                                                                       \
        hipExtLaunchKernelGGL((cats_gemm_skinny_bf16<TBV, 8, 1, GEMM_ST, true, 2>), grid, block, 0, st,      \
                              ev_start, ev_stop, 0, a);                                                 \
    else                                                                                                \
        hipExtLaunchKernelGGL((cats_gemm_skinny_bf16<TBV, 8, 1, GEMM_ST, false, 2>), grid, block, 0, st,     \
                              ev_start, ev_stop, 0, a)
    if (a.plan.ts == 2) {   // make_gemm_plan grants it beyond 96 rows: two blocks of X per workgroup
        CATS_LAUNCH_TS(2);
    } else if (nwr == 4 && kgs == 2) {
        if (tb == 1) {
            CATS_LAUNCH_V(1, 4, 2);
        } else {
            CATS_LAUNCH_V(2, 4, 2);
        }
    } else if (nwr == 4) {
        if (tb == 1) {
            CATS_LAUNCH_V(1, 4, 1);
        } else {
            CATS_LAUNCH_V(2, 4, 1);
        }
    } else {
        if (tb == 1) {
            CATS_LAUNCH_V(1, 8, 1);
        } else if (tb == 2) {
            CATS_LAUNCH_V(2, 8, 1);
        } else {   // up to 96 rows (beyond that the plan asks for pairs)
            CATS_LAUNCH_V(3, 8, 1);
        }
    }
#undef CATS_LAUNCH_V
#undef CATS_LAUNCH_TS
}
