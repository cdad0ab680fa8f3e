// Skinny bf16 GEMM on MFMA: the weight stream of the verification pass
// (paper Sec. 3.2, "Target verification pass": the layer weights are brought in
// once and applied to every tree token in a single batched forward).
//
// Y[t][n] = sum_k X[t][k] W[n][k], T <= 128 rows, N and K large.  Every weight
// element is loaded from HBM exactly once, straight into the MFMA B-operand
// registers by 128-bit loads; the T activations of the current K chunk are
// staged in LDS and reused by the four waves of the workgroup.  Each wave owns
// 32 weight rows, the workgroup 128; the K range is cut into `splits` slices
// (grid.y) so that enough workgroups exist to fill 256 CUs, and the float32
// partial sums go to part[split][t][n] for the following epilogue kernel to
// add up in a fixed order.
#include "common.hpp"

namespace {

constexpr int XS_ROW = GEMM_KC / 8 + 1;  // u32x4 per staged row: 256 B of data + 16 B pad

// MFMA 32x32x16 bf16 operand layout (wave64): lane l supplies, for A, row l%32
// and k = 8*(l/32)..+7; for B, column l%32 and the same k; the 16 results of a
// lane are D[8*(r/4) + 4*(l/32) + r%4][l%32].
template <int TB>
__global__ __launch_bounds__(256) void cats_gemm_skinny_bf16(GemmArgs a) {
    __shared__ u32x4 xs[2][TB * 32][XS_ROW];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;

    const int n = blockIdx.x * GEMM_BN + wave * 32 + col;
    const bool n_ok = n < a.N;
    const int nn = n_ok ? n : a.N - 1;
    const int seg = nn / a.seg_rows;
    const bf16_t* wseg = seg == 0 ? a.w[0] : (seg == 1 ? a.w[1] : a.w[2]);
    const bf16_t* wrow = wseg + static_cast<size_t>(nn - seg * a.seg_rows) * a.K;

    const int k_begin = blockIdx.y * a.k_per_split;
    const int k_end = min(a.K, k_begin + a.k_per_split);
    const int n_chunks = (k_end - k_begin + GEMM_KC - 1) / GEMM_KC;

    // staging assignment: thread -> (row, 16-byte column) of the X tile
    const int xr = tid >> 4, xc = tid & 15;

    u32x4 wreg[8];
    u32x4 xreg[TB * 2];
    const u32x4 zero4 = u32x4{0u, 0u, 0u, 0u};

#define CATS_LOAD_W(k0)                                                                     \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                         \
        const int kk = (k0) + 16 * j + 8 * g;                                               \
        wreg[j] = kk < k_end ? *reinterpret_cast<const u32x4*>(wrow + kk) : zero4;          \
    }
#define CATS_LOAD_X(k0)                                                                     \
    _Pragma("unroll") for (int p = 0; p < TB * 2; ++p) {                                    \
        const int r = xr + 16 * p;                                                          \
        const int kk = (k0) + 8 * xc;                                                       \
        xreg[p] = (r < a.T && kk < k_end)                                                   \
                      ? *reinterpret_cast<const u32x4*>(a.x + static_cast<size_t>(r) * a.K + kk) \
                      : zero4;                                                              \
    }

    f32x16 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tb][r] = 0.f;

    if (n_chunks > 0) {
        CATS_LOAD_W(k_begin)
        CATS_LOAD_X(k_begin)
    }
    int buf = 0;
    for (int c = 0; c < n_chunks; ++c) {
#pragma unroll
        for (int p = 0; p < TB * 2; ++p) xs[buf][xr + 16 * p][xc] = xreg[p];
        __syncthreads();
        u32x4 wcur[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) wcur[j] = wreg[j];
        if (c + 1 < n_chunks) {
            const int k0 = k_begin + (c + 1) * GEMM_KC;
            CATS_LOAD_W(k0)
            CATS_LOAD_X(k0)
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bf16x8 b = as_bf16x8(wcur[j]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const bf16x8 av = as_bf16x8(xs[buf][tb * 32 + col][2 * j + g]);
                acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, b, acc[tb], 0, 0, 0);
            }
        }
        buf ^= 1;
    }

    if (n_ok) {
        float* out = a.part + static_cast<size_t>(blockIdx.y) * a.T * a.N + n;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int t = tb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (t < a.T) out[static_cast<size_t>(t) * a.N] = acc[tb][r];
            }
    }
}

}  // namespace

void launch_gemm(const GemmArgs& a, int splits, hipStream_t st) {
    dim3 grid((a.N + GEMM_BN - 1) / GEMM_BN, splits);
    const int tb = (a.T + 31) / 32;
    switch (tb) {
        case 1: hipLaunchKernelGGL(cats_gemm_skinny_bf16<1>, grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL(cats_gemm_skinny_bf16<2>, grid, dim3(256), 0, st, a); break;
        case 3: hipLaunchKernelGGL(cats_gemm_skinny_bf16<3>, grid, dim3(256), 0, st, a); break;
        default: hipLaunchKernelGGL(cats_gemm_skinny_bf16<4>, grid, dim3(256), 0, st, a); break;
    }
}
