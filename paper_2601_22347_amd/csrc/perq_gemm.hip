// Reference consumer of the packed codes: out = (s_a c_a)(s_w c_w)^T for symmetric INT4 operands.
//
// With P and the block rotation merged into the weights (Remark "Merging Permutations",
// Section 4: W~ = R~^T P^T W), the product of the two quantized operands stands for X W.  This
// kernel is the plain integer product, 8 codes per v_dot8_i32_i4; it exists to show that the
// packed layout is directly consumable and to check the identity end to end, not to be fast.
#include "perq.h"

#include <hip/hip_runtime.h>

namespace perq {
namespace {

constexpr int kTileT = 64, kTileN = 64;       // outputs per workgroup; 4 x 4 per thread

__global__ void __launch_bounds__(256)
w4a4_gemm_kernel(const uint8_t* __restrict__ a_codes, const float* __restrict__ a_scales, int64_t T,
                 const uint8_t* __restrict__ w_codes, const float* __restrict__ w_scales, int32_t N, int32_t d,
                 float* __restrict__ out, int64_t ldo) {
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t t0 = (int64_t)blockIdx.y * kTileT + ty * 4;
    const int32_t n0 = (int32_t)blockIdx.x * kTileN + tx * 4;
    const int64_t row_bytes = d >> 1;
    const uint4* ap[4];
    const uint4* wp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // rows past the end re-read the last row; their results are not stored
        const int64_t t = t0 + i < T ? t0 + i : T - 1;
        const int32_t n = n0 + i < N ? n0 + i : N - 1;
        ap[i] = reinterpret_cast<const uint4*>(a_codes + t * row_bytes);
        wp[i] = reinterpret_cast<const uint4*>(w_codes + (int64_t)n * row_bytes);
    }
    int acc[4][4] = {};
    for (int k = 0; k < (d >> 5); ++k) {                  // 32 codes = 16 bytes per step
        uint4 a[4], w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = ap[i][k]; w[i] = wp[i][k]; }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int s = acc[i][j];
                s = __builtin_amdgcn_sdot8((int)a[i].x, (int)w[j].x, s, false);
                s = __builtin_amdgcn_sdot8((int)a[i].y, (int)w[j].y, s, false);
                s = __builtin_amdgcn_sdot8((int)a[i].z, (int)w[j].z, s, false);
                s = __builtin_amdgcn_sdot8((int)a[i].w, (int)w[j].w, s, false);
                acc[i][j] = s;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (t0 + i >= T) continue;
        const float sa = a_scales[t0 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (n0 + j < N) out[(t0 + i) * ldo + n0 + j] = (float)acc[i][j] * sa * w_scales[n0 + j];
        }
    }
}

}  // namespace
}  // namespace perq

extern "C" perq_status_t perq_w4a4_gemm_ref(const uint8_t* a_codes, const float* a_scales, int64_t T,
                                            const uint8_t* w_codes, const float* w_scales, int32_t N, int32_t d,
                                            float* out, int64_t ldo, void* hip_stream) {
    if (T < 0 || N < 0 || d <= 0 || d % 32 != 0 || ldo < N) return PERQ_ERR_INVALID_ARG;
    if (d > PERQ_MAX_D) return PERQ_ERR_UNSUPPORTED;
    if (T == 0 || N == 0) return PERQ_OK;
    if (!a_codes || !a_scales || !w_codes || !w_scales || !out) return PERQ_ERR_INVALID_ARG;
    if (((reinterpret_cast<uintptr_t>(a_codes) | reinterpret_cast<uintptr_t>(w_codes)) & 15u) != 0 ||
        ((reinterpret_cast<uintptr_t>(a_scales) | reinterpret_cast<uintptr_t>(w_scales) | reinterpret_cast<uintptr_t>(out)) & 3u) != 0)
        return PERQ_ERR_UNSUPPORTED;
    const int64_t gy = (T + perq::kTileT - 1) / perq::kTileT;
    if (gy > 65535) return PERQ_ERR_UNSUPPORTED;          // one launch, no splitting of T here
    const dim3 grid((unsigned)((N + perq::kTileN - 1) / perq::kTileN), (unsigned)gy);
    hipLaunchKernelGGL(perq::w4a4_gemm_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(hip_stream), a_codes, a_scales,
                       T, w_codes, w_scales, N, d, out, ldo);
    return hipGetLastError() == hipSuccess ? PERQ_OK : PERQ_ERR_LAUNCH;
}
