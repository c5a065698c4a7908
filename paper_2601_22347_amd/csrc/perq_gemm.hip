// Reference consumers of the packed codes: out = (s_a c_a)(s_w c_w)^T for symmetric INT4 operands,
// and the same product for MXFP4 operands on the scaled matrix instruction.
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

// ---- MXFP4 operands: the scaled matrix instruction of gfx950 consumes them as they are --------
// v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in the fp4 format: lane (i, h), i = lane & 31,
// h = lane >> 5, supplies 32 consecutive e2m1 codes (16 bytes, element 2k in the low nibble of byte
// k) of row i (A) or column i (B) for the contraction indices 32 h .. 32 h + 31, and one e8m0 byte
// that scales exactly those 32 -- a 32-group of the packed output and its scale byte, unchanged.
// One wave computes a 32 x 32 tile of the output, 64 contraction indices per instruction.
typedef int mx_v8i __attribute__((ext_vector_type(8)));
typedef float mx_v16f __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(64)
w4a4_mxfp4_gemm_kernel(const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales, int64_t T,
                       const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int32_t N, int32_t d,
                       float* __restrict__ out, int64_t ldo) {
    const int lane = threadIdx.x, i = lane & 31, h = lane >> 5;
    const int64_t t0 = (int64_t)blockIdx.y * 32;
    const int32_t n0 = (int32_t)blockIdx.x * 32;
    // rows and columns past the end re-read the last one; their results are not stored
    const int64_t t = t0 + i < T ? t0 + i : T - 1;
    const int64_t n = n0 + i < N ? n0 + i : N - 1;
    const uint8_t* ac = a_codes + t * (d >> 1);
    const uint8_t* wc = w_codes + n * (d >> 1);
    const uint8_t* as = a_scales + t * (d >> 5);
    const uint8_t* ws = w_scales + n * (d >> 5);
    mx_v16f acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (int k0 = 0; k0 < d; k0 += 64) {
        const int k = k0 + 32 * h;                       // this lane's 32-group
        uint4 a = make_uint4(0, 0, 0, 0), w = make_uint4(0, 0, 0, 0);
        int sa = 127, sw = 127;
        if (k < d) {                                     // (d need only be a multiple of 32)
            a = *reinterpret_cast<const uint4*>(ac + (k >> 1));
            w = *reinterpret_cast<const uint4*>(wc + (k >> 1));
            sa = as[k >> 5];
            sw = ws[k >> 5];
        }
        const mx_v8i va = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
        const mx_v8i vw = {(int)w.x, (int)w.y, (int)w.z, (int)w.w, 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vw, acc, 4 /* A: fp4 */, 4 /* B: fp4 */, 0, sa, 0, sw);
    }
    // accumulator j of lane (i, h): row 8 (j >> 2) + 4 h + (j & 3), column i
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int64_t row = t0 + 8 * (j >> 2) + 4 * h + (j & 3);
        if (row < T && n0 + i < N) out[row * ldo + n0 + i] = acc[j];
    }
}

}  // namespace
}  // namespace perq

extern "C" perq_status_t perq_w4a4_mxfp4_gemm_ref(const uint8_t* a_codes, const uint8_t* a_scales, int64_t T,
                                                  const uint8_t* w_codes, const uint8_t* w_scales, int32_t N,
                                                  int32_t d, float* out, int64_t ldo, void* hip_stream) {
    if (T < 0 || N < 0 || d <= 0 || d % 32 != 0 || ldo < N) return PERQ_ERR_INVALID_ARG;
    if (d > PERQ_MAX_D) return PERQ_ERR_UNSUPPORTED;
    if (T == 0 || N == 0) return PERQ_OK;
    if (!a_codes || !a_scales || !w_codes || !w_scales || !out) return PERQ_ERR_INVALID_ARG;
    if (((reinterpret_cast<uintptr_t>(a_codes) | reinterpret_cast<uintptr_t>(w_codes)) & 15u) != 0 ||
        (reinterpret_cast<uintptr_t>(out) & 3u) != 0)
        return PERQ_ERR_UNSUPPORTED;
    const int64_t gy = (T + 31) / 32;
    if (gy > 65535) return PERQ_ERR_UNSUPPORTED;          // one launch, no splitting of T here
    const dim3 grid((unsigned)((N + 31) / 32), (unsigned)gy);
    hipLaunchKernelGGL(perq::w4a4_mxfp4_gemm_kernel, grid, dim3(64), 0, static_cast<hipStream_t>(hip_stream), a_codes,
                       a_scales, T, w_codes, w_scales, N, d, out, ldo);
    return hipGetLastError() == hipSuccess ? PERQ_OK : PERQ_ERR_LAUNCH;
}

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
