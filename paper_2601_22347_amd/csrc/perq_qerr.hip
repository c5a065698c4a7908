// Per-token quantization error of the fused path's output (Section 3: the worst-case l2 error of a
// q-bit quantizer is sqrt(d) / (2^q - 2) times the row's largest magnitude, which is why suppressing
// outliers pays): from the pre-quantization values y (perq_permute_rotate_f32) and the codes and
// scales perq_permute_rotate_quant wrote for the same input,
//     out[t] = ( ||y_t - Q(y_t)||_2,  ||y_t||_2,  ||y_t||_inf )
// with Q(y) the value the codes stand for.  One workgroup per token; every thread adds its elements
// in index order and the 256 partial sums are added in a fixed tree, so the result does not depend on
// scheduling.  Sums are fp32.
#include "perq.h"
#include "perq_launch.h"

namespace perq {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float e2m1_value(uint32_t nib) {
    // sign | 2 exponent bits (bias 1) | 1 mantissa bit; exponent 0 is the subnormal 0 / 0.5
    const uint32_t e = (nib >> 1) & 3u, m = nib & 1u;
    const float mag = e == 0 ? 0.5f * (float)m : (1.0f + 0.5f * (float)m) * (float)(1u << (e - 1u));
    return (nib & 8u) ? -mag : mag;
}

template <int FMT>
__global__ void __launch_bounds__(kThreads)
quant_error_kernel(const float* __restrict__ y, int64_t T, int32_t d, const uint8_t* __restrict__ codes,
                   const void* __restrict__ scales, float* __restrict__ out) {
    __shared__ float red[3][kThreads];
    const int64_t row = blockIdx.x;
    const float* yr = y + row * (int64_t)d;
    const uint8_t* cr = codes + row * (int64_t)(d >> 1);
    float step = 0.0f, zero = 0.0f;
    if constexpr (FMT == PERQ_FMT_INT4_SYM_TOKEN || FMT == PERQ_FMT_FP4_TOKEN) step = static_cast<const float*>(scales)[row];
    if constexpr (FMT == PERQ_FMT_INT4_ASYM_TOKEN) {
        step = static_cast<const float*>(scales)[2 * row];
        zero = static_cast<const float*>(scales)[2 * row + 1];
    }
    float err = 0.0f, nrm = 0.0f, amax = 0.0f;
    // a thread takes byte k = two adjacent elements; consecutive threads take consecutive bytes
    for (int k = threadIdx.x; k < (d >> 1); k += kThreads) {
        const uint32_t byte = cr[k];
        const float2 v = *reinterpret_cast<const float2*>(yr + 2 * k);
        float q0, q1;
        const uint32_t n0 = byte & 15u, n1 = byte >> 4;
        if constexpr (FMT == PERQ_FMT_INT4_SYM_TOKEN) {
            q0 = step * (float)((int)(n0 ^ 8u) - 8);          // two's complement nibble
            q1 = step * (float)((int)(n1 ^ 8u) - 8);
        } else if constexpr (FMT == PERQ_FMT_INT4_ASYM_TOKEN) {
            q0 = step * ((float)n0 + zero);
            q1 = step * ((float)n1 + zero);
        } else if constexpr (FMT == PERQ_FMT_FP4_TOKEN) {
            q0 = step * e2m1_value(n0);
            q1 = step * e2m1_value(n1);
        } else {
            const uint32_t E = static_cast<const uint8_t*>(scales)[row * (int64_t)(d >> 5) + (k >> 4)];
            const float s = __uint_as_float(E << 23);         // 2^(E - 127); E = 0 stands for 2^-127
            const float s0 = E == 0 ? 0x1p-127f : s;
            q0 = s0 * e2m1_value(n0);
            q1 = s0 * e2m1_value(n1);
        }
        const float e0 = v.x - q0, e1 = v.y - q1;
        err = __builtin_fmaf(e0, e0, err);
        err = __builtin_fmaf(e1, e1, err);
        nrm = __builtin_fmaf(v.x, v.x, nrm);
        nrm = __builtin_fmaf(v.y, v.y, nrm);
        amax = fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y)));
    }
    red[0][threadIdx.x] = err;
    red[1][threadIdx.x] = nrm;
    red[2][threadIdx.x] = amax;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            red[0][threadIdx.x] += red[0][threadIdx.x + w];
            red[1][threadIdx.x] += red[1][threadIdx.x + w];
            red[2][threadIdx.x] = fmaxf(red[2][threadIdx.x], red[2][threadIdx.x + w]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out[3 * row] = sqrtf(red[0][0]);
        out[3 * row + 1] = sqrtf(red[1][0]);
        out[3 * row + 2] = red[2][0];
    }
}

}  // namespace
}  // namespace perq

extern "C" perq_status_t perq_quant_error(const float* y, int64_t T, int32_t d, const uint8_t* codes,
                                          const void* scales, perq_fmt_t fmt, float* out, void* hip_stream) {
    if (T < 0 || d <= 0 || d % 32 != 0) return PERQ_ERR_INVALID_ARG;
    if (fmt != PERQ_FMT_INT4_SYM_TOKEN && fmt != PERQ_FMT_MXFP4 && fmt != PERQ_FMT_INT4_ASYM_TOKEN &&
        fmt != PERQ_FMT_FP4_TOKEN && fmt != PERQ_FMT_FP4_TOKEN_AMAX7)
        return PERQ_ERR_INVALID_ARG;
    if (T == 0) return PERQ_OK;
    if (y == nullptr || codes == nullptr || scales == nullptr || out == nullptr) return PERQ_ERR_INVALID_ARG;
    if (T >= ((int64_t)1 << 31)) return PERQ_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(y) & 7u) != 0 || (reinterpret_cast<uintptr_t>(out) & 3u) != 0 ||
        (reinterpret_cast<uintptr_t>(scales) & (fmt == PERQ_FMT_MXFP4 ? 0u : 3u)) != 0)
        return PERQ_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const dim3 grid((unsigned)T), block(perq::kThreads);
    switch (fmt) {
        case PERQ_FMT_INT4_SYM_TOKEN:
            hipLaunchKernelGGL(perq::quant_error_kernel<PERQ_FMT_INT4_SYM_TOKEN>, grid, block, 0, stream, y, T, d, codes, scales, out);
            break;
        case PERQ_FMT_MXFP4:
            hipLaunchKernelGGL(perq::quant_error_kernel<PERQ_FMT_MXFP4>, grid, block, 0, stream, y, T, d, codes, scales, out);
            break;
        case PERQ_FMT_INT4_ASYM_TOKEN:
            hipLaunchKernelGGL(perq::quant_error_kernel<PERQ_FMT_INT4_ASYM_TOKEN>, grid, block, 0, stream, y, T, d, codes, scales, out);
            break;
        default:
            hipLaunchKernelGGL(perq::quant_error_kernel<PERQ_FMT_FP4_TOKEN>, grid, block, 0, stream, y, T, d, codes, scales, out);
            break;
    }
    return hipGetLastError() == hipSuccess ? PERQ_OK : PERQ_ERR_LAUNCH;
}
