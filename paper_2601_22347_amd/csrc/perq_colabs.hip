// a_i = (1/M) sum_k |x[k,i]|  -- the sort key of Algorithm 1 -- as two deterministic passes; the
// same two passes with max in place of + give max_k |x[k,i]|, the statistic of the "absmax" and
// ZigZag permutations of the ablation (Appendix C).
//
// Pass 1: the M rows are cut into S slices; workgroup (column tile, slice) adds |x| over its
// rows, each lane owning 8 adjacent columns (one 16-byte bf16 load per row), and writes fp32
// partial sums part[slice][column].  Pass 2: one lane per column adds the S partials in slice
// order (in double) and divides by M.  No atomics: the result is independent of scheduling.
// Rounding: at most rows_per_slice - 1 fp32 additions of non-negative terms per partial, so the
// relative error of a_i is below (rows_per_slice + 1) * 2^-24.
#include "perq.h"
#include "perq_launch.h"

#include <mutex>

namespace perq {
namespace {

constexpr int kColsPerLane = 8;
constexpr int kThreads = 256;
constexpr int kTileCols = kColsPerLane * kThreads;   // 2048

struct ColabsPlan {
    int col_tiles;
    int slices;
    int rows_per_slice;
};

ColabsPlan colabs_plan(int64_t M, int32_t d) {
    ColabsPlan pl;
    pl.col_tiles = (d + kTileCols - 1) / kTileCols;
    int64_t want = 512 / pl.col_tiles;           // ~2 workgroups per CU: longer row loops, small partials
    if (want < 1) want = 1;
    int64_t rps = (M + want - 1) / want;
    if (rps < 8) rps = 8;                        // at least a few rows per lane
    pl.rows_per_slice = (int)rps;
    pl.slices = (int)((M + rps - 1) / rps);
    return pl;
}

template <bool MAXSTAT>
__global__ void __launch_bounds__(kThreads)
colabs_partial_kernel(const uint16_t* __restrict__ x, int64_t M, int32_t d, int64_t ldx,
                      int rows_per_slice, float* __restrict__ part) {
    const int col = blockIdx.x * kTileCols + threadIdx.x * kColsPerLane;
    if (col >= d) return;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_slice;
    const int64_t r1 = r0 + rows_per_slice < M ? r0 + rows_per_slice : M;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const uint16_t* px = x + col;
#pragma unroll 4
    for (int64_t r = r0; r < r1; ++r) {
        const uint4 w = *reinterpret_cast<const uint4*>(px + r * ldx);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float lo = fabsf(bf16lo_to_f32(ww[q])), hi = fabsf(bf16hi_to_f32(ww[q]));
            acc[2 * q] = MAXSTAT ? fmaxf(acc[2 * q], lo) : acc[2 * q] + lo;
            acc[2 * q + 1] = MAXSTAT ? fmaxf(acc[2 * q + 1], hi) : acc[2 * q + 1] + hi;
        }
    }
    float4* out = reinterpret_cast<float4*>(part + (int64_t)blockIdx.y * d + col);
    out[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    out[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
}

// Pass 2: 32 columns per workgroup, 8 lanes per column.  Lane j of a column adds slices
// j, j+8, ... in double; the 8 sub-sums are then added in lane order.  Fixed order throughout.
constexpr int kFinishCols = 32;
constexpr int kFinishWays = kThreads / kFinishCols;   // 8

template <bool MAXSTAT>
__global__ void __launch_bounds__(kThreads)
colabs_finish_kernel(const float* __restrict__ part, int slices, int32_t d, float m_rows,
                     float* __restrict__ out) {
    __shared__ double red[kFinishWays][kFinishCols];
    const int cl = threadIdx.x % kFinishCols, way = threadIdx.x / kFinishCols;
    const int col = blockIdx.x * kFinishCols + cl;
    double s = 0.0;
    if (col < d) {
#pragma unroll 8
        for (int k = way; k < slices; k += kFinishWays) {
            const double v = (double)part[(int64_t)k * d + col];
            s = MAXSTAT ? (v > s ? v : s) : s + v;
        }
    }
    red[way][cl] = s;
    __syncthreads();
    if (way == 0 && col < d) {
        double t = red[0][cl];
#pragma unroll
        for (int j = 1; j < kFinishWays; ++j) t = MAXSTAT ? (red[j][cl] > t ? red[j][cl] : t) : t + red[j][cl];
        out[col] = MAXSTAT ? (float)t : (float)(t / (double)m_rows);
    }
}

}  // namespace
}  // namespace perq

extern "C" size_t perq_colabs_mean_workspace_bytes(int64_t M, int32_t d) {
    if (M <= 0 || d <= 0) return 0;
    const perq::ColabsPlan pl = perq::colabs_plan(M, d);
    return (size_t)pl.slices * (size_t)d * sizeof(float);
}

// Partial sums of perq_colabs_mean_static, for callers that cannot hand over device memory of their
// own.  In host code this name only stands for the array: its device address is looked up once per
// device (scratch_of_current_device) and that pointer is what kernels are given.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) float scratch[kStaticScratchBytes / sizeof(float)];

namespace perq {
namespace {
perq_status_t colabs_check(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx, const float* out) {
    if (x_bf16 == nullptr || out == nullptr) return PERQ_ERR_INVALID_ARG;
    if (M <= 0 || d <= 0 || ldx < d) return PERQ_ERR_INVALID_ARG;
    if (d % 8 != 0 || ldx % 8 != 0 || (reinterpret_cast<uintptr_t>(x_bf16) & 15u) != 0)
        return PERQ_ERR_UNSUPPORTED;
    return PERQ_OK;
}

template <bool MAXSTAT>
perq_status_t colabs_launch(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx, float* out, float* part,
                            void* hip_stream) {
    const ColabsPlan pl = colabs_plan(M, d);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(colabs_partial_kernel<MAXSTAT>, dim3(pl.col_tiles, pl.slices), dim3(kThreads), 0, stream, x_bf16,
                       M, d, ldx, pl.rows_per_slice, part);
    if (hipGetLastError() != hipSuccess) return PERQ_ERR_LAUNCH;
    hipLaunchKernelGGL(colabs_finish_kernel<MAXSTAT>, dim3((d + kFinishCols - 1) / kFinishCols), dim3(kThreads), 0,
                       stream, part, pl.slices, d, (float)M, out);
    if (hipGetLastError() != hipSuccess) return PERQ_ERR_LAUNCH;
    return PERQ_OK;
}

template <bool MAXSTAT>
perq_status_t colabs_stat(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx, float* out, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    const perq_status_t st = colabs_check(x_bf16, M, d, ldx, out);
    if (st != PERQ_OK) return st;
    const size_t need = perq_colabs_mean_workspace_bytes(M, d);
    if (workspace == nullptr || workspace_bytes < need) return PERQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 15u) != 0) return PERQ_ERR_INVALID_ARG;
    return colabs_launch<MAXSTAT>(x_bf16, M, d, ldx, out, static_cast<float*>(workspace), hip_stream);
}

// Device address of `scratch` on the current device: every device holds its own copy of the array
// at an address of its own, looked up at the first call with that device current.
perq_status_t scratch_of_current_device(float** out) {
    static std::mutex mu;
    static float* known[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PERQ_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (known[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return PERQ_ERR_LAUNCH;
        }
        known[dev] = static_cast<float*>(ptr);
    }
    *out = known[dev];
    return PERQ_OK;
}
}  // namespace
}  // namespace perq

extern "C" perq_status_t perq_colabs_mean(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx,
                                          float* out_mean, void* workspace, size_t workspace_bytes,
                                          void* hip_stream) {
    return perq::colabs_stat<false>(x_bf16, M, d, ldx, out_mean, workspace, workspace_bytes, hip_stream);
}

extern "C" perq_status_t perq_colabs_absmax(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx,
                                            float* out_max, void* workspace, size_t workspace_bytes,
                                            void* hip_stream) {
    return perq::colabs_stat<true>(x_bf16, M, d, ldx, out_max, workspace, workspace_bytes, hip_stream);
}

extern "C" perq_status_t perq_colabs_mean_static(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx,
                                                 float* out_mean, void* hip_stream) {
    const perq_status_t st = perq::colabs_check(x_bf16, M, d, ldx, out_mean);
    if (st != PERQ_OK) return st;
    if (perq_colabs_mean_workspace_bytes(M, d) > kStaticScratchBytes) return PERQ_ERR_UNSUPPORTED;
    float* part = nullptr;
    const perq_status_t sp = perq::scratch_of_current_device(&part);
    if (sp != PERQ_OK) return sp;
    return perq::colabs_launch<false>(x_bf16, M, d, ldx, out_mean, part, hip_stream);
}
