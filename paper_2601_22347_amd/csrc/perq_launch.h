// Host-side launch plumbing shared by the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>

#include "perq_device.h"

namespace perq {

struct LaunchInfo {
    int num_cus;
    int lds_per_cu;   // bytes
};

// Properties of the current device (queried once per process and device).
const LaunchInfo& launch_info();

// Number of workgroups of `kern` (threads per workgroup, dynamic LDS bytes) that one CU keeps
// resident; on first use per device also raises the kernel's dynamic-LDS limit to lds_bytes.
// Asked of the runtime once per kernel, device and configuration, then remembered.
hipError_t resident_blocks(const void* kern, int threads, uint32_t lds_bytes, int* per_cu);

// Kernel families behind perq_permute_rotate_quant / perq_permute_rotate_f32.
hipError_t launch_butterfly(const ApplyParams& p, int out_kind, hipStream_t stream);
bool mfma_supports(const ApplyParams& p);
// Whether the matrix-core kernel is the faster of the two for this call (measured crossovers).
bool mfma_preferred(const ApplyParams& p, int out_kind);
hipError_t launch_mfma(const ApplyParams& p, int out_kind, hipStream_t stream);
// Block sizes 2^k' * 4t, 4t = 12, 28 or 76 (non-power-of-two rotation), one family of kernels per base.
bool npo2_supports(const ApplyParams& p);
hipError_t launch_npo2(const ApplyParams& p, int out_kind, hipStream_t stream);
hipError_t launch_npo2_28(const ApplyParams& p, int out_kind, hipStream_t stream);
hipError_t launch_npo2_12(const ApplyParams& p, int out_kind, hipStream_t stream);
hipError_t launch_npo2_76(const ApplyParams& p, int out_kind, hipStream_t stream);
// The same chunked kernel with H_32 as base: power-of-two b > 4096 on d = 8192, 16384.
bool chunked_pow2_supports(const ApplyParams& p);
hipError_t launch_npo2_32(const ApplyParams& p, int out_kind, hipStream_t stream);

}  // namespace perq
