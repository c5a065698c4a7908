// Non-power-of-two rotation (Appendix A.1): the kernels for the 12-dimensional base
// (d = 3072, 6144, 12288: the Qwen3 0.6B, 1.7B and 8B down-projection widths).
#include "perq_npo2_impl.h"

namespace perq {

hipError_t launch_npo2_12(const ApplyParams& p, int out_kind, hipStream_t stream) {
    return launch_npo2_base_impl<12>(p, out_kind, stream);
}

}  // namespace perq
