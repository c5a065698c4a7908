// Non-power-of-two rotation (Appendix A.1): the kernels for the 76-dimensional base
// (d = 2432, 4864, 9728: the last is the Qwen3 4B down-projection width).
#include "perq_npo2_impl.h"

namespace perq {

hipError_t launch_npo2_76(const ApplyParams& p, int out_kind, hipStream_t stream) {
    return launch_npo2_base_impl<76>(p, out_kind, stream);
}

}  // namespace perq
