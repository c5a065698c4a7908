// Power-of-two blocks above 4096 (b = 8192 .. 32768 on d = 8192, 16384, 32768: among them the
// full-vector rotation at the Llama3 1B/3B width) through the chunked kernel, with Sylvester's H_32
// as its base matrix.
#include "perq_npo2_impl.h"

namespace perq {

hipError_t launch_npo2_32(const ApplyParams& p, int out_kind, hipStream_t stream) {
    return launch_npo2_base_impl<32>(p, out_kind, stream);
}

bool chunked_pow2_supports(const ApplyParams& p) {
    const int chunk_pos = npo2_chunk_pos<32>();       // 4096
    if (p.d != 2 * chunk_pos && p.d != 4 * chunk_pos && p.d != 8 * chunk_pos) return false;
    return p.b > 4096 && p.b <= p.d && (p.b & (p.b - 1)) == 0 && p.ldx < ((int64_t)1 << 28);
}

}  // namespace perq
