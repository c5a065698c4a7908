// Non-power-of-two rotation (Appendix A.1): the kernels for the 28-dimensional base
// (d = 3584, 7168, 14336, the Llama3-8B width) and the choice among the bases.
#include "perq_npo2_impl.h"

namespace perq {

hipError_t launch_npo2_28(const ApplyParams& p, int out_kind, hipStream_t stream) {
    return launch_npo2_base_impl<28>(p, out_kind, stream);
}

namespace {

// b = 2^k' * 4t, t odd: the order 4t of the base, 0 if b is a power of two or 2t
int base_order(int32_t b) {
    int32_t t = b;
    while (t % 2 == 0) t /= 2;
    return (t == 1 || b / t < 4) ? 0 : 4 * t;
}

}  // namespace

bool npo2_supports(const ApplyParams& p) {
    int chunk_pos;
    switch (base_order(p.b)) {
        case 28: chunk_pos = npo2_chunk_pos<28>(); break;
        case 12: chunk_pos = npo2_chunk_pos<12>(); break;
        case 76: chunk_pos = npo2_chunk_pos<76>(); break;
        default: return false;
    }
    if (p.d != chunk_pos && p.d != 2 * chunk_pos && p.d != 4 * chunk_pos &&
        !(base_order(p.b) == 28 && p.d == 8 * chunk_pos))
        return false;
    // row offsets inside a unit of up to four rows are kept in 32 bits
    return p.d % p.b == 0 && p.ldx < ((int64_t)1 << 28);
}

hipError_t launch_npo2(const ApplyParams& p, int out_kind, hipStream_t stream) {
    switch (base_order(p.b)) {
        case 28: return launch_npo2_28(p, out_kind, stream);
        case 12: return launch_npo2_12(p, out_kind, stream);
        case 76: return launch_npo2_76(p, out_kind, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace perq
