// C-ABI entry points of the fused apply path: argument checks, kernel choice, launch.
#include "perq.h"
#include "perq_base.h"
#include "perq_launch.h"
#include "perq_layout.h"

#include <cmath>
#include <map>
#include <mutex>
#include <tuple>

namespace perq {

const LaunchInfo& launch_info() {
    static LaunchInfo info[64];
    static bool known[64] = {};
    static std::mutex mu;
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev < 0 || dev >= 64) dev = 0;
    std::lock_guard<std::mutex> lock(mu);
    if (!known[dev]) {
        int cus = 0, lds = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess ||
            lds <= 0)
            lds = 64 * 1024;
        info[dev].num_cus = cus;
        info[dev].lds_per_cu = lds;
        known[dev] = true;
    }
    return info[dev];
}

hipError_t resident_blocks(const void* kern, int threads, uint32_t lds_bytes, int* per_cu) {
    static std::map<std::tuple<const void*, int, int, uint32_t>, int> known;
    static std::mutex mu;
    int dev = 0;
    (void)hipGetDevice(&dev);
    const auto key = std::make_tuple(kern, dev, threads, lds_bytes);
    std::lock_guard<std::mutex> lock(mu);
    const auto it = known.find(key);
    if (it != known.end()) {
        *per_cu = it->second;
        return hipSuccess;
    }
    // the limit is only ever raised: an earlier, larger configuration of the same kernel stays valid
    static std::map<std::pair<const void*, int>, uint32_t> limit;
    hipError_t e = hipSuccess;
    uint32_t& lim = limit[std::make_pair(kern, dev)];
    if (lds_bytes > lim) {
        e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        lim = lds_bytes;
    }
    int n = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, lds_bytes);
    if (e != hipSuccess) return e;
    if (n < 1) n = 1;
    known[key] = n;
    *per_cu = n;
    return hipSuccess;
}

namespace {

bool is_pow2(int32_t v) { return v > 0 && (v & (v - 1)) == 0; }

// Shared checks of the apply entry points; fills the kernel parameters.
perq_status_t check_apply(const uint16_t* x, int64_t T, int32_t d, int64_t ldx, const int32_t* perm,
                          int32_t b, ApplyParams* p) {
    if (T < 0 || d <= 0 || ldx < d) return PERQ_ERR_INVALID_ARG;
    if (b < 16 || b > d || d % b != 0) return PERQ_ERR_INVALID_ARG;
    if (!is_pow2(b)) {
        // b = 2^k' * 4t, t odd: a rotation exists for the library iff it can build the 4t-dim base
        int32_t t = b;
        while (t % 2 == 0) t /= 2;
        if (b / t < 4 || hadamard_base_kind(4 * t) == 0) return PERQ_ERR_INVALID_ARG;
    }
    if (d % 32 != 0) return PERQ_ERR_INVALID_ARG;
    if (d > PERQ_MAX_D) return PERQ_ERR_UNSUPPORTED;
    p->T = T;
    if (T == 0) return PERQ_OK;               // nothing to read or write: pointers may be null
    if (x == nullptr) return PERQ_ERR_INVALID_ARG;
    if (ldx % 8 != 0 || (reinterpret_cast<uintptr_t>(x) & 15u) != 0) return PERQ_ERR_UNSUPPORTED;
    if (perm != nullptr && (reinterpret_cast<uintptr_t>(perm) & 15u) != 0) return PERQ_ERR_UNSUPPORTED;
    int log2b = 0;
    while ((1 << log2b) < b) ++log2b;
    p->x = x;
    p->T = T;
    p->ldx = ldx;
    p->perm = perm;
    p->place = nullptr;
    p->lane_table = nullptr;
    p->codes = nullptr;
    p->scales = nullptr;
    p->y = nullptr;
    p->d = d;
    p->b = b;
    p->log2b = log2b;
    p->rsqrt_b = (float)(1.0 / std::sqrt((double)b));
    p->odd_norm = (log2b & 1) ? (float)std::sqrt(0.5) : 1.0f;
    p->half_log2b = log2b / 2;
    p->inv_7sqrt_b = 1.0 / (7.0 * std::sqrt((double)b));
    p->inv_15sqrt_b = 1.0 / (15.0 * std::sqrt((double)b));
    p->fp4_qmax = 6.0f;
    p->inv_fp4sqrt_b = 1.0 / (6.0 * std::sqrt((double)b));
    return PERQ_OK;
}

perq_status_t dispatch(const ApplyParams& p, int out_kind, perq_algo_t algo, hipStream_t stream) {
    if (p.T == 0) return PERQ_OK;
    hipError_t e;
    if (!is_pow2(p.b)) {
        if (algo != PERQ_ALGO_AUTO || !npo2_supports(p)) return PERQ_ERR_UNSUPPORTED;
        return launch_npo2(p, out_kind, stream) == hipSuccess ? PERQ_OK : PERQ_ERR_LAUNCH;
    }
    switch (algo) {
        case PERQ_ALGO_AUTO:
            // The matrix-core kernel wins wherever its 4096-wide wave tiles are filled (measured:
            // rocprofv3 summaries under profiles/); b > 4096 on rows of 8192, 16384 or 32768 goes to the
            // chunked matrix-core kernel; other narrow rows and odd widths take the butterflies.
            if (chunked_pow2_supports(p)) e = launch_npo2_32(p, out_kind, stream);
            else e = mfma_preferred(p, out_kind) ? launch_mfma(p, out_kind, stream) : launch_butterfly(p, out_kind, stream);
            break;
        case PERQ_ALGO_BUTTERFLY:
            e = launch_butterfly(p, out_kind, stream);
            break;
        case PERQ_ALGO_MFMA:
            if (!mfma_supports(p)) return PERQ_ERR_UNSUPPORTED;
            e = launch_mfma(p, out_kind, stream);
            break;
        default:
            return PERQ_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? PERQ_OK : PERQ_ERR_LAUNCH;
}

}  // namespace
}  // namespace perq

namespace perq {
namespace {
perq_status_t quant_entry(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx, const int32_t* perm,
                          const void* prepared, int32_t b, perq_fmt_t fmt, perq_algo_t algo, uint8_t* codes,
                          void* scales, void* hip_stream) {
    ApplyParams p;
    int out_kind;
    switch (fmt) {
        case PERQ_FMT_INT4_SYM_TOKEN: out_kind = OUT_INT4; break;
        case PERQ_FMT_MXFP4: out_kind = OUT_MXFP4; break;
        case PERQ_FMT_INT4_ASYM_TOKEN: out_kind = OUT_INT4_ASYM; break;
        case PERQ_FMT_FP4_TOKEN: out_kind = OUT_FP4_TOKEN; break;
        case PERQ_FMT_FP4_TOKEN_AMAX7: out_kind = OUT_FP4_TOKEN; break;
        default: return PERQ_ERR_INVALID_ARG;
    }
    if (algo != PERQ_ALGO_AUTO && algo != PERQ_ALGO_BUTTERFLY && algo != PERQ_ALGO_MFMA)
        return PERQ_ERR_INVALID_ARG;
    const perq_status_t st = check_apply(x_bf16, T, d, ldx, perm, b, &p);
    if (st != PERQ_OK || p.T == 0) return st;
    if (codes == nullptr || scales == nullptr) return PERQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(codes) & 15u) != 0) return PERQ_ERR_UNSUPPORTED;
    const uintptr_t scale_align = fmt == PERQ_FMT_MXFP4 ? 1u : (fmt == PERQ_FMT_INT4_ASYM_TOKEN ? 8u : 4u);
    if ((reinterpret_cast<uintptr_t>(scales) & (scale_align - 1u)) != 0) return PERQ_ERR_UNSUPPORTED;
    if (prepared != nullptr && (reinterpret_cast<uintptr_t>(prepared) & 15u) != 0) return PERQ_ERR_UNSUPPORTED;
    p.codes = codes;
    p.scales = scales;
    // The prepared form belongs to the matrix-core kernel's staging of whole rows of d >= 4096 through
    // perm (the same shapes perq_perm_prepare accepts); every other shape takes perm as it is.
    //   Its tables of operand offsets in lane order spare every launch the work of turning perm into
    // LDS addresses.  Its placement pays on rows of three tiles or more, where the operand reads keep
    // the LDS busiest (d = 14336: 3 - 4 % less run time); the lookup that has to come before a
    // workgroup's first row loads costs rows of one or two tiles more than the reads gain (d = 4096,
    // 8192: + 1 - 1.5 %), so those stay in the fixed layout (layout::placement_applies, which the
    // tables follow).
    if (prepared != nullptr && perm != nullptr && algo == PERQ_ALGO_AUTO && d >= 4096 && d % 512 == 0 && is_pow2(b) &&
        b >= 16 && b <= 4096 && mfma_supports(p)) {
        // [int32 place of the channel of every position][uint16 granule of every slot][uint16 lane tables]
        const int32_t* places = static_cast<const int32_t*>(prepared);
        if (layout::placement_applies(d)) {
            p.perm = places;
            p.place = reinterpret_cast<const uint16_t*>(places + d);
        }
        p.lane_table = reinterpret_cast<const uint16_t*>(places + d) + d / 8;
    }
    if (fmt == PERQ_FMT_FP4_TOKEN_AMAX7) {
        p.fp4_qmax = 7.0f;
        p.inv_fp4sqrt_b = 1.0 / (7.0 * std::sqrt((double)b));
    }
    return dispatch(p, out_kind, algo, static_cast<hipStream_t>(hip_stream));
}
}  // namespace
}  // namespace perq

extern "C" perq_status_t perq_permute_rotate_quant_algo(const uint16_t* x_bf16, int64_t T, int32_t d,
                                                        int64_t ldx, const int32_t* perm, int32_t b,
                                                        perq_fmt_t fmt, perq_algo_t algo, uint8_t* codes,
                                                        void* scales, void* hip_stream) {
    return perq::quant_entry(x_bf16, T, d, ldx, perm, nullptr, b, fmt, algo, codes, scales, hip_stream);
}

extern "C" perq_status_t perq_permute_rotate_quant(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                                   const int32_t* perm, int32_t b, perq_fmt_t fmt,
                                                   uint8_t* codes, void* scales, void* hip_stream) {
    return perq::quant_entry(x_bf16, T, d, ldx, perm, nullptr, b, fmt, PERQ_ALGO_AUTO, codes, scales, hip_stream);
}

extern "C" perq_status_t perq_permute_rotate_quant_prepared(const uint16_t* x_bf16, int64_t T, int32_t d,
                                                            int64_t ldx, const int32_t* perm,
                                                            const void* prepared, int32_t b, perq_fmt_t fmt,
                                                            uint8_t* codes, void* scales, void* hip_stream) {
    return perq::quant_entry(x_bf16, T, d, ldx, perm, prepared, b, fmt, PERQ_ALGO_AUTO, codes, scales, hip_stream);
}

extern "C" perq_status_t perq_permute_rotate_f32(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                                 const int32_t* perm, int32_t b, perq_algo_t algo, float* y,
                                                 void* hip_stream) {
    perq::ApplyParams p;
    if (algo != PERQ_ALGO_AUTO && algo != PERQ_ALGO_BUTTERFLY && algo != PERQ_ALGO_MFMA)
        return PERQ_ERR_INVALID_ARG;
    const perq_status_t st = perq::check_apply(x_bf16, T, d, ldx, perm, b, &p);
    if (st != PERQ_OK || p.T == 0) return st;
    if (y == nullptr) return PERQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(y) & 15u) != 0) return PERQ_ERR_UNSUPPORTED;
    p.y = y;
    return perq::dispatch(p, perq::OUT_F32, algo, static_cast<hipStream_t>(hip_stream));
}

extern "C" perq_status_t perq_block_diagnostics(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                                const int32_t* perm, int32_t b, float* out, void* hip_stream) {
    perq::ApplyParams p;
    const perq_status_t st = perq::check_apply(x_bf16, T, d, ldx, perm, b, &p);
    if (st != PERQ_OK || p.T == 0) return st;
    if (out == nullptr) return PERQ_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(out) & 15u) != 0) return PERQ_ERR_UNSUPPORTED;
    if (!perq::is_pow2(b)) return PERQ_ERR_UNSUPPORTED;
    p.y = out;
    return perq::launch_butterfly(p, perq::OUT_DIAG, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? PERQ_OK
               : PERQ_ERR_LAUNCH;
}
