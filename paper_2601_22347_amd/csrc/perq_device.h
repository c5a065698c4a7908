// Device-side building blocks shared by the PeRQ apply kernels (gfx950, wave64).
//
//  - bf16 <-> fp32 bit moves
//  - lane-xor butterflies on DPP / swizzle / permlane-swap
//  - the three epilogues on a run of 32 contiguous rotated outputs held by one lane:
//      INT4 symmetric per token   (Section 3; Appendix B Eq. 4, z = 0)
//      MXFP4                      (Appendix B Eq. 5: e2m1 + one power-of-two scale per 32)
//      INT4 asymmetric per token  (Appendix B, INT4 paragraph: step (max-min)/15, integer zero point)
//      FP4 per token              (Appendix B, (MX)FP4 paragraph: e2m1 with one real scale per token)
//      fp32 dump                  (test entry)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace perq {

enum OutKind { OUT_INT4 = 0, OUT_MXFP4 = 1, OUT_F32 = 2, OUT_INT4_ASYM = 3, OUT_FP4_TOKEN = 4, OUT_DIAG = 5 };

struct ApplyParams {
    const uint16_t* x;      // bf16 [T, ldx]
    int64_t T;
    int64_t ldx;
    const int32_t* perm;    // int32 [d] or nullptr
    const uint16_t* place;  // prepared placement: granule of the row in every LDS slot (then perm holds places), or nullptr
    const uint16_t* lane_table;  // prepared operand offsets in the matrix-core kernel's lane order (two tables), or nullptr
    uint8_t* codes;         // [T, d/2]
    void* scales;           // float [T], uint8 [T, d/32] or float [T][2] (step, zero point)
    float* y;               // [T, d] (test entry), or [T, 4] (diagnostics)
    int32_t d;
    int32_t b;
    int32_t log2b;
    float rsqrt_b;          // fl32(1/sqrt(b))
    float odd_norm;         // 1.0 if log2b even, fl32(1/sqrt(2)) if odd
    int32_t half_log2b;     // floor(log2b / 2)
    double inv_7sqrt_b;     // 1 / (7 sqrt(b)) in double
    double inv_15sqrt_b;    // 1 / (15 sqrt(b))
    double inv_fp4sqrt_b;   // 1 / (c sqrt(b)), c = fp4_qmax
    float fp4_qmax;         // per-token FP4: the row maximum maps to this many steps (6, or 7 as printed)
};

// Streaming (non-temporal) 16-byte global accesses: every input byte is read once and every
// output byte written once, so neither should displace anything in the caches.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void store_stream16(void* p, uint4 v) {
    const u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
}

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_stream8(void* p, uint32_t a, uint32_t b) {
    const u32x2_t t = {a, b};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x2_t*>(p));
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits for every
// outstanding global load and store of the wave, which would expose the latency of loads issued
// ahead of their use once per barrier.
__device__ __forceinline__ void workgroup_barrier_lds() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// ---- lane-xor exchange: value held by lane (l ^ M) ---------------------------------------
template <int M>
__device__ __forceinline__ float lane_xor(float v) {
    const int iv = __float_as_int(v);
    if constexpr (M == 1) {
        return __int_as_float(__builtin_amdgcn_update_dpp(iv, iv, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    } else if constexpr (M == 2) {
        return __int_as_float(__builtin_amdgcn_update_dpp(iv, iv, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    } else if constexpr (M == 4) {
        return __int_as_float(__builtin_amdgcn_ds_swizzle(iv, 0x101F));                      // xor 4 inside 32 lanes
    } else if constexpr (M == 8) {
        return __int_as_float(__builtin_amdgcn_update_dpp(iv, iv, 0x128, 0xF, 0xF, false));  // row_ror:8
    } else if constexpr (M == 16) {
        return __int_as_float(__builtin_amdgcn_ds_swizzle(iv, 0x401F));                      // xor 16 inside 32 lanes
    } else {
        return __shfl_xor(v, 32, 64);
    }
}

// max(v, value of lane l ^ M) as one step of a reduction that runs M = 1, 2, 4, ... upwards: for
// M = 4 the lanes l ^ 1, l ^ 2 must already hold the same v (the mirror inside 8 lanes then reaches
// the other quad).  Vector-ALU data movement only: a trip through the LDS crossbar would also wait
// for every LDS read the wave has in flight.
template <int M>
__device__ __forceinline__ float lane_max(float v) {
    if constexpr (M == 4) {
        const int iv = __float_as_int(v);
        return fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(iv, iv, 0x141, 0xF, 0xF, false)));   // row_half_mirror
    } else if constexpr (M == 16) {
        const uint32_t u = __float_as_uint(v);
        auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);      // [r0 r0 r2 r2], [r1 r1 r3 r3]
        return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    } else if constexpr (M == 32) {
        const uint32_t u = __float_as_uint(v);
        auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);      // [lo lo], [hi hi]
        return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    } else {
        return fmaxf(v, lane_xor<M>(v));
    }
}

// One radix-2 butterfly stage across lanes for N registers: v <- (lane & M) ? p - v : p + v,
// p = value of lane ^ M.  `sgn` is -1 in lanes with bit M set, +1 elsewhere.
template <int M, int N>
__device__ __forceinline__ void lane_stage(float (&v)[N], float sgn) {
    if constexpr (M == 16 || M == 32) {
        // Two registers at a time through a half-wave (or odd/even row) swap: after the first
        // swap every lane holds both operands of one butterfly, after the second each result
        // is back with its owner.  Pure VALU, no LDS crossbar.
#pragma unroll
        for (int i = 0; i < N; i += 2) {
            const uint32_t u = __float_as_uint(v[i]), w = __float_as_uint(v[i + 1]);
            uint32_t r0, r1;
            if constexpr (M == 32) {
                auto r = __builtin_amdgcn_permlane32_swap(u, w, false, false); r0 = r[0]; r1 = r[1];
            } else {
                auto r = __builtin_amdgcn_permlane16_swap(u, w, false, false); r0 = r[0]; r1 = r[1];
            }
            const float s = __uint_as_float(r0) + __uint_as_float(r1);
            const float t = __uint_as_float(r0) - __uint_as_float(r1);
            uint32_t q0, q1;
            if constexpr (M == 32) {
                auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(t), false, false);
                q0 = q[0]; q1 = q[1];
            } else {
                auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(s), __float_as_uint(t), false, false);
                q0 = q[0]; q1 = q[1];
            }
            v[i] = __uint_as_float(q0);
            v[i + 1] = __uint_as_float(q1);
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = __builtin_fmaf(v[i], sgn, lane_xor<M>(v[i]));
    }
}

// In-register radix-2 stages on a run of N = 2^k contiguous elements, strides 1 .. hmax/2.
template <int N>
__device__ __forceinline__ void reg_stages(float (&v)[N], int hmax) {
#pragma unroll
    for (int h = 1; h < N; h <<= 1) {
        if (h < hmax) {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                if ((i & h) == 0) {
                    const float a = v[i], c = v[i | h];
                    v[i] = a + c;
                    v[i | h] = a - c;
                }
            }
        }
    }
}

template <int N>
__device__ __forceinline__ float absmax(const float (&v)[N]) {
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < N; ++i) m = fmaxf(m, fabsf(v[i]));
    return m;
}

// ---- rows of vanishing magnitude -----------------------------------------------------------
// The per-token formats multiply every value by qmax / (row maximum) (or 15 / (max - min)).  Below
// an extent of 2^-100 -- a row of bf16 subnormals -- that quotient leaves the fp32 range, so such a
// row is multiplied by 2^100 first: exact, and the codes depend on ratios only.  The scale written
// out is computed from the extent as it was.
constexpr float kTinyRow = 0x1p-100f, kTinyRowLift = 0x1p100f;
__device__ __forceinline__ bool tiny_row(float extent) {
    return __builtin_expect(extent < kTinyRow && extent > 0.0f, 0);
}
template <int N>
__device__ __forceinline__ void lift_values(float (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] *= kTinyRowLift;
}

// ---- INT4: 8 values -> one dword of two's-complement nibbles, element 0 in bits 3:0 ------
// fma(y, inv, 1.5*2^23 + 8) rounds y*inv to an integer c (ties to even) in one step and leaves
// the word 0x4B400000 + (c + 8): the low nibble is c in offset binary (1..15, so nothing
// carries out of it) and every higher bit is the same constant for all elements.  Eight such
// words are merged with shift-adds; the constant parts add up to kInt4Bias, which is removed
// once, and flipping bit 3 of every nibble turns offset binary into two's complement.
constexpr uint32_t kInt4Bias = (uint32_t)(0x4B400000ull * 0x11111111ull);
__device__ __forceinline__ uint32_t int4_pack8(const float* v, float inv) {
    uint32_t acc = __float_as_uint(__builtin_fmaf(v[7], inv, 12582920.0f));
#pragma unroll
    for (int i = 6; i >= 0; --i) acc = (acc << 4) + __float_as_uint(__builtin_fmaf(v[i], inv, 12582920.0f));
    return (acc - kInt4Bias) ^ 0x88888888u;
}

// ---- INT4 asymmetric: 8 values -> one dword of unsigned nibbles (code = rne(y*inv) - z) -----
// Same rounding word as above without the +8: 0x4B400000 + c, c = rne(y*inv) (possibly negative;
// all arithmetic is modulo 2^32 and linear).  As long as every c - z lies in [0, 15] the eight
// words can be merged first and K + z * 0x11111111 removed once.  c - z = 16 happens only for
// values within half a step of the row maximum, and only in rows whose two ends round 16 steps
// apart; such rows take the second routine, which clamps element by element (see Int4Asym).
constexpr uint32_t kInt4AsymBias = (uint32_t)(0x4B400000ull * 0x11111111ull);
__device__ __forceinline__ uint32_t int4a_pack8(const float* v, float inv, uint32_t z_nibbles) {
    uint32_t acc = __float_as_uint(__builtin_fmaf(v[7], inv, 12582912.0f));
#pragma unroll
    for (int i = 6; i >= 0; --i) acc = (acc << 4) + __float_as_uint(__builtin_fmaf(v[i], inv, 12582912.0f));
    return acc - kInt4AsymBias - z_nibbles;
}
struct Int4Asym;
__device__ __forceinline__ uint32_t int4a_pack8_clamped(const float* v, const Int4Asym& q);

// ---- FP4 with a real-valued scale: 8 values -> one dword of e2m1 nibbles --------------------
// y * inv (inv = 6 / row maximum) is handed to the same convert with scale 1.
__device__ __forceinline__ uint32_t fp4_pack8(const float* v, float inv) {
    uint32_t w = 0;
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[0] * inv, v[1] * inv, 1.0f, 0);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[2] * inv, v[3] * inv, 1.0f, 1);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[4] * inv, v[5] * inv, 1.0f, 2);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[6] * inv, v[7] * inv, 1.0f, 3);
    const uint32_t mag = w & 0x77777777u;
    const uint32_t nz = (mag + 0x77777777u) & 0x88888888u;
    return mag | (w & nz);
}

// Per-row quantities of the asymmetric INT4 quantizer from the row's extremes (unnormalised
// rotation outputs; the missing 1/sqrt(b) cancels in every ratio).
struct Int4Asym {
    float inv;          // 15 / (hi - lo), 0 for a constant row
    int z;              // rne(lo * inv), rounded by the very instruction that rounds the elements
    int mode;           // 0: eight elements at a time (int4a_pack8); 1: the two ends round 16 steps apart,
                        // element-wise with a clip; 2: an offset row, element-wise in double
    float range;        // hi - lo
};
__device__ __forceinline__ int int4a_round(float y, float inv) {
    return (int)(__float_as_uint(__builtin_fmaf(y, inv, 12582912.0f)) - 0x4B400000u);
}
// The rounding word is an integer only while |y * inv| < 2^22.  A row that is a large offset plus a
// small spread (every block one value at its first position, tiny values elsewhere: the rotated row
// is nearly constant) leaves that range: |lo| * 15 / (hi - lo) can reach 15 * 2^24, the spread being
// at least one fp32 step of the offset.  Such rows are rounded in double, where lo * inv, y * inv and
// their difference are exact integers after rint (hi - lo is exact in fp32 there: both ends lie
// within a factor of two).  z stays below 2^28 and is written out as a float: exact up to 2^24.
constexpr float kInt4AsymFast = 0x1p21f;
__device__ __forceinline__ Int4Asym int4_asym_row(float lo, float hi) {
    Int4Asym q;
    q.range = hi - lo;
    q.inv = q.range > 0.0f ? 15.0f / q.range : 0.0f;
    if (__builtin_expect(fmaxf(fabsf(lo), fabsf(hi)) * q.inv < kInt4AsymFast, 1)) {
        // (the rounding is monotonic, so every element of the row lands in [z, round(hi)])
        q.z = int4a_round(lo, q.inv);
        q.mode = int4a_round(hi, q.inv) - q.z > 15 ? 1 : 0;
    } else {
        q.z = (int)__builtin_rint((double)lo * (15.0 / (double)q.range));
        q.mode = 2;
    }
    return q;
}
__device__ __forceinline__ uint32_t int4a_pack8_clamped(const float* v, const Int4Asym& q) {
    uint32_t acc = 0;
    if (q.mode == 2) {
        const double invd = 15.0 / (double)q.range;
#pragma unroll
        for (int i = 7; i >= 0; --i) {
            const int c = (int)(__builtin_rint((double)v[i] * invd) - (double)q.z);
            acc = (acc << 4) | (uint32_t)(c < 0 ? 0 : (c > 15 ? 15 : c));
        }
        return acc;
    }
#pragma unroll
    for (int i = 7; i >= 0; --i) {
        const int c = int4a_round(v[i], q.inv) - q.z;
        acc = (acc << 4) | (uint32_t)(c < 0 ? 0 : (c > 15 ? 15 : c));
    }
    return acc;
}

template <int N>
__device__ __forceinline__ void minmax(const float (&v)[N], float& lo, float& hi) {
    lo = v[0]; hi = v[0];
#pragma unroll
    for (int i = 1; i < N; ++i) { lo = fminf(lo, v[i]); hi = fmaxf(hi, v[i]); }
}

// ---- MXFP4: 8 values -> one dword of e2m1 nibbles ----------------------------------------
// The hardware convert divides by 2^(exponent field of `scale` - 127), rounds to nearest even
// on the e2m1 grid and saturates at 6.  A value that rounds to zero keeps its sign bit, so
// nibbles 0x8 are rewritten to 0x0 (zero is always stored as +0).
__device__ __forceinline__ uint32_t mxfp4_pack8(const float* v, float scale) {
    uint32_t w = 0;
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[0], v[1], scale, 0);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[2], v[3], scale, 1);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[4], v[5], scale, 2);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[6], v[7], scale, 3);
    const uint32_t mag = w & 0x77777777u;
    const uint32_t nz = (mag + 0x77777777u) & 0x88888888u;   // bit 3 of a nibble set iff magnitude != 0
    return mag | (w & nz);
}

// Shared exponent of one 32-group from its (already normalised up to 2^-k) maximum:
// E = clamp(expfield(amax) - k - 2, 0, 254); an all-zero or subnormal maximum gives E = 0.
__device__ __forceinline__ int mx_shared_exponent(float amax_scaled, int k) {
    int e = (int)((__float_as_uint(amax_scaled) >> 23) & 0xFFu) - k - 2;
    e = e < 0 ? 0 : e;
    return e > 254 ? 254 : e;
}

}  // namespace perq
