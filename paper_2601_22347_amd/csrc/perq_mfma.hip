// Matrix-core kernel for X -> quantize(XP R~), b <= 4096, d a multiple of 512.
//
// The low five index bits of the rotation are one dense product on the MFMA unit; what is left
// (b > 32) are a few +-1 butterflies on the accumulators.
//
// Work split.  A wave owns a tile of 4096 contiguous positions of one (permuted) row, seen as
// 128 sub-blocks of 32.  Lane l = (c, h), c = l & 31, h = l >> 5, owns sub-blocks 4c .. 4c+3.
// For sub-block q of the lane, v_mfma_f32_32x32x16_bf16 computes  D = A * B  with
//     B[k][c]  = the data, element k of the lane's sub-block (lane (c,h) supplies k = 16kt+8h+e),
//     A[i][k]  = +-1: row sigma(i) of the Sylvester matrix H_32 (of I_2 (x) H_16 when b = 16),
// so column c of D is the rotated sub-block.  sigma is chosen so that the 16 accumulators of
// lane (c,h) are the contiguous outputs 16h .. 16h+15 of the sub-block.  bf16 x (+-1) products
// are exact and accumulate in fp32.
//     b = 64, 128     : butterflies between the lane's four accumulator tiles (registers only)
//     b = 256 .. 4096 : butterflies across lanes on c (DPP / swizzle / permlane swap)
//
// Data movement.  The raw bf16 rows go global -> LDS with 16-byte direct-to-LDS loads (no
// registers, no ds_write), streaming policy; they are the only HBM reads.  The B operands are
// read back from LDS either as one 16-byte read per fragment (P = I) or element by element
// through `perm`, whose LDS byte addresses each lane computes once and keeps for every row.
// 16-byte granule g of a row lives in slot g ^ f((g >> 4) & 7), which spreads both patterns
// over all banks; the swizzle is applied on the global side of the direct-to-LDS load.
#include "perq_device.h"
#include "perq_launch.h"

namespace perq {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 4096;     // elements per wave tile
constexpr int kQ = 4;           // sub-blocks of 32 per lane

struct MfmaGeom {
    int tiles_per_row;   // power of two >= ceil(d / 4096)
    int rows;            // rows per workgroup iteration = waves / tiles_per_row
    int nload;           // direct-to-LDS load instructions per lane per iteration
    uint32_t row_bytes;  // d * 2
    uint32_t red_off;    // byte offset of the cross-wave reduction scratch
};

// granule -> slot inside a row (an involution: bits 4..6 select the xor pattern for bits 0..2)
__device__ __forceinline__ uint32_t granule_slot(uint32_t g) {
    const uint32_t c = (g >> 4) & 7u;
    return g ^ (((c & 3u) << 1) | (c >> 2));
}

__device__ __forceinline__ uint32_t popc_parity(uint32_t v) { return __builtin_popcount(v) & 1u; }

template <int OUT, bool PERM, int NWAVES>
__global__ void __launch_bounds__(NWAVES * 64)
mfma_kernel(ApplyParams p, MfmaGeom g) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, h = lane >> 5;
    const int d = p.d, b = p.b;
    const int rr = wave / g.tiles_per_row;                 // row slot of this wave
    const int tile_base = (wave % g.tiles_per_row) * kTile;
    int tile_len = d - tile_base;
    tile_len = tile_len < 0 ? 0 : (tile_len > kTile ? kTile : tile_len);
    const bool full_tile = tile_len == kTile;

    // ---- A operand: rows sigma(i) of the +-1 matrix, two K steps of 16 ---------------------
    bf16x8_t afrag[2];
    {
        const uint32_t i = (uint32_t)lane & 31u;
        const uint32_t n = 16u * ((i >> 2) & 1u) + 4u * (i >> 3) + (i & 3u);
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t k = 16u * kt + 8u * h + e;
                uint32_t bits;
                if (b >= 32) bits = popc_parity(n & k) ? 0xBF80u : 0x3F80u;
                else bits = (n >> 4) != (k >> 4) ? 0u : (popc_parity(n & k & 15u) ? 0xBF80u : 0x3F80u);
                if (e & 1) w[e >> 1] |= bits << 16; else w[e >> 1] = bits;
            }
            afrag[kt] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
        }
    }

    // ---- LDS addresses of this lane's operands (fixed for the whole launch) ----------------
    // PERM: one address per element; identity: one per 16-byte fragment.
    uint32_t src[PERM ? 64 : 8];
    bool qvalid[kQ];
#pragma unroll
    for (int q = 0; q < kQ; ++q) {
        const int sb = c * kQ + q;
        qvalid[q] = sb * 32 < tile_len;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const uint32_t pos = (uint32_t)tile_base + (uint32_t)sb * 32u + 16u * kt + 8u * h;
            if constexpr (PERM) {
                int4 e0 = make_int4(0, 0, 0, 0), e1 = make_int4(0, 0, 0, 0);
                if (qvalid[q]) {
                    e0 = *reinterpret_cast<const int4*>(p.perm + pos);
                    e1 = *reinterpret_cast<const int4*>(p.perm + pos + 4);
                }
                const uint32_t ch[8] = {(uint32_t)e0.x, (uint32_t)e0.y, (uint32_t)e0.z, (uint32_t)e0.w,
                                        (uint32_t)e1.x, (uint32_t)e1.y, (uint32_t)e1.z, (uint32_t)e1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    src[(q * 2 + kt) * 8 + e] =
                        (uint32_t)rr * g.row_bytes + ((granule_slot(ch[e] >> 3) << 4) | ((ch[e] & 7u) << 1));
            } else {
                src[q * 2 + kt] = (uint32_t)rr * g.row_bytes + (qvalid[q] ? (granule_slot(pos >> 3) << 4) : 0u);
            }
        }
    }

    // -1 / +1 of the cross-lane butterflies on c
    float sgn[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) sgn[k] = (c >> k) & 1 ? -1.0f : 1.0f;

    const int64_t ngroups = (p.T + g.rows - 1) / g.rows;
    const uint32_t gpr = (uint32_t)d >> 3;                    // granules per row (multiple of 64)

    // One direct-to-LDS instruction moves 64 consecutive slots (1 KiB) of one row.
    auto issue_loads = [&](int64_t grp) {
        for (int k = 0; k < g.nload; ++k) {
            const uint32_t s0 = (uint32_t)(k * NWAVES + wave) * 64u;         // first slot, wave-uniform
            const uint32_t rslot = s0 / gpr;
            const int64_t row = grp * g.rows + rslot;
            if (rslot < (uint32_t)g.rows && row < p.T) {
                const uint32_t gs = s0 - rslot * gpr + (uint32_t)lane;          // slot inside the row
                const uint16_t* src_g = p.x + row * p.ldx + (int64_t)granule_slot(gs) * 8;
                __builtin_amdgcn_global_load_lds(src_g, lds + (size_t)s0 * 16u, 16, 0, 2 /* nt */);
            }
        }
    };

    if ((int64_t)blockIdx.x < ngroups) issue_loads(blockIdx.x);

    for (int64_t grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
        const int64_t row = grp * g.rows + rr;
        const bool row_live = rr < g.rows && row < p.T;

        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's direct-to-LDS loads have landed
        __syncthreads();

        // ---- B operands out of LDS ----------------------------------------------------------
        uint4 bfrag[kQ][2];
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                if constexpr (PERM) {
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const uint32_t lo = *reinterpret_cast<const uint16_t*>(lds + src[(q * 2 + kt) * 8 + e]);
                        const uint32_t hi = *reinterpret_cast<const uint16_t*>(lds + src[(q * 2 + kt) * 8 + e + 1]);
                        w[e >> 1] = lo | (hi << 16);
                    }
                    bfrag[q][kt] = make_uint4(w[0], w[1], w[2], w[3]);
                } else {
                    bfrag[q][kt] = *reinterpret_cast<const uint4*>(lds + src[q * 2 + kt]);
                }
            }
        }
        if (!full_tile) {
#pragma unroll
            for (int q = 0; q < kQ; ++q)
                if (!qvalid[q]) bfrag[q][0] = bfrag[q][1] = make_uint4(0, 0, 0, 0);
        }
        __syncthreads();                          // every wave has its operands: LDS may be refilled
        if (grp + gridDim.x < ngroups) issue_loads(grp + gridDim.x);

        // ---- low five bits on the matrix cores ------------------------------------------------
        float v[64];
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            f32x16_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[0], __builtin_bit_cast(bf16x8_t, bfrag[q][0]), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[1], __builtin_bit_cast(bf16x8_t, bfrag[q][1]), acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 16; ++r) v[q * 16 + r] = acc[r];
        }

        // ---- remaining butterflies --------------------------------------------------------------
        if (b >= 64) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float a0 = v[r], a1 = v[16 + r], a2 = v[32 + r], a3 = v[48 + r];
                v[r] = a0 + a1; v[16 + r] = a0 - a1; v[32 + r] = a2 + a3; v[48 + r] = a2 - a3;
            }
        }
        if (b >= 128) {
#pragma unroll
            for (int r = 0; r < 32; ++r) {
                const float a0 = v[r], a2 = v[32 + r];
                v[r] = a0 + a2; v[32 + r] = a0 - a2;
            }
        }
        if (b >= 256) lane_stage<1>(v, sgn[0]);
        if (b >= 512) lane_stage<2>(v, sgn[1]);
        if (b >= 1024) lane_stage<4>(v, sgn[2]);
        if (b >= 2048) lane_stage<8>(v, sgn[3]);
        if (b >= 4096) lane_stage<16>(v, sgn[4]);

        // ---- epilogue: lane (c,h) holds outputs 16h..16h+15 of sub-blocks 4c..4c+3 -------------
        if constexpr (OUT == OUT_F32) {
#pragma unroll
            for (int q = 0; q < kQ; ++q) {
                if (row_live && qvalid[q]) {
                    float4* yo = reinterpret_cast<float4*>(p.y + row * (int64_t)d + tile_base + (c * kQ + q) * 32 + 16 * h);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        yo[j] = make_float4(v[q * 16 + 4 * j] * p.rsqrt_b, v[q * 16 + 4 * j + 1] * p.rsqrt_b,
                                            v[q * 16 + 4 * j + 2] * p.rsqrt_b, v[q * 16 + 4 * j + 3] * p.rsqrt_b);
                }
            }
        } else {
            uint32_t pk[kQ][2];
            uint32_t ebytes = 0;
            float row_max = 0.0f;
            if constexpr (OUT == OUT_MXFP4) {
                if (p.odd_norm != 1.0f) {
#pragma unroll
                    for (int i = 0; i < 64; ++i) v[i] *= p.odd_norm;
                }
#pragma unroll
                for (int q = 0; q < kQ; ++q) {
                    float m = 0.0f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) m = fmaxf(m, fabsf(v[q * 16 + r]));
                    m = fmaxf(m, lane_xor<32>(m));                   // the other half of the 32-group
                    const int E = mx_shared_exponent(m, p.half_log2b);
                    const float scale = __uint_as_float((uint32_t)(E + p.half_log2b) << 23);
                    pk[q][0] = mxfp4_pack8(v + q * 16, scale);
                    pk[q][1] = mxfp4_pack8(v + q * 16 + 8, scale);
                    ebytes |= (uint32_t)E << (8 * q);
                }
            } else {
                float m = absmax(v);
                m = fmaxf(m, lane_xor<1>(m));
                m = fmaxf(m, lane_xor<2>(m));
                m = fmaxf(m, lane_xor<4>(m));
                m = fmaxf(m, lane_xor<8>(m));
                m = fmaxf(m, lane_xor<16>(m));
                m = fmaxf(m, lane_xor<32>(m));
                if (g.tiles_per_row > 1) {
                    float* red = reinterpret_cast<float*>(lds + g.red_off);
                    if (lane == 0) red[wave] = m;
                    __syncthreads();
                    const int w0 = rr * g.tiles_per_row;
                    for (int w = 0; w < g.tiles_per_row; ++w) m = fmaxf(m, red[w0 + w]);
                }
                row_max = m;
                const float inv = m > 0.0f ? 7.0f / m : 0.0f;
#pragma unroll
                for (int q = 0; q < kQ; ++q) {
                    pk[q][0] = int4_pack8(v + q * 16, inv);
                    pk[q][1] = int4_pack8(v + q * 16 + 8, inv);
                }
            }
            // Give lane (c,0) the whole of sub-blocks 4c, 4c+1 and lane (c,1) the whole of 4c+2, 4c+3:
            // the half-wave swap exchanges (q, h=1) of the low lanes' tiles with (q+2, h=0).
            uint32_t out[2][4];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    auto s = __builtin_amdgcn_permlane32_swap(pk[q][j], pk[q + 2][j], false, false);
                    out[q][j] = s[0];
                    out[q][2 + j] = s[1];
                }
            }
            if (row_live) {
                uint8_t* crow = p.codes + row * (int64_t)(d >> 1) + ((tile_base + (c * kQ + 2 * h) * 32) >> 1);
                const bool ok0 = (c * kQ + 2 * h) * 32 < tile_len, ok1 = (c * kQ + 2 * h + 1) * 32 < tile_len;
                if (ok0) store_stream16(crow, make_uint4(out[0][0], out[0][1], out[0][2], out[0][3]));
                if (ok1) store_stream16(crow + 16, make_uint4(out[1][0], out[1][1], out[1][2], out[1][3]));
                if constexpr (OUT == OUT_MXFP4) {
                    if (h == 0 && qvalid[0])
                        *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(p.scales) + row * (int64_t)(d >> 5) +
                                                     (tile_base >> 5) + c * kQ) = ebytes;
                } else {
                    if (lane == 0 && tile_base == 0)
                        static_cast<float*>(p.scales)[row] = (float)((double)row_max * p.inv_7sqrt_b);
                }
            }
        }
    }
}

template <int OUT, int NWAVES>
hipError_t launch_mfma_nw(const ApplyParams& p, hipStream_t stream) {
    MfmaGeom g;
    const int tiles = (p.d + kTile - 1) / kTile;
    g.tiles_per_row = 1;
    while (g.tiles_per_row < tiles) g.tiles_per_row <<= 1;
    g.rows = NWAVES / g.tiles_per_row;
    g.row_bytes = (uint32_t)p.d * 2u;
    const uint32_t stage_bytes = (uint32_t)g.rows * g.row_bytes;
    const uint32_t slots = stage_bytes / 16u;
    g.nload = (int)((slots + NWAVES * 64u - 1u) / (NWAVES * 64u));
    g.red_off = stage_bytes;
    const uint32_t lds_bytes = stage_bytes + 64u * sizeof(float);

    auto kern = p.perm ? mfma_kernel<OUT, true, NWAVES> : mfma_kernel<OUT, false, NWAVES>;
    if (lds_bytes > 64u * 1024u) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    int per_cu = 0;
    hipError_t oe = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, NWAVES * 64, lds_bytes);
    if (oe != hipSuccess) return oe;
    if (per_cu < 1) per_cu = 1;
    const int64_t ngroups = (p.T + g.rows - 1) / g.rows;
    int64_t grid = (int64_t)launch_info().num_cus * per_cu;
    if (grid > ngroups) grid = ngroups;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NWAVES * 64), lds_bytes, stream, p, g);
    return hipGetLastError();
}

}  // namespace

bool mfma_supports(const ApplyParams& p) { return p.b <= kTile && p.d % 512 == 0 && p.d <= 32768; }

hipError_t launch_mfma(const ApplyParams& p, int out_kind, hipStream_t stream) {
    const bool wide = p.d > 4 * kTile;        // up to 8 tiles per row -> 8 waves
    switch (out_kind) {
        case OUT_INT4:
            return wide ? launch_mfma_nw<OUT_INT4, 8>(p, stream) : launch_mfma_nw<OUT_INT4, 4>(p, stream);
        case OUT_MXFP4:
            return wide ? launch_mfma_nw<OUT_MXFP4, 8>(p, stream) : launch_mfma_nw<OUT_MXFP4, 4>(p, stream);
        default:
            return wide ? launch_mfma_nw<OUT_F32, 8>(p, stream) : launch_mfma_nw<OUT_F32, 4>(p, stream);
    }
}

}  // namespace perq
