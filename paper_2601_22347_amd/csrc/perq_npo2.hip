// Rotation with a block size that is not a power of two: b = 2^k' * 28 (Appendix A.1, the
// Llama3-8B width 14336 = 2^9 * 28), then the same quantizers as the other kernels.
//
// A block of the (permuted) row is a [2^k'][28] array Z (position a*28 + r); the rotation is
// H_{2^k'} Z H_28 / sqrt(b).
//
//   1. Z H_28 and two bits of a (5 and 6) are one dense product on the MFMA unit
//      (v_mfma_f32_32x32x16_bf16): the data are the A operand, row m = a & 31, contraction
//      index k = 32 ((a >> 5) & 3) + r (r padded from 28 to 32 by zero rows of B); accumulator
//      tile n (n = 0..3: the output's bits 5, 6) takes, k-step by k-step, the base matrix or its
//      negative as B, according to H_4.  bf16 x (+-1) is exact, sums are fp32.  A lane (c, h) then holds
//      column r' = c of 16 rows per tile.  The matrix unit is nearly idle in this kernel, the
//      vector ALU is what limits it: every stage moved into the product is two VALU per element less.
//   2. The rest of the Sylvester factor: a wave owns a chunk of 128 consecutive a; a-bits
//      0,1,3,4 (accumulator index) are in-register butterflies, bit 2 (the half-wave) one swap
//      stage.  Bits 7 and up join different waves' chunks: every wave leaves its chunk in LDS
//      as fp32 in position order, and after a barrier each thread collects 16 consecutive
//      positions of every chunk of its row and finishes the remaining one or two stages in
//      registers.
//   3. In that layout (16 consecutive outputs per thread and chunk) the row statistics, the
//      rounding and the nibble packing are those of the other kernels.
//
// A workgroup of four waves handles 4 chunks per iteration: one row of d = 14336, two of 7168,
// four of 3584.  The raw rows go global -> registers (issued one iteration ahead) -> LDS; each
// chunk's bf16 data lie at the start of the fp32 area of the same chunk, which only the owning
// wave reads (P = I) before overwriting it.
#include "perq_base.h"
#include "perq_device.h"
#include "perq_launch.h"

#include <cmath>
#include <type_traits>

namespace perq {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kBase = 28;                      // rows of the base matrix
constexpr int kChunkA = 128;                   // a-values per wave chunk
constexpr int kChunkPos = kChunkA * kBase;     // 3584 positions
constexpr int kGroups = kChunkPos / 16;        // 224 runs of 16 positions per chunk
constexpr int kChunks = 4;                     // chunks per workgroup iteration
constexpr int kThreads = 256;
constexpr int kGranules = kChunks * kChunkPos * 2 / 16;   // 1792 16-byte pieces of raw input
constexpr int kPre = kGranules / kThreads;                // 7 per thread

struct Npo2Geom {
    uint32_t hrow[32];   // bit c of hrow[r]: entry (r, c) of the base matrix is -1; rows 28.. unused
    int32_t kp;          // k' = log2(b / 28)
    float norm256;       // fl32(256 / sqrt(b))
};

// NCH = chunks per row (d = NCH * 3584); rows per iteration = 4 / NCH.
// STG >= 0: the block spans whole chunks (k' = 7 + STG): all seven in-chunk stages and STG stages
// across chunks, unconditionally.  STG = -1: k' < 7 is read at run time (a stage that may or may
// not run costs a register copy per element on top of its two operations).
template <int OUT, bool PERM, int NCH, int STG>
__global__ void __launch_bounds__(kThreads, 2)
npo2_kernel(const ApplyParams p, const Npo2Geom g) {
    constexpr int kRows = kChunks / NCH;
    constexpr int kThreadsPerRow = 64 * NCH;
    constexpr int kIts = (kGroups + kThreadsPerRow - 1) / kThreadsPerRow;   // 1, 2, 4
    constexpr int kRowGranules = NCH * kChunkPos * 2 / 16;                  // 448 * NCH

    __shared__ __attribute__((aligned(16))) float ex[kChunks * kChunkPos];  // 56 KiB
    __shared__ float red[2][8];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int d = p.d;
    const int kp = STG >= 0 ? 7 + STG : g.kp;
    const int my_row = wave / NCH;          // row of the iteration this wave works on
    const int my_chunk = wave % NCH;        // chunk of that row (phase 1)
    unsigned char* const ex_bytes = reinterpret_cast<unsigned char*>(ex);

    // ---- B operand: lane (c, h) supplies r = 16 half + 8 h + e of column c; both signs -----------
    bf16x8_t bpos[2], bneg[2];
    uint32_t hrow[32];                          // (copied first: uniform values, selected by lane below)
#pragma unroll
    for (int k = 0; k < 32; ++k) hrow[k] = g.hrow[k];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            uint32_t pair = 0;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int k_lo = 16 * half + 2 * e2 + s;             // h = 0
                const int k_hi = k_lo + 8;                           // h = 1
                const uint32_t bits = h ? hrow[k_hi] : hrow[k_lo];
                const bool live = (h ? k_hi : k_lo) < kBase && c < kBase;
                const uint32_t val = live ? (((bits >> c) & 1u) ? 0xBF80u : 0x3F80u) : 0u;
                pair |= val << (16 * s);
            }
            w[e2] = pair;
        }
        bpos[half] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
        // (a zero entry stays +0 or becomes -0: either way it contributes nothing)
        bneg[half] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0] ^ 0x80008000u, w[1] ^ 0x80008000u,
                                                              w[2] ^ 0x80008000u, w[3] ^ 0x80008000u));
    }

    // ---- gather table (P != I): LDS byte address, relative to the row's first chunk, of the
    //      source channel of every A element of this lane; 16-bit, two per register ---------------
    uint32_t tab[PERM ? 32 : 1];
    if constexpr (PERM) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)          // (a >> 5) & 3
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    uint32_t pair = 0;
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const int r = 16 * kt + 8 * h + 2 * e2 + s;
                        uint32_t off = 0xFFFFu;
                        if (r < kBase) {
                            const int pos = my_chunk * kChunkPos + (32 * mt + c) * kBase + r;
                            const int ch = p.perm[pos];
                            off = (uint32_t)(ch / kChunkPos) * (uint32_t)(kChunkPos * 4) + (uint32_t)(ch % kChunkPos) * 2u;
                        }
                        pair |= off << (16 * s);
                    }
                    tab[(mt * 2 + kt) * 4 + e2] = pair;
                }
    } else {
        tab[0] = 0;
    }

    const int64_t n_units = (p.T + kRows - 1) / kRows;
    // 16-byte piece i of this thread: which row of the unit, where in the row, where in LDS.
    // Kept in registers across rows where registers are to spare (P = I), recomputed otherwise.
    constexpr bool kHoist = !PERM;
    auto piece_row = [&](int i) { return (tid + kThreads * i) / kRowGranules; };
    auto piece_goff = [&](int i) {
        const int gi = tid + kThreads * i;
        return (uint32_t)(gi / kRowGranules) * (uint32_t)(p.ldx * 2) + 16u * (uint32_t)(gi % kRowGranules);
    };
    auto piece_loff = [&](int i) {
        const int gi = tid + kThreads * i;
        return (uint32_t)(gi / (kChunkPos * 2 / 16)) * (uint32_t)(kChunkPos * 4) + 16u * (uint32_t)(gi % (kChunkPos * 2 / 16));
    };
    uint32_t g_off[kHoist ? kPre : 1], l_off[kHoist ? kPre : 1];
    if constexpr (kHoist) {
#pragma unroll
        for (int i = 0; i < kPre; ++i) {
            g_off[i] = piece_goff(i);
            l_off[i] = piece_loff(i);
        }
    } else {
        g_off[0] = 0;
        l_off[0] = 0;
    }

    auto issue_loads = [&](uint4 (&pre)[kPre], int64_t unit) {
        // rows of the unit that exist (uniform); the unit's first row as a scalar base address
        const int64_t left = p.T - unit * kRows;
        const int live = unit < n_units ? (left < kRows ? (int)left : kRows) : 0;
        const unsigned char* base = reinterpret_cast<const unsigned char*>(p.x) + unit * kRows * p.ldx * 2;
#pragma unroll
        for (int i = 0; i < kPre; ++i) {
            pre[i] = make_uint4(0, 0, 0, 0);
            if (piece_row(i) < live) pre[i] = load_stream16(base + (kHoist ? g_off[i] : piece_goff(i)));
        }
    };
    auto stage_rows = [&](const uint4 (&pre)[kPre]) {
#pragma unroll
        for (int i = 0; i < kPre; ++i)
            *reinterpret_cast<uint4*>(ex_bytes + (kHoist ? l_off[i] : piece_loff(i))) = pre[i];
    };

    // Raw rows are requested one unit ahead of their use.  (The barriers below wait for LDS only,
    // so these loads stay in flight across them; a second unit of prefetch was measured: no gain.)
    const int64_t stride = gridDim.x;
    uint4 pre[kPre];

    auto body = [&](int64_t unit) {
        workgroup_barrier_lds();                                   // raw rows of this unit are in LDS
        // ---- phase 1: base product and the in-wave stages on one chunk -------------------------
        const unsigned char* stage = ex_bytes + wave * (kChunkPos * 4);
        const unsigned char* row_stage = ex_bytes + my_row * NCH * (kChunkPos * 4);
        // afrag[al][half]: row c of A is a & 31 = c, the k-step covers (a >> 5) & 3 = al, r = 16 half + 8 h + e
        // (lane pitch 56 bytes: the 32 rows of one read fall into different banks)
        bf16x8_t afrag[4][2];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                uint32_t w[4];
                if constexpr (!PERM) {
                    const unsigned char* src = stage + ((32 * mt + c) * kBase + 16 * kt + 8 * h) * 2;
                    const uint2 lo = *reinterpret_cast<const uint2*>(src);
                    uint2 hi = *reinterpret_cast<const uint2*>(src + 8);
                    if (kt == 1 && h == 1) hi = make_uint2(0, 0);          // r = 28 .. 31 do not exist
                    w[0] = lo.x; w[1] = lo.y; w[2] = hi.x; w[3] = hi.y;
                } else {
#pragma unroll
                    for (int e2 = 0; e2 < 4; ++e2) {
                        const uint32_t pair = tab[(mt * 2 + kt) * 4 + e2];
                        const uint32_t o0 = pair & 0xFFFFu, o1 = pair >> 16;
                        const uint32_t v0 = o0 == 0xFFFFu ? 0u : *reinterpret_cast<const uint16_t*>(row_stage + o0);
                        const uint32_t v1 = o1 == 0xFFFFu ? 0u : *reinterpret_cast<const uint16_t*>(row_stage + o1);
                        w[e2] = v0 | (v1 << 16);
                    }
                }
                afrag[mt][kt] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
            }
        }

        // Accumulator tile nt collects the outputs with (a >> 5) & 3 = nt: the sum over al of
        // H[al][nt] * (Z_al H_28), H = H_4 when the block spans the whole chunk (k' >= 7),
        // I_2 (x) H_2 for k' = 6 and I_4 below.
        f32x16_t acc[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[nt] = f32x16_t{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        // keep: those of a-bits 5, 6 that lie above the block (they must agree between input and output)
        auto products = [&](auto keep_const) {
            constexpr int keep = decltype(keep_const)::value;
#pragma unroll
            for (int al = 0; al < 4; ++al) {
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    if (((al ^ nt) & keep) == 0) {
                        const bool minus = (__builtin_popcount(al & nt & ~keep) & 1) != 0;
#pragma unroll
                        for (int half = 0; half < 2; ++half)
                            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[al][half], minus ? bneg[half] : bpos[half],
                                                                              acc[nt], 0, 0, 0);
                    }
                }
            }
        };
        if (STG >= 0) products(std::integral_constant<int, 0>{});
        else if (kp == 6) products(std::integral_constant<int, 2>{});
        else products(std::integral_constant<int, 3>{});
        float v[64];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int j = 0; j < 16; ++j) v[nt * 16 + j] = acc[nt][j];
        // accumulator j of tile nt in lane (c, h): a = 32 nt + 8 (j >> 2) + 4 h + (j & 3)
        auto pair_stage = [&](int bit_in_index) {
#pragma unroll
            for (int i = 0; i < 64; ++i) {
                if ((i & bit_in_index) == 0) {
                    const float s = v[i], t = v[i | bit_in_index];
                    v[i] = s + t;
                    v[i | bit_in_index] = s - t;
                }
            }
        };
        if (STG >= 0 || kp > 0) pair_stage(1);       // a bit 0
        if (STG >= 0 || kp > 1) pair_stage(2);       // a bit 1
        if (STG >= 0 || kp > 3) pair_stage(4);       // a bit 3
        if (STG >= 0 || kp > 4) pair_stage(8);       // a bit 4
        // a bit 2 separates the half-waves.  One half-wave swap per register pair (i, i+1) hands
        // the low lanes both halves of register i and the high lanes both halves of register i+1;
        // sum and difference stay there.  Afterwards the half-wave tells a bit 0 and the slot in
        // the pair a bit 2.  Without this stage (k' <= 2) the same swap only re-sorts the values,
        // so that the addresses below hold either way.
        const bool stage2 = STG >= 0 || kp > 2;
#pragma unroll
        for (int i = 0; i < 64; i += 2) {
            auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[i]), __float_as_uint(v[i + 1]), false, false);
            const float lo = __uint_as_float(sw[0]), hi = __uint_as_float(sw[1]);
            v[i] = stage2 ? lo + hi : lo;
            v[i + 1] = stage2 ? lo - hi : hi;
        }
        if constexpr (PERM) workgroup_barrier_lds();   // every wave has gathered its operands: the chunks may be overwritten
        if (c < kBase) {
            float* dst = ex + wave * kChunkPos + h * kBase + c;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    dst[(32 * nt + 8 * (j >> 2) + 4 * (j & 1) + (j & 2)) * kBase] = v[nt * 16 + j];
        }
        workgroup_barrier_lds();                                   // all chunks of all rows are in LDS

        // ---- phase 2: 16 consecutive positions of every chunk of the row per thread ------------
        const int t_row = tid - my_row * kThreadsPerRow;
        const int64_t row = unit * kRows + my_row;
        const bool row_live = row < p.T;
        float f[kIts][NCH][16];
#pragma unroll
        for (int it = 0; it < kIts; ++it) {
            const int gI = t_row + kThreadsPerRow * it;
            const bool live = gI < kGroups;
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const float4* src = reinterpret_cast<const float4*>(ex + (my_row * NCH + ch) * kChunkPos + 16 * (live ? gI : 0));
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 t4 = src[q];
                    f[it][ch][4 * q] = t4.x; f[it][ch][4 * q + 1] = t4.y;
                    f[it][ch][4 * q + 2] = t4.z; f[it][ch][4 * q + 3] = t4.w;
                }
            }
            if constexpr (NCH >= 2) {
                if (STG >= 1) {
#pragma unroll
                    for (int ch = 0; ch < NCH; ch += 2)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const float s = f[it][ch][e], t = f[it][ch + 1][e];
                            f[it][ch][e] = s + t;
                            f[it][ch + 1][e] = s - t;
                        }
                }
            }
            if constexpr (NCH >= 4) {
                if (STG >= 2) {
#pragma unroll
                    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const float s = f[it][ch][e], t = f[it][ch + 2][e];
                            f[it][ch][e] = s + t;
                            f[it][ch + 2][e] = s - t;
                        }
                }
            }
        }

        // ---- row statistics (per-token formats) -------------------------------------------------
        constexpr bool kTokenStat = OUT == OUT_INT4 || OUT == OUT_INT4_ASYM || OUT == OUT_FP4_TOKEN;
        constexpr int kRed = OUT == OUT_INT4_ASYM ? 2 : 1;
        float m[2] = {0.0f, 0.0f};
        if constexpr (kTokenStat) {
            if constexpr (OUT == OUT_INT4_ASYM) { m[0] = -3.0e38f; m[1] = -3.0e38f; }
#pragma unroll
            for (int it = 0; it < kIts; ++it) {
                if (t_row + kThreadsPerRow * it < kGroups) {
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            if constexpr (OUT == OUT_INT4_ASYM) {
                                m[0] = fmaxf(m[0], f[it][ch][e]);
                                m[1] = fmaxf(m[1], -f[it][ch][e]);
                            } else {
                                m[0] = fmaxf(m[0], fabsf(f[it][ch][e]));
                            }
                        }
                }
            }
#pragma unroll
            for (int j = 0; j < kRed; ++j) {
                m[j] = fmaxf(m[j], lane_xor<1>(m[j]));
                m[j] = fmaxf(m[j], lane_xor<2>(m[j]));
                m[j] = fmaxf(m[j], lane_xor<4>(m[j]));
                m[j] = fmaxf(m[j], lane_xor<8>(m[j]));
                m[j] = fmaxf(m[j], lane_xor<16>(m[j]));
                m[j] = fmaxf(m[j], lane_xor<32>(m[j]));
            }
            if (lane == 0) {
#pragma unroll
                for (int j = 0; j < kRed; ++j) red[j][wave] = m[j];
            }
        }
        workgroup_barrier_lds();            // statistics visible; nobody reads the fp32 chunks any more
        stage_rows(pre);            // the next unit's raw rows
        if constexpr (!PERM) issue_loads(pre, unit + 2 * stride);
        if constexpr (kTokenStat) {
#pragma unroll
            for (int j = 0; j < kRed; ++j) {
                float t = red[j][my_row * NCH];
#pragma unroll
                for (int w = 1; w < NCH; ++w) t = fmaxf(t, red[j][my_row * NCH + w]);
                m[j] = t;
            }
        }

        // ---- quantize, pack, store ---------------------------------------------------------------
        float inv = 0.0f;
        Int4Asym qa = {0.0f, 0, false};
        if constexpr (OUT == OUT_INT4) inv = m[0] > 0.0f ? 7.0f / m[0] : 0.0f;
        if constexpr (OUT == OUT_FP4_TOKEN) inv = m[0] > 0.0f ? 6.0f / m[0] : 0.0f;
        if constexpr (OUT == OUT_INT4_ASYM) qa = int4_asym_row(-m[1], m[0]);
#pragma unroll
        for (int it = 0; it < kIts; ++it) {
            const int gI = t_row + kThreadsPerRow * it;
            if (gI < kGroups && row_live) {
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const int pos = ch * kChunkPos + 16 * gI;
                    float* val = f[it][ch];
                    if constexpr (OUT == OUT_F32) {
                        float4* yo = reinterpret_cast<float4*>(p.y + row * (int64_t)d + pos);
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            yo[q] = make_float4(val[4 * q] * p.rsqrt_b, val[4 * q + 1] * p.rsqrt_b,
                                                val[4 * q + 2] * p.rsqrt_b, val[4 * q + 3] * p.rsqrt_b);
                    } else {
                        uint32_t lo, hi;
                        if constexpr (OUT == OUT_INT4) {
                            lo = int4_pack8(val, inv);
                            hi = int4_pack8(val + 8, inv);
                        } else if constexpr (OUT == OUT_FP4_TOKEN) {
                            lo = fp4_pack8(val, inv);
                            hi = fp4_pack8(val + 8, inv);
                        } else if constexpr (OUT == OUT_INT4_ASYM) {
                            if (!qa.clamp) {
                                const uint32_t zn = (uint32_t)qa.z * 0x11111111u;
                                lo = int4a_pack8(val, qa.inv, zn);
                                hi = int4a_pack8(val + 8, qa.inv, zn);
                            } else {
                                lo = int4a_pack8_clamped(val, qa.inv, qa.z);
                                hi = int4a_pack8_clamped(val + 8, qa.inv, qa.z);
                            }
                        } else {
                            // MXFP4: values normalised by 256 / sqrt(b), so the exponent field handed to
                            // the convert is never zero; the other half of the 32-group is the
                            // neighbouring thread's run
                            float gm = 0.0f;
#pragma unroll
                            for (int e = 0; e < 16; ++e) {
                                val[e] *= g.norm256;
                                gm = fmaxf(gm, fabsf(val[e]));
                            }
                            gm = fmaxf(gm, lane_xor<1>(gm));
                            const int E = mx_shared_exponent(gm, 8);
                            const float scale = __uint_as_float((uint32_t)(E + 8) << 23);
                            lo = mxfp4_pack8(val, scale);
                            hi = mxfp4_pack8(val + 8, scale);
                            if ((gI & 1) == 0)
                                static_cast<uint8_t*>(p.scales)[row * (int64_t)(d >> 5) + (pos >> 5)] = (uint8_t)E;
                        }
                        *reinterpret_cast<uint2*>(p.codes + row * (int64_t)(d >> 1) + (pos >> 1)) = make_uint2(lo, hi);
                    }
                }
            }
        }
        if (row_live && t_row == 0) {
            if constexpr (OUT == OUT_INT4)
                static_cast<float*>(p.scales)[row] = (float)((double)m[0] * p.inv_7sqrt_b);
            if constexpr (OUT == OUT_FP4_TOKEN)
                static_cast<float*>(p.scales)[row] = (float)((double)m[0] * p.inv_6sqrt_b);
            if constexpr (OUT == OUT_INT4_ASYM)
                static_cast<float2*>(p.scales)[row] =
                    make_float2((float)((double)(m[0] + m[1]) * p.inv_15sqrt_b), (float)qa.z);
        }
        // (with a gather table held, the registers are free again only here)
        if constexpr (PERM) issue_loads(pre, unit + 2 * stride);
    };

    int64_t unit = blockIdx.x;
    issue_loads(pre, unit);
    stage_rows(pre);
    issue_loads(pre, unit + stride);
    for (; unit < n_units; unit += stride) body(unit);
}

template <int OUT, bool PERM, int NCH>
hipError_t launch_stg(const ApplyParams& p, const Npo2Geom& g, dim3 grid, hipStream_t stream) {
    const int stg = g.kp - 7;
    if (stg < 0) {
        hipLaunchKernelGGL((npo2_kernel<OUT, PERM, NCH, -1>), grid, dim3(kThreads), 0, stream, p, g);
    } else if (stg == 0) {
        hipLaunchKernelGGL((npo2_kernel<OUT, PERM, NCH, 0>), grid, dim3(kThreads), 0, stream, p, g);
    } else if constexpr (NCH >= 2) {
        if (stg == 1) {
            hipLaunchKernelGGL((npo2_kernel<OUT, PERM, NCH, 1>), grid, dim3(kThreads), 0, stream, p, g);
        } else if constexpr (NCH >= 4) {
            hipLaunchKernelGGL((npo2_kernel<OUT, PERM, NCH, 2>), grid, dim3(kThreads), 0, stream, p, g);
        } else {
            return hipErrorInvalidValue;
        }
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int OUT, bool PERM>
hipError_t launch_nch(const ApplyParams& p, const Npo2Geom& g, int nch, dim3 grid, hipStream_t stream) {
    switch (nch) {
        case 1: return launch_stg<OUT, PERM, 1>(p, g, grid, stream);
        case 2: return launch_stg<OUT, PERM, 2>(p, g, grid, stream);
        default: return launch_stg<OUT, PERM, 4>(p, g, grid, stream);
    }
}

template <int OUT>
hipError_t launch_perm(const ApplyParams& p, const Npo2Geom& g, int nch, dim3 grid, hipStream_t stream) {
    return p.perm != nullptr ? launch_nch<OUT, true>(p, g, nch, grid, stream)
                             : launch_nch<OUT, false>(p, g, nch, grid, stream);
}

}  // namespace

bool npo2_supports(const ApplyParams& p) {
    if (p.d != kChunkPos && p.d != 2 * kChunkPos && p.d != 4 * kChunkPos) return false;
    if (p.b % kBase != 0) return false;
    const int32_t a = p.b / kBase;
    // row offsets inside a unit of up to four rows are kept in 32 bits
    return a > 0 && (a & (a - 1)) == 0 && p.d % p.b == 0 && p.ldx < ((int64_t)1 << 28);
}

hipError_t launch_npo2(const ApplyParams& p, int out_kind, hipStream_t stream) {
    Npo2Geom g;
    const int kind = hadamard_base_kind(kBase);
    for (int r = 0; r < 32; ++r) {
        uint32_t bits = 0;
        if (r < kBase)
            for (int c = 0; c < kBase; ++c)
                if (hadamard_base_entry(kBase, kind, r, c) < 0) bits |= 1u << c;
        g.hrow[r] = bits;
    }
    g.kp = 0;
    while ((kBase << g.kp) < p.b) ++g.kp;
    g.norm256 = (float)(256.0 / std::sqrt((double)p.b));
    const int nch = p.d / kChunkPos;
    const int64_t rows_per_unit = kChunks / nch;
    const int64_t n_units = (p.T + rows_per_unit - 1) / rows_per_unit;
    const int64_t max_grid = 2 * (int64_t)launch_info().num_cus;
    const dim3 grid((unsigned)(n_units < max_grid ? n_units : max_grid));
    switch (out_kind) {
        case OUT_INT4: return launch_perm<OUT_INT4>(p, g, nch, grid, stream);
        case OUT_MXFP4: return launch_perm<OUT_MXFP4>(p, g, nch, grid, stream);
        case OUT_INT4_ASYM: return launch_perm<OUT_INT4_ASYM>(p, g, nch, grid, stream);
        case OUT_FP4_TOKEN: return launch_perm<OUT_FP4_TOKEN>(p, g, nch, grid, stream);
        case OUT_F32: return launch_perm<OUT_F32>(p, g, nch, grid, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace perq
