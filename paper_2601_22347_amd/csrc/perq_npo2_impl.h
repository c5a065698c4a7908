// Rotation with a block size that is not a power of two: b = 2^k' * MB, MB = 4t the order of the
// base matrix (Appendix A.1: 28 for the Llama3-8B width 14336 = 2^9 * 28; 12 and 76 for the Qwen3
// widths), then the same quantizers as the other kernels.  With Sylvester's H_32 in the place of the
// base the same kernel takes power-of-two blocks above 4096.  One translation unit per MB includes
// this file and instantiates launch_npo2_base_impl<MB>.
//
// A block of the (permuted) row is a [2^k'][MB] array Z (position a*MB + r); the rotation is
// H_{2^k'} Z H_MB / sqrt(b).
//
//   1. Z H_MB is a dense product on the MFMA unit (v_mfma_f32_32x32x16_bf16): the data are the A
//      operand, the +-1 base matrix is B; bf16 x (+-1) is exact, sums are fp32.  The contraction
//      index also takes those bits of a that cost nothing extra there (see Base<MB>): the matrix
//      unit is far from busy in this kernel, the vector ALU is what limits it, and every stage
//      moved into the product is two VALU per element less.  A lane (c, h) then holds one column
//      of 16 rows per accumulator tile.
//   2. The rest of the Sylvester factor inside a wave's chunk: the a-bits held in the accumulator
//      index are in-register butterflies, the bit that separates the half-waves is one swap stage.
//      Bits above the chunk join different waves' chunks: every wave leaves its chunk in LDS as
//      fp32 in position order (for the bases 28 and 32 one half of it at a time, so that the exchange
//      area is no larger than the raw rows and three workgroups stay resident), and after a barrier
//      each thread collects 8 consecutive positions of every chunk of its row and finishes the
//      remaining one to three stages in registers.
//   3. In that layout (8 consecutive outputs per thread and chunk: one dword of codes) the row
//      statistics, the rounding and the nibble packing are those of the other kernels.
//
// A workgroup of four waves handles 4 chunks per iteration: one row of 4 chunks, two of 2, four of 1;
// rows of 8 chunks (d = 28672 and 32768 for the bases 28 and 32) take workgroups of eight waves.
// The raw rows go global -> registers (issued one iteration ahead) -> LDS; each chunk's bf16 data
// lie at the start of the fp32 area of the same chunk; the owning wave puts them there and, without
// a gather, is the only one to read them before it overwrites them: two barriers per row (four
// where the chunks go through LDS in two halves).
#pragma once
#include "perq_base.h"
#include "perq_device.h"
#include "perq_launch.h"

#include <cmath>
#include <type_traits>

namespace perq {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// How one base order maps onto 32x32x16 products.  Rows of A are 32 values of a; a k-step holds 16
// contraction indices, lane (c, h) supplying 8 h .. 8 h + 7 of them.
//   kA0  a-values side by side in the 32 output columns (2: column c = 16 (a & 1) + r', and the
//        two k-steps of a product are a & 1 = 0, 1: bit 0 of a is part of the product)
//   kKS  k-steps that cover r (kA0 = 1) or a & 1 (kA0 = 2)
//   kNT  column tiles of 32 that cover r'
//   kAL  row tiles of one chunk that are contracted against each other (4: two more bits of a in
//        the product, the k-steps of tile al entering output tile al' with the sign of H_4)
template <int MB> struct Base;
template <> struct Base<28> { static constexpr int kA0 = 1, kKS = 2, kNT = 1, kAL = 4; };
template <> struct Base<12> { static constexpr int kA0 = 2, kKS = 2, kNT = 1, kAL = 4; };
template <> struct Base<76> { static constexpr int kA0 = 1, kKS = 5, kNT = 3, kAL = 1; };
// Sylvester's H_32 as the base: power-of-two blocks above what the 4096-wide tiles of the other
// matrix-core kernel hold (b = 8192 .. 32768 on d = 8192, 16384, 32768) take the same path.
template <> struct Base<32> { static constexpr int kA0 = 1, kKS = 2, kNT = 1, kAL = 4; };

// Waves per workgroup = chunks per workgroup iteration: four, or eight for rows of eight chunks.
constexpr int npo2_waves(int nch) { return nch == 8 ? 8 : 4; }

template <int MB>
struct Npo2Geom {
    uint32_t hrow[16 * (Base<MB>::kA0 == 2 ? 1 : Base<MB>::kKS)][Base<MB>::kNT];   // bit c of word w of row r: entry (r, 32 w + c) is -1
    int32_t kp;          // k' = log2(b / MB)
    float norm256;       // fl32(256 / sqrt(b))
};

// NCH = chunks per row (1, 2, 4, 8); rows per iteration = waves / NCH.
// STG >= 0: the block spans whole chunks: every in-chunk stage and STG stages across chunks,
// unconditionally.  STG = -1: a smaller block, k' is read at run time (a stage that may or may
// not run costs a register copy per element on top of its two operations).
template <int OUT, bool PERM, int MB, int NCH, int STG>
__global__ void __launch_bounds__(64 * npo2_waves(NCH), NCH == 8 ? 1 : 2)
npo2_kernel(const ApplyParams p, const Npo2Geom<MB> g) {
    using B = Base<MB>;
    constexpr int kA0 = B::kA0, kKS = B::kKS, kNT = B::kNT, kAL = B::kAL;
    constexpr int kSh = kA0 == 2 ? 1 : 0;                 // a-bit of row bit 0 of a product
    constexpr int kColMask = 32 / kA0 - 1;                // column -> r' inside a tile
    constexpr int kTileA = 32 * kA0;                      // a-values per row tile
    constexpr int kChunkA = kTileA * kAL;                 // a-values per wave chunk: 128, 256, 32
    constexpr int kChunkBits = (kChunkA == 32 ? 5 : (kChunkA == 128 ? 7 : 8));
    constexpr int kChunkPos = kChunkA * MB;               // 3584, 3072, 2432; 4096 for H_32
    // consecutive positions per thread and chunk in phase 2 (16 was measured too: no faster where
    // it fills every lane, and slower with a gather table in registers)
    constexpr int kRun = 8;
    constexpr int kGroups = kChunkPos / kRun;             // runs per chunk
    constexpr int kChunkGranules = kChunkPos * 2 / 16;    // 16-byte pieces of raw input per chunk
    constexpr int kPre = (kChunkGranules + 63) / 64;      // pieces per lane: every wave stages its own chunk
    constexpr bool kPreExact = kChunkGranules % 64 == 0;
    constexpr int kTiles = kAL * kNT;                     // accumulator tiles per lane
    constexpr int kVals = 16 * kTiles;
    constexpr int kNpo2Chunks = npo2_waves(NCH);
    constexpr int kRows = kNpo2Chunks / NCH;
    constexpr int kThreadsPerRow = 64 * NCH;
    // The chunks go through LDS in kRounds parts (a part = the row tiles 0, 1 or 2, 3 of every chunk, a
    // contiguous half of its positions): the exchange area holds one part of every chunk, which is
    // also the size of a chunk's raw bf16 data, and a third workgroup fits beside two
    // (d = b = 14336: 275 -> 262 us).
    // (one part where four whole chunks already leave room for three workgroups, the base 12: the two
    //  extra barriers per row cost 1 % there; and for rows of eight chunks, whose workgroups of eight
    //  waves are alone on a CU by their registers and would idle half their threads in every part)
    constexpr int kRounds = (kAL == 4 && NCH <= 4 && 4 * kChunkPos * 4 > 160 * 1024 / 3) ? 2 : 1;
    constexpr int kAreaPos = kChunkPos / kRounds;         // positions of a chunk in LDS at a time
    constexpr int kGroupsR = kGroups / kRounds;           // runs per chunk and part
    constexpr int kItsR = (kGroupsR + kThreadsPerRow - 1) / kThreadsPerRow;
    constexpr int kIts = kRounds * kItsR;
    static_assert(kGroups % kRounds == 0 && kGroupsR % 4 == 0, "a part holds whole 32-groups and whole quads of runs");
    // (a run of 8 is one dword of codes; where runs of 16 would leave 12 .. 40 % of the lanes of every
    //  wave idle in the last pass, whole waves skip it with runs of 8 instead)
    static_assert(kGroups % (32 / kRun) == 0 && kChunkPos % 32 == 0, "a 32-group is two or four neighbouring threads' runs");
    // MB = 32: a row of the A operand is 64 bytes, so rows four apart would share their banks.  The
    // 16-byte piece q of row a is kept at piece q ^ ((a >> 2) & 3) of the row instead (raw data only).
    constexpr bool kSwz = MB == 32;

    __shared__ __attribute__((aligned(16))) float ex[kNpo2Chunks * kAreaPos];
    __shared__ float red[2][8];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int d = p.d;
    const int kp = STG >= 0 ? kChunkBits + STG : g.kp;
    const int my_row = wave / NCH;          // row of the iteration this wave works on
    const int my_chunk = wave % NCH;        // chunk of that row (phase 1)
    unsigned char* const ex_bytes = reinterpret_cast<unsigned char*>(ex);

    // index r of the base matrix that element e of k-step ks holds in this lane
    auto r_of = [&](int ks, int e) { return (kA0 == 2 ? 0 : 16 * ks) + 8 * h + e; };

    // ---- B operand: lane (c, h) supplies column c, both signs where tiles are contracted ---------
    bf16x8_t bpos[kNT][kKS], bneg[kAL > 1 ? kNT : 1][kAL > 1 ? kKS : 1];
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt) {
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {
            uint32_t w[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                uint32_t pair = 0;
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int e = 2 * e2 + s;
                    const int r_lo = (kA0 == 2 ? 0 : 16 * ks) + e, r_hi = r_lo + 8;     // h = 0, 1
                    const uint32_t bits = h ? g.hrow[r_hi][nt] : g.hrow[r_lo][nt];
                    const int rr = h ? r_hi : r_lo;
                    const int rc = 32 * nt + (c & kColMask);                             // r'
                    uint32_t val = (rr < MB && rc < MB) ? (((bits >> (c & kColMask)) & 1u) ? 0xBF80u : 0x3F80u) : 0u;
                    if constexpr (kA0 == 2) {
                        // H_2 between the a & 1 of the k-step and the a & 1 of the column; the identity
                        // when bit 0 of a lies above the block (k' = 0)
                        const int a_in = ks, a_out = c >> 4;
                        if (kp > 0) val ^= (a_in & a_out) ? 0x8000u : 0u;
                        else if (a_in != a_out) val = 0u;
                        if (val == 0x8000u) val = 0u;
                    }
                    pair |= val << (16 * s);
                }
                w[e2] = pair;
            }
            bpos[nt][ks] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
            if constexpr (kAL > 1)      // (a zero entry stays +0 or becomes -0: either way it contributes nothing)
                bneg[nt][ks] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0] ^ 0x80008000u, w[1] ^ 0x80008000u,
                                                                       w[2] ^ 0x80008000u, w[3] ^ 0x80008000u));
        }
    }

    // a inside the chunk of row c of tile al, k-step ks
    auto a_of = [&](int al, int ks) { return kTileA * al + kA0 * c + (kA0 == 2 ? ks : 0); };

    // ---- gather table (P != I): LDS byte address, relative to the row's first chunk, of the
    //      source channel of every A element of this lane; 16-bit (halved), two per register ------
    constexpr int kTab = kAL * kKS * 4;
    uint32_t tab[PERM ? kTab : 1];
    if constexpr (PERM) {
#pragma unroll
        for (int al = 0; al < kAL; ++al)
#pragma unroll
            for (int ks = 0; ks < kKS; ++ks)
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    uint32_t pair = 0;
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        // (an index past the end of the base meets a zero row of B: it is pointed at the
                        //  a-value's first element, finite like all input, so that every read below is
                        //  unconditional)
                        const int r = r_of(ks, 2 * e2 + s);
                        const int pos = my_chunk * kChunkPos + a_of(al, ks) * MB + (r < MB ? r : 0);
                        const int ch = p.perm[pos];
                        const uint32_t cl = (uint32_t)(ch % kChunkPos);
                        // (in units of two bytes: eight chunks of fp32 pass 64 KiB)
                        const uint32_t off = (uint32_t)(ch / kChunkPos) * (uint32_t)(kAreaPos * 2) +
                                             (kSwz ? ((cl >> 5) * 4u + (((cl >> 3) & 3u) ^ ((cl >> 7) & 3u))) * 8u + (cl & 7u) : cl);
                        pair |= off << (16 * s);
                    }
                    tab[(al * kKS + ks) * 4 + e2] = pair;
                }
    } else {
        tab[0] = 0;
    }

    const int64_t n_units = (p.T + kRows - 1) / kRows;
    // Every wave loads and stages the raw data of its own chunk (16-byte piece lane + 64 i of the
    // chunk's 2 * kChunkPos bytes), so without a gather nobody else's data are needed in phase 1.
    auto piece_live = [&](int i) { return kPreExact || i + 1 < kPre || lane + 64 * i < kChunkGranules; };
    const uint32_t g_base = (uint32_t)my_row * (uint32_t)(p.ldx * 2) + (uint32_t)my_chunk * (uint32_t)(kChunkPos * 2) + 16u * (uint32_t)lane;
    // (swizzled: piece lane + 64 i belongs to row (lane >> 2) + 16 i, whose bits 2, 3 are those of lane >> 4)
    unsigned char* const l_base = ex_bytes + wave * (kAreaPos * 4) +
                                  16 * (kSwz ? ((lane & ~3) | ((lane & 3) ^ ((lane >> 4) & 3))) : lane);

    auto issue_loads = [&](uint4 (&pre)[kPre], int64_t unit) {
        // the unit's first row as a scalar base address; rows past the end are read as zeros
        const bool live = unit < n_units && unit * kRows + my_row < p.T;
        const unsigned char* base = reinterpret_cast<const unsigned char*>(p.x) + unit * kRows * p.ldx * 2 + g_base;
        // (one test per unit, not a cleared register set per load)
        if (live) {
#pragma unroll
            for (int i = 0; i < kPre; ++i) {
                if (piece_live(i)) pre[i] = load_stream16(base + 1024 * i);
                else pre[i] = make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kPre; ++i) pre[i] = make_uint4(0, 0, 0, 0);
        }
    };
    auto stage_rows = [&](const uint4 (&pre)[kPre]) {
#pragma unroll
        for (int i = 0; i < kPre; ++i)
            if (piece_live(i)) *reinterpret_cast<uint4*>(l_base + 1024 * i) = pre[i];
    };

    // Raw rows are requested one unit ahead of their use.  (The barriers below wait for LDS only,
    // so these loads stay in flight across them; a second unit of prefetch was measured: no gain.)
    const int64_t stride = gridDim.x;
    uint4 pre[kPre];

    auto body = [&](int64_t unit) {
        if constexpr (PERM) workgroup_barrier_lds();               // the gather reads other waves' chunks too
        // ---- phase 1: base product and the in-wave stages on one chunk -------------------------
        const unsigned char* stage = ex_bytes + wave * (kAreaPos * 4);
        const unsigned char* row_stage = ex_bytes + my_row * NCH * (kAreaPos * 4);
        bf16x8_t afrag[kAL][kKS];
#pragma unroll
        for (int al = 0; al < kAL; ++al) {
#pragma unroll
            for (int ks = 0; ks < kKS; ++ks) {
                uint32_t w[4];
                if constexpr (!PERM) {
                    // 8 consecutive r of one a: two 8-byte reads (the pitch between lanes is MB * kA0 * 2
                    // bytes: 56, 48 or 152, so the 32 rows of a read fall into different banks)
                    const unsigned char* src =
                        kSwz ? stage + a_of(al, ks) * 64 + (((2 * ks + h) ^ ((c >> 2) & 3)) * 16)
                             : stage + (a_of(al, ks) * MB + r_of(ks, 0)) * 2;
                    const uint2 lo = *reinterpret_cast<const uint2*>(src);
                    uint2 hi = *reinterpret_cast<const uint2*>(src + 8);
                    if (r_of(ks, 4) >= MB) hi = make_uint2(0, 0);          // past the end of the base
                    w[0] = lo.x; w[1] = lo.y; w[2] = hi.x; w[3] = hi.y;
                } else {
#pragma unroll
                    for (int e2 = 0; e2 < 4; ++e2) {
                        const uint32_t pair = tab[(al * kKS + ks) * 4 + e2];
                        const uint32_t o0 = pair & 0xFFFFu, o1 = pair >> 16;
                        const uint32_t v0 = *reinterpret_cast<const uint16_t*>(row_stage + 2u * o0);
                        const uint32_t v1 = *reinterpret_cast<const uint16_t*>(row_stage + 2u * o1);
                        w[e2] = v0 | (v1 << 16);
                    }
                }
                afrag[al][ks] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
            }
        }

        // Accumulator tile (al', nt): outputs whose a lies in row tile al', columns 32 nt ..: the sum
        // over al of H[al][al'] * (Z_al H_MB), H = H_4 when the block spans the whole chunk,
        // I_2 (x) H_2 when it spans half of it, I_4 below.
        // The products of one output tile at a time, and the in-register stages of a tile while the
        // matrix unit works on the next one: a wave issues in order, so the stages' instructions are
        // placed between the products (one product keeps the unit busy for about as long as eight
        // vector instructions take).
        float v[kVals];
        // accumulator j of tile (al', nt) in lane (c, h): row m = 8 (j >> 2) + 4 h + (j & 3) of the
        // product, a = kTileA al' + kA0 m (+ c >> 4 when kA0 = 2); row bit q is a-bit q + kSh
        const bool stage2 = STG >= 0 || kp > kSh + 2;
        auto tile_stages = [&](int t) {
            float* w = v + 16 * t;
            auto pair_stage = [&](int bit_in_index) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if ((i & bit_in_index) == 0) {
                        const float s = w[i], u = w[i | bit_in_index];
                        w[i] = s + u;
                        w[i | bit_in_index] = s - u;
                    }
                }
            };
            if (STG >= 0 || kp > kSh + 0) pair_stage(1);       // row bit 0
            if (STG >= 0 || kp > kSh + 1) pair_stage(2);       // row bit 1
            if (STG >= 0 || kp > kSh + 3) pair_stage(4);       // row bit 3
            if (STG >= 0 || kp > kSh + 4) pair_stage(8);       // row bit 4
            // Row bit 2 separates the half-waves.  One half-wave swap per register pair (i, i+1) hands
            // the low lanes both halves of register i and the high lanes both halves of register i+1;
            // sum and difference stay there.  Afterwards the half-wave tells row bit 0 and the slot in
            // the pair row bit 2.  Without this stage the same swap only re-sorts the values, so that
            // the addresses below hold either way.
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(w[i]), __float_as_uint(w[i + 1]), false, false);
                const float lo = __uint_as_float(sw[0]), hi = __uint_as_float(sw[1]);
                w[i] = stage2 ? lo + hi : lo;
                w[i + 1] = stage2 ? lo - hi : hi;
            }
        };
        // Accumulator tile (al', nt): outputs whose a lies in row tile al', columns 32 nt ..: the sum
        // over al of H[al][al'] * (Z_al H_MB), H = H_4 when the block spans the whole chunk,
        // I_2 (x) H_2 when it spans half of it, I_4 below.
        // keep: those of the two tile bits that lie above the block (they must agree between input and output)
        auto phase1 = [&](auto keep_const) {
            constexpr int keep = decltype(keep_const)::value;
#pragma unroll
            for (int t = 0; t < kTiles; ++t) {
                const int ao = t / kNT, nt = t % kNT;
                f32x16_t acc = f32x16_t{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int al = 0; al < kAL; ++al) {
                    if (((al ^ ao) & keep) == 0) {
                        const bool minus = (__builtin_popcount(al & ao & ~keep) & 1) != 0;
#pragma unroll
                        for (int ks = 0; ks < kKS; ++ks) {
                            if constexpr (kAL > 1)
                                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[al][ks], minus ? bneg[nt][ks] : bpos[nt][ks], acc, 0, 0, 0);
                            else
                                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[al][ks], bpos[nt][ks], acc, 0, 0, 0);
                        }
                    }
                }
                if (t > 0) tile_stages(t - 1);
#pragma unroll
                for (int j = 0; j < 16; ++j) v[t * 16 + j] = acc[j];
                // one product, then a share of the stage's instructions, until the tile's products are out
                constexpr int kProducts = kAL > 1 ? (keep == 0 ? kAL : (keep == 3 ? 1 : 2)) * kKS : kKS;
                if (t > 0) {
#pragma unroll
                    for (int i = 0; i < kProducts; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one matrix instruction
                        __builtin_amdgcn_sched_group_barrier(0x002, 96 / kProducts, 0);          // vector instructions
                    }
                }
            }
            tile_stages(kTiles - 1);
        };
        if (kAL == 1 || STG >= 0) phase1(std::integral_constant<int, 0>{});
        else if (kp == kChunkBits - 1) phase1(std::integral_constant<int, 2>{});
        else phase1(std::integral_constant<int, 3>{});
        // ---- the chunks through LDS, a part at a time; phase 2: runs of kRun = 8 consecutive positions
        //      of every chunk of the row per thread ---------------------------------------------------
        const int t_row = tid - my_row * kThreadsPerRow;
        const int64_t row = unit * kRows + my_row;
        const bool row_live = row < p.T;
        // pass `it` of a thread: run gI of every chunk (run_live: the thread has one in this pass)
        auto run_live = [&](int it) { return t_row + kThreadsPerRow * (it % kItsR) < kGroupsR; };
        auto run_of = [&](int it) { return (it / kItsR) * kGroupsR + t_row + kThreadsPerRow * (it % kItsR); };
        float f[kIts][NCH][kRun];
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            // r = 0: every wave has gathered its operands (the raw chunks may be overwritten);
            // r = 1: every thread has read its runs of the first part
            if (PERM || r > 0) workgroup_barrier_lds();
            {
                const int rl = c & kColMask;                // r' inside a column tile
                float* dst = ex + wave * kAreaPos + (kA0 * h + (kA0 == 2 ? (c >> 4) : 0)) * MB + rl;
#pragma unroll
                for (int ao = r * (kAL / kRounds); ao < (r + 1) * (kAL / kRounds); ++ao)
#pragma unroll
                    for (int nt = 0; nt < kNT; ++nt) {
                        if (32 * nt + rl < MB) {
#pragma unroll
                            for (int j = 0; j < 16; ++j)
                                dst[(kTileA * (ao - r * (kAL / kRounds)) + kA0 * (8 * (j >> 2) + 4 * (j & 1) + (j & 2))) * MB + 32 * nt] =
                                    v[(ao * kNT + nt) * 16 + j];
                        }
                    }
            }
            workgroup_barrier_lds();                                   // this part of all chunks of all rows is in LDS
#pragma unroll
            for (int it = r * kItsR; it < (r + 1) * kItsR; ++it) {
                const int gl = t_row + kThreadsPerRow * (it - r * kItsR);     // run inside the part
                const bool live = gl < kGroupsR;
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const float4* src = reinterpret_cast<const float4*>(ex + (my_row * NCH + ch) * kAreaPos + kRun * (live ? gl : 0));
#pragma unroll
                    for (int q = 0; q < kRun / 4; ++q) {
                        const float4 t4 = src[q];
                        f[it][ch][4 * q] = t4.x; f[it][ch][4 * q + 1] = t4.y;
                        f[it][ch][4 * q + 2] = t4.z; f[it][ch][4 * q + 3] = t4.w;
                    }
                }
                // stages across chunks: bit s of the chunk index, s < STG
#pragma unroll
                for (int sb = 0; sb < 3; ++sb) {
                    if (sb < STG && (2 << sb) <= NCH) {
#pragma unroll
                        for (int ch = 0; ch < NCH; ++ch) {
                            if ((ch & (1 << sb)) == 0) {
#pragma unroll
                                for (int e = 0; e < kRun; ++e) {
                                    const float s = f[it][ch][e], t = f[it][ch | (1 << sb)][e];
                                    f[it][ch][e] = s + t;
                                    f[it][ch | (1 << sb)][e] = s - t;
                                }
                            }
                        }
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
                if (run_live(it)) {
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
                        for (int e = 0; e < kRun; ++e) {
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
                m[j] = lane_max<1>(m[j]);
                m[j] = lane_max<2>(m[j]);
                m[j] = lane_max<4>(m[j]);
                m[j] = lane_max<8>(m[j]);
                m[j] = lane_max<16>(m[j]);
                m[j] = lane_max<32>(m[j]);
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
        if constexpr (kTokenStat) {
            float hi = m[0], lo = OUT == OUT_INT4_ASYM ? -m[1] : 0.0f;
            if (tiny_row(hi - lo)) {
#pragma unroll
                for (int it = 0; it < kIts; ++it) {
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) lift_values(f[it][ch]);
                }
                hi *= kTinyRowLift;
                lo *= kTinyRowLift;
            }
            if constexpr (OUT == OUT_INT4) inv = hi > 0.0f ? 7.0f / hi : 0.0f;
            if constexpr (OUT == OUT_FP4_TOKEN) inv = hi > 0.0f ? p.fp4_qmax / hi : 0.0f;
            if constexpr (OUT == OUT_INT4_ASYM) qa = int4_asym_row(lo, hi);
        }
        // Rows of four chunks with 4-bit codes: a thread's four dwords of one pass belong to four chunks,
        // those of the four threads of a quad to four consecutive runs of each.  A 4 x 4 transposition
        // inside the quad (two exchange steps) hands thread q the 16 consecutive bytes of chunk q, so a
        // pass ends in one 16-byte store per thread instead of four 4-byte ones.
        constexpr bool kQuadStore = NCH == 4 && OUT != OUT_F32 && kRun == 8;
#pragma unroll
        for (int it = 0; it < kIts; ++it) {
            const int gI = run_of(it);
            uint32_t wq[kQuadStore ? 4 : 1];
            if (run_live(it) && row_live) {
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const int pos = ch * kChunkPos + kRun * gI;
                    float* val = f[it][ch];
                    if constexpr (OUT == OUT_F32) {
                        float4* yo = reinterpret_cast<float4*>(p.y + row * (int64_t)d + pos);
#pragma unroll
                        for (int q = 0; q < kRun / 4; ++q)
                            yo[q] = make_float4(val[4 * q] * p.rsqrt_b, val[4 * q + 1] * p.rsqrt_b,
                                                val[4 * q + 2] * p.rsqrt_b, val[4 * q + 3] * p.rsqrt_b);
                    } else {
                        uint32_t w[kRun / 8];
                        if constexpr (OUT == OUT_MXFP4) {
                            // values normalised by 256 / sqrt(b), so the exponent field handed to the
                            // convert is never zero; the rest of the 32-group are the runs of the
                            // neighbouring threads
                            float gm = 0.0f;
#pragma unroll
                            for (int e = 0; e < kRun; ++e) {
                                val[e] *= g.norm256;
                                gm = fmaxf(gm, fabsf(val[e]));
                            }
                            gm = lane_max<1>(gm);
                            if constexpr (kRun == 8) gm = lane_max<2>(gm);
                            const int E = mx_shared_exponent(gm, 8);
                            const float scale = __uint_as_float((uint32_t)(E + 8) << 23);
#pragma unroll
                            for (int k = 0; k < kRun / 8; ++k) w[k] = mxfp4_pack8(val + 8 * k, scale);
                            if ((gI & (32 / kRun - 1)) == 0)
                                static_cast<uint8_t*>(p.scales)[row * (int64_t)(d >> 5) + (pos >> 5)] = (uint8_t)E;
                        } else {
#pragma unroll
                            for (int k = 0; k < kRun / 8; ++k) {
                                if constexpr (OUT == OUT_INT4) {
                                    w[k] = int4_pack8(val + 8 * k, inv);
                                } else if constexpr (OUT == OUT_FP4_TOKEN) {
                                    w[k] = fp4_pack8(val + 8 * k, inv);
                                } else {
                                    if (qa.mode == 0) w[k] = int4a_pack8(val + 8 * k, qa.inv, (uint32_t)qa.z * 0x11111111u);
                                    else w[k] = int4a_pack8_clamped(val + 8 * k, qa);
                                }
                            }
                        }
                        if constexpr (kQuadStore) {
                            wq[ch] = w[0];
                        } else {
                            uint8_t* dst = p.codes + row * (int64_t)(d >> 1) + (pos >> 1);
                            if constexpr (kRun == 16) *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
                            else *reinterpret_cast<uint32_t*>(dst) = w[0];
                        }
                    }
                }
                if constexpr (kQuadStore) {
                    // (the threads of a quad are live together: kGroups is a multiple of 4 and so is a row's first thread)
                    const int q = lane & 3;
                    auto exchange = [&](uint32_t& keep_lo, uint32_t& keep_hi, bool upper, auto ctrl) {
                        // the thread with the lower number keeps lo and receives the partner's lo in hi's place
                        const uint32_t give = upper ? keep_lo : keep_hi;
                        const uint32_t got = (uint32_t)__builtin_amdgcn_update_dpp((int)give, (int)give, decltype(ctrl)::value, 0xF, 0xF, false);
                        if (upper) keep_lo = got; else keep_hi = got;
                    };
                    exchange(wq[0], wq[1], (q & 1) != 0, std::integral_constant<int, 0xB1>{});     // quad_perm [1,0,3,2]
                    exchange(wq[2], wq[3], (q & 1) != 0, std::integral_constant<int, 0xB1>{});
                    exchange(wq[0], wq[2], (q & 2) != 0, std::integral_constant<int, 0x4E>{});     // quad_perm [2,3,0,1]
                    exchange(wq[1], wq[3], (q & 2) != 0, std::integral_constant<int, 0x4E>{});
                    // thread q now holds chunk q's dwords of runs gI - q .. gI - q + 3
                    uint8_t* dst = p.codes + row * (int64_t)(d >> 1) + ((q * kChunkPos + kRun * (gI - q)) >> 1);
                    store_stream16(dst, make_uint4(wq[0], wq[1], wq[2], wq[3]));
                }
            }
        }
        if (row_live && t_row == 0) {
            if constexpr (OUT == OUT_INT4)
                static_cast<float*>(p.scales)[row] = (float)((double)m[0] * p.inv_7sqrt_b);
            if constexpr (OUT == OUT_FP4_TOKEN)
                static_cast<float*>(p.scales)[row] = (float)((double)m[0] * p.inv_fp4sqrt_b);
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

template <int MB>
constexpr int npo2_chunk_pos() { return 32 * Base<MB>::kA0 * Base<MB>::kAL * MB; }
template <int MB>
constexpr int npo2_chunk_bits() { return Base<MB>::kAL == 1 ? 5 : (Base<MB>::kA0 == 1 ? 7 : 8); }

// Entry (r, c) of the base: Sylvester's matrix for 32, Paley's constructions otherwise.
template <int MB>
int base_entry(int kind, int r, int c) {
    if constexpr (MB == 32) return (__builtin_popcount((unsigned)(r & c)) & 1) ? -1 : 1;
    else return hadamard_base_entry(MB, kind, r, c);
}

// A persistent grid: as many workgroups as stay resident (two per CU by the size of the fp32 exchange
// area for the bases 28 and 32, three for the smaller chunks of 12 and 76 where the registers allow).
template <class Kern, int MB>
hipError_t launch_resident(Kern kern, int threads, const ApplyParams& p, const Npo2Geom<MB>& g, int64_t n_units, hipStream_t stream) {
    int per_cu = 0;
    const hipError_t e = resident_blocks(reinterpret_cast<const void*>(kern), threads, 0, &per_cu);
    if (e != hipSuccess) return e;
    const int64_t max_grid = (int64_t)per_cu * launch_info().num_cus;
    hipLaunchKernelGGL(kern, dim3((unsigned)(n_units < max_grid ? n_units : max_grid)), dim3(threads), 0, stream, p, g);
    return hipGetLastError();
}

template <int OUT, bool PERM, int MB, int NCH>
hipError_t launch_stg(const ApplyParams& p, const Npo2Geom<MB>& g, int64_t n_units, hipStream_t stream) {
    const int stg = g.kp - npo2_chunk_bits<MB>();
    constexpr int threads = 64 * npo2_waves(NCH);
    if (stg < 0) return launch_resident(npo2_kernel<OUT, PERM, MB, NCH, -1>, threads, p, g, n_units, stream);
    if (stg == 0) return launch_resident(npo2_kernel<OUT, PERM, MB, NCH, 0>, threads, p, g, n_units, stream);
    if constexpr (NCH >= 2) {
        if (stg == 1) return launch_resident(npo2_kernel<OUT, PERM, MB, NCH, 1>, threads, p, g, n_units, stream);
    }
    if constexpr (NCH >= 4) {
        if (stg == 2) return launch_resident(npo2_kernel<OUT, PERM, MB, NCH, 2>, threads, p, g, n_units, stream);
    }
    if constexpr (NCH >= 8) {
        if (stg == 3) return launch_resident(npo2_kernel<OUT, PERM, MB, NCH, 3>, threads, p, g, n_units, stream);
    }
    return hipErrorInvalidValue;
}

// Rows of eight chunks (d = 28672, 32768) exist for the bases 28 and 32 only.
template <int MB>
constexpr bool npo2_has_eight() { return MB == 28 || MB == 32; }

template <int OUT, bool PERM, int MB>
hipError_t launch_nch(const ApplyParams& p, const Npo2Geom<MB>& g, int nch, int64_t n_units, hipStream_t stream) {
    switch (nch) {
        case 1: return launch_stg<OUT, PERM, MB, 1>(p, g, n_units, stream);
        case 2: return launch_stg<OUT, PERM, MB, 2>(p, g, n_units, stream);
        case 4: return launch_stg<OUT, PERM, MB, 4>(p, g, n_units, stream);
        case 8:
            if constexpr (npo2_has_eight<MB>()) return launch_stg<OUT, PERM, MB, 8>(p, g, n_units, stream);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

template <int OUT, int MB>
hipError_t launch_perm(const ApplyParams& p, const Npo2Geom<MB>& g, int nch, int64_t n_units, hipStream_t stream) {
    return p.perm != nullptr ? launch_nch<OUT, true, MB>(p, g, nch, n_units, stream)
                             : launch_nch<OUT, false, MB>(p, g, nch, n_units, stream);
}

// The caller has checked npo2_supports(p) and that b / MB is a power of two.
template <int MB>
hipError_t launch_npo2_base_impl(const ApplyParams& p, int out_kind, hipStream_t stream) {
    // the sign bits of the base matrix are worked out once per process
    static const Npo2Geom<MB> base_bits = [] {
        Npo2Geom<MB> t{};
        constexpr int kRowsPad = sizeof(t.hrow) / sizeof(t.hrow[0]);
        const int kind = MB == 32 ? 0 : hadamard_base_kind(MB);
        for (int r = 0; r < kRowsPad; ++r)
            for (int w = 0; w < Base<MB>::kNT; ++w) {
                uint32_t bits = 0;
                if (r < MB)
                    for (int c = 0; c < 32 && 32 * w + c < MB; ++c)
                        if (base_entry<MB>(kind, r, 32 * w + c) < 0) bits |= 1u << c;
                t.hrow[r][w] = bits;
            }
        return t;
    }();
    Npo2Geom<MB> g = base_bits;
    g.kp = 0;
    while ((MB << g.kp) < p.b) ++g.kp;
    g.norm256 = (float)(256.0 / std::sqrt((double)p.b));
    const int nch = p.d / npo2_chunk_pos<MB>();
    const int64_t rows_per_unit = npo2_waves(nch) / nch;
    const int64_t n_units = (p.T + rows_per_unit - 1) / rows_per_unit;
    switch (out_kind) {
        case OUT_INT4: return launch_perm<OUT_INT4, MB>(p, g, nch, n_units, stream);
        case OUT_MXFP4: return launch_perm<OUT_MXFP4, MB>(p, g, nch, n_units, stream);
        case OUT_INT4_ASYM: return launch_perm<OUT_INT4_ASYM, MB>(p, g, nch, n_units, stream);
        case OUT_FP4_TOKEN: return launch_perm<OUT_FP4_TOKEN, MB>(p, g, nch, n_units, stream);
        case OUT_F32: return launch_perm<OUT_F32, MB>(p, g, nch, n_units, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace
}  // namespace perq
