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
//     b = 64, 128     : the product is widened to H_64 / H_128: accumulator tile q sums the
//                       +-H_32 products of the 2 / 4 sub-blocks of its block (more MFMAs, no VALU)
//     b = 256, 512    : H_128 as above, then one or two butterfly stages across lanes on c
//                       (DPP quad_perm)
//     b = 1024 .. 4096: the roles are turned round.  The data become the A operand: row m of A
//                       collects position bits 0..3 and bit 11 of the tile, the contraction index
//                       K position bits 4..10 (A[m][K] = x[(m & 15) + 16 K + 2048 (m >> 4)]), and
//                       the product with the +-1 matrix I (x) H_{b/16} contracts those seven
//                       middle bits (16 .. 32 MFMAs per tile).  A lane then holds, for 4
//                       transformed K, 16 contiguous positions, whose four low bits are finished by
//                       in-register butterflies (4 VALU per element).  Bit 11 separates the two
//                       half-waves; it belongs to the block only for b = 4096, which alone pays
//                       one half-wave swap stage.
//
// Data movement.  The raw bf16 rows go global -> LDS with 16-byte direct-to-LDS loads (no
// registers, no ds_write), streaming policy; they are the only HBM reads.  The B operands are
// read back from LDS either as one 16-byte read per fragment (P = I) or element by element
// through `perm`, whose LDS byte addresses each lane computes once and keeps for every row.
// 16-byte granule g of a row lives in slot g ^ f((g >> 4) & 7), which spreads both patterns
// over all banks; the swizzle is applied on the global side of the direct-to-LDS load.
#include "perq.h"
#include "perq_device.h"
#include "perq_launch.h"
#include "perq_layout.h"
#include "perq_schedule.h"

#include <map>
#include <mutex>
#include <thread>
#include <tuple>
#include <type_traits>

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
    uint32_t ctr_set;    // which set of ticket counters this launch draws from
    uint32_t dynamic;    // 1: units dealt at run time through the ticket counters; 0: fixed stride
    uint32_t fold_mask;  // rows folded into 4096-wide ones: width of a real row - 1; else all ones
    int32_t row_c_bits;  // low bits of c = lane & 31 that stay inside one real row: 5, or 2..4 when folded
    int32_t row_per_half; // 1: folded rows of 2048 in the high-K modes, one real row per half-wave
};

// Ticket counters of the run-time row schedule (perq_schedule.h): kSets sets of kQueues counters,
// each counter on a 256-byte line of its own.  Zero at load; every launch leaves its set at zero.
// A set belongs to one stream for the life of the process (see stream_counter_set below): launches
// of one stream run one after the other, so no two launches ever draw from the same set at the same
// time, whatever the streams do between them.
using schedule::kQueues;
using schedule::kSets;
__device__ uint32_t work_ctr[kSets][kQueues][64];

// Which set of counters a launch on `stream` draws from, or -1: none, the launch takes the fixed
// stride.  A stream keeps the set it was given first; a launch being captured into a graph gets
// none (the graph may be replayed on any stream, beside anything), nor does a stream that comes
// when every set of its device is taken.  The per-thread default stream is a different stream in
// every host thread and is told apart by the thread.
struct StreamKey {
    int device;
    hipStream_t stream;
    std::thread::id thread;
    bool operator<(const StreamKey& o) const {
        return std::tie(device, stream, thread) < std::tie(o.device, o.stream, o.thread);
    }
};
std::mutex sched_mu;
std::map<StreamKey, int> sched_sets;
int sched_taken[64] = {};          // sets handed out so far, per device

int stream_counter_set(hipStream_t stream) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    if (cs != hipStreamCaptureStatusNone) return -1;
    StreamKey key;
    key.device = 0;
    (void)hipGetDevice(&key.device);
    if (key.device < 0 || key.device >= 64) return -1;
    key.stream = stream;
    key.thread = stream == hipStreamPerThread ? std::this_thread::get_id() : std::thread::id();
    std::lock_guard<std::mutex> lock(sched_mu);
    const auto it = sched_sets.find(key);
    if (it != sched_sets.end()) return it->second;
    if (sched_taken[key.device] >= (int)kSets) return -1;
    const int set = sched_taken[key.device]++;
    sched_sets[key] = set;
    return set;
}

__global__ void clear_counters_kernel() {
    uint32_t* c = &work_ctr[0][0][0];
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < kSets * kQueues * 64u; i += gridDim.x * blockDim.x) c[i] = 0u;
}

using layout::granule_slot;      // granule -> slot inside a staged row
using layout::hk_pos;            // high-K mode: position inside the tile of row m, contraction index K

__device__ __forceinline__ uint32_t popc_parity(uint32_t v) { return __builtin_popcount(v) & 1u; }


// Stores to LDS and workgroup barriers of the main loop, written as instructions.  The compiler
// makes every LDS store it knows of wait until no direct-to-LDS load is outstanding (it cannot
// tell that the staging buffers and these small scratch areas are disjoint), and its barrier waits
// for all memory traffic; either would drain the loads that are meant to stay in flight across
// iterations.  LDS instructions of one wave execute in order, so a later read of the same wave
// sees the store without a wait; across waves the barrier below waits for the wave's own LDS
// traffic first.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}
__device__ __forceinline__ void lds_store16(void* p, uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const u32x4_t v = {a, b, c, d};
    asm volatile("ds_write_b128 %0, %1" ::"v"(lds_addr(p)), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_store4(void* p, float v) {
    asm volatile("ds_write_b32 %0, %1" ::"v"(lds_addr(p)), "v"(v) : "memory");
}
// two 16-byte reads, complete on return
__device__ __forceinline__ void lds_load16x2(const void* p0, const void* p1, uint4& v0, uint4& v1) {
    u32x4_t a, b;
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a), "=&v"(b)
                 : "v"(lds_addr(p0)), "v"(lds_addr(p1))
                 : "memory");
    v0 = make_uint4(a.x, a.y, a.z, a.w);
    v1 = make_uint4(b.x, b.y, b.z, b.w);
}
__device__ __forceinline__ uint32_t lds_load4(const void* p) {
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(lds_addr(p)) : "memory");
    return v;
}

// Element-wise operand gather, written as instructions.  gather8 issues the eight 2-byte reads of
// one operand fragment (byte addresses a[0..7], plus a constant offset that selects the staging
// buffer) and returns with them in flight; the values may be used only after a gather_wait that
// names them.  Reads of LDS return in issue order, so "at most N operations outstanding" proves
// every read but the last N complete.  Through the compiler the same reads came with a mask of
// every result and a byte permute per pair (96 vector instructions per tile where 32 do), and all
// 64 were waited for before the first product could start.
template <uint32_t OFF>
__device__ __forceinline__ void gather8(uint32_t (&t)[8], const uint32_t* a) {
    asm volatile(
        "ds_read_u16 %0, %8 offset:%16\n\t"
        "ds_read_u16 %1, %9 offset:%16\n\t"
        "ds_read_u16 %2, %10 offset:%16\n\t"
        "ds_read_u16 %3, %11 offset:%16\n\t"
        "ds_read_u16 %4, %12 offset:%16\n\t"
        "ds_read_u16 %5, %13 offset:%16\n\t"
        "ds_read_u16 %6, %14 offset:%16\n\t"
        "ds_read_u16 %7, %15 offset:%16"
        : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7])
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]), "n"(OFF)
        : "memory");
}
// Wait until at most N LDS operations of this wave are outstanding; the sixteen values of the two
// fragments named are valid afterwards (they are operands of the statements so that no use of
// them can be moved ahead of the wait).
template <int N>
__device__ __forceinline__ void gather_wait(uint32_t (&t0)[8], uint32_t (&t1)[8]) {
    static_assert(N == 0 || N == 12, "");
    if constexpr (N == 0)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(t0[0]), "+v"(t0[1]), "+v"(t0[2]), "+v"(t0[3]), "+v"(t0[4]), "+v"(t0[5]), "+v"(t0[6]), "+v"(t0[7])
                     :: "memory");
    else
        asm volatile("s_waitcnt lgkmcnt(12)"
                     : "+v"(t0[0]), "+v"(t0[1]), "+v"(t0[2]), "+v"(t0[3]), "+v"(t0[4]), "+v"(t0[5]), "+v"(t0[6]), "+v"(t0[7])
                     :: "memory");
    asm volatile(""
                 : "+v"(t1[0]), "+v"(t1[1]), "+v"(t1[2]), "+v"(t1[3]), "+v"(t1[4]), "+v"(t1[5]), "+v"(t1[6]), "+v"(t1[7])
                 :: "memory");
}
// The same for the eight values of one fragment, N = 0 or 8, with the four shift-or instructions
// that pack them in the same statement: left to the compiler they sink to where the operands are
// used, a whole epilogue later, and the eight unpacked values of every fragment stay live until then.
template <int N>
__device__ __forceinline__ uint4 gather_wait8_pack(const uint32_t (&t)[8]) {
    static_assert(N == 0 || N == 8, "");
    uint32_t w0, w1, w2, w3;
    if constexpr (N == 0)
        asm volatile("s_waitcnt lgkmcnt(0)\n\t"
                     "v_lshl_or_b32 %0, %5, 16, %4\n\t"
                     "v_lshl_or_b32 %1, %7, 16, %6\n\t"
                     "v_lshl_or_b32 %2, %9, 16, %8\n\t"
                     "v_lshl_or_b32 %3, %11, 16, %10"
                     : "=&v"(w0), "=&v"(w1), "=&v"(w2), "=&v"(w3)
                     : "v"(t[0]), "v"(t[1]), "v"(t[2]), "v"(t[3]), "v"(t[4]), "v"(t[5]), "v"(t[6]), "v"(t[7])
                     : "memory");
    else
        asm volatile("s_waitcnt lgkmcnt(8)\n\t"
                     "v_lshl_or_b32 %0, %5, 16, %4\n\t"
                     "v_lshl_or_b32 %1, %7, 16, %6\n\t"
                     "v_lshl_or_b32 %2, %9, 16, %8\n\t"
                     "v_lshl_or_b32 %3, %11, 16, %10"
                     : "=&v"(w0), "=&v"(w1), "=&v"(w2), "=&v"(w3)
                     : "v"(t[0]), "v"(t[1]), "v"(t[2]), "v"(t[3]), "v"(t[4]), "v"(t[5]), "v"(t[6]), "v"(t[7])
                     : "memory");
    return make_uint4(w0, w1, w2, w3);
}
__device__ __forceinline__ uint4 pack_fragment(const uint32_t (&t)[8]) {
    return make_uint4(t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16));
}

// STAGES = number of +-1 butterfly stages after the matrix product: log2(b) - 5, 0 for b <= 32.
// A template parameter so that the accumulators stay in registers along one straight path.
// SHARED: d = 4096 exactly with a permutation: the four waves of a workgroup, each on whole rows of
// its own, build one table of operand addresses together (see below).
// PIPE: the element-wise gather runs one unit ahead of the arithmetic (see the main loop).
template <int OUT, bool PERM, int NWAVES, int STAGES, bool SHARED, bool PIPE>
// (two 4-wave workgroups fit a CU's LDS, so the register budget is that of 2 waves per SIMD)
__global__ void __launch_bounds__(NWAVES * 64, NWAVES == 4 ? 2 : 1) __attribute__((amdgpu_num_vgpr(248)))
mfma_kernel(ApplyParams p, MfmaGeom g) {
    // The dynamic array holds nothing but the row staging buffers, the targets of the
    // direct-to-LDS loads.  Everything the kernel writes to LDS with ordinary stores lives in
    // arrays of its own: the compiler makes a store to LDS wait for every direct-to-LDS load
    // that may write the same memory, and with one shared array that was all loads in flight.
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ __align__(16) unsigned char out_stage[NWAVES * 2048];   // per-wave output staging
    __shared__ float red_scratch[64];                                  // row extremes across waves
    __shared__ uint32_t unit_box[1];                                   // next unit of the workgroup
    // Two staging buffers when a row group fits 32 KiB (4 waves): the loads of the next group are
    // in flight during the whole of the current one.  The buffer is selected by a compile-time
    // offset on the LDS instructions (loop unrolled by two).  8-wave groups use one buffer.
    constexpr bool kDouble = NWAVES == 4;
    constexpr uint32_t kBufStride = 32768;

    // Every kernel argument the set-up needs, fetched in one round trip: left to itself the compiler
    // loads each where it is first used, four to five trips to the argument segment one after the
    // other (about half a microsecond each on a launch's cold scalar cache) ahead of the first row loads
    // (first loads issued 2.7 -> 1.9 us after the launch at d = 4096, 4.4 -> 2.8 us at d = 14336;
    // T = 2048, d = 8192: 14.1 -> 13.9 us, d = 14336, b = 128: 201.0 -> 199.6 us).  Not in the high-K
    // variants, whose main loops came out 0.3 - 0.6 % slower with the arguments held in registers.
    if constexpr (STAGES < 5)
        asm volatile("; kernel arguments are in registers" ::"s"(p.x), "s"(p.T), "s"(p.ldx), "s"(p.perm), "s"(p.place),
                     "s"(p.lane_table), "s"(p.d), "s"(p.b), "s"(g.tiles_per_row), "s"(g.rows), "s"(g.nload), "s"(g.row_bytes),
                     "s"(g.ctr_set), "s"(g.dynamic), "s"(g.fold_mask), "s"(g.row_c_bits), "s"(g.row_per_half));
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, h = lane >> 5;
    const int d = p.d, b = p.b;
    const int rr = wave / g.tiles_per_row;                 // row slot of this wave
    const int tile_base = (wave % g.tiles_per_row) * kTile;
    int tile_len = d - tile_base;
    tile_len = tile_len < 0 ? 0 : (tile_len > kTile ? kTile : tile_len);
    // one tile per row: every wave stages and consumes its own row, no workgroup barrier needed
    const bool wave_local = SHARED || g.tiles_per_row == 1;

    // ---- A operand: rows sigma(i) of the +-1 matrix, two K steps of 16 ---------------------
    // high-K mode (b >= 1024): the constant is the B operand, column j = lane & 31 unpermuted
    constexpr bool kHighK = STAGES >= 5;
    constexpr bool kElem = PERM || kHighK;          // operands gathered element by element
    bf16x8_t afrag[2], afrag_neg[2];
    const uint32_t sigma_i = layout::lane_sigma((uint32_t)lane & 31u);
    // -1 / +1 of the cross-lane butterflies on c
    float sgn[5];
    // Filled in once the first row loads are on their way: nothing ahead of them needs these, and a
    // launch is as long as its first loads are late (d = 4096, b = 128: 57.8 -> 56.9 us; T = 2048,
    // d = 8192: 14.4 -> 14.1 us).  The high-K variants with the gather one unit ahead keep them up here:
    // with them further down the same main loop came out 2 % slower (d = 14336, b = 2048: 208.9 -> 213.7 us).
    constexpr bool kConstantsFirst = STAGES >= 5 && PIPE;
    auto build_constants = [&]() {
        const uint32_t n = kHighK ? ((uint32_t)lane & 31u) : sigma_i;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t k = 16u * kt + 8u * h + e;
                uint32_t bits;
                if (b >= 32) bits = popc_parity(n & k) ? 0xBF80u : 0x3F80u;   // H_32 is symmetric
                else bits = (n >> 4) != (k >> 4) ? 0u : (popc_parity(n & k & 15u) ? 0xBF80u : 0x3F80u);
                if (e & 1) w[e >> 1] |= bits << 16; else w[e >> 1] = bits;
            }
            afrag[kt] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
            afrag_neg[kt] = __builtin_bit_cast(bf16x8_t, make_uint4(w[0] ^ 0x80008000u, w[1] ^ 0x80008000u,
                                                                   w[2] ^ 0x80008000u, w[3] ^ 0x80008000u));
        }
#pragma unroll
        for (int k = 0; k < 5; ++k) sgn[k] = (c >> k) & 1 ? -1.0f : 1.0f;
    };
    if constexpr (kConstantsFirst) build_constants();

    // ---- LDS addresses of this lane's operands (fixed for the whole launch) ----------------
    // PERM: one address per element; identity: one per 16-byte fragment.
    // Sub-blocks past the end of a ragged last tile read a 16-byte slot that is kept at zero
    // (the last 16 bytes of each staging buffer; a ragged row never fills its buffer).
    constexpr uint32_t kZeroSlot = (kDouble ? kBufStride : 65536u) - 16u;
    uint32_t src[kElem ? 64 : 8];
    bool qvalid[kQ];
    // (filled in after the first loads have been issued, see the end of the kernel)
    // sub-block (32 positions) of the tile that accumulator tile q of this lane ends up holding
    auto sbq = [&](int q) -> int { return c * kQ + q; };                            // (low-K modes)
    // high-K mode: first position of the 16 contiguous outputs in accumulator tile q of this lane
    // (b = 4096: after the stage on position bit 11 a lane holds both halves of two tiles instead
    //  of its own half of four; run 2 q' + hb is tile 2 h + q', half hb)
    auto hk_run = [&](int q) -> int {
        if constexpr (STAGES == 7) return 16 * ((2 * h + (q >> 1)) * 32 + c) + 2048 * (q & 1);
        return 16 * (q * 32 + c) + 2048 * h;
    };

    const uint32_t gpr = (uint32_t)d >> 3;                    // granules per row (multiple of 64)
    // Where a granule of the row sits in its staging buffer: the fixed swizzle, or the placement the
    // caller prepared for this permutation (perq_perm_prepare).  In that case p.perm holds, per
    // position, the channel's place in the staged row (slot * 8 + channel % 8) instead of the channel,
    // and p.place the granule of the row that every slot takes (inside the slot's line of 8; entries
    // are clipped to the row).
    const uint16_t* const place = p.place;
    auto slot_of = [&](uint32_t granule) -> uint32_t { return place == nullptr ? granule_slot(granule) : granule; };
    auto granule_at = [&](uint32_t slot) -> uint32_t {
        if (place == nullptr) return granule_slot(slot);
        const uint32_t v = place[slot];
        return v < gpr ? v : gpr - 1u;
    };

    // One direct-to-LDS instruction moves 64 consecutive slots (1 KiB) of one row.  On rows of its
    // own, wave w fills row slot w; otherwise the instructions are dealt round-robin to the waves
    // (a row group is then one or two rows).  Everything but the unit is fixed for the launch: per
    // instruction k a per-lane byte offset from the unit's first row (the swizzle lives here, and
    // the row stride for a load of the second row), an LDS offset lds_base0 + k * lds_stride, and
    // two bit masks saying which k belong to the first and to the second row.
    constexpr int kMaxLoad = 8;
    uint32_t ld_lane_off[kMaxLoad];
    uint32_t mask_row0 = 0, mask_row1 = 0;
    const uint32_t lds_base0 = wave_local ? (uint32_t)wave * g.row_bytes : (uint32_t)wave * 1024u;
    const uint32_t lds_stride = wave_local ? 1024u : NWAVES * 1024u;
#pragma unroll
    for (int k = 0; k < kMaxLoad; ++k) {
        uint32_t in_row, rslot;
        bool ok;
        if (wave_local) {
            rslot = 0;
            in_row = (uint32_t)k * 64u;
            ok = in_row < gpr;
        } else {
            const uint32_t s0 = (uint32_t)(k * NWAVES + wave) * 64u;
            rslot = s0 / gpr;
            in_row = s0 - rslot * gpr;
            ok = rslot < (uint32_t)g.rows;
        }
        ok = ok && k < g.nload;
        ld_lane_off[k] = (ok ? granule_at(in_row + (uint32_t)lane) : 0u) * 16u + rslot * (uint32_t)(p.ldx * 2);
        if (ok) (rslot == 0 ? mask_row0 : mask_row1) |= 1u << k;
    }
    const unsigned char* xbytes = reinterpret_cast<const unsigned char*>(p.x);
    const int64_t ldx_bytes = p.ldx * 2;
    // unit = what one worker takes at a time: a row for a wave on rows of its own, else a row group
    // of the workgroup
    auto issue_loads = [&](uint32_t unit, uint32_t buf_off) -> int {
        const int64_t row0 = wave_local ? (int64_t)unit : (int64_t)unit * g.rows;
        const unsigned char* rp = xbytes + row0 * ldx_bytes;
        const uint32_t m = row0 + 1 < p.T ? (mask_row0 | mask_row1) : mask_row0;
        auto load = [&](int k) {
            __builtin_amdgcn_global_load_lds(rp + ld_lane_off[k], lds + buf_off + lds_base0 + (uint32_t)k * lds_stride,
                                             16, 0, 2 /* nt */);
        };
#pragma unroll
        for (int k = 0; k < kMaxLoad; ++k) {
            if ((m >> k) & 1u) load(k);
        }
        return __builtin_popcount(m);
    };

    // Wait until at most n of this wave's vector-memory operations are outstanding.  They retire
    // in issue order, so once no more than the n operations issued after a group's loads remain,
    // that group has landed.  n must not exceed the true count; a smaller n only waits longer.
    auto wait_vm_le = [&](int n) {
        // (vmcnt is a six-bit count, split over bits 3:0 and 15:14 of the operand)
#define PERQ_VMCNT(N) case N: __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14)); break;
        switch (n < 0 ? 0 : (n > 63 ? 63 : n)) {
            PERQ_VMCNT(0) PERQ_VMCNT(1) PERQ_VMCNT(2) PERQ_VMCNT(3) PERQ_VMCNT(4) PERQ_VMCNT(5) PERQ_VMCNT(6) PERQ_VMCNT(7)
            PERQ_VMCNT(8) PERQ_VMCNT(9) PERQ_VMCNT(10) PERQ_VMCNT(11) PERQ_VMCNT(12) PERQ_VMCNT(13) PERQ_VMCNT(14) PERQ_VMCNT(15)
            PERQ_VMCNT(16) PERQ_VMCNT(17) PERQ_VMCNT(18) PERQ_VMCNT(19) PERQ_VMCNT(20) PERQ_VMCNT(21) PERQ_VMCNT(22) PERQ_VMCNT(23)
            PERQ_VMCNT(24) PERQ_VMCNT(25) PERQ_VMCNT(26) PERQ_VMCNT(27) PERQ_VMCNT(28) PERQ_VMCNT(29) PERQ_VMCNT(30) PERQ_VMCNT(31)
            PERQ_VMCNT(32) PERQ_VMCNT(33) PERQ_VMCNT(34) PERQ_VMCNT(35) PERQ_VMCNT(36) PERQ_VMCNT(37) PERQ_VMCNT(38) PERQ_VMCNT(39)
            PERQ_VMCNT(40) PERQ_VMCNT(41) PERQ_VMCNT(42) PERQ_VMCNT(43) PERQ_VMCNT(44) PERQ_VMCNT(45) PERQ_VMCNT(46) PERQ_VMCNT(47)
            PERQ_VMCNT(48) PERQ_VMCNT(49) PERQ_VMCNT(50) PERQ_VMCNT(51) PERQ_VMCNT(52) PERQ_VMCNT(53) PERQ_VMCNT(54) PERQ_VMCNT(55)
            PERQ_VMCNT(56) PERQ_VMCNT(57) PERQ_VMCNT(58) PERQ_VMCNT(59) PERQ_VMCNT(60) PERQ_VMCNT(61) PERQ_VMCNT(62)
            default: __builtin_amdgcn_s_waitcnt(0x0F70 | 15 | (3 << 14)); break;
        }
#undef PERQ_VMCNT
    };
    // Loads issued after those of the unit about to be consumed.  (The stores issued in between are
    // not counted: that only makes the wait stricter, and counting them measured no faster.)
    int n_behind = 0;

    // ---- schedule ----------------------------------------------------------------------------
    // The XCDs of the chip do not get equal shares of the memory bandwidth, and which of them falls
    // behind changes from launch to launch; with a fixed split the launch lasts as long as the
    // slowest one.  So, given enough units, only the first two of every worker are fixed (worker w
    // takes w and w + W); every further unit is drawn from one of kQueues ticket counters
    // (queue q owns units 2W + q + kQueues * t).  A queue is shared by the workgroups 8k .. 8k+7
    // for a few k, one per XCD each, so every queue balances across XCDs, while one counter sees
    // only 1/kQueues of the atomics (same-address atomics from different XCDs retire at roughly
    // 90 per microsecond).
    //   A ticket is drawn right before the loads of an iteration are issued and read at the end of
    // that iteration, after the wait that leaves only those loads outstanding: vector-memory
    // operations retire in order, so the wait covers the atomic, and the ticket comes for free.
    // The atomic is written as an instruction with its result in v255, a register the compiler is
    // told nothing about and cannot allocate (the kernel is limited to 248 VGPRs): its own atomic
    // would wait for everything in flight, and a result it knew of it might move while pending.
    //   A worker stops drawing at its first ticket past the end, so queue q hands out exactly
    // units_q + workers_q tickets per launch; whoever draws the last one puts the counter back to
    // zero for the next launch.
    const bool dyn = g.dynamic != 0;
    const bool whole_wave_row = g.row_c_bits == 5 && !g.row_per_half;     // no folded rows in a wave
    const uint32_t unit_rows = wave_local ? 1u : (uint32_t)g.rows;
    const uint32_t n_workers = wave_local ? gridDim.x * NWAVES : gridDim.x;
    const uint32_t worker = wave_local ? blockIdx.x * NWAVES + (uint32_t)wave : blockIdx.x;
    const uint32_t n_units = (uint32_t)((p.T + unit_rows - 1) / unit_rows);      // (T < 2^31 here)
    const uint32_t qid = schedule::queue_of_block(blockIdx.x);
    const schedule::QueuePlan qp = schedule::queue_plan(n_units, n_workers, qid);
    uint32_t* ctr = &work_ctr[g.ctr_set][qid][0];
    bool drawing = dyn && (wave_local || wave == 0);     // one wave draws for a workgroup
    uint32_t own_next = 2;                               // fixed stride: place in the worker's own sequence
    auto draw = [&]() {
        if (lane == 0) asm volatile("global_atomic_add v255, %0, %1, off sc0" ::"v"(ctr), "v"(1u) : "v255", "memory");
    };
    // the worker's next unit (n_units: none); call once per iteration, after the wait
    auto fetch_next = [&]() -> uint32_t {
        if (dyn) {
            if (!drawing) return n_units;
            uint32_t t;
            asm volatile("v_readfirstlane_b32 %0, v255" : "=s"(t)::"memory");
            if (t == qp.last_ticket && lane == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (t < qp.units) return schedule::unit_of_ticket(qp, t);
            drawing = false;
            return n_units;
        }
        const uint32_t u = worker + own_next * n_workers;
        ++own_next;
        return u < n_units ? u : n_units;
    };
    const bool boxed = dyn && !wave_local;               // the drawing wave passes the unit on through LDS
    uint32_t u_cur = worker, u_nxt = worker + n_workers, u_new = n_units;

    // ---- one unit out of staging buffer BUF --------------------------------------------------
    // P = I with b <= 512 (16-byte operand reads): on entry the unit's loads have landed (waited for
    // at the end of the iteration before); operands are read, the buffer is refilled, then the
    // arithmetic.
    // Gathered operands (kElem): the gather runs one unit ahead of the arithmetic.  On entry F holds
    // the operands of u_cur, its buffer BUF has been refilled already, and u_nxt sits in the other
    // buffer.  The products of u_cur are issued, then the wave waits for u_nxt to have landed and
    // reads its operands into FN in nine small steps placed between the parts of u_cur's epilogue
    // (64 two-byte reads that meet in the LDS banks take as long as the vector work they now hide
    // behind), and the other buffer is refilled as soon as the last read has returned.
    constexpr bool kPiped = kElem && PIPE;
    uint4 F[kPiped ? 8 : 1];
    auto body = [&](auto buf_const) {
        constexpr uint32_t kOff = kDouble ? decltype(buf_const)::value * kBufStride : 0u;
        constexpr uint32_t kOffN = kDouble ? (1u - decltype(buf_const)::value) * kBufStride : 0u;   // buffer of u_nxt
        const int64_t row = wave_local ? (int64_t)u_cur : (int64_t)u_cur * g.rows + rr;
        const bool row_live = row < p.T;
        uint32_t u_after = n_units;            // (piped) the unit the other buffer is refilled with

        if (!kPiped && !wave_local) {
            workgroup_barrier_lds();
            if (boxed) u_new = __builtin_amdgcn_readfirstlane(lds_load4(unit_box));   // (uniform: keep it scalar)
        }

        // The refill of a buffer, once its operands are in registers.  With two buffers the unit
        // after next goes here, so two units' loads are in flight during the arithmetic.
        auto refill = [&]() {
            if (!wave_local) workgroup_barrier_lds();
            const uint32_t u_load = kPiped ? (kDouble ? u_after : u_new) : (kDouble ? u_new : u_nxt);
            if (drawing) draw();
            n_behind = u_load < n_units ? issue_loads(u_load, kPiped ? kOffN : kOff) : 0;
        };
        // (piped) steps A .. B-1 of the next unit's gather: step i < 8 issues the reads of fragment i,
        // step i > 0 waits for fragment i-1 (everything but the eight reads just issued) and packs it;
        // after step 8 the other buffer is free and is refilled
        uint4 FN[kPiped ? 8 : 1];
        uint32_t tg[2][8];
        auto gather_steps = [&](auto first, auto last) {
            if constexpr (kPiped) {
#pragma unroll
                for (int i = decltype(first)::value; i < decltype(last)::value; ++i) {
                    if (i < 8) gather8<kOffN>(tg[i & 1], src + 8 * i);
                    if (i >= 1) {
                        if (i < 8) FN[i - 1] = gather_wait8_pack<8>(tg[(i - 1) & 1]);
                        else FN[i - 1] = gather_wait8_pack<0>(tg[(i - 1) & 1]);
                    }
                    if (i == 8) refill();
                }
                __builtin_amdgcn_sched_barrier(0);     // the steps stay where they were put
            }
        };
#define PERQ_GATHER_STEPS(A, B) gather_steps(std::integral_constant<int, (A)>{}, std::integral_constant<int, (B)>{})
        const f32x16_t zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        float v[64];
        if constexpr (!kElem) {
            // ---- P = I, b <= 512: one 16-byte read per operand fragment --------------------------
            uint4 bfrag[kQ][2];
#pragma unroll
            for (int q = 0; q < kQ; ++q) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt) bfrag[q][kt] = *reinterpret_cast<const uint4*>(lds + kOff + src[q * 2 + kt]);
            }
            refill();
            // H_32 (b <= 32), H_64 or H_128: accumulator tile qo = sum over the sub-blocks qi of its
            // block of (+-H_32) * X_qi, the sign being entry (qo, qi) of the Sylvester matrix of
            // order kDense
            constexpr int kDense = STAGES == 0 ? 1 : (STAGES == 1 ? 2 : 4);
#pragma unroll
            for (int qo = 0; qo < kQ; ++qo) {
                f32x16_t acc = zero16;
#pragma unroll
                for (int j = 0; j < kDense; ++j) {
                    const int qi = (qo & ~(kDense - 1)) | j;
                    const bool neg = __builtin_popcount(qo & qi & (kDense - 1)) & 1;
#pragma unroll
                    for (int kt = 0; kt < 2; ++kt)
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(neg ? afrag_neg[kt] : afrag[kt],
                                                                      __builtin_bit_cast(bf16x8_t, bfrag[qi][kt]), acc, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) v[qo * 16 + r] = acc[r];
            }
        } else {
            // ---- operands gathered element by element, four groups of two fragments ---------------
            // Low-K modes: group g holds sub-block qi = g of the lane; accumulator tile qo of the same
            // block of kDense sub-blocks takes (+-H_32) * X_qi, the sign being entry (qo, qi) of the
            // Sylvester matrix of order kDense.
            // High-K modes: D[m][n] = sum_K X[m][K] * S[K][n], S = I (x) H_{b/16} on the 128 middle
            // indices (H_64 (x) I_2 ... for b = 1024, H_128 for b >= 2048).  With K = 32 Kh + Kl and
            // n = 32 nt + j the entry is H_kHi[Kh][nt] (zero off the block diagonal) times H_32[Kl][j];
            // the latter is the constant fragment, and group g holds Kh = g.
            // Every accumulator sums its products in ascending (group, fragment) order.
            constexpr int kGroup = kHighK ? (STAGES == 5 ? 2 : 4) : (STAGES == 0 ? 1 : (STAGES == 1 ? 2 : 4));
            f32x16_t acc[kQ] = {zero16, zero16, zero16, zero16};
            auto products = [&](int g, const uint4& f0, const uint4& f1) {
#pragma unroll
                for (int o = 0; o < kQ; ++o) {
                    if ((o / kGroup) != (g / kGroup)) continue;
                    const bool neg = __builtin_popcount((o % kGroup) & (g % kGroup)) & 1;
                    const bf16x8_t d0 = __builtin_bit_cast(bf16x8_t, f0), d1 = __builtin_bit_cast(bf16x8_t, f1);
                    if constexpr (!kHighK) {
                        acc[o] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(neg ? afrag_neg[0] : afrag[0], d0, acc[o], 0, 0, 0);
                        acc[o] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(neg ? afrag_neg[1] : afrag[1], d1, acc[o], 0, 0, 0);
                    } else {
                        acc[o] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(d0, neg ? afrag_neg[0] : afrag[0], acc[o], 0, 0, 0);
                        acc[o] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(d1, neg ? afrag_neg[1] : afrag[1], acc[o], 0, 0, 0);
                    }
                }
            };
            if constexpr (kPiped) {
                // u_nxt has landed (in the other buffer), and with it the ticket drawn at the last refill
                auto next_unit_landed = [&]() {
                    wait_vm_le(kDouble ? n_behind : 0);
                    u_after = fetch_next();
                    if (!wave_local) {
                        if (boxed && wave == 0 && lane == 0) lds_store4(unit_box, __uint_as_float(u_after));
                        workgroup_barrier_lds();
                        if (boxed) u_after = __builtin_amdgcn_readfirstlane(lds_load4(unit_box));   // (uniform: keep it scalar)
                    }
                    __builtin_amdgcn_sched_barrier(0);
                };
#pragma unroll
                for (int gq = 0; gq < kQ; ++gq) products(gq, F[2 * gq], F[2 * gq + 1]);
                next_unit_landed();
                PERQ_GATHER_STEPS(0, kHighK ? 2 : 3);
            } else {
                // the products of a group are issued while the reads of the next two groups are on their way
                uint32_t t[4][2][8];
                gather8<kOff>(t[0][0], src + 0);
                gather8<kOff>(t[0][1], src + 8);
                gather8<kOff>(t[1][0], src + 16);
                gather8<kOff>(t[1][1], src + 24);
#pragma unroll
                for (int gq = 0; gq < kQ; ++gq) {
                    // 32 reads were issued after those of group gq (none after the last group's): with at
                    // most 12 outstanding, group gq has arrived
                    if (gq < kQ - 1) gather_wait<12>(t[gq][0], t[gq][1]);
                    else gather_wait<0>(t[gq][0], t[gq][1]);
                    const uint4 f0 = pack_fragment(t[gq][0]), f1 = pack_fragment(t[gq][1]);
                    if (gq + 2 < kQ) {
                        gather8<kOff>(t[gq + 2][0], src + 16 * (gq + 2));
                        gather8<kOff>(t[gq + 2][1], src + 16 * (gq + 2) + 8);
                    }
                    if (gq == kQ - 1) refill();
                    products(gq, f0, f1);
                    // (keeps the compiler from moving these products behind the next group's wait)
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int o = 0; o < kQ; ++o) {
#pragma unroll
                for (int r = 0; r < 16; ++r) v[o * 16 + r] = acc[o][r];
            }
        }
        if constexpr (kHighK) {
            // position bits 0..3: the 16 contiguous outputs of every accumulator tile
#pragma unroll
            for (int hh = 1; hh < 16; hh <<= 1) {
#pragma unroll
                for (int i = 0; i < 64; ++i) {
                    if ((i & hh) == 0) {
                        const float a0 = v[i], a1 = v[i | hh];
                        v[i] = a0 + a1;
                        v[i | hh] = a0 - a1;
                    }
                }
                if (hh == 1) PERQ_GATHER_STEPS(2, 3);
                if (hh == 2) PERQ_GATHER_STEPS(3, 4);
                if (hh == 4) PERQ_GATHER_STEPS(4, 5);
                if (hh == 8) PERQ_GATHER_STEPS(5, 6);
            }
            if constexpr (STAGES == 7) {
                // position bit 11 (b = 4096 only): one half-wave swap hands the low lanes both halves
                // of tiles 0 and 1 and the high lanes both halves of tiles 2 and 3; sum and
                // difference stay where they are computed (see hk_run), so nothing is swapped back
                float w[64];
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[qp * 16 + r]),
                                                                   __float_as_uint(v[(qp + 2) * 16 + r]), false, false);
                        const float lo = __uint_as_float(sw[0]), hi = __uint_as_float(sw[1]);
                        w[qp * 32 + r] = lo + hi;
                        w[qp * 32 + 16 + r] = lo - hi;
                    }
                }
#pragma unroll
                for (int i = 0; i < 64; ++i) v[i] = w[i];
            }
            PERQ_GATHER_STEPS(6, 7);
        }
        constexpr int kG0 = kHighK ? 7 : 3;        // (piped) gather steps of the next unit done so far

        // ---- butterflies across lanes for b = 256, 512 ------------------------------------------
        if constexpr (STAGES == 3 || STAGES == 4) lane_stage<1>(v, sgn[0]);
        if constexpr (STAGES == 4) lane_stage<2>(v, sgn[1]);

        // ---- epilogue: lane (c,h) holds outputs 16h..16h+15 of sub-blocks 4c..4c+3 (low-K modes),
        //      or the 16 outputs from hk_run(q) on of every accumulator tile q (high-K mode) -------
        if constexpr (OUT == OUT_F32) {
            PERQ_GATHER_STEPS(kG0, 9);
#pragma unroll
            for (int q = 0; q < kQ; ++q) {
                if (row_live && qvalid[q]) {
                    float4* yo = reinterpret_cast<float4*>(p.y + row * (int64_t)d + tile_base + (kHighK ? hk_run(q) : sbq(q) * 32 + 16 * h));
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        yo[j] = make_float4(v[q * 16 + 4 * j] * p.rsqrt_b, v[q * 16 + 4 * j + 1] * p.rsqrt_b,
                                            v[q * 16 + 4 * j + 2] * p.rsqrt_b, v[q * 16 + 4 * j + 3] * p.rsqrt_b);
                }
            }
        } else {
            uint32_t pk[kQ][2];
            uint32_t ebytes = 0;
            float row_max = 0.0f;     // the row's maximum, or hi - lo for the asymmetric quantizer
            int row_zero = 0;
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
                    // the other half of the 32-group: the other half-wave, or the neighbouring lane
                    m = kHighK ? lane_max<1>(m) : lane_max<32>(m);
                    const int E = mx_shared_exponent(m, p.half_log2b);
                    const float scale = __uint_as_float((uint32_t)(E + p.half_log2b) << 23);
                    pk[q][0] = mxfp4_pack8(v + q * 16, scale);
                    pk[q][1] = mxfp4_pack8(v + q * 16 + 8, scale);
                    ebytes |= (uint32_t)E << (8 * q);
                    if constexpr (kHighK) {
                        if (q == 0) PERQ_GATHER_STEPS(7, 8);
                        if (q == 1) PERQ_GATHER_STEPS(8, 9);
                    } else {
                        if (q == 0) PERQ_GATHER_STEPS(3, 5);
                        if (q == 1) PERQ_GATHER_STEPS(5, 7);
                        if (q == 2) PERQ_GATHER_STEPS(7, 8);
                        if (q == 3) PERQ_GATHER_STEPS(8, 9);
                    }
                }
            } else {
                // per-token extremes: m[0] = max |y| (symmetric INT4, FP4) or max y (asymmetric
                // INT4), m[1] = max -y; the zeros read for absent sub-blocks of a ragged tile take
                // no part in a minimum or maximum
                constexpr int kRed = OUT == OUT_INT4_ASYM ? 2 : 1;
                float m[2] = {0.0f, 0.0f};
                if constexpr (OUT == OUT_INT4_ASYM) {
                    m[0] = -3.0e38f;
                    m[1] = -3.0e38f;
#pragma unroll
                    for (int q = 0; q < kQ; ++q) {
                        if (qvalid[q]) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                m[0] = fmaxf(m[0], v[q * 16 + r]);
                                m[1] = fmaxf(m[1], -v[q * 16 + r]);
                            }
                        }
                    }
                } else {
                    m[0] = absmax(v);
                }
                PERQ_GATHER_STEPS(kG0, kHighK ? 8 : 5);
#pragma unroll
                // (folded rows, low-K modes only: a real row is 4, 8 or 16 neighbouring values of c and
                //  both half-waves, so the exchange stops at the row's edge)
                for (int j = 0; j < kRed; ++j) {
                    m[j] = lane_max<1>(m[j]);
                    m[j] = lane_max<2>(m[j]);
                    if (whole_wave_row) {
                        m[j] = lane_max<4>(m[j]);
                        m[j] = lane_max<8>(m[j]);
                        m[j] = lane_max<16>(m[j]);
                        m[j] = lane_max<32>(m[j]);
                    } else {
                        if (g.row_c_bits > 2) m[j] = lane_max<4>(m[j]);
                        if (g.row_c_bits > 3) m[j] = lane_max<8>(m[j]);
                        if (g.row_c_bits > 4) m[j] = lane_max<16>(m[j]);
                        if (!g.row_per_half) m[j] = lane_max<32>(m[j]);
                    }
                }
                if (!wave_local) {
                    // extremes across the row's waves; scratch alternates with the group parity so
                    // that one barrier per group is enough
                    float* red = red_scratch + decltype(buf_const)::value * 32;
                    if (lane == 0) {
#pragma unroll
                        for (int j = 0; j < kRed; ++j) lds_store4(red + 2 * wave + j, m[j]);
                    }
                    workgroup_barrier_lds();
                    const int w0 = rr * g.tiles_per_row;
                    for (int w = 0; w < g.tiles_per_row; ++w) {
#pragma unroll
                        for (int j = 0; j < kRed; ++j) m[j] = fmaxf(m[j], red[2 * (w0 + w) + j]);
                    }
                }
                PERQ_GATHER_STEPS(kHighK ? 8 : 5, kHighK ? 9 : 8);
                if constexpr (OUT == OUT_INT4) {
                    row_max = m[0];
                    float mx = m[0];
                    if (tiny_row(mx)) { lift_values(v); mx *= kTinyRowLift; }
                    const float inv = mx > 0.0f ? 7.0f / mx : 0.0f;
#pragma unroll
                    for (int q = 0; q < kQ; ++q) {
                        pk[q][0] = int4_pack8(v + q * 16, inv);
                        pk[q][1] = int4_pack8(v + q * 16 + 8, inv);
                    }
                } else if constexpr (OUT == OUT_FP4_TOKEN) {
                    row_max = m[0];
                    float mx = m[0];
                    if (tiny_row(mx)) { lift_values(v); mx *= kTinyRowLift; }
                    const float inv = mx > 0.0f ? p.fp4_qmax / mx : 0.0f;
#pragma unroll
                    for (int q = 0; q < kQ; ++q) {
                        pk[q][0] = fp4_pack8(v + q * 16, inv);
                        pk[q][1] = fp4_pack8(v + q * 16 + 8, inv);
                    }
                } else {
                    row_max = m[0] + m[1];                 // hi - lo
                    float lo = -m[1], hi = m[0];
                    if (tiny_row(row_max)) { lift_values(v); lo *= kTinyRowLift; hi *= kTinyRowLift; }
                    const Int4Asym qa = int4_asym_row(lo, hi);
                    row_zero = qa.z;
                    if (qa.mode == 0) {
                        const uint32_t zn = (uint32_t)qa.z * 0x11111111u;
#pragma unroll
                        for (int q = 0; q < kQ; ++q) {
                            pk[q][0] = int4a_pack8(v + q * 16, qa.inv, zn);
                            pk[q][1] = int4a_pack8(v + q * 16 + 8, qa.inv, zn);
                        }
                    } else {
#pragma unroll
                        for (int q = 0; q < kQ; ++q) {
                            pk[q][0] = int4a_pack8_clamped(v + q * 16, qa);
                            pk[q][1] = int4a_pack8_clamped(v + q * 16 + 8, qa);
                        }
                    }
                }
            }
            // Low-K modes: the wave's 2 KiB of codes take one trip through LDS so that each store
            // instruction writes 1 KiB of consecutive bytes (lane l -> 16 bytes at 16 l) instead of short
            // pieces at a pitch.  16-byte slot s sits at s ^ ((s >> 3) & 7).
            // High-K modes: a lane's 16 codes of an accumulator tile are 8 consecutive bytes and the 32
            // lanes of a half-wave hold 256 consecutive bytes, whole cache lines, so the codes are stored
            // from the registers (four 8-byte stores instead of two 16-byte ones, and no wait for a
            // round trip through an LDS queue that the other waves' operand reads keep long;
            // d = 14336, b = 2048: 222 -> 215 us).
            if constexpr (!kHighK && OUT != OUT_MXFP4) PERQ_GATHER_STEPS(8, 9);
            uint4 o0, o1;
            if constexpr (!kHighK) {
                unsigned char* ob = out_stage + (uint32_t)wave * 2048u;
                // Give lane (c,0) the whole of its sub-blocks q = 0, 1 and lane (c,1) the whole of
                // q = 2, 3: the half-wave swap exchanges (q, h=1) of the low lanes' tiles with (q+2, h=0).
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
                const uint32_t s0 = (uint32_t)sbq(2 * h), s1 = (uint32_t)sbq(2 * h + 1);
                lds_store16(ob + ((s0 ^ ((s0 >> 3) & 7u)) << 4), out[0][0], out[0][1], out[0][2], out[0][3]);
                lds_store16(ob + ((s1 ^ ((s1 >> 3) & 7u)) << 4), out[1][0], out[1][1], out[1][2], out[1][3]);
                const uint32_t r0 = (uint32_t)lane, r1 = 64u + (uint32_t)lane;
                lds_load16x2(ob + ((r0 ^ ((r0 >> 3) & 7u)) << 4), ob + ((r1 ^ ((r1 >> 3) & 7u)) << 4), o0, o1);
            }
            if (row_live) {
                uint8_t* ctile = p.codes + row * (int64_t)(d >> 1) + (tile_base >> 1);
                if constexpr (!kHighK) {
                    if (lane * 32 < tile_len) store_stream16(ctile + lane * 16, o0);
                    if (2048 + lane * 32 < tile_len) store_stream16(ctile + lane * 16 + 1024, o1);
                } else {
#pragma unroll
                    for (int q = 0; q < kQ; ++q)
                        if (qvalid[q]) store_stream8(ctile + ((uint32_t)hk_run(q) >> 1), pk[q][0], pk[q][1]);
                }
                if constexpr (OUT == OUT_MXFP4) {
                    uint8_t* srow = static_cast<uint8_t*>(p.scales) + row * (int64_t)(d >> 5) + (tile_base >> 5);
                    if constexpr (!kHighK) {
                        if (h == 0 && qvalid[0]) *reinterpret_cast<uint32_t*>(srow + c * kQ) = ebytes;
                    } else {
#pragma unroll
                        for (int q = 0; q < kQ; ++q)
                            if ((c & 1) == 0 && qvalid[q]) srow[hk_run(q) >> 5] = (uint8_t)(ebytes >> (8 * q));
                    }
                } else {
                    // one scale per real row: the first lane of the row writes it (a folded tile holds
                    // 32 >> row_c_bits rows)
                    const int in_row = c & ((1 << g.row_c_bits) - 1);
                    const int64_t real_row = g.row_per_half ? 2 * row + h : (row << (5 - g.row_c_bits)) + (c >> g.row_c_bits);
                    if (in_row == 0 && (h == 0 || g.row_per_half) && tile_base == 0) {
                        if constexpr (OUT == OUT_INT4_ASYM)
                            static_cast<float2*>(p.scales)[real_row] =
                                make_float2((float)((double)row_max * p.inv_15sqrt_b), (float)row_zero);
                        else
                            static_cast<float*>(p.scales)[real_row] =
                                (float)((double)row_max * (OUT == OUT_INT4 ? p.inv_7sqrt_b : p.inv_fp4sqrt_b));
                    }
                }
            }
        }

        if constexpr (kPiped) {
            u_cur = u_nxt;
            u_nxt = u_new;
            u_new = u_after;
#pragma unroll
            for (int f = 0; f < 8; ++f) F[f] = FN[f];
        } else {
            // ---- the next unit's loads have landed, and the ticket with them -------------------
            wait_vm_le(kDouble ? n_behind : 0);
            u_cur = u_nxt;
            u_nxt = u_new;
            u_new = fetch_next();
            if (boxed && wave == 0 && lane == 0) lds_store4(unit_box, __uint_as_float(u_new));
        }
#undef PERQ_GATHER_STEPS
    };

    // Operand addresses through `perm`, shared case: when every wave of the workgroup owns a whole
    // row of exactly one tile (d = 4096), all four waves need the same 64 addresses per lane up to
    // the row's base.  Wave w then looks up only fragments 2w and 2w+1 (16 channels per lane),
    // leaves their byte offsets inside a row in LDS as 16-bit numbers (fragment f of lane l: 16
    // bytes at f * 1024 + 16 l of the second staging buffer, not yet in use), and after the
    // barrier below every lane collects its eight fragments.  All of this comes before the first
    // row loads: nothing queues behind those, and no ordinary LDS access meets a pending
    // direct-to-LDS load.
    constexpr bool shared_src = SHARED;
    const bool use_table = PERM && p.lane_table != nullptr;      // operand addresses prepared by the caller, see below
    static_assert(!SHARED || (PERM && NWAVES == 4), "the shared table is for four waves with the same tile");
    if constexpr (SHARED) {
        if (!use_table) {
            uint32_t ch[16];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t f = 2u * (uint32_t)wave + j;
                if constexpr (!kHighK) {
                    const uint32_t pos = ((uint32_t)c * kQ + (f >> 1)) * 32u + 16u * (f & 1u) + 8u * h;
                    const int4 e0 = *reinterpret_cast<const int4*>(p.perm + (pos & g.fold_mask));
                    const int4 e1 = *reinterpret_cast<const int4*>(p.perm + (pos & g.fold_mask) + 4);
                    const uint32_t fb = pos & ~g.fold_mask;          // first channel of the real row
                    ch[8 * j + 0] = fb + e0.x; ch[8 * j + 1] = fb + e0.y; ch[8 * j + 2] = fb + e0.z; ch[8 * j + 3] = fb + e0.w;
                    ch[8 * j + 4] = fb + e1.x; ch[8 * j + 5] = fb + e1.y; ch[8 * j + 6] = fb + e1.z; ch[8 * j + 7] = fb + e1.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t pos = hk_pos(sigma_i, 16u * f + 8u * h + e);
                        ch[8 * j + e] = (uint32_t)p.perm[pos & g.fold_mask] + (pos & ~g.fold_mask);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const uint32_t a0 = ch[8 * j + e], a1 = ch[8 * j + e + 1];
                    const uint32_t o0 = (slot_of(a0 >> 3) << 4) | ((a0 & 7u) << 1);
                    const uint32_t o1 = (slot_of(a1 >> 3) << 4) | ((a1 & 7u) << 1);
                    w[e >> 1] = o0 | (o1 << 16);
                }
                *reinterpret_cast<uint4*>(lds + kBufStride + (2u * (uint32_t)wave + j) * 1024u + 16u * (uint32_t)lane) =
                    make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    }

    // Operand addresses through `perm`, general case with two staging buffers: see below.
    constexpr bool kLdsTable = PERM && !SHARED && kDouble;
    // Operand addresses the caller prepared (perq_perm_prepare): the eight fragments of a lane are eight
    // 16-byte reads of the tile's table.  They are issued ahead of the first row loads and waited for
    // by count, so they arrive while the rows are on their way.  The reads and the wait are written as
    // instructions: the compiler's own wait for a load it knows would cover every row load behind it.
    auto src_from_table = [&](auto&& issue_rows) {
        if constexpr (PERM) {
            const uint32_t tiles = ((uint32_t)d + (uint32_t)kTile - 1u) / (uint32_t)kTile;
            const bool have = tile_len > 0;                                     // (uniform in a wave)
            const uint4* tb = reinterpret_cast<const uint4*>(p.lane_table) +
                              ((kHighK ? tiles : 0u) + (have ? (uint32_t)tile_base / (uint32_t)kTile : 0u)) * 512u + (uint32_t)lane;
            u32x4_t t[8];
#pragma unroll
            for (int f = 0; f < 8; ++f) asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(t[f]) : "v"(tb + f * 64) : "memory");
            const int n_after = issue_rows();        // vector-memory operations issued behind the table reads (or fewer)
            // (the count is waited for in a branch of its own; the statement after it is where the
            //  compiler is told that the eight registers have their values, on one path for all counts)
#define PERQ_TABLE_WAIT(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
            switch (n_after < 0 ? 0 : n_after) {
                PERQ_TABLE_WAIT(1) PERQ_TABLE_WAIT(2) PERQ_TABLE_WAIT(3) PERQ_TABLE_WAIT(4) PERQ_TABLE_WAIT(5) PERQ_TABLE_WAIT(6)
                PERQ_TABLE_WAIT(7) PERQ_TABLE_WAIT(8) PERQ_TABLE_WAIT(9) PERQ_TABLE_WAIT(10) PERQ_TABLE_WAIT(11) PERQ_TABLE_WAIT(12)
                PERQ_TABLE_WAIT(13) PERQ_TABLE_WAIT(14) PERQ_TABLE_WAIT(15) PERQ_TABLE_WAIT(16)
                default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
            }
#undef PERQ_TABLE_WAIT
            asm volatile("; table reads have landed in %0 %1 %2 %3 %4 %5 %6 %7"
                         : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]), "+v"(t[4]), "+v"(t[5]), "+v"(t[6]), "+v"(t[7])::"memory");
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < kQ; ++q) qvalid[q] = kHighK ? hk_run(q) < tile_len : (c * kQ + q) * 32 < tile_len;
            const uint32_t base = (uint32_t)rr * g.row_bytes;
#pragma unroll
            for (int f = 0; f < 8; ++f) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t w = t[f][e >> 1];
                    const uint32_t off = (e & 1) ? w >> 16 : w & 0xFFFFu;
                    src[f * 8 + e] = !have || off == 0xFFFFu ? kZeroSlot : base + off;     // (0xFFFF: past the row's end)
                }
            }
        }
    };
    if (tid < 4) {
        *reinterpret_cast<uint32_t*>(lds + kZeroSlot + 4 * tid) = 0u;
        if (kDouble && (!kLdsTable || use_table)) *reinterpret_cast<uint32_t*>(lds + kBufStride + kZeroSlot + 4 * tid) = 0u;
    }
    __syncthreads();
    // (returns the number of row loads issued: the ticket's atomic, issued between them, is not counted)
    auto first_loads = [&]() -> int {
        const int n0 = u_cur < n_units ? issue_loads(u_cur, 0u) : 0;
        if (drawing) draw();
        if constexpr (kDouble) n_behind = u_nxt < n_units ? issue_loads(u_nxt, kBufStride) : 0;
        if constexpr (!kConstantsFirst) build_constants();
        return n0 + (kDouble ? n_behind : 0);
    };
    if constexpr (!SHARED && !kLdsTable) {
        if (!use_table) first_loads();
    }

    // Shared case: collect the eight fragments of addresses the four waves have left in LDS.
    if constexpr (SHARED) {
        if (!use_table) {
            const uint32_t base = (uint32_t)rr * g.row_bytes;
#pragma unroll
            for (int q = 0; q < kQ; ++q) qvalid[q] = true;
#pragma unroll
            for (int f = 0; f < 8; ++f) {
                const uint4 t = *reinterpret_cast<const uint4*>(lds + kBufStride + (uint32_t)f * 1024u + 16u * (uint32_t)lane);
                const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    src[f * 8 + e] = base + (w[e >> 1] & 0xFFFFu);
                    src[f * 8 + e + 1] = base + (w[e >> 1] >> 16);
                }
            }
            __syncthreads();      // the table's place is about to be loaded over
        }
    }
    if constexpr (SHARED) {
        if (use_table) src_from_table(first_loads);
        else first_loads();
    }
    // Otherwise every wave builds its own addresses (and reads `perm`) while the first row groups
    // are already on their way from HBM.  All sixteen 16-byte reads of `perm` are issued together
    // (absent sub-blocks re-read position 0 and are redirected to the zero slot).
    if constexpr (shared_src) {
        // done above
    } else if (use_table) {
        src_from_table(first_loads);
    } else if constexpr (kLdsTable) {
        // The first unit is requested, then the tile of `perm` is read in order (16-byte loads,
        // 1 KiB per instruction: read lane by lane along the operand layout the same entries cost
        // eight times as many cache-line requests), every entry is turned into the 16-bit LDS
        // offset of its channel inside a row, and the 4096 offsets of a tile are kept in a quarter
        // of the second staging buffer, still unused.  Every lane then picks its 64 offsets from
        // there.  Only after that is the second unit requested into that buffer.
        if (u_cur < n_units) issue_loads(u_cur, 0u);
        if constexpr (!kConstantsFirst) build_constants();
        // Waves on the same tile (the rows of a row group; all four on rows of their own) share one
        // table and read a part of the tile's entries each.
        const uint32_t tile_id = (uint32_t)wave % (uint32_t)g.tiles_per_row;
        const uint32_t share = (uint32_t)NWAVES / (uint32_t)g.tiles_per_row;      // 1, 2 or 4 waves per table
        unsigned char* tab = lds + kBufStride + tile_id * 8192u;
        {
            int4 pe[16];
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                if ((uint32_t)jj * share < 16u) {
                    const uint32_t t = (((uint32_t)jj * share + (uint32_t)rr) * 64u + (uint32_t)lane) * 4u;   // entry inside the tile
                    const uint32_t pos = (uint32_t)tile_base + t;
                    pe[jj] = (int)t < tile_len ? *reinterpret_cast<const int4*>(p.perm + (pos & g.fold_mask)) : make_int4(0, 0, 0, 0);
                }
            }
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) {
                if ((uint32_t)jj * share < 16u) {
                    const uint32_t t = (((uint32_t)jj * share + (uint32_t)rr) * 64u + (uint32_t)lane) * 4u;
                    const uint32_t fb = ((uint32_t)tile_base + t) & ~g.fold_mask;       // first channel of the real row
                    const uint32_t ch[4] = {fb + pe[jj].x, fb + pe[jj].y, fb + pe[jj].z, fb + pe[jj].w};
                    uint32_t o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (slot_of(ch[e] >> 3) << 4) | ((ch[e] & 7u) << 1);
                    *reinterpret_cast<uint2*>(tab + 2u * t) = make_uint2(o[0] | (o[1] << 16), o[2] | (o[3] << 16));
                }
            }
        }
        __syncthreads();      // the tables are complete
        const uint32_t base = (uint32_t)rr * g.row_bytes;
        if constexpr (!kHighK) {
#pragma unroll
            for (int q = 0; q < kQ; ++q) qvalid[q] = (c * kQ + q) * 32 < tile_len;
#pragma unroll
            for (int f = 0; f < kQ * 2; ++f) {
                const uint32_t in_tile = ((uint32_t)c * kQ + (f >> 1)) * 32u + 16u * (f & 1) + 8u * h;
                const uint4 t4 = *reinterpret_cast<const uint4*>(tab + 2u * in_tile);
                const uint32_t w[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    src[f * 8 + e] = qvalid[f >> 1] ? base + (w[e >> 1] & 0xFFFFu) : kZeroSlot;
                    src[f * 8 + e + 1] = qvalid[f >> 1] ? base + (w[e >> 1] >> 16) : kZeroSlot;
                }
            }
        } else {
#pragma unroll
            for (int q = 0; q < kQ; ++q) qvalid[q] = hk_run(q) < tile_len;
#pragma unroll
            for (int f = 0; f < 8; ++f) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t in_tile = hk_pos(sigma_i, 16u * f + 8u * h + e);
                    const bool ok = (int)in_tile < tile_len;
                    const uint32_t off = *reinterpret_cast<const uint16_t*>(tab + 2u * (ok ? in_tile : 0u));
                    src[f * 8 + e] = ok ? base + off : kZeroSlot;
                }
            }
        }
        // The zero slot of the second buffer lies in the fourth table.  The last wave, the only reader
        // of that table, clears the slot once it has its offsets and before the barrier: a clear issued
        // after the barrier could land behind another wave's row data on a launch whose code is still cold.
        if (wave == NWAVES - 1 && lane < 4) *reinterpret_cast<uint32_t*>(lds + kBufStride + kZeroSlot + 4 * lane) = 0u;
        __syncthreads();      // every wave has its offsets: the tables' place may be written
        if (drawing) draw();
        n_behind = u_nxt < n_units ? issue_loads(u_nxt, kBufStride) : 0;
    } else if constexpr (!kHighK) {
        int4 pe[kQ * 2][2];
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            const int sb = c * kQ + q;
            qvalid[q] = sb * 32 < tile_len;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const uint32_t pos = (uint32_t)tile_base + (uint32_t)sb * 32u + 16u * kt + 8u * h;
                if constexpr (PERM) {
                    const int32_t* pp = p.perm + (qvalid[q] ? (pos & g.fold_mask) : 0u);
                    pe[q * 2 + kt][0] = *reinterpret_cast<const int4*>(pp);
                    pe[q * 2 + kt][1] = *reinterpret_cast<const int4*>(pp + 4);
                } else {
                    src[q * 2 + kt] = qvalid[q] ? (uint32_t)rr * g.row_bytes + (granule_slot(pos >> 3) << 4) : kZeroSlot;
                }
            }
        }
        if constexpr (PERM) {
#pragma unroll
            for (int f = 0; f < kQ * 2; ++f) {
                const int4 e0 = pe[f][0], e1 = pe[f][1];
                const uint32_t fb = ((uint32_t)tile_base + ((uint32_t)c * kQ + (f >> 1)) * 32u) & ~g.fold_mask;
                const uint32_t ch[8] = {fb + e0.x, fb + e0.y, fb + e0.z, fb + e0.w, fb + e1.x, fb + e1.y, fb + e1.z, fb + e1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    src[f * 8 + e] =
                        qvalid[f >> 1] ? (uint32_t)rr * g.row_bytes + ((slot_of(ch[e] >> 3) << 4) | ((ch[e] & 7u) << 1))
                                       : kZeroSlot;
            }
        }
    } else {
        // high-K mode: fragment kt, element e of lane (i, h) is position hk_pos(sigma(i), K) of the
        // tile, K = 16 kt + 8 h + e; all 64 channel numbers are fetched before any is used
#pragma unroll
        for (int q = 0; q < kQ; ++q) qvalid[q] = hk_run(q) < tile_len;
        uint32_t ch[64];
#pragma unroll
        for (int f = 0; f < 8; ++f) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t in_tile = hk_pos(sigma_i, 16u * f + 8u * h + e);
                const uint32_t pos = (uint32_t)tile_base + in_tile;
                const bool ok = (int)in_tile < tile_len;
                if constexpr (PERM) ch[f * 8 + e] = (uint32_t)p.perm[ok ? (pos & g.fold_mask) : 0u] + (pos & ~g.fold_mask);
                else ch[f * 8 + e] = pos;
            }
        }
#pragma unroll
        for (int f = 0; f < 8; ++f) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool ok = (int)hk_pos(sigma_i, 16u * f + 8u * h + e) < tile_len;
                const uint32_t cc = ch[f * 8 + e];
                src[f * 8 + e] = ok ? (uint32_t)rr * g.row_bytes + ((slot_of(cc >> 3) << 4) | ((cc & 7u) << 1)) : kZeroSlot;
            }
        }
    }

    // the element-wise gather hands these to its read instructions as they are: LDS addresses, not
    // offsets into the staging buffers
    if constexpr (kElem) {
        const uint32_t staging = lds_addr(lds);
#pragma unroll
        for (int i = 0; i < 64; ++i) src[i] += staging;
    }

    // the first unit has landed; the ticket drawn behind its loads says which unit comes third
    wait_vm_le(kDouble ? n_behind : 0);
    u_new = fetch_next();
    if (boxed && wave == 0 && lane == 0) lds_store4(unit_box, __uint_as_float(u_new));
    if constexpr (kPiped) {
        // the operands of the first unit, and the first refill of its buffer
        if (!wave_local) {
            workgroup_barrier_lds();
            if (boxed) u_new = __builtin_amdgcn_readfirstlane(lds_load4(unit_box));
        }
        uint32_t t0[8], t1[8];
#pragma unroll
        for (int f = 0; f < 8; f += 2) {
            gather8<0u>(t0, src + 8 * f);
            gather8<0u>(t1, src + 8 * f + 8);
            gather_wait<0>(t0, t1);
            F[f] = pack_fragment(t0);
            F[f + 1] = pack_fragment(t1);
        }
        if (!wave_local) workgroup_barrier_lds();
        const uint32_t u_load = kDouble ? u_new : u_nxt;
        if (drawing) draw();
        n_behind = u_load < n_units ? issue_loads(u_load, 0u) : 0;
    }

    while (u_cur < n_units) {
        body(std::integral_constant<uint32_t, 0>{});
        if (u_cur < n_units) body(std::integral_constant<uint32_t, 1>{});
    }
}

template <int OUT, int NWAVES, int STAGES>
hipError_t launch_mfma_st(const ApplyParams& p, uint32_t fold_mask, hipStream_t stream) {
    MfmaGeom g;
    const int tiles = (p.d + kTile - 1) / kTile;
    g.tiles_per_row = 1;
    while (g.tiles_per_row < tiles) g.tiles_per_row <<= 1;
    g.rows = NWAVES / g.tiles_per_row;
    g.row_bytes = (uint32_t)p.d * 2u;
    const uint32_t stage_bytes = (uint32_t)g.rows * g.row_bytes;
    const uint32_t gpr = (uint32_t)p.d / 8u;
    g.nload = g.tiles_per_row == 1 ? (int)(gpr / 64u)
                                   : (int)((stage_bytes / 16u + NWAVES * 64u - 1u) / (NWAVES * 64u));
    const uint32_t lds_bytes = 65536u;                  // dynamic part: the staging buffers (incl. the zero slot)
    g.ctr_set = 0;
    g.dynamic = 0;
    g.fold_mask = fold_mask;
    g.row_c_bits = 5;
    g.row_per_half = 0;
    if (fold_mask != 0xFFFFFFFFu) {
        if (STAGES >= 5) g.row_per_half = 1;        // (high-K modes fold rows of 2048 only, see folds())
        else for (g.row_c_bits = 2; (128u << g.row_c_bits) < fold_mask + 1u; ++g.row_c_bits) {}
    }

    const int64_t ngroups = (p.T + g.rows - 1) / g.rows;
    auto kern = p.perm ? mfma_kernel<OUT, true, NWAVES, STAGES, false, false> : mfma_kernel<OUT, false, NWAVES, STAGES, false, false>;
    if constexpr (NWAVES == 4) {
        if (p.perm && p.d == kTile) kern = mfma_kernel<OUT, true, NWAVES, STAGES, true, false>;
        // Rows of four tiles with one scale per token (a barrier for the row's extremes in every
        // iteration) run faster with the gather one unit ahead: d = 14336, b = 2048 with a
        // permutation 245 -> 234 us, b = 128 226 -> 222 us; rows of one or two tiles and MXFP4 do not.
        if constexpr (OUT != OUT_MXFP4) {
            if (g.tiles_per_row == 4) {
                if (p.perm) kern = mfma_kernel<OUT, true, NWAVES, STAGES, false, true>;
                else if constexpr (STAGES >= 5) kern = mfma_kernel<OUT, false, NWAVES, STAGES, false, true>;
            }
        }
    }
    // (static and dynamic LDS together pass 64 KiB)
    int per_cu = 0;
    hipError_t e = resident_blocks(reinterpret_cast<const void*>(kern), NWAVES * 64, lds_bytes, &per_cu);
    if (e != hipSuccess) return e;
    int64_t grid = (int64_t)launch_info().num_cus * per_cu;
    if (grid > ngroups) grid = ngroups;
    // Units are dealt at run time when every worker (a wave on rows of its own, else a workgroup)
    // gets at least its two fixed ones and the workgroups fill the ticket queues evenly.
    {
        const bool wave_local = g.tiles_per_row == 1;
        const int64_t workers = wave_local ? grid * NWAVES : grid;
        const int64_t units = wave_local ? p.T : ngroups;
        g.dynamic = 0;
        if (schedule::queues_usable(grid, workers, units)) {
            const int set = stream_counter_set(stream);
            if (set >= 0) {
                g.dynamic = 1;
                g.ctr_set = (uint32_t)set;
            }
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NWAVES * 64), lds_bytes, stream, p, g);
    return hipGetLastError();
}

template <int OUT, int NWAVES>
hipError_t launch_mfma_nw(const ApplyParams& p, uint32_t fold_mask, hipStream_t stream) {
    switch (p.log2b <= 5 ? 0 : p.log2b - 5) {
        case 0: return launch_mfma_st<OUT, NWAVES, 0>(p, fold_mask, stream);
        case 1: return launch_mfma_st<OUT, NWAVES, 1>(p, fold_mask, stream);
        case 2: return launch_mfma_st<OUT, NWAVES, 2>(p, fold_mask, stream);
        case 3: return launch_mfma_st<OUT, NWAVES, 3>(p, fold_mask, stream);
        case 4: return launch_mfma_st<OUT, NWAVES, 4>(p, fold_mask, stream);
        case 5: return launch_mfma_st<OUT, NWAVES, 5>(p, fold_mask, stream);
        case 6: return launch_mfma_st<OUT, NWAVES, 6>(p, fold_mask, stream);
        default: return launch_mfma_st<OUT, NWAVES, 7>(p, fold_mask, stream);
    }
}

}  // namespace

bool mfma_supports(const ApplyParams& p) {
    // (32-bit unit numbers and row strides)
    return p.b <= kTile && p.d % 512 == 0 && p.d <= 32768 && p.T < ((int64_t)1 << 31) && p.ldx < ((int64_t)1 << 30);
}

// Narrow rows stored back to back can be folded into 4096-wide ones (a wave's tile is 4096 wide
// whatever d is): blocks and 32-groups do not straddle rows, and codes, e8m0 bytes and fp32 outputs
// of consecutive rows are contiguous, so only the operand addresses through `perm` know about it.
// Rows of 512, 1024 or 2048 fold.  The formats with one scale per token need the row's extremes:
// their exchange between lanes follows the real rows where a lane's values lie inside one row
// (b <= 512, and rows of 2048 for b >= 1024).  Rows that do not fill a last 4096-wide one (fewer
// than 4096 / d of them) take a second, unfolded launch.
static bool folds(const ApplyParams& p, int out_kind) {
    const bool per_token = out_kind == OUT_INT4 || out_kind == OUT_INT4_ASYM || out_kind == OUT_FP4_TOKEN;
    // (b >= 1024: a half-wave holds positions 2048 h .. 2048 h + 2047, one real row when d = 2048; rows
    //  of 1024 would split a lane's registers between two rows)
    if (per_token && p.b > 512 && p.d != 2048) return false;
    return out_kind != OUT_DIAG && p.d >= 512 && p.d < kTile && kTile % p.d == 0 && p.ldx == p.d &&
           p.T >= kTile / p.d;
}

bool mfma_preferred(const ApplyParams& p, int out_kind) {
    if (!mfma_supports(p)) return false;
    if (p.d >= kTile) return true;            // its 4096-wide wave tiles are filled
    // folded narrow rows: ahead from b = 128 on, and for any b once the launch is long
    return folds(p, out_kind) && (p.b >= 128 || p.T * (int64_t)p.d >= ((int64_t)1 << 26));
}

hipError_t launch_mfma(const ApplyParams& p0, int out_kind, hipStream_t stream) {
    ApplyParams p = p0;
    uint32_t fold_mask = 0xFFFFFFFFu;
    if (folds(p, out_kind)) {
        const int64_t per_tile = kTile / p.d, rest = p.T % per_tile;
        if (rest != 0) {
            // the last rows, too few for a 4096-wide one: a launch of their own, unfolded (folds() says no
            // to fewer rows than fill one)
            ApplyParams q = p0;
            const int64_t done = p.T - rest;
            q.T = rest;
            q.x = p0.x + done * p0.ldx;
            if (p0.codes != nullptr) q.codes = p0.codes + done * (p0.d >> 1);
            if (p0.y != nullptr) q.y = p0.y + done * p0.d;
            if (p0.scales != nullptr) {
                const int64_t per_row = out_kind == OUT_MXFP4 ? (p0.d >> 5) : (out_kind == OUT_INT4_ASYM ? 8 : 4);
                q.scales = static_cast<unsigned char*>(p0.scales) + done * per_row;
            }
            const hipError_t e = launch_mfma(q, out_kind, stream);
            if (e != hipSuccess) return e;
        }
        fold_mask = (uint32_t)p.d - 1u;
        p.T = p.T / per_tile;
        p.d = kTile;
        p.ldx = kTile;
    }
    const bool wide = p.d > 4 * kTile;        // up to 8 tiles per row -> 8 waves
    switch (out_kind) {
        case OUT_INT4:
            return wide ? launch_mfma_nw<OUT_INT4, 8>(p, fold_mask, stream) : launch_mfma_nw<OUT_INT4, 4>(p, fold_mask, stream);
        case OUT_MXFP4:
            return wide ? launch_mfma_nw<OUT_MXFP4, 8>(p, fold_mask, stream) : launch_mfma_nw<OUT_MXFP4, 4>(p, fold_mask, stream);
        case OUT_INT4_ASYM:
            return wide ? launch_mfma_nw<OUT_INT4_ASYM, 8>(p, fold_mask, stream)
                        : launch_mfma_nw<OUT_INT4_ASYM, 4>(p, fold_mask, stream);
        case OUT_FP4_TOKEN:
            return wide ? launch_mfma_nw<OUT_FP4_TOKEN, 8>(p, fold_mask, stream)
                        : launch_mfma_nw<OUT_FP4_TOKEN, 4>(p, fold_mask, stream);
        default:
            return wide ? launch_mfma_nw<OUT_F32, 8>(p, fold_mask, stream) : launch_mfma_nw<OUT_F32, 4>(p, fold_mask, stream);
    }
}

}  // namespace perq

extern "C" int32_t perq_schedule_set(void* hip_stream) {
    return perq::stream_counter_set(static_cast<hipStream_t>(hip_stream));
}

extern "C" perq_status_t perq_reset_schedule(void* hip_stream) {
    hipLaunchKernelGGL(perq::clear_counters_kernel, dim3(64), dim3(256), 0, static_cast<hipStream_t>(hip_stream));
    return hipGetLastError() == hipSuccess ? PERQ_OK : PERQ_ERR_LAUNCH;
}
