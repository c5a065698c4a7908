// Shuffle-butterfly kernel for X -> quantize(XP R~): every shape the C ABI accepts.
//
// Layout.  A row of d = 32*nt elements is spread over nt lanes; lane t owns the 32 contiguous
// positions [32t, 32t+32) of the permuted row.  Index bits 0..4 are therefore in registers,
// bits 5..10 are the lane number inside a wave, bits 11.. are the wave number inside the row:
//
//    stages 1..16   in registers                       (b = 16, 32 need nothing else)
//    stages 32..1024 across lanes: DPP, swizzle, permlane swaps
//    stages 2048..  across waves through LDS           (b >= 4096)
//
// The raw bf16 row is staged once in LDS with perfectly coalesced 16-byte global loads (the
// only HBM read); the gather through `perm` is a 2-byte LDS read per element whose byte
// address is computed once per lane and kept in registers for every row the workgroup
// processes.  With one lane per 32 outputs an MXFP4 group is lane-local and each lane stores
// 16 contiguous bytes of codes.
//
// Rows narrower than 8192 are packed several to a 256-thread workgroup when nt is a power of
// two; otherwise a workgroup of ceil(nt/64) waves handles one row at a time.
#include "perq_device.h"
#include "perq_launch.h"

namespace perq {

namespace {

// 16-byte granule g of a row is stored at granule slot g ^ ((g >> 3) & 3): both the coalesced
// writer (consecutive lanes, consecutive g) and the reader (lane t reads granules 4t..4t+3,
// one per instruction) then touch 8 distinct 16-byte bank groups per 8 lanes.
__device__ __forceinline__ uint32_t granule_slot(uint32_t g) { return g ^ ((g >> 3) & 3u); }

struct BflyGeom {
    int nt;              // lanes per row = d / 32
    int rows;            // rows per workgroup iteration
    int waves_per_row;   // ceil(nt / 64)
    uint32_t row_bytes;  // d * 2
    uint32_t red_off;    // byte offset of the reduction scratch in LDS
};

template <int OUT, bool PERM, int MAXT>
__global__ void __launch_bounds__(MAXT)
butterfly_kernel(ApplyParams p, BflyGeom g) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int r = tid / g.nt < g.rows ? tid / g.nt : g.rows - 1;   // row slot of this thread
    const int t = g.rows > 1 ? tid % g.nt : tid;                   // lane index inside the row
    const bool active = t < g.nt && tid < g.rows * g.nt;
    const int ta = active ? t : 0;
    const int d = p.d, b = p.b;

    // -1 / +1 per butterfly distance, in lane units
    float sgn[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) sgn[k] = (t >> k) & 1 ? -1.0f : 1.0f;

    // LDS byte address (inside one staged row) of each of this lane's 32 source elements
    uint32_t src_addr[PERM ? 32 : 1];
    if constexpr (PERM) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int4 e4 = *reinterpret_cast<const int4*>(p.perm + 32 * (active ? t : 0) + 4 * q);
            const int e[4] = {e4.x, e4.y, e4.z, e4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t ee = (uint32_t)e[j];
                src_addr[4 * q + j] = (granule_slot(ee >> 3) << 4) | ((ee & 7u) << 1);
            }
        }
    }

    const int64_t ngroups = (p.T + g.rows - 1) / g.rows;
    unsigned char* my_row = lds + (uint32_t)r * g.row_bytes;

    auto load_group = [&](int64_t grp, uint4 (&buf)[4]) {
        const int64_t row = grp * g.rows + r;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            buf[k] = make_uint4(0, 0, 0, 0);
            if (active && row < p.T)
                buf[k] = load_stream16(p.x + row * p.ldx + (int64_t)(t + k * g.nt) * 8);
        }
    };

    uint4 stage[4];
    if (blockIdx.x < ngroups) load_group(blockIdx.x, stage);

    for (int64_t grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
        const int64_t row = grp * g.rows + r;
        const bool live = active && row < p.T;

        // ---- stage the raw rows in LDS ----------------------------------------------------
        if (active) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                *reinterpret_cast<uint4*>(my_row + (granule_slot((uint32_t)(t + k * g.nt)) << 4)) = stage[k];
        }
        __syncthreads();
        if (grp + gridDim.x < ngroups) load_group(grp + gridDim.x, stage);   // prefetch next rows

        // ---- this lane's 32 permuted elements -> fp32 --------------------------------------
        // (lanes past the end of the row read slot 0 and are never stored)
        float v[32];
        if constexpr (PERM) {
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const uint32_t h = *reinterpret_cast<const uint16_t*>(my_row + src_addr[i]);
                v[i] = __uint_as_float(h << 16);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint4 w = *reinterpret_cast<const uint4*>(my_row + (granule_slot((uint32_t)(4 * ta + j)) << 4));
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v[8 * j + 2 * q] = bf16lo_to_f32(ww[q]);
                    v[8 * j + 2 * q + 1] = bf16hi_to_f32(ww[q]);
                }
            }
        }

        // ---- diagnostics: statistics of the permuted, not yet rotated values ------------------
        float dg_amax = 0.0f, dg_l1 = 0.0f, dg_blk = 0.0f;
        if constexpr (OUT == OUT_DIAG) {
            float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) { s0 += fabsf(v[i]); s1 += fabsf(v[16 + i]); }
            if (active) {
                dg_amax = absmax(v);
                dg_l1 = s0 + s1;
                dg_blk = b == 16 ? fmaxf(s0, s1) : dg_l1;     // b >= 64: summed over lanes below
            }
            if (b >= 64) {
                float* sums = reinterpret_cast<float*>(lds + g.red_off) + 64;
                if (active) sums[r * g.nt + t] = dg_l1;
            }
        }

        // ---- rotation: unnormalised +-1 butterflies ----------------------------------------
        reg_stages<32>(v, b);                               // distances 1..16 (16 only if b >= 32)
        if (b >= 64) lane_stage<1>(v, sgn[0]);
        if (b >= 128) lane_stage<2>(v, sgn[1]);
        if (b >= 256) lane_stage<4>(v, sgn[2]);
        if (b >= 512) lane_stage<8>(v, sgn[3]);
        if (b >= 1024) lane_stage<16>(v, sgn[4]);
        if (b >= 2048) lane_stage<32>(v, sgn[5]);
        if (b >= 4096) {
            // distances 2048.. : partner lane is in another wave; exchange all 32 values through
            // LDS (aliasing the staged rows, which are dead by now).  Granule j of lane t sits at
            // slot t*8 + (j ^ (t & 7)) so that 8 consecutive lanes cover all banks.
            float4* xbuf = reinterpret_cast<float4*>(lds) + (size_t)r * (d >> 2);
            for (int m = 64; 32 * m < b; m <<= 1) {
                __syncthreads();
                if (active) {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        xbuf[t * 8 + (j ^ (t & 7))] = make_float4(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
                }
                __syncthreads();
                const int pt = t ^ m;
                const float s = (t & m) ? -1.0f : 1.0f;
                if (active) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float4 q = xbuf[pt * 8 + (j ^ (pt & 7))];
                        v[4 * j] = __builtin_fmaf(v[4 * j], s, q.x);
                        v[4 * j + 1] = __builtin_fmaf(v[4 * j + 1], s, q.y);
                        v[4 * j + 2] = __builtin_fmaf(v[4 * j + 2], s, q.z);
                        v[4 * j + 3] = __builtin_fmaf(v[4 * j + 3], s, q.w);
                    }
                }
            }
        }

        // ---- epilogue -------------------------------------------------------------------------
        if constexpr (OUT == OUT_F32) {
            if (live) {
                float4* yo = reinterpret_cast<float4*>(p.y + row * (int64_t)d + 32 * t);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    yo[j] = make_float4(v[4 * j] * p.rsqrt_b, v[4 * j + 1] * p.rsqrt_b,
                                        v[4 * j + 2] * p.rsqrt_b, v[4 * j + 3] * p.rsqrt_b);
            }
        } else if constexpr (OUT == OUT_DIAG) {
            // per token: ||x||_inf, ||x||_1, largest block l1 of the permuted row, ||y||_inf
            __syncthreads();                    // the lane sums are in LDS
            if (b >= 64) {
                const int lanes = b >> 5;       // lanes per block; the first of each adds them in order
                const float* sums = reinterpret_cast<const float*>(lds + g.red_off) + 64;
                dg_blk = 0.0f;
                if (active && (t & (lanes - 1)) == 0) {
                    for (int k = 0; k < lanes; ++k) dg_blk += sums[r * g.nt + t + k];
                }
            }
            float m[4] = {dg_amax, dg_l1, dg_blk, active ? absmax(v) * p.rsqrt_b : 0.0f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // sums and maxima of non-negative numbers; lanes past the row hold zeros
#define PERQ_DIAG_STEP(M)                                              \
    if (g.nt > M) { const float o = lane_xor<M>(m[j]); m[j] = j == 1 ? m[j] + o : fmaxf(m[j], o); }
                PERQ_DIAG_STEP(1) PERQ_DIAG_STEP(2) PERQ_DIAG_STEP(4) PERQ_DIAG_STEP(8) PERQ_DIAG_STEP(16) PERQ_DIAG_STEP(32)
#undef PERQ_DIAG_STEP
            }
            if (g.waves_per_row > 1) {
                float* red = reinterpret_cast<float*>(lds + g.red_off);
                const int wave = tid >> 6;
                if (lane == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) red[4 * wave + j] = m[j];
                }
                __syncthreads();
                const int w0 = (r * g.nt) >> 6;
#pragma unroll
                for (int j = 0; j < 4; ++j) m[j] = 0.0f;
                for (int w = 0; w < g.waves_per_row; ++w) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float o = red[4 * (w0 + w) + j];
                        m[j] = j == 1 ? m[j] + o : fmaxf(m[j], o);
                    }
                }
            }
            if (live && t == 0) reinterpret_cast<float4*>(p.y)[row] = make_float4(m[0], m[1], m[2], m[3]);
        } else if constexpr (OUT == OUT_MXFP4) {
            if (p.odd_norm != 1.0f) {
#pragma unroll
                for (int i = 0; i < 32; ++i) v[i] *= p.odd_norm;
            }
            const int E = mx_shared_exponent(absmax(v), p.half_log2b);
            const float scale = __uint_as_float((uint32_t)(E + p.half_log2b) << 23);
            if (live) {
                const uint4 c = make_uint4(mxfp4_pack8(v, scale), mxfp4_pack8(v + 8, scale),
                                           mxfp4_pack8(v + 16, scale), mxfp4_pack8(v + 24, scale));
                store_stream16(p.codes + row * (int64_t)(d >> 1) + 16 * t, c);
                static_cast<uint8_t*>(p.scales)[row * (int64_t)(d >> 5) + t] = (uint8_t)E;
            }
        } else {
            // per-token extremes: lanes of the row inside this wave, then the row's waves.
            // m[0] = max |y| (symmetric INT4, FP4) or max y (asymmetric INT4), m[1] = max -y.
            constexpr int kRed = OUT == OUT_INT4_ASYM ? 2 : 1;
            float m[2] = {0.0f, 0.0f};
            if constexpr (OUT == OUT_INT4_ASYM) {
                float lo, hi;
                minmax(v, lo, hi);
                m[0] = active ? hi : -3.0e38f;
                m[1] = active ? -lo : -3.0e38f;
            } else {
                m[0] = active ? absmax(v) : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kRed; ++j) {
                if (g.nt > 1) m[j] = lane_max<1>(m[j]);
                if (g.nt > 2) m[j] = lane_max<2>(m[j]);
                if (g.nt > 4) m[j] = lane_max<4>(m[j]);
                if (g.nt > 8) m[j] = lane_max<8>(m[j]);
                if (g.nt > 16) m[j] = lane_max<16>(m[j]);
                if (g.nt > 32) m[j] = lane_max<32>(m[j]);
            }
            if (g.waves_per_row > 1) {
                float* red = reinterpret_cast<float*>(lds + g.red_off);
                const int wave = tid >> 6;
                __syncthreads();               // red[] of the previous row has been consumed
                if (lane == 0) {
#pragma unroll
                    for (int j = 0; j < kRed; ++j) red[2 * wave + j] = m[j];
                }
                __syncthreads();
                const int w0 = (r * g.nt) >> 6;
                for (int w = 0; w < g.waves_per_row; ++w) {
#pragma unroll
                    for (int j = 0; j < kRed; ++j) m[j] = fmaxf(m[j], red[2 * (w0 + w) + j]);
                }
            }
            uint8_t* crow = p.codes + row * (int64_t)(d >> 1) + 16 * t;
            if constexpr (OUT == OUT_INT4) {
                float mx = m[0];
                if (tiny_row(mx)) { lift_values(v); mx *= kTinyRowLift; }
                const float inv = mx > 0.0f ? 7.0f / mx : 0.0f;
                if (live) {
                    const uint4 c = make_uint4(int4_pack8(v, inv), int4_pack8(v + 8, inv),
                                               int4_pack8(v + 16, inv), int4_pack8(v + 24, inv));
                    store_stream16(crow, c);
                    if (t == 0) static_cast<float*>(p.scales)[row] = (float)((double)m[0] * p.inv_7sqrt_b);
                }
            } else if constexpr (OUT == OUT_FP4_TOKEN) {
                float mx = m[0];
                if (tiny_row(mx)) { lift_values(v); mx *= kTinyRowLift; }
                const float inv = mx > 0.0f ? p.fp4_qmax / mx : 0.0f;
                if (live) {
                    const uint4 c = make_uint4(fp4_pack8(v, inv), fp4_pack8(v + 8, inv),
                                               fp4_pack8(v + 16, inv), fp4_pack8(v + 24, inv));
                    store_stream16(crow, c);
                    if (t == 0) static_cast<float*>(p.scales)[row] = (float)((double)m[0] * p.inv_fp4sqrt_b);
                }
            } else {
                float lo = -m[1], hi = m[0];
                const float range = hi - lo;
                if (tiny_row(range)) { lift_values(v); lo *= kTinyRowLift; hi *= kTinyRowLift; }
                const Int4Asym q = int4_asym_row(lo, hi);
                if (live) {
                    uint4 c;
                    if (q.mode == 0) {
                        const uint32_t zn = (uint32_t)q.z * 0x11111111u;
                        c = make_uint4(int4a_pack8(v, q.inv, zn), int4a_pack8(v + 8, q.inv, zn),
                                       int4a_pack8(v + 16, q.inv, zn), int4a_pack8(v + 24, q.inv, zn));
                    } else {
                        c = make_uint4(int4a_pack8_clamped(v, q), int4a_pack8_clamped(v + 8, q),
                                       int4a_pack8_clamped(v + 16, q), int4a_pack8_clamped(v + 24, q));
                    }
                    store_stream16(crow, c);
                    if (t == 0) {
                        float2* so = static_cast<float2*>(p.scales) + row;
                        *so = make_float2((float)((double)range * p.inv_15sqrt_b), (float)q.z);
                    }
                }
            }
        }
        __syncthreads();   // LDS is rewritten by the next iteration
    }
}

template <int OUT>
hipError_t launch_butterfly_out(const ApplyParams& p, hipStream_t stream) {
    BflyGeom g;
    g.nt = p.d / 32;
    const bool pow2 = (g.nt & (g.nt - 1)) == 0;
    int threads;
    if (pow2 && g.nt <= 256) {
        g.rows = 256 / g.nt;
        threads = 256;
    } else {
        g.rows = 1;
        threads = ((g.nt + 63) / 64) * 64;
    }
    g.waves_per_row = (g.nt + 63) / 64;
    g.row_bytes = (uint32_t)p.d * 2u;
    const uint32_t stage_bytes = (uint32_t)g.rows * g.row_bytes;
    const uint32_t xchg_bytes = p.b >= 4096 ? (uint32_t)g.rows * (uint32_t)p.d * 4u : 0u;
    g.red_off = stage_bytes > xchg_bytes ? stage_bytes : xchg_bytes;
    // (+ one float per lane of every row: the lane sums of the diagnostics kernel)
    const uint32_t lds_bytes = g.red_off + 64u * sizeof(float) + (OUT == OUT_DIAG ? (uint32_t)(g.rows * g.nt) * 4u : 0u);

    // register budget follows the workgroup size: 256 threads for rows up to 8192, 512 up to
    // 16384, 1024 beyond
    auto kern = threads <= 256   ? (p.perm ? butterfly_kernel<OUT, true, 256> : butterfly_kernel<OUT, false, 256>)
                : threads <= 512 ? (p.perm ? butterfly_kernel<OUT, true, 512> : butterfly_kernel<OUT, false, 512>)
                                 : (p.perm ? butterfly_kernel<OUT, true, 1024> : butterfly_kernel<OUT, false, 1024>);
    // Persistent grid: as many workgroups as the device keeps resident, each walking the rows.
    int per_cu = 0;
    const hipError_t oe = resident_blocks(reinterpret_cast<const void*>(kern), threads, lds_bytes, &per_cu);
    if (oe != hipSuccess) return oe;
    const int64_t ngroups = (p.T + g.rows - 1) / g.rows;
    int64_t grid = (int64_t)launch_info().num_cus * per_cu;
    if (grid > ngroups) grid = ngroups;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3((unsigned)threads), lds_bytes, stream, p, g);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_butterfly(const ApplyParams& p, int out_kind, hipStream_t stream) {
    switch (out_kind) {
        case OUT_INT4: return launch_butterfly_out<OUT_INT4>(p, stream);
        case OUT_MXFP4: return launch_butterfly_out<OUT_MXFP4>(p, stream);
        case OUT_INT4_ASYM: return launch_butterfly_out<OUT_INT4_ASYM>(p, stream);
        case OUT_FP4_TOKEN: return launch_butterfly_out<OUT_FP4_TOKEN>(p, stream);
        case OUT_DIAG: return launch_butterfly_out<OUT_DIAG>(p, stream);
        default: return launch_butterfly_out<OUT_F32>(p, stream);
    }
}

}  // namespace perq
