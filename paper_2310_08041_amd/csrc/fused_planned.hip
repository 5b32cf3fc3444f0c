// The fast fused kernel: norm + channel disassembly + channel assembly + per-token quantization
// (steps a1..a4; Sec. 4.3, Eq. 3, Eq. 4, Eq. 2) for maps that come with a plan.
//
// Shape of the computation
//   * Persistent workgroups: grid = (CUs x resident workgroups), each workgroup walks rows
//     blockIdx, blockIdx + grid, ...  What depends only on the map and on gamma -- the lane's share of
//     gamma, of the plan's group descriptors, pass bits and general-group entries -- is loaded once
//     into registers and reused for every row.
//   * HBM: a row is read exactly once, 16 bytes per lane, consecutive lanes on consecutive addresses;
//     the loads of the workgroup's next row are issued before the current row is processed, so they
//     are in flight during its arithmetic.  Codes leave as one coalesced store per lane and group.
//   * LDS: y (fp32) is staged "transposed by 8": channel c at float (c & 7) * S + (c >> 3).  A lane
//     that owns channels 8i..8i+7 writes 8 dwords next to its neighbours' (no bank conflicts), and a
//     lane that needs 8 consecutive channels starting anywhere reads 8 dwords next to its neighbours'.
//     S is a compile-time constant, so all 16 addresses are one register plus an immediate.
//   * min/max of the reassembled row without materialising it: every reassembled channel is either
//     an unscaled copy of an input channel (those inputs carry a pass bit and enter min/max when y is
//     produced) or a channel of a "general" group (sub-channels, merged channels and their
//     neighbours), whose values are computed from LDS by whichever lane the item falls to, kept in a
//     small second LDS area, and enter min/max there.  min and max do not depend on order.
//   * Codes: one fused multiply-add against 1.5 * 2^23 rounds x * inv to the nearest-even integer in
//     the low mantissa bits; a signed median clamps; shift-and-add packs.  Plain groups whose source
//     offset is not a multiple of 8 are read rotated and the packed word is rotated back.
//
// Compiled with -ffp-contract=off (see fused_nrq.hip).
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "qllm.h"
#include "fused_common.h"

using namespace qllm_detail;

namespace {

// work-list entries (see qllm_plan_map_host): kind << 28 | group << 15 | d
constexpr int KIND_PLAIN = 0, KIND_GENERAL = 1, KIND_PAD = 2, KIND_NONE = 3;
constexpr int32_t WORK_NONE = KIND_NONE << 28;
constexpr int32_t ITEM_LONG = -2; // first word of a plan item whose entries are in the table of long rows

template <typename XT>
struct Raw; // 8 input elements as they sit in memory
template <>
struct Raw<uint16_t> {
    uint4 q;
};
template <>
struct Raw<float> {
    float4 lo, hi;
};

// The planned kernel is only launched for rows that are 16-byte aligned and whole chunks long
// (C % 8 == 0); everything else goes to the plain kernel.
__device__ __forceinline__ void load_raw(Raw<uint16_t> &r, const uint16_t *xr, int c0)
{
    r.q = *reinterpret_cast<const uint4 *>(xr + c0);
}

__device__ __forceinline__ void load_raw(Raw<float> &r, const float *xr, int c0)
{
    r.lo = *reinterpret_cast<const float4 *>(xr + c0);
    r.hi = *reinterpret_cast<const float4 *>(xr + c0 + 4);
}

__device__ __forceinline__ void widen(const Raw<uint16_t> &r, float *v)
{
    const uint32_t w[4] = {r.q.x, r.q.y, r.q.z, r.q.w};
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        v[2 * p] = __uint_as_float(w[p] << 16);
        v[2 * p + 1] = __uint_as_float(w[p] & 0xffff0000u);
    }
}

__device__ __forceinline__ void widen(const Raw<float> &r, float *v)
{
    v[0] = r.lo.x; v[1] = r.lo.y; v[2] = r.lo.z; v[3] = r.lo.w;
    v[4] = r.hi.x; v[5] = r.hi.y; v[6] = r.hi.z; v[7] = r.hi.w;
}

// Hides the register contents from the optimiser, so that widening a chunk a second time really is
// redone (two shifts per pair) instead of keeping 8 widened floats per chunk alive across the
// statistics reduction.
__device__ __forceinline__ void forget(Raw<uint16_t> &r)
{
    asm volatile("" : "+v"(r.q.x), "+v"(r.q.y), "+v"(r.q.z), "+v"(r.q.w));
}
__device__ __forceinline__ void forget(Raw<float> &) {}

// (float)(1 / sqrt(t)) for t > 0: the hardware's reciprocal-square-root estimate refined by two Newton
// steps in fp64 (relative error of a few 1e-16), then rounded to fp32.  It equals the fp32 rounding of
// the exact value unless that lies within ~1e-16 (relative) of a rounding boundary of fp32.
__device__ __forceinline__ float rsqrt_to_f32(double t)
{
    double r = __builtin_amdgcn_rsq(t);
    const double h = 0.5 * t;
#pragma unroll
    for (int n = 0; n < 2; ++n) {
        const double e = __builtin_fma(-(h * r), r, 0.5);
        r = __builtin_fma(r, e, r);
    }
    return (float)r;
}

// ---- wavefront reductions on the data-parallel-primitive path (no LDS round trips).
// Four butterfly steps inside each row of 16 lanes, then the four row results are combined from
// lanes 0, 16, 32, 48.  The order of the additions is fixed, so the result is reproducible.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    const uint64_t u = __double_as_longlong(v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xf, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xf, 0xf, false);
    return __longlong_as_double((long long)((uint64_t)lo | ((uint64_t)hi << 32)));
}
constexpr int DPP_XOR1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i <-> 7 - i inside each half row
constexpr int DPP_MIRROR = 0x140;      // lane i <-> 15 - i inside each row
constexpr int DPP_WAVE_SHR1 = 0x138;   // lane i <- lane i - 1 across the whole wavefront (lane 0 keeps `old`)

__device__ __forceinline__ float lane_f32(float v, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ double lane_f64(double v, int l)
{
    const uint64_t u = __double_as_longlong(v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), l);
    return __longlong_as_double((long long)((uint64_t)lo | ((uint64_t)hi << 32)));
}

__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_f64<DPP_XOR1>(v);
    v += dpp_f64<DPP_XOR2>(v);
    v += dpp_f64<DPP_HALF_MIRROR>(v);
    v += dpp_f64<DPP_MIRROR>(v);
    return (lane_f64(v, 0) + lane_f64(v, 16)) + (lane_f64(v, 32) + lane_f64(v, 48));
}
__device__ __forceinline__ void wave_minmax(float &mn, float &mx)
{
    mn = fminf(mn, dpp_f32<DPP_XOR1>(mn)); mx = fmaxf(mx, dpp_f32<DPP_XOR1>(mx));
    mn = fminf(mn, dpp_f32<DPP_XOR2>(mn)); mx = fmaxf(mx, dpp_f32<DPP_XOR2>(mx));
    mn = fminf(mn, dpp_f32<DPP_HALF_MIRROR>(mn)); mx = fmaxf(mx, dpp_f32<DPP_HALF_MIRROR>(mx));
    mn = fminf(mn, dpp_f32<DPP_MIRROR>(mn)); mx = fmaxf(mx, dpp_f32<DPP_MIRROR>(mx));
    mn = fminf(fminf(lane_f32(mn, 0), lane_f32(mn, 16)), fminf(lane_f32(mn, 32), lane_f32(mn, 48)));
    mx = fmaxf(fmaxf(lane_f32(mx, 0), lane_f32(mx, 16)), fmaxf(lane_f32(mx, 32), lane_f32(mx, 48)));
}
__device__ __forceinline__ int32_t wave_sum_i32(int32_t v)
{
    v += __builtin_amdgcn_update_dpp(0, v, DPP_XOR1, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, DPP_XOR2, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, DPP_HALF_MIRROR, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, DPP_MIRROR, 0xf, 0xf, false);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

// Sum over the workgroup: one LDS slot per wave, one barrier, then lane w of every wave fetches slot w
// (one LDS access instead of a dependent chain of them) and the wave adds the slots in slot order.
// The slot array holds 16 entries, zero where there is no wave, and is not reused before another
// barrier has passed.
__device__ __forceinline__ double block_sum(double v, double *slots, int wave, int lane)
{
    v = wave_sum(v);
    if (lane == 0) slots[wave] = v;
    __syncthreads();
    const double mine = slots[lane & 15];
    double s = lane_f64(mine, 0);
#pragma unroll
    for (int w = 1; w < 16; ++w) s += lane_f64(mine, w);
    return s;
}

// gamma of one 8-channel chunk (held in registers for the lifetime of the workgroup).  NORM_NONE runs
// as "rstd = 1, gamma = 1": both multiplications are exact, so y == x bit for bit.
__device__ __forceinline__ void load_gamma(float *g, const float *gamma, int c0, int C, bool use)
{
#pragma unroll
    for (int j = 0; j < GROUP; ++j) g[j] = 1.0f;
    if (!use || c0 >= C) return;
    const float4 g0 = *reinterpret_cast<const float4 *>(gamma + c0);
    const float4 g1 = *reinterpret_cast<const float4 *>(gamma + c0 + 4);
    g[0] = g0.x; g[1] = g0.y; g[2] = g0.z; g[3] = g0.w;
    g[4] = g1.x; g[5] = g1.y; g[6] = g1.z; g[7] = g1.w;
}

// 8 values of a plain group whose first source channel is 8*u + V, V known at compile time:
// channel 8u + V + j sits in LDS row (V + j) & 7, column u + ((V + j) >> 3); slot k = LDS row k.
template <int S_T, int V>
__device__ __forceinline__ void read_plain(const float *ycol, float *val)
{
#pragma unroll
    for (int k = 0; k < GROUP; ++k) val[k] = ycol[k * S_T + (k < V ? 1 : 0)];
}

// Eq. (2) for a row whose quotients are too large for the fused-multiply-add trick.
__device__ __noinline__ uint32_t slow_code(float x, float inv, int32_t beta, int32_t qmax)
{
    const double q = rne_product_slow(x, inv) + (double)beta;
    return (uint32_t)fmin(fmax(q, 0.0), (double)qmax);
}

// Quantizes the 8 slots of one group (Eq. 2), packs them, rotates slot order back into channel order
// and stores.  Returns the sum of the codes.
//
// Fast form: b = bits(fma(x, inv, MAGIC)) is MAGIC_BITS + rne(x*inv); clamping b to [lo, lo + qmax]
// with lo = MAGIC_BITS - beta (one median-of-three) leaves lo + code.  The 8 (or 4) values are packed with shift-and-add
// in wrapping 32-bit arithmetic and the common offset lo * (1 + 2^BITS + 2^(2 BITS) + ...) is taken
// off once.
template <int BITS>
__device__ __forceinline__ int32_t pack_store(const float *val, uint32_t live, int rot, int32_t fast, float inv,
                                              int32_t beta, uint8_t *out_row, int g)
{
    constexpr int QMAX = (1 << BITS) - 1;
    uint32_t c[GROUP], bias = 0;
    if (fast) {
        // floats in [2^23, 2^24) are integers and order like their bit patterns: clamp them as floats
        const float lo = __int_as_float(MAGIC_BITS - beta), hi = __int_as_float(MAGIC_BITS - beta + QMAX);
        bias = (uint32_t)(MAGIC_BITS - beta);
#pragma unroll
        for (int k = 0; k < GROUP; ++k)
            c[k] = __float_as_uint(__builtin_amdgcn_fmed3f(__builtin_fmaf(val[k], inv, MAGIC), lo, hi));
    } else {
#pragma unroll 1
        for (int k = 0; k < GROUP; ++k) c[k] = slow_code(val[k], inv, beta, QMAX); // rare; kept out of line
    }
    if (live != 0xffu) {
#pragma unroll
        for (int k = 0; k < GROUP; ++k) c[k] = (live >> k & 1u) ? c[k] : bias;
    }
    if constexpr (BITS == 4) {
        uint32_t p = 0;
#pragma unroll
        for (int k = GROUP - 1; k >= 0; --k) p = (p << 4) + c[k];
        p -= bias * 0x11111111u;
        reinterpret_cast<uint32_t *>(out_row)[g] = __builtin_amdgcn_alignbit(p, p, rot * 4); // rotate right
        return (int32_t)__builtin_amdgcn_udot8(p, 0x11111111u, 0u, false);
    } else if constexpr (BITS == 8) {
        uint32_t p0 = 0, p1 = 0;
#pragma unroll
        for (int k = 3; k >= 0; --k) {
            p0 = (p0 << 8) + c[k];
            p1 = (p1 << 8) + c[k + 4];
        }
        p0 -= bias * 0x01010101u;
        p1 -= bias * 0x01010101u;
        const uint64_t p = (uint64_t)p0 | ((uint64_t)p1 << 32);
        const int sh = rot * 8;
        reinterpret_cast<uint64_t *>(out_row)[g] = (p >> sh) | (p << ((64 - sh) & 63));
        return (int32_t)__builtin_amdgcn_udot4(p0, 0x01010101u, __builtin_amdgcn_udot4(p1, 0x01010101u, 0u, false), false);
    } else {
        uint32_t h0 = 0, h1 = 0; // four 6-bit codes each
#pragma unroll
        for (int k = 3; k >= 0; --k) {
            h0 = (h0 << 6) + c[k];
            h1 = (h1 << 6) + c[k + 4];
        }
        h0 = (h0 - bias * 0x41041u) & 0xffffffu;
        h1 = (h1 - bias * 0x41041u) & 0xffffffu;
        uint64_t p = (uint64_t)h0 | ((uint64_t)h1 << 24);
        const int sh = rot * 6;
        p = ((p >> sh) | (p << (48 - sh))) & 0xffffffffffffull;
        uint16_t *o16 = reinterpret_cast<uint16_t *>(out_row + (int64_t)g * 6);
        o16[0] = (uint16_t)p;
        o16[1] = (uint16_t)(p >> 16);
        o16[2] = (uint16_t)(p >> 32);
        const uint32_t f = (h0 & 0x3f03fu) + ((h0 >> 6) & 0x3f03fu) + (h1 & 0x3f03fu) + ((h1 >> 6) & 0x3f03fu);
        return (int32_t)((f & 0xfffu) + (f >> 12));
    }
}

// GAM_REG: the lane's share of gamma stays in registers for the lifetime of the workgroup; otherwise it
// is re-read (from L2) for every row, which frees 8 registers per chunk.
template <typename XT, int BITS, int S_T, int ITERS, int NT_MAX, bool GAM_REG, bool LAYER>
__global__ __launch_bounds__(NT_MAX) void fused_planned_kernel(const FusedArgs a)
{
    extern __shared__ float lds[];
    float *ylds = lds;              // [8 * S_T]        y, transposed by 8
    float *exc = lds + GROUP * S_T; // [8 * n_general]  reassembled channels of the general groups
    float *zero = exc + GROUP * a.n_general; // [4] a zero: the "second source" of single-entry items
    int4 *longs = reinterpret_cast<int4 *>(zero + 4); // [n_long] {LDS index of src, dest, scale, pos} of long rows
    __shared__ double red_d[2][16];
    __shared__ float red_f[32];
    __shared__ int32_t red_i[16];
    // bf16 rows are prefetched one row ahead; fp32 rows would need twice the registers and are not
    constexpr bool PREFETCH = sizeof(XT) == 2;
    constexpr int ITEMS_REG = ITERS >= 4 ? ITERS : ITERS + 1; // general-group entries a lane keeps in registers

    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6, nwaves = nt >> 6;
    const int n_chunks = (a.C + GROUP - 1) / GROUP;
    const int n_items = a.n_general * GROUP;
    const float inf = __builtin_inff();
    constexpr bool layer = LAYER;

    // ---- per-lane state that outlives the rows
    float gam[GAM_REG ? ITERS : 1][GROUP];
    uint32_t pass[ITERS];
    int32_t desc[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int i = tid + it * nt;
        pass[it] = i < n_chunks ? (uint32_t)a.passes[i] : 0u;
        desc[it] = i < a.n_groups_pad ? a.desc[i] : WORK_NONE; // work-list entry of this lane and step
        if constexpr (GAM_REG) load_gamma(gam[it], a.gamma, i * GROUP, a.C, a.norm != QLLM_NORM_NONE);
    }
    for (int j = tid; j < a.n_long; j += nt) {
        int4 le = reinterpret_cast<const int4 *>(a.longs)[j];
        le.x = (le.x & 7) * S_T + (le.x >> 3);
        longs[j] = le;
    }
    if (tid < 4) zero[tid] = 0.0f;
    if (tid < 16) { // reduction slots of waves that do not exist hold the identity
        red_d[0][tid] = 0.0;
        red_d[1][tid] = 0.0;
        red_f[tid] = inf;
        red_f[16 + tid] = -inf;
        red_i[tid] = 0;
    }
    __syncthreads();
    // general-group entries of this lane: {LDS index of source 0 | LDS index of source 1 << 16, scale}
    // (the second index of a single-entry item points at the zero); for a long row (bit m of long_mask)
    // the second word is first | count << 24 into the table of long rows
    int2 item[ITEMS_REG];
    uint32_t long_mask = 0;
#pragma unroll
    for (int m = 0; m < ITEMS_REG; ++m) {
        const int j = tid + m * nt;
        item[m] = make_int2(0, 0);
        if (j < n_items) {
            const int2 e = reinterpret_cast<const int2 *>(a.items)[j];
            item[m].y = e.y;
            if (e.x == ITEM_LONG) {
                long_mask |= 1u << m;
            } else {
                const uint32_t s0 = (uint32_t)e.x & 0xffffu, s1 = (uint32_t)e.x >> 16;
                const uint32_t i0 = (s0 & 7) * S_T + (s0 >> 3);
                const uint32_t i1 = s1 == 0xffffu ? (uint32_t)(zero - lds) : (s1 & 7) * S_T + (s1 >> 3);
                item[m].x = (int32_t)(i0 | (i1 << 16)); // float indices into lds, both below 65536
            }
        }
    }

    const XT *xbase = reinterpret_cast<const XT *>(a.x);
    Raw<XT> raw[ITERS], ahead[PREFETCH ? ITERS : 1];
    int64_t row = blockIdx.x;
    if (PREFETCH && row < a.N) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = tid + it * nt;
            if (i < n_chunks) load_raw(ahead[PREFETCH ? it : 0], xbase + row * a.ldx, i * GROUP);
        }
    }

    for (; row < a.N; row += gridDim.x) {
        // Everything derived from the plan (LDS addresses, masks, shifts) costs a handful of
        // instructions per row to recompute, but a register each to keep: make the optimiser
        // recompute it by hiding that the plan registers do not change from row to row.
#pragma unroll
        for (int it = 0; it < ITERS; ++it) asm volatile("" : "+v"(desc[it]), "+v"(pass[it]));
#pragma unroll
        for (int m = 0; m < ITEMS_REG; ++m) asm volatile("" : "+v"(item[m].x), "+v"(item[m].y));

        // ---- step a1.  Take this row (already on its way); put the next row's loads in flight.
        if constexpr (PREFETCH) {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) raw[it] = ahead[it];
            const int64_t next = row + gridDim.x;
            if (next < a.N) {
#pragma unroll
                for (int it = 0; it < ITERS; ++it) {
                    const int i = tid + it * nt;
                    if (i < n_chunks) load_raw(ahead[it], xbase + next * a.ldx, i * GROUP);
                }
            }
        } else {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int i = tid + it * nt;
                if (i < n_chunks) load_raw(raw[it], xbase + row * a.ldx, i * GROUP);
            }
        }

        // row statistics in fp64 (chunks past C hold zeros: load_raw pads)
        float mu = 0.0f, rstd = 1.0f;
        if (!LAYER && a.norm == QLLM_NORM_RMS) {
            double q = 0.0;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                if (tid + it * nt < n_chunks) {
                    float v[GROUP];
                    widen(raw[it], v);
#pragma unroll
                    for (int j = 0; j < GROUP; ++j) {
                        const double d = (double)v[j];
                        q = __builtin_fma(d, d, q);
                    }
                }
            }
            q = block_sum(q, red_d[0], wave, lane);
            rstd = rsqrt_to_f32(q * a.inv_C + (double)a.eps);
        } else if constexpr (LAYER) {
            double s = 0.0;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                if (tid + it * nt < n_chunks) {
                    float v[GROUP];
                    widen(raw[it], v);
#pragma unroll
                    for (int j = 0; j < GROUP; ++j) s += (double)v[j];
                }
            }
            s = block_sum(s, red_d[0], wave, lane);
            const double mu64 = s * a.inv_C;
            double q = 0.0;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int c0 = (tid + it * nt) * GROUP;
                if (c0 < a.C) {
                    float v[GROUP];
                    widen(raw[it], v);
#pragma unroll
                    for (int j = 0; j < GROUP; ++j) {
                        const double d = (double)v[j] - mu64;
                        q = __builtin_fma(d, d, q);
                    }
                }
            }
            q = block_sum(q, red_d[1], wave, lane);
            mu = (float)mu64;
            rstd = rsqrt_to_f32(q * a.inv_C + (double)a.eps);
        }

        // ---- y into LDS; min/max over the channels that pass unscaled
        float mn = inf, mx = -inf;
        const bool shift = LAYER && a.beta != nullptr;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = tid + it * nt;
            float gjit[GROUP];
            if constexpr (!GAM_REG) load_gamma(gjit, a.gamma, i * GROUP, a.C, a.norm != QLLM_NORM_NONE);
            const float *g8 = GAM_REG ? gam[GAM_REG ? it : 0] : gjit;
            if (i < n_chunks) {
                float y[GROUP];
                forget(raw[it]);
                widen(raw[it], y);
#pragma unroll
                for (int j = 0; j < GROUP; ++j) {
                    float t = y[j];
                    if constexpr (LAYER) t = t - mu;
                    t = t * rstd;
                    t = t * g8[j];
                    if constexpr (LAYER) {
                        if (shift) t = t + a.beta[i * GROUP + j];
                    }
                    y[j] = t;
                    ylds[j * S_T + i] = t;
                }
                if (pass[it] == 0xffu) {
#pragma unroll
                    for (int j = 0; j < GROUP; ++j) {
                        mn = fminf(mn, y[j]);
                        mx = fmaxf(mx, y[j]);
                    }
                }
            }
        }
        // Chunks in which some channel does not pass (an outlier that is split, a merged source) are
        // few, but nearly every wave has a lane with one: handled here, one per lane and turn, so a
        // wave spends as many turns as its busiest lane has such chunks (one or two), not ITERS.
        // A lane re-reads its own LDS writes: in order, no barrier needed.
        {
            uint32_t todo = 0;
#pragma unroll
            for (int it = 0; it < ITERS; ++it)
                if (pass[it] != 0xffu && pass[it] != 0u) todo |= 1u << it;
            while (todo) {
                const int it = __builtin_ctz(todo);
                todo &= todo - 1;
                uint32_t m = pass[0];
#pragma unroll
                for (int q = 1; q < ITERS; ++q) m = it == q ? pass[q] : m;
                const float *col = ylds + tid + it * nt;
#pragma unroll
                for (int j = 0; j < GROUP; ++j) {
                    const float yv = col[j * S_T];
                    const bool in = m >> j & 1u;
                    mn = fminf(mn, in ? yv : inf);
                    mx = fmaxf(mx, in ? yv : -inf);
                }
            }
        }
        __syncthreads(); // y complete

        // ---- steps a2 + a3 for the general groups: sub-channels (scale 1/T), merged channels
        //      (scale 1/g each) and the plain channels that share a group of 8 with them.
        //      All LDS reads are issued before any of them is used.
        {
            float y0[ITEMS_REG], y1[ITEMS_REG];
#pragma unroll
            for (int m = 0; m < ITEMS_REG; ++m) { // long rows and unused slots read index 0, harmlessly
                const uint32_t p = (uint32_t)item[m].x;
                y0[m] = lds[p & 0xffffu];
                y1[m] = lds[p >> 16];
            }
#pragma unroll
            for (int m = 0; m < ITEMS_REG; ++m) {
                const int j = tid + m * nt;
                const float sc = __int_as_float(item[m].y);
                float xv = sc * y0[m];
                xv = xv + sc * y1[m];
                const bool real = j < n_items && !(long_mask >> m & 1u);
                mn = fminf(mn, real ? xv : inf);
                mx = fmaxf(mx, real ? xv : -inf);
                if (real) exc[j] = xv;
            }
            // Long rows (a channel merged from three or more, Eq. 4).  The sum runs left to right in
            // fp32, so its order is fixed; its latency need not be.  Entry e of the table belongs to lane
            // e % 64 and a row sits in consecutive lanes of one wavefront: every lane forms its product,
            // then "value of the lane below + own product" is repeated; the lane of entry number pos is
            // final after pos repeats (repeating it again changes nothing) and the row's last lane
            // ends up with the row's value.
            for (int base = 0; base < a.n_long; base += nt) {
                const int e = base + tid;
                int4 le = make_int4(0, -1, 0, 0);
                if (e < a.n_long) le = longs[e];
                const float p = __int_as_float(le.z) * lds[le.x];
                float acc = p;
                for (int t = 1; __builtin_amdgcn_ballot_w64(le.w >= t) != 0; ++t) {
                    const float below = dpp_f32<DPP_WAVE_SHR1>(acc);
                    acc = le.w > 0 ? below + p : p;
                }
                if (le.y >= 0) {
                    exc[le.y] = acc;
                    mn = fminf(mn, acc);
                    mx = fmaxf(mx, acc);
                }
            }
        }

        // ---- per-token range (Eq. 2)
        wave_minmax(mn, mx);
        if (lane == 0) {
            red_f[wave] = mn;
            red_f[16 + wave] = mx;
        }
        __syncthreads(); // also: exc complete
        mn = red_f[lane & 15];
        mx = red_f[16 + (lane & 15)];
        mn = fminf(mn, dpp_f32<DPP_XOR1>(mn)); mx = fmaxf(mx, dpp_f32<DPP_XOR1>(mx));
        mn = fminf(mn, dpp_f32<DPP_XOR2>(mn)); mx = fmaxf(mx, dpp_f32<DPP_XOR2>(mx));
        mn = fminf(mn, dpp_f32<DPP_HALF_MIRROR>(mn)); mx = fmaxf(mx, dpp_f32<DPP_HALF_MIRROR>(mx));
        mn = fminf(mn, dpp_f32<DPP_MIRROR>(mn)); mx = fmaxf(mx, dpp_f32<DPP_MIRROR>(mx));
        mn = lane_f32(mn, 0);
        mx = lane_f32(mx, 0);
        constexpr int QMAX = (1 << BITS) - 1;
        const float range = mx - mn;
        const float alpha = range > 0.0f ? range / (float)QMAX : 1.0f;
        const float inv = 1.0f / alpha;
        const int32_t fast = fabsf(mn * inv) < FAST_LIMIT && fabsf(mx * inv) < FAST_LIMIT;
        int32_t beta;
        if (fast) beta = -rne_product_fast(mn, inv);
        else beta = (int32_t)fmin(fmax(-rne_product_slow(mn, inv), -2147483647.0), 2147483647.0);

        // ---- step a4: codes
        int32_t sum = 0;
        uint8_t *out_row = a.codes + row * a.row_bytes;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int32_t e = desc[it];
            const int kind = (uint32_t)e >> 28;
            if (kind != KIND_NONE) {
                const int g = (e >> 15) & 0x1fff, d = e & 0x7fff;
                float val[GROUP];
                uint32_t live = 0xffu;
                const int vv = d & 7;
                int rot = vv;
                const int v0 = __builtin_amdgcn_readfirstlane(vv);
                if (__all(kind == KIND_PLAIN && vv == v0)) {
                    // the usual case (the work list is sorted for it): the whole wave reads plain groups
                    // with the same misalignment, every address is one register plus an immediate
                    const float *ycol = ylds + (d >> 3);
                    switch (v0) {
                    case 0: read_plain<S_T, 0>(ycol, val); break;
                    case 1: read_plain<S_T, 1>(ycol, val); break;
                    case 2: read_plain<S_T, 2>(ycol, val); break;
                    case 3: read_plain<S_T, 3>(ycol, val); break;
                    case 4: read_plain<S_T, 4>(ycol, val); break;
                    case 5: read_plain<S_T, 5>(ycol, val); break;
                    case 6: read_plain<S_T, 6>(ycol, val); break;
                    default: read_plain<S_T, 7>(ycol, val); break;
                    }
                } else if (kind == KIND_PLAIN) {
                    const int u = d >> 3;
#pragma unroll
                    for (int k = 0; k < GROUP; ++k) val[k] = ylds[k * S_T + u + (k < vv ? 1 : 0)];
                } else if (kind == KIND_GENERAL) {
                    const float4 e0 = *reinterpret_cast<const float4 *>(exc + d * GROUP);
                    const float4 e1 = *reinterpret_cast<const float4 *>(exc + d * GROUP + 4);
                    val[0] = e0.x; val[1] = e0.y; val[2] = e0.z; val[3] = e0.w;
                    val[4] = e1.x; val[5] = e1.y; val[6] = e1.z; val[7] = e1.w;
                    rot = 0;
                    const int left = a.C_out - g * GROUP;
                    if (left < GROUP) live = (1u << left) - 1u;
                } else {
                    rot = 0;
                    live = 0u;
#pragma unroll
                    for (int k = 0; k < GROUP; ++k) val[k] = 0.0f;
                }
                sum += pack_store<BITS>(val, live, rot, fast, inv, beta, out_row, g);
            }
        }
        sum = wave_sum_i32(sum);
        if (lane == 0) red_i[wave] = sum;
        __syncthreads(); // row done: LDS may be overwritten, red_i is complete
        if (wave == 0) {
            int32_t s = red_i[lane & 15];
            s += __builtin_amdgcn_update_dpp(0, s, DPP_XOR1, 0xf, 0xf, false);
            s += __builtin_amdgcn_update_dpp(0, s, DPP_XOR2, 0xf, 0xf, false);
            s += __builtin_amdgcn_update_dpp(0, s, DPP_HALF_MIRROR, 0xf, 0xf, false);
            s += __builtin_amdgcn_update_dpp(0, s, DPP_MIRROR, 0xf, 0xf, false);
            if (lane == 0) {
            a.alpha[row] = alpha;
            a.zero[row] = beta;
            a.rowsum[row] = s;
            }
        }
    }
}

struct Shape {
    int s_t, iters, nt;
};

// Smallest compiled (S, ITERS) that holds `units` 8-channel groups, and the workgroup size for it.
Shape pick_shape(int units)
{
    Shape s;
    if (units <= 256) s = {256, 1, 0};
    else if (units <= 1024) s = {1024, 2, 0};
    else if (units <= 2048) s = {2048, 2, 0};
    else s = {4096, 4, 0};
    s.nt = ((units + s.iters - 1) / s.iters + 63) / 64 * 64;
    return s;
}

int cu_count()
{
    static int cached = 0;
    if (cached) return cached;
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        n <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    cached = n;
    return n;
}

template <typename K>
int32_t launch(K kernel, const FusedArgs &a, const Shape &sh, size_t lds, hipStream_t stream)
{
    if (lds > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            qllm_note_hip_error("planned fused kernel: raising the LDS limit", hipGetErrorName(e));
            return QLLM_ERR_HIP;
        }
    }
    // resident workgroups per CU: bounded by LDS (160 KB) and by 2048 lanes
    int per_cu = (int)((160 * 1024) / (lds + 1024));
    per_cu = per_cu < 2048 / sh.nt ? per_cu : 2048 / sh.nt;
    if (per_cu < 1) per_cu = 1;
    int64_t grid = (int64_t)cu_count() * per_cu;
    if (grid > a.N) grid = a.N;
    (void)hipGetLastError();
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3((unsigned)sh.nt), lds, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error("planned fused kernel: launch", hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}

template <typename XT, int BITS, bool LAYER>
int32_t dispatch(const FusedArgs &a, const Shape &sh, size_t lds, hipStream_t stream)
{
    if (sh.s_t == 256) return launch(fused_planned_kernel<XT, BITS, 256, 1, 256, true, LAYER>, a, sh, lds, stream);
    if (sh.s_t == 1024) return launch(fused_planned_kernel<XT, BITS, 1024, 2, 512, true, LAYER>, a, sh, lds, stream);
    if (sh.s_t == 2048) return launch(fused_planned_kernel<XT, BITS, 2048, 2, 1024, true, LAYER>, a, sh, lds, stream);
    return launch(fused_planned_kernel<XT, BITS, 4096, 4, 1024, true, LAYER>, a, sh, lds, stream);
}

template <typename XT>
int32_t dispatch_bits(const FusedArgs &a, int bits, const Shape &sh, size_t lds, hipStream_t stream)
{
    if (a.norm == QLLM_NORM_LAYER) {
        if (bits == 4) return dispatch<XT, 4, true>(a, sh, lds, stream);
        if (bits == 6) return dispatch<XT, 6, true>(a, sh, lds, stream);
        return dispatch<XT, 8, true>(a, sh, lds, stream);
    }
    if (bits == 4) return dispatch<XT, 4, false>(a, sh, lds, stream);
    if (bits == 6) return dispatch<XT, 6, false>(a, sh, lds, stream);
    return dispatch<XT, 8, false>(a, sh, lds, stream);
}

} // namespace

int32_t qllm_launch_fused_planned(const FusedArgs &a, int32_t x_dtype, int32_t bits, hipStream_t stream)
{
    const int n_chunks = (a.C + GROUP - 1) / GROUP;
    const int units = n_chunks > a.n_groups_pad ? n_chunks : a.n_groups_pad;
    if (units > 4096 || !a.vec_ok || a.C % GROUP != 0) return QLLM_ERR_WORKSPACE;
    const Shape sh = pick_shape(units);
    const size_t lds = ((size_t)sh.s_t + (size_t)a.n_general) * GROUP * sizeof(float) + 16 + (size_t)a.n_long * 16;
    if (lds + 1024 > 160 * 1024) return QLLM_ERR_WORKSPACE;
    const int items_reg = sh.iters >= 4 ? sh.iters : sh.iters + 1;
    if ((int64_t)a.n_general * GROUP > (int64_t)items_reg * sh.nt) return QLLM_ERR_WORKSPACE; // general-group entries live in registers
    if (x_dtype == QLLM_BF16) return dispatch_bits<uint16_t>(a, bits, sh, lds, stream);
    return dispatch_bits<float>(a, bits, sh, lds, stream);
}
