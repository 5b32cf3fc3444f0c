// The fast fused kernel: norm + channel disassembly + channel assembly + per-token quantization
// (steps a1..a4; Sec. 4.3, Eq. 3, Eq. 4, Eq. 2) for maps that come with a plan.
//
// Shape of the computation
//   * Persistent workgroups: grid = (CUs x resident workgroups), each workgroup walks rows
//     blockIdx, blockIdx + grid, ...  What depends only on the map and on gamma -- the lane's share of
//     gamma and of the plan -- is loaded once into registers and reused for every row.
//   * HBM: a row is read exactly once, 16 bytes per lane, consecutive lanes on consecutive addresses;
//     the loads of the workgroup's next row are issued before the current row is processed, so they
//     are in flight during its arithmetic.  Codes leave as one coalesced store per lane and group.
//   * y stays in the registers of the lane that loaded its chunk of 8 channels, from the norm until
//     that same lane quantizes it.  A code does not depend on where its channel ends up, so chunks are
//     quantized and packed in INPUT order and only the packed words (4 to 8 bytes per chunk) go through
//     LDS.  Nearly all groups of 8 output channels are "plain": 8 consecutive input channels, unscaled,
//     starting anywhere; such a group is two neighbouring packed words funnel-shifted by its
//     misalignment: two LDS reads and one shift per group, whatever the misalignment.
//   * The other ("general") groups hold sub-channels (Eq. 3, scale 1/T), merged channels (Eq. 4) and
//     the unscaled channels that share a group of 8 with them.  The plan lists the input chunks they
//     read; only those chunks' y (fp32) is staged in LDS.  Their values are computed by whichever lane
//     the entry falls to, kept in a second small LDS area, and quantized by the lane that stores the
//     group.
//   * min/max of the reassembled row without materialising it: every reassembled channel is either
//     an unscaled copy of an input channel (those inputs carry a pass bit and enter min/max when y is
//     produced) or a channel of a general group (enters where it is computed).
//   * Codes: one fused multiply-add against 1.5 * 2^23 rounds x * inv to the nearest-even integer in
//     the low mantissa bits; a median-of-three clamps; shift-and-add packs.
//   * Four barriers per row (five with LayerNorm): statistics, staged y complete, range, packed
//     words complete.  The first also separates a row's last LDS reads from the next row's writes.
//
// Compiled with -ffp-contract=off (see fused_nrq.hip).
#include <hip/hip_runtime.h>

#include <stdint.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "qllm.h"
#include "fused_common.h"
#include "plan_budget.h"

using namespace qllm_detail;

namespace {

// work-list entries (see qllm_plan_map_host): kind << 30 | group << 17 | field
constexpr int KIND_PLAIN = 0, KIND_COMP = 1, KIND_PAD = 2, KIND_NONE = 3;
constexpr int32_t WORK_NONE = (int32_t)(3u << 30);

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

__device__ __forceinline__ float widen_one(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float widen_one(float f) { return f; }

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

// dst = src as a copy the optimiser has to make here and now: the registers of src are then free for
// the next load, instead of the copy being postponed to the end of the loop body, behind that load.
__device__ __forceinline__ void move_up(Raw<uint16_t> &dst, const Raw<uint16_t> &src)
{
    asm volatile("v_mov_b32 %0, %1" : "=v"(dst.q.x) : "v"(src.q.x));
    asm volatile("v_mov_b32 %0, %1" : "=v"(dst.q.y) : "v"(src.q.y));
    asm volatile("v_mov_b32 %0, %1" : "=v"(dst.q.z) : "v"(src.q.z));
    asm volatile("v_mov_b32 %0, %1" : "=v"(dst.q.w) : "v"(src.q.w));
}
__device__ __forceinline__ void move_up(Raw<float> &dst, const Raw<float> &src) { dst = src; }

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

// ---- wavefront reductions on the data-parallel-primitive (DPP) path: no LDS round trips.
// Four butterfly steps inside each row of 16 lanes, then the four row results are combined from
// lanes 0, 16, 32, 48.  The order of the additions is fixed, so the result is reproducible.
// Each step is ONE instruction that takes its first operand from another lane.  They are written
// out because the optimiser, given the lane movement as a builtin, spends four instructions a step
// (a zeroed destination, the move, a NaN-quieting pass, the operation).  Every lane of the wavefront
// must be active; the s_nop covers the two wait states a DPP operand needs after it was written.
#define QLLM_DPP_STEP(fn, type, cons, op, ctrl)                                                          \
    __device__ __forceinline__ type fn(type v)                                                           \
    {                                                                                                    \
        type r;                                                                                          \
        asm("s_nop 1\n\t" op " %0, %1, %1 " ctrl " row_mask:0xf bank_mask:0xf" : "=" cons(r) : cons(v)); \
        return r;                                                                                        \
    }
#define QLLM_DPP_FAMILY(name, type, op)                                  \
    QLLM_DPP_STEP(name##_xor1, type, "v", op, "quad_perm:[1,0,3,2]")     \
    QLLM_DPP_STEP(name##_xor2, type, "v", op, "quad_perm:[2,3,0,1]")     \
    QLLM_DPP_STEP(name##_half_mirror, type, "v", op, "row_half_mirror")  \
    QLLM_DPP_STEP(name##_mirror, type, "v", op, "row_mirror")            \
    __device__ __forceinline__ type name##_row16(type v) /* all 16 lanes of a row end with the row's result */ \
    {                                                                    \
        return name##_mirror(name##_half_mirror(name##_xor2(name##_xor1(v)))); \
    }
QLLM_DPP_FAMILY(dpp_min, float, "v_min_f32_dpp")
QLLM_DPP_FAMILY(dpp_max, float, "v_max_f32_dpp")
QLLM_DPP_FAMILY(dpp_add, int32_t, "v_add_u32_dpp")

// value of the lane below (lane 0: zero), across the whole wavefront
__device__ __forceinline__ float below(float v)
{
    float r;
    asm("s_nop 1\n\tv_mov_b32_dpp %0, %1 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0" : "=v"(r) : "v"(v));
    return r;
}

// One step of the lane-by-lane addition of a long row: (value of the lane below) * keep + p in one rounding,
// the shift folded into the multiply-add.  The copy of p does not depend on the step before, so only the
// multiply-add (and the two idle states a DPP read needs after the write of its source) sit on the chain.
__device__ __forceinline__ float chain_step(float acc, float keep, float p)
{
    float t;
    asm("v_mov_b32 %0, %3\n\ts_nop 0\n\tv_fmac_f32_dpp %0, %1, %2 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0"
        : "=&v"(t)
        : "v"(acc), "v"(keep), "v"(p));
    return t;
}

// v + (v of the partner lane) in fp64: the two halves move separately, the addition is ordinary
#define QLLM_DPP_ADD_F64(fn, ctrl)                                                                           \
    __device__ __forceinline__ double fn(double v)                                                           \
    {                                                                                                        \
        const uint64_t u = __double_as_longlong(v);                                                          \
        uint32_t lo, hi;                                                                                     \
        asm("s_nop 1\n\tv_mov_b32_dpp %0, %2 " ctrl " row_mask:0xf bank_mask:0xf\n\t"                        \
            "v_mov_b32_dpp %1, %3 " ctrl " row_mask:0xf bank_mask:0xf"                                       \
            : "=&v"(lo), "=&v"(hi)                                                                           \
            : "v"((uint32_t)u), "v"((uint32_t)(u >> 32)));                                                   \
        return v + __longlong_as_double((long long)((uint64_t)lo | ((uint64_t)hi << 32)));                   \
    }
QLLM_DPP_ADD_F64(dpp_addd_xor1, "quad_perm:[1,0,3,2]")
QLLM_DPP_ADD_F64(dpp_addd_xor2, "quad_perm:[2,3,0,1]")
QLLM_DPP_ADD_F64(dpp_addd_half_mirror, "row_half_mirror")
QLLM_DPP_ADD_F64(dpp_addd_mirror, "row_mirror")
__device__ __forceinline__ double dpp_addd_row16(double v)
{
    return dpp_addd_mirror(dpp_addd_half_mirror(dpp_addd_xor2(dpp_addd_xor1(v))));
}

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
    v = dpp_addd_row16(v);
    return (lane_f64(v, 0) + lane_f64(v, 16)) + (lane_f64(v, 32) + lane_f64(v, 48));
}
__device__ __forceinline__ void wave_minmax(float &mn, float &mx)
{
    mn = dpp_min_row16(mn);
    mx = dpp_max_row16(mx);
    mn = fminf(fminf(lane_f32(mn, 0), lane_f32(mn, 16)), fminf(lane_f32(mn, 32), lane_f32(mn, 48)));
    mx = fmaxf(fmaxf(lane_f32(mx, 0), lane_f32(mx, 16)), fmaxf(lane_f32(mx, 32), lane_f32(mx, 48)));
}
__device__ __forceinline__ int32_t wave_sum_i32(int32_t v)
{
    v = dpp_add_row16(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

// Sum of the 16 per-wave slots (zero where there is no wave): lane w of every row of 16 lanes fetches
// slot w and a butterfly adds them, so every lane ends with the same total without a dependent chain
// of LDS reads.  The slots are not reused before another barrier has passed.
__device__ __forceinline__ double total16(const double *slots, int lane)
{
    return dpp_addd_row16(slots[lane & 15]);
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

// Eq. (2) for a row whose quotients are too large for the fused-multiply-add trick.
__device__ __noinline__ uint32_t slow_code(float x, float inv, int32_t beta, int32_t qmax)
{
    const double q = rne_product_slow(x, inv) + (double)beta;
    return (uint32_t)fmin(fmax(q, 0.0), (double)qmax);
}

// bit k of m8 -> the k-th code field of a packed chunk, all ones
template <int BITS>
__device__ __forceinline__ uint64_t widen_mask(uint32_t m8)
{
    uint64_t m = 0;
#pragma unroll
    for (int k = 0; k < GROUP; ++k)
        if (m8 >> k & 1u) m |= (uint64_t)((1u << BITS) - 1u) << (BITS * k);
    return m;
}

// dwords of LDS per packed chunk of 8 codes (6-bit chunks take 48 of the 64 bits)
template <int BITS>
constexpr int PKW = BITS == 4 ? 1 : 2;

// Quantizes 8 values (Eq. 2) and packs their codes, first value lowest.
//
// Fast form: b = bits(fma(x, inv, MAGIC)) is MAGIC_BITS + rne(x*inv); clamping b to [lo, lo + qmax]
// with lo = MAGIC_BITS - beta (one median-of-three) leaves lo + code.  The values are packed with
// shift-and-add in wrapping 32-bit arithmetic and the common offset lo * (1 + 2^BITS + 2^(2 BITS) + ...)
// is taken off once.  `live`: bit k clear forces code k to 0 (channels past the end of the row).
template <int BITS>
__device__ __forceinline__ void quant_pack(const float *val, uint32_t live, int32_t fast, float inv, int32_t beta,
                                           uint32_t &w0, uint32_t &w1)
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
#pragma unroll
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
        w0 = p - bias * 0x11111111u;
        w1 = 0;
    } else if constexpr (BITS == 8) {
        uint32_t p0 = 0, p1 = 0;
#pragma unroll
        for (int k = 3; k >= 0; --k) {
            p0 = (p0 << 8) + c[k];
            p1 = (p1 << 8) + c[k + 4];
        }
        w0 = p0 - bias * 0x01010101u;
        w1 = p1 - bias * 0x01010101u;
    } else {
        uint32_t h0 = 0, h1 = 0; // four 6-bit codes each
#pragma unroll
        for (int k = 3; k >= 0; --k) {
            h0 = (h0 << 6) + c[k];
            h1 = (h1 << 6) + c[k + 4];
        }
        h0 = (h0 - bias * 0x41041u) & 0xffffffu;
        h1 = (h1 - bias * 0x41041u) & 0xffffffu;
        w0 = h0 | (h1 << 24);
        w1 = h1 >> 8;
    }
}

// Sum of the 8 codes of a packed group.
template <int BITS>
__device__ __forceinline__ int32_t code_sum(uint32_t w0, uint32_t w1)
{
    if constexpr (BITS == 4) {
        return (int32_t)__builtin_amdgcn_udot8(w0, 0x11111111u, 0u, false);
    } else if constexpr (BITS == 8) {
        return (int32_t)__builtin_amdgcn_udot4(w0, 0x01010101u, __builtin_amdgcn_udot4(w1, 0x01010101u, 0u, false), false);
    } else {
        const uint32_t h0 = w0 & 0xffffffu, h1 = (w0 >> 24) | (w1 << 8);
        const uint32_t f = (h0 & 0x3f03fu) + ((h0 >> 6) & 0x3f03fu) + (h1 & 0x3f03fu) + ((h1 >> 6) & 0x3f03fu);
        return (int32_t)((f & 0xfffu) + (f >> 12));
    }
}

// Packed codes of output group g into the row.
template <int BITS>
__device__ __forceinline__ void store_group(uint8_t *out_row, int g, uint32_t w0, uint32_t w1)
{
    if constexpr (BITS == 4) {
        reinterpret_cast<uint32_t *>(out_row)[g] = w0;
    } else if constexpr (BITS == 8) {
        reinterpret_cast<uint2 *>(out_row)[g] = make_uint2(w0, w1);
    } else { // 6 bytes, 2-byte aligned
        uint16_t *o16 = reinterpret_cast<uint16_t *>(out_row + (int64_t)g * 6);
        o16[0] = (uint16_t)w0;
        o16[1] = (uint16_t)(w0 >> 16);
        o16[2] = (uint16_t)w1;
    }
}

// The 8 codes that start v codes into packed chunk u (0 <= v < 8): chunks u and u + 1 funnel-shifted.
// The word after the last chunk exists (and is only ever shifted out), and so does the one before the first.
// In two halves, so that the LDS reads can be issued long before the words are needed.
template <int BITS>
struct Window {
    uint32_t a0, a1, b0, b1; // chunk u, chunk u + 1 (a1, b1: 6 and 8 bits only)
};

template <int BITS>
__device__ __forceinline__ Window<BITS> funnel_fetch(const uint32_t *pk, int u)
{
    Window<BITS> w;
    if constexpr (BITS == 4) {
        w.a0 = pk[u];
        w.b0 = pk[u + 1];
        w.a1 = w.b1 = 0;
    } else {
        const uint2 a = reinterpret_cast<const uint2 *>(pk)[u], b = reinterpret_cast<const uint2 *>(pk)[u + 1];
        w.a0 = a.x; w.a1 = a.y; w.b0 = b.x; w.b1 = b.y;
    }
    return w;
}

// `vb` = BITS * v in its low 6 bits (whatever sits above them is ignored)
template <int BITS>
__device__ __forceinline__ void funnel_shift(const Window<BITS> &w, uint32_t vb, uint32_t &w0, uint32_t &w1)
{
    if constexpr (BITS == 4) {
        w0 = __builtin_amdgcn_alignbit(w.b0, w.a0, vb); // ({hi, lo} >> 4v), low 32 bits; the instruction reads 5 bits of vb
        w1 = 0;
    } else {
        const uint64_t A = (uint64_t)w.a0 | ((uint64_t)w.a1 << 32), B = (uint64_t)w.b0 | ((uint64_t)w.b1 << 32);
        const uint32_t sh = vb & 63u;
        uint64_t r;
        if constexpr (BITS == 6) {
            r = ((A >> sh) | (B << (48 - sh))) & 0xffffffffffffull;
        } else {
            const uint64_t up = B << ((64 - sh) & 63);
            r = (A >> sh) | (sh ? up : 0ull);
        }
        w0 = (uint32_t)r;
        w1 = (uint32_t)(r >> 32);
    }
}

template <int BITS>
__device__ __forceinline__ void funnel(const uint32_t *pk, int u, int v, uint32_t &w0, uint32_t &w1)
{
    funnel_shift<BITS>(funnel_fetch<BITS>(pk, u), (uint32_t)(BITS * v), w0, w1);
}

// The row loop is software-pipelined over three phases with TWO barriers per row, so that work bound by
// latency (LDS round trips, cross-lane reductions, dependent scalar chains) has dense arithmetic of another
// step of the path next to it between the same two barriers:
//   phase 1   step a1 of row r, first half: widen the row (it was requested one row earlier), request
//             row r + 1, x of the chunks that hold a source of a computed channel staged in LDS,
//             partial sums of the row statistics.
//   -- barrier (also: every wave has finished phase 3 of row r - 1)
//   phase 2   the LAST step of row r - 1: its output groups are assembled from the packed words and stored;
//             rstd (mu) from the partial sums; y = norm(x) in registers; min/max; steps a2 + a3 for the
//             computed channels, which normalise the staged x of their sources themselves (gamma and
//             beta of the staged chunks sit in LDS for the lifetime of the workgroup), so that no
//             barrier separates them from the rest of the row.
//   -- barrier
//   phase 3   range (Eq. 2), codes of the lane's own chunks packed in input order, codes of the
//             computed channels; runs on into phase 1 of row r + 1 without a barrier.
// Every buffer in LDS is written in one phase and read in the next, with one of the two barriers in between,
// and written again no earlier than a barrier after its last read: the packed words and the computed
// channels' codes of row r are written in its phase 3, read in phase 2 of row r + 1 (behind the first barrier)
// and written again in phase 3 of row r + 1 (behind the second).
// LayerNorm has one more barrier inside phase 2 (the mean has to be known before the squared
// deviations are summed).
//
// Every lane owns ITERS chunks of the row and as many plain output groups: the regular, dense part.  The
// irregular part -- computed channels, long rows, composite output groups -- is a few hundred items per row,
// dealt out over the lanes in order.  (Giving it to two extra wavefronts of its own was measured with 14 + 2
// wavefronts at the 70B shape: they take longer over the long rows and the composite groups than the others
// take over the row, 66 against 57 us.)
//
// Input channels that no output channel copies (split channels, channels merged away or into) must stay
// out of min/max, and their codes must not spill into their neighbours' bits.  The lane's own copy of
// gamma holds a NaN for them: y is then a NaN, which min/max skip and which the clamp of the quantizer
// turns into code 0, at no cost per row.
//
// NORM: QLLM_NORM_NONE / LAYER / RMS.  GAM_REG: the lane's share of gamma stays in registers for the
// lifetime of the workgroup; otherwise it is re-read (from L2) for every row, which frees 8 registers per chunk.
// FULL: the row fills the workgroup exactly (chunks = ITERS x lanes): no bounds tests.
// STREAM: for maps whose lists do not fit in LDS next to the row (a 28 672-channel row with a few thousand
// computed channels).  The lists of the irregular part stay in global memory (every workgroup reads the same
// few hundred KB: they live in L2), every chunk of the row is staged, in the input's own type, at its own
// position (the plan then has n_pub == n_chunks, so a staged position IS the channel number), and gamma /
// beta of a source are read from global memory by that number.
template <typename XT, int BITS, int ITERS, int NT_MAX, bool GAM_REG, int NORM, bool FULL, bool STREAM = false>
__global__ __launch_bounds__(NT_MAX) void fused_planned_kernel(const FusedArgs a)
{
    constexpr bool LAYER = NORM == QLLM_NORM_LAYER, RMS = NORM == QLLM_NORM_RMS;
    constexpr int W = PKW<BITS>;
    constexpr int QMAX = (1 << BITS) - 1;
    constexpr uint32_t NOT_PUBLISHED = 0xffffffu;
    extern __shared__ __align__(16) float lds[];
    const bool shift = LAYER && a.beta != nullptr;
    const int n_stage = GROUP * a.n_pub + 4;  // staged positions: the chunks that hold sources, then a zero
    const int goff = NORM != QLLM_NORM_NONE ? n_stage : 0, boff = goff + (shift ? n_stage : 0);
    float *pub = lds;                          // [n_stage] x of the staged chunks; [8 n_pub ..] stays zero
    float *pubg = lds + goff;                  // [n_stage] gamma at the same positions, 0 for the zero (not with NORM_NONE)
    float *pubb = lds + boff;                  // [n_stage] beta likewise (LayerNorm with a shift only)
    XT *pubx = reinterpret_cast<XT *>(lds);    // STREAM: [C + 8] the row as it came; [C ..] stays zero
    const int n_stage_words = STREAM ? (int)(((size_t)(a.C + GROUP) * sizeof(XT) + 15) / 16 * 4) : boff + n_stage;
    float *specv = lds + n_stage_words;        // [n_dest4] values of the computed channels
    const int n_dest4 = (a.n_dest + 3) & ~3;
    // the lists of the irregular part: copies in LDS, or (STREAM) the plan's own in global memory
    int4 *longs_w = reinterpret_cast<int4 *>(specv + n_dest4);         // [n_long] entries of the long rows
    uint4 *rec_w = reinterpret_cast<uint4 *>(longs_w + a.n_long);      // [n_comp][2] a composite group: its first two segments, its number
    int2 *spec_w = reinterpret_cast<int2 *>(rec_w + 2 * a.n_comp);     // [n_spec] {staged sources, scale}
    uint32_t *ins = STREAM ? reinterpret_cast<uint32_t *>(specv + n_dest4)
                           : reinterpret_cast<uint32_t *>(spec_w + a.n_spec); // [n_comp * W] codes of the computed channels, in place
    uint32_t *pk = ins + a.n_comp * W + W;                             // [-1 .. n_chunks] * W packed codes, input order; both ends zero
    int32_t *dest_w = reinterpret_cast<int32_t *>(pk + (a.n_chunks + 1) * W); // [n_dest] composite group << 3 | position
    uint32_t *segs_w = reinterpret_cast<uint32_t *>(dest_w + a.n_dest); // [n_segw] segments of the composite groups
    uint32_t *chunkw = STREAM ? pk + (a.n_chunks + 1) * W : segs_w + a.n_segw; // [ITERS * lanes] pass bits | staging slot << 8
    // [ITERS * lanes] the lanes' output slots, ready to use: {byte offset of the first of the group's two packed
    // chunks from pk (a plain group; else that of the zero chunk before pk), BITS * position in that chunk (6 bits) |
    // group or composite number << 8 | kind << 30}
    int2 *work = reinterpret_cast<int2 *>(chunkw + ((ITERS * blockDim.x + ((chunkw - reinterpret_cast<uint32_t *>(lds)) & 1)) )); // 8-byte aligned
    const int4 *longs = longs_w;
    const uint4 *rec = rec_w;
    const int2 *spec = spec_w;
    const int32_t *dest = dest_w;
    const uint32_t *segs = segs_w;
    if constexpr (STREAM) {
        longs = reinterpret_cast<const int4 *>(a.longs);
        rec = reinterpret_cast<const uint4 *>(a.recs);
        spec = reinterpret_cast<const int2 *>(a.spec);
        dest = a.dest;
        segs = reinterpret_cast<const uint32_t *>(a.segs);
    }
    __shared__ double red_d[2][16];
    __shared__ float red_f[32];
    __shared__ int32_t red_i[16];
    // bf16 rows are prefetched one row ahead; fp32 rows would need twice the registers and are not
    constexpr bool PREFETCH = sizeof(XT) == 2;
    // The streamed form puts the output groups of the row before together in phase 1 and pays a third barrier at
    // the end of phase 3 for it: its phase 2 is the long one (long rows, lists from L2), and the composite groups'
    // records come from L2 as well.
    constexpr bool OUT_IN_PHASE_1 = STREAM;

    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6;
    const int n_chunks = a.n_chunks;
    const float inf = __builtin_inff(), nan = __uint_as_float(0xffffffffu);

    // ---- the plan, once per workgroup.  Every lane first requests all it is going to need -- the first row,
    //      gamma, its shares of the plan's lists -- and only then starts to put things into LDS, so that the set-up
    //      costs about one trip to memory and not one per list.
    const XT *xbase = reinterpret_cast<const XT *>(a.x);
    Raw<XT> raw[ITERS];
    int64_t row = blockIdx.x;
    if (PREFETCH && row < a.N) { // the first row
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = tid + it * nt;
            load_raw(raw[it], xbase + row * a.ldx, (FULL || i < n_chunks ? i : n_chunks - 1) * GROUP);
        }
    }
    // composite groups that have a slot in the lanes' last pass, and those that have not
    const int comp_slot0 = max(a.n_work - a.n_comp, (ITERS - 1) * nt);
    const int n_loop = max(0, a.n_comp - max(0, ITERS * nt - comp_slot0));
    // The plan lists plain groups, then composite groups, then padding.  Plain and padding groups keep
    // the plan's order in the lanes' slots (slot it * lanes + lane), so that neighbouring lanes store
    // neighbouring groups.  Composite groups take the slots that are left in the lanes' last pass, as
    // kind << 30 | number; those that do not fit there (the first n_loop) are dealt out in a loop of their own.
    const int n_p = a.n_groups - a.n_comp, n_np = a.n_work - a.n_comp;
    uint32_t cw0[ITERS];
    int32_t we0[ITERS];
    float gam[GAM_REG ? ITERS : 1][GROUP];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int sl = tid + it * nt;
        cw0[it] = sl < n_chunks ? (uint32_t)a.chunks[sl] : (NOT_PUBLISHED << 8);
        we0[it] = WORK_NONE;
        if (sl < n_np) we0[it] = a.work[sl < n_p ? sl : sl + a.n_comp];
        else if (sl >= comp_slot0 && sl - comp_slot0 < a.n_comp - n_loop) we0[it] = (int32_t)((1u << 30) | (uint32_t)(n_loop + sl - comp_slot0));
        if constexpr (GAM_REG) load_gamma(gam[it], a.gamma, sl * GROUP, a.C, NORM != QLLM_NORM_NONE);
    }
    // the first lanes' worth of every list in flight at once; what is left of a longer list follows below
    const bool has_long = !STREAM && tid < a.n_long, has_spec = !STREAM && tid < a.n_spec, has_dest = !STREAM && tid < a.n_dest,
               has_rec = !STREAM && tid < a.n_comp;
    int4 l0 = make_int4(0, 0, 0, 0);
    int2 s0 = make_int2(0, 0);
    int32_t d0 = 0;
    uint4 ra = make_uint4(0, 0, 0, 0), rb = ra;
    if (has_long) l0 = reinterpret_cast<const int4 *>(a.longs)[tid];
    if (has_spec) s0 = reinterpret_cast<const int2 *>(a.spec)[tid];
    if (has_dest) d0 = a.dest[tid];
    if (has_rec) {
        ra = reinterpret_cast<const uint4 *>(a.recs)[2 * tid];
        rb = reinterpret_cast<const uint4 *>(a.recs)[2 * tid + 1];
    }
    uint32_t sg0[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) sg0[it] = !STREAM && tid + it * nt < a.n_segw ? (uint32_t)a.segs[tid + it * nt] : 0u;

    // A composite group's record {count | list << 8, d0, mask0, d1, mask1, group}: masks widened to code fields,
    // laid out for one pair of wide LDS reads.  The list itself (for groups of more than two segments) stays as
    // it is: {d, mask, -} per segment, widened where it is used.
    auto put_rec = [&](int c, const uint4 &p, const uint4 &q) {
        const uint64_t m0 = widen_mask<BITS>(p.z), m1 = widen_mask<BITS>(q.x);
        rec_w[2 * c] = make_uint4(p.x, p.y, (uint32_t)m0, (uint32_t)(m0 >> 32));
        rec_w[2 * c + 1] = make_uint4(p.w, (uint32_t)m1, (uint32_t)(m1 >> 32), q.y);
    };
    for (int j = tid; j < a.n_comp * W; j += nt) ins[j] = 0u;
    if constexpr (STREAM) {
        if (tid < GROUP) pubx[a.C + tid] = (XT)0; // the zero (bf16 bits or a float); gamma and beta of it read as 0
    } else if (tid < 4) { // the zero: x = 0, gamma = 0, beta = 0, so that its y is a zero whatever the row's statistics
        pub[GROUP * a.n_pub + tid] = 0.0f;
        if (NORM != QLLM_NORM_NONE) pubg[GROUP * a.n_pub + tid] = 0.0f;
        if (shift) pubb[GROUP * a.n_pub + tid] = 0.0f;
    }
    if (tid < W) {
        pk[n_chunks * W + tid] = 0u;
        pk[tid - W] = 0u;
    }
    if (tid < 16) { // reduction slots of waves that do not exist (or take no part) hold the identity
        red_d[0][tid] = 0.0;
        red_d[1][tid] = 0.0;
        red_f[tid] = inf;
        red_f[16 + tid] = inf; // minus the maximum
        red_i[tid] = 0;
    }
    if (has_long) longs_w[tid] = l0;
    if (has_spec) spec_w[tid] = s0;
    if (has_dest) dest_w[tid] = d0;
    if (has_rec) put_rec(tid, ra, rb);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int sl = tid + it * nt;
        chunkw[sl] = cw0[it];
        {
            const uint32_t e = (uint32_t)we0[it], kind = e >> 30;
            const int d = kind == KIND_PLAIN ? (int)(e & 0x1ffffu) : -GROUP; // non-plain: the zero chunk, not shifted
            const uint32_t number = kind == KIND_COMP ? e & 0x1ffffu : (e >> 17) & 0x1fffu;
            work[sl] = make_int2((d >> 3) * (W * 4), (int32_t)((uint32_t)(BITS * (d & 7)) | (number << 8) | (kind << 30)));
        }
        if (!STREAM && sl < a.n_segw) segs_w[sl] = sg0[it];
    }
    if constexpr (!STREAM) {
        for (int j = tid + nt; j < a.n_long; j += nt) longs_w[j] = reinterpret_cast<const int4 *>(a.longs)[j];
        for (int j = tid + nt; j < a.n_spec; j += nt) spec_w[j] = reinterpret_cast<const int2 *>(a.spec)[j];
        for (int j = tid + nt; j < a.n_dest; j += nt) dest_w[j] = a.dest[j];
        for (int j = tid + nt; j < a.n_comp; j += nt) put_rec(j, reinterpret_cast<const uint4 *>(a.recs)[2 * j], reinterpret_cast<const uint4 *>(a.recs)[2 * j + 1]);
        for (int j = tid + ITERS * nt; j < a.n_segw; j += nt) segs_w[j] = (uint32_t)a.segs[j];
    }
    // norm parameters of the staged chunks
    if constexpr (NORM != QLLM_NORM_NONE && !STREAM) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int sl = tid + it * nt;
            const uint32_t slot = cw0[it] >> 8;
            if (slot != NOT_PUBLISHED) {
                float g8[GROUP];
                if constexpr (GAM_REG) {
#pragma unroll
                    for (int k = 0; k < GROUP; ++k) g8[k] = gam[it][k];
                } else {
                    load_gamma(g8, a.gamma, sl * GROUP, a.C, true);
                }
#pragma unroll
                for (int k = 0; k < GROUP; ++k) pubg[slot * GROUP + k] = g8[k];
                if (shift) {
                    load_gamma(g8, a.beta, sl * GROUP, a.C, true);
#pragma unroll
                    for (int k = 0; k < GROUP; ++k) pubb[slot * GROUP + k] = g8[k];
                }
            }
        }
    }
    // gamma of the lane's chunks; NaN where the input channel is copied by no output channel (see above)
    // and for chunks past the end of the row.  NORM_NONE multiplies by 1 (exact) or NaN.
    auto mask_gamma = [&](float *g, uint32_t passes) {
#pragma unroll
        for (int j = 0; j < GROUP; ++j) g[j] = (passes >> j & 1u) ? g[j] : nan;
    };
    if constexpr (GAM_REG) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) mask_gamma(gam[it], tid + it * nt < n_chunks ? cw0[it] & 0xffu : 0u);
        // gamma has to have arrived before the row loop is entered: a load still pending there would make
        // every pass of the loop wait for whatever was requested last, the next row's prefetch included.
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
#pragma unroll
            for (int j = 0; j < GROUP; ++j) asm volatile("" : "+v"(gam[it][j]));
        }
    }

    // The reduction slots were set by the first lanes of wave 0; the other waves write theirs before
    // the first barrier of the first row, so the set-up has to be over for everybody first.
    __syncthreads();

    const uint32_t zero_at = (uint32_t)(GROUP * a.n_pub);
    // `prev`: the row whose output groups are still to be stored.  At first the first row itself: its place in
    // the output then receives codes made of whatever LDS holds, and the real ones one pass later.
    int64_t prev = row;

    // rowsum of a finished row: the waves' partial sums are complete once a barrier has passed
    auto finish_rowsum = [&](int64_t r) {
        if (wave == 0) {
            const int32_t s = dpp_add_row16(red_i[lane & 15]);
            if (lane == 0) a.rowsum[r] = s;
        }
    };
    // Eq. (2) for one value
    auto one_code = [&](float v, int32_t fast, float inv, int32_t beta) -> uint32_t {
        if (fast) {
            const float lo = __int_as_float(MAGIC_BITS - beta), hi = __int_as_float(MAGIC_BITS - beta + QMAX);
            return __float_as_uint(__builtin_amdgcn_fmed3f(__builtin_fmaf(v, inv, MAGIC), lo, hi)) - (uint32_t)(MAGIC_BITS - beta);
        }
        return slow_code(v, inv, beta, QMAX);
    };

    // ---- step a4, second half, of the row before: the output groups.  A plain group is two neighbouring
    //      packed words funnel-shifted; a composite group is several such windows, each masked to the
    //      channels it supplies, plus the codes of its computed channels.
    struct RecPair {
        uint4 r0, r1;
    };
    auto rec_fetch = [&](int comp) -> RecPair { return RecPair{rec[2 * comp], rec[2 * comp + 1]}; };
    auto composite_of = [&](const RecPair &rp, int comp, uint32_t &w0, uint32_t &w1) -> int {
        uint4 r0 = rp.r0, r1 = rp.r1; // {count | list << 8, d0, mask0}, {d1, mask1, group}
        if constexpr (STREAM) { // the plan's own record {count | list << 8, d0, mask0, d1}, {mask1, group, -, -}: masks still one bit per code
            const uint64_t m0 = widen_mask<BITS>(r0.z), m1 = widen_mask<BITS>(r1.x);
            r1 = make_uint4(r0.w, (uint32_t)m1, (uint32_t)(m1 >> 32), r1.y);
            r0 = make_uint4(r0.x, r0.y, (uint32_t)m0, (uint32_t)(m0 >> 32));
        }
        uint32_t i0 = ins[comp * W], i1 = 0u;
        ins[comp * W] = 0u; // ready for the next row's codes
        if constexpr (W == 2) {
            i1 = ins[comp * W + 1];
            ins[comp * W + 1] = 0u;
        }
        uint32_t f0, f1, g0, g1;
        funnel<BITS>(pk, (int)r0.y >> 3, r0.y & 7, f0, f1);
        funnel<BITS>(pk, (int)r1.x >> 3, r1.x & 7, g0, g1);
        i0 |= (f0 & r0.z) | (g0 & r1.y);
        if constexpr (W == 2) i1 |= (f1 & r0.w) | (g1 & r1.z);
        const int n_seg = r0.x & 0xffu, off = r0.x >> 8;
        for (int sg = 2; sg < n_seg; ++sg) {
            const int ds = (int)segs[off + 1 + 3 * sg];
            const uint64_t m = widen_mask<BITS>(segs[off + 2 + 3 * sg]);
            funnel<BITS>(pk, ds >> 3, ds & 7, f0, f1);
            i0 |= f0 & (uint32_t)m;
            if constexpr (W == 2) i1 |= f1 & (uint32_t)(m >> 32);
        }
        w0 = i0;
        w1 = i1;
        return (int)r1.w;
    };
    auto composite = [&](int comp, uint32_t &w0, uint32_t &w1) -> int { return composite_of(rec_fetch(comp), comp, w0, w1); };
    // The output pass in pieces, so that the row loop can put other work between its LDS reads and their use.
    struct OutState {
        int2 e[ITERS];
        Window<BITS> win[ITERS];
        RecPair rp; // STREAM: the record of the last slot's composite group, requested together with the packed words
    };
    auto out_read_work = [&](OutState &o, int ltid) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) o.e[it] = work[ltid + it * nt];
        if constexpr (STREAM) { // the record of the last slot's composite group comes from global memory: asked for early
            const bool comp = ((uint32_t)o.e[ITERS - 1].y >> 30) == KIND_COMP;
            o.rp = rec_fetch(comp ? (o.e[ITERS - 1].y >> 8) & 0x3fffff : 0);
        }
    };
    auto out_read_codes = [&](OutState &o) { // padding and composite groups read the row's first words and drop them
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            o.win[it] = funnel_fetch<BITS>(reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(pk) + o.e[it].x), 0);
        }
    };
    auto out_store = [&](OutState &o, int64_t prev, int ltid) {
        int32_t sum = 0;
        uint8_t *out_row = a.codes + prev * a.row_bytes;
        int g[ITERS];
        uint32_t w0[ITERS], w1[ITERS];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            funnel_shift<BITS>(o.win[it], (uint32_t)o.e[it].y, w0[it], w1[it]); // not a plain group: all zero
            g[it] = (o.e[it].y >> 8) & 0x3fffff;
        }
        // composite groups sit in slots of the last pass only
        if (((uint32_t)o.e[ITERS - 1].y >> 30) == KIND_COMP) {
            const int comp = g[ITERS - 1];
            if constexpr (STREAM) g[ITERS - 1] = composite_of(o.rp, comp, w0[ITERS - 1], w1[ITERS - 1]);
            else g[ITERS - 1] = composite(comp, w0[ITERS - 1], w1[ITERS - 1]);
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            if (FULL || ((uint32_t)o.e[it].y >> 30) != KIND_NONE) {
                store_group<BITS>(out_row, g[it], w0[it], w1[it]);
                sum += code_sum<BITS>(w0[it], w1[it]);
            }
        }
        if (n_loop > 0) { // more composite groups than free slots; the next one's record is under way while this one is put together
            RecPair next = rec_fetch(ltid < n_loop ? ltid : 0);
            for (int comp = ltid; comp < n_loop; comp += nt) {
                const RecPair cur = next;
                if (comp + nt < n_loop) next = rec_fetch(comp + nt);
                uint32_t c0, c1;
                const int gc = composite_of(cur, comp, c0, c1);
                store_group<BITS>(out_row, gc, c0, c1);
                sum += code_sum<BITS>(c0, c1);
            }
        }
        return sum;
    };

    for (; row < a.N; row += gridDim.x) {
        // Addresses derived from the lane's number cost an instruction or two per row to recompute, but a
        // register each to keep: hide from the optimiser that the number does not change from row to row.
        int ltid = threadIdx.x;
        asm volatile("" : "+v"(ltid));

        // ================= phase 1
        // In the order the hardware should see it (scheduling fences in between): LDS reads first, dense
        // arithmetic while they are under way, and the next row's loads spread out between blocks of
        // arithmetic instead of in one burst (a dozen wavefronts asking for 57 KB at once queue up in the address unit).
        OutState o;
        uint32_t slot[ITERS];
        if constexpr (OUT_IN_PHASE_1) {
            out_read_work(o, ltid);
            out_read_codes(o);
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) slot[it] = chunkw[ltid + it * nt] >> 8;
        __builtin_amdgcn_sched_barrier(0);

        // ---- step a1, first half.  A bf16 row is already here (it was requested while the row before it
        //      was worked on): widen it; the next one goes into the same registers further down.
        float y[ITERS][GROUP]; // x until phase 2 turns it into y in place
        if constexpr (!PREFETCH) {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int i = ltid + it * nt;
                if (FULL || i < n_chunks) load_raw(raw[it], xbase + row * a.ldx, i * GROUP);
            }
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            if (FULL || ltid + it * nt < n_chunks) {
                widen(raw[it], y[it]);
                if constexpr (STREAM) *reinterpret_cast<Raw<XT> *>(pubx + (ltid + it * nt) * GROUP) = raw[it]; // the whole row is staged
            } else {
#pragma unroll
                for (int j = 0; j < GROUP; ++j) y[it][j] = 0.0f;
            }
            // here and now: the optimiser would rather widen where x is first used, further down, and
            // keep the row's packed form alive next to the registers the next row is loaded into
#pragma unroll
            for (int j = 0; j < GROUP; ++j) asm volatile("" : "+v"(y[it][j]));
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- row statistics in fp64 (two interleaved partial sums per lane: the additions do not wait for one
        //      another; the order is fixed, so the result is reproducible; slots past the row hold 0), with
        //      the next row's loads in between.  Those are unconditional, so that the loaded registers ARE the
        //      next pass's row (a load under a condition would be merged with the old contents at the end of
        //      the condition, which waits for it): the last pass requests its own row again, lanes past the end
        //      of the row the row's last chunk.  They come before the stores of the row before: loads and stores
        //      retire through one counter, and a wait for the row placed after those stores would wait for them too.
        double s0 = 0.0, s1 = 0.0;
        {
            const int64_t next = row + gridDim.x, again = next < a.N ? next : row;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                if constexpr (PREFETCH) {
                    const int i = ltid + it * nt;
                    load_raw(raw[it], xbase + again * a.ldx, (FULL || i < n_chunks ? i : n_chunks - 1) * GROUP);
                }
                if constexpr (NORM != QLLM_NORM_NONE) {
#pragma unroll
                    for (int j = 0; j < GROUP; j += 2) {
                        const double d0 = (double)y[it][j], d1 = (double)y[it][j + 1];
                        if constexpr (RMS) {
                            s0 = __builtin_fma(d0, d0, s0);
                            s1 = __builtin_fma(d1, d1, s1);
                        } else {
                            s0 += d0;
                            s1 += d1;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        if constexpr (OUT_IN_PHASE_1) {
            int32_t sum = out_store(o, prev, ltid);
            sum = wave_sum_i32(sum);
            if (lane == 0) red_i[wave] = sum;
        }
        // ---- x of the chunks that hold a source of a computed channel (normalised by its readers in phase 2)
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            if (!STREAM && slot[it] != NOT_PUBLISHED) {
                float4 *dst = reinterpret_cast<float4 *>(pub + slot[it] * GROUP);
                dst[0] = make_float4(y[it][0], y[it][1], y[it][2], y[it][3]);
                dst[1] = make_float4(y[it][4], y[it][5], y[it][6], y[it][7]);
            }
        }
        // ---- the wavefront's shares of the two sums
        if constexpr (NORM != QLLM_NORM_NONE) {
            const double s = wave_sum(s0 + s1);
            if (lane == 0) red_d[0][wave] = s;
        }
        __syncthreads(); // partial statistics, staged x; and every wave is done with phase 3 of the row before:
                         // its packed words and the codes of its computed channels are complete

        // ================= phase 2
        // ---- step a4, second half, of the row before: the words its output groups are made of are requested
        //      first and put together further down, after the dense arithmetic of this row
        if constexpr (OUT_IN_PHASE_1) finish_rowsum(prev);
        else out_read_work(o, ltid);
        // What a computed channel reads does not depend on the row's statistics: the first pass's entries and
        // the staged x, gamma (beta) of their sources are requested now and used after rstd is known.
        struct Staged {
            float x, g, b;
        };
        auto staged_fetch = [&](uint32_t pos) -> Staged {
            Staged v;
            if constexpr (STREAM) {
                const bool real = pos < (uint32_t)a.C; // else the zero
                v.x = widen_one(pubx[pos]);
                v.g = NORM != QLLM_NORM_NONE ? (real ? a.gamma[pos] : 0.0f) : 1.0f;
                v.b = shift && real ? a.beta[pos] : 0.0f;
            } else {
                v.x = pub[pos];
                v.g = NORM != QLLM_NORM_NONE ? pubg[pos] : 1.0f;
                v.b = shift ? pubb[pos] : 0.0f;
            }
            return v;
        };
        const bool spec0 = ltid < a.n_spec;
        const int2 item0 = spec0 ? spec[ltid] : make_int2((int32_t)(zero_at | (zero_at << 16)), 0);
        const Staged src0 = staged_fetch((uint32_t)item0.x & 0xffffu), src1 = staged_fetch((uint32_t)item0.x >> 16);

        float mu = 0.0f, rstd = 1.0f;
        if constexpr (RMS) {
            rstd = rsqrt_to_f32(total16(red_d[0], lane) * a.inv_C + (double)a.eps);
        } else if constexpr (LAYER) {
            const double mu64 = total16(red_d[0], lane) * a.inv_C;
            double q = 0.0;
            {
                double q0 = 0.0, q1 = 0.0;
#pragma unroll
                for (int it = 0; it < ITERS; ++it) {
                    if (FULL || ltid + it * nt < n_chunks) {
#pragma unroll
                        for (int j = 0; j < GROUP; j += 2) {
                            const double d0 = (double)y[it][j] - mu64, d1 = (double)y[it][j + 1] - mu64;
                            q0 = __builtin_fma(d0, d0, q0);
                            q1 = __builtin_fma(d1, d1, q1);
                        }
                    }
                }
                q = q0 + q1;
            }
            q = wave_sum(q);
            if (lane == 0) red_d[1][wave] = q;
            __syncthreads();
            mu = (float)mu64;
            rstd = rsqrt_to_f32(total16(red_d[1], lane) * a.inv_C + (double)a.eps);
        }

        // y of a staged position (a source of a computed channel), normalised exactly as its owner does below
        auto staged_norm = [&](const Staged &v) -> float {
            float t = v.x;
            if constexpr (NORM != QLLM_NORM_NONE) {
                if constexpr (LAYER) t = t - mu;
                t = t * rstd;
                t = t * v.g;
                if constexpr (LAYER) {
                    if (shift) t = t + v.b;
                }
            }
            return t;
        };
        auto staged_y = [&](uint32_t pos) -> float { return staged_norm(staged_fetch(pos)); };

        // ---- y in registers, in place; min/max over the channels that some output channel copies (all
        //      others are NaN by now)
        float mn = inf, mx = -inf;
        {
            const float *gamma_row = a.gamma, *beta_row = a.beta; // opaque, so that per-row loads stay per row
            asm volatile("" : "+s"(gamma_row), "+s"(beta_row));
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int i = ltid + it * nt;
                float gjit[GROUP];
                if constexpr (!GAM_REG) {
                    load_gamma(gjit, gamma_row, i * GROUP, a.C, NORM != QLLM_NORM_NONE);
                    mask_gamma(gjit, chunkw[i] & 0xffu);
                }
                const float *g8 = GAM_REG ? gam[GAM_REG ? it : 0] : gjit;
                float bj[GROUP];
                if constexpr (LAYER) load_gamma(bj, beta_row, i * GROUP, a.C, shift); // beta: re-read (from L2) for every row
#pragma unroll
                for (int j = 0; j < GROUP; ++j) {
                    float t = y[it][j];
                    if constexpr (LAYER) t = t - mu;
                    if constexpr (NORM != QLLM_NORM_NONE) t = t * rstd;
                    t = t * g8[j];
                    if constexpr (LAYER) {
                        if (shift) t = t + bj[j];
                    }
                    y[it][j] = t;
                }
#pragma unroll
                for (int j = 0; j < GROUP; j += 2) {
                    mn = fminf(fminf(mn, y[it][j]), y[it][j + 1]);
                    mx = fmaxf(fmaxf(mx, y[it][j]), y[it][j + 1]);
                }
            }
        }

        // ---- step a4, second half, of the row before: its output groups put together and stored; the wavefront's
        //      share of that row's code sum goes through the same barrier as this row's min/max
        if constexpr (!OUT_IN_PHASE_1) {
            out_read_codes(o);
            int32_t sum = out_store(o, prev, ltid);
            sum = wave_sum_i32(sum);
            if (lane == 0) red_i[wave] = sum;
        }

        {
            // ---- steps a2 + a3 for the computed channels of one entry (sub-channels, scale 1/T, Eq. 3) or of
            //      two entries of equal scale (a merged pair, Eq. 4); one per lane and pass.
            {
                const float sc = __int_as_float(item0.y);
                float xv = sc * staged_norm(src0);
                xv = xv + sc * staged_norm(src1);
                if (spec0) {
                    mn = fminf(mn, xv);
                    mx = fmaxf(mx, xv);
                    specv[ltid] = xv;
                }
            }
            if (a.n_spec > nt)
            for (int j = ltid + nt; j < a.n_spec; j += nt) {
                const int2 item = spec[j];
                const float sc = __int_as_float(item.y);
                float xv = sc * staged_y((uint32_t)item.x & 0xffffu);
                xv = xv + sc * staged_y((uint32_t)item.x >> 16);
                mn = fminf(mn, xv);
                mx = fmaxf(mx, xv);
                specv[j] = xv;
            }
            // Long rows (a channel merged from three or more, Eq. 4).  The sum runs left to right in
            // fp32, so its order is fixed; its latency need not be.  Entry e of the table belongs to lane
            // e % 64 and a row sits in consecutive lanes of one wavefront: every lane forms its product,
            // then "value of the lane below + own product" is repeated; the lane of entry number pos is
            // final after pos repeats (repeating it again changes nothing) and the row's last lane
            // ends up with the row's value.  Every entry carries the largest pos of its wavefront.
            for (int base = 0; base < a.n_long; base += nt) {
                const int e = base + ltid;
                int4 le = make_int4((int32_t)zero_at, -1, 0, 0);
                if (e < a.n_long) le = longs[e];
                const float p = __int_as_float(le.z) * staged_y((uint32_t)le.x);
                // keep = 1 takes the value of the lane below, keep = 0 (a row's first entry) drops it: fma(v, 1, p) is
                // the correctly rounded v + p, fma(v, 0, p) is p
                const float keep = (le.w & 0xff) > 0 ? 1.0f : 0.0f;
                const int steps = __builtin_amdgcn_readfirstlane(le.w >> 8);
                float acc = p;
                int t = 0;
                for (; t + 4 <= steps; t += 4) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc = chain_step(acc, keep, p);
                }
                for (; t < steps; ++t) acc = chain_step(acc, keep, p);
                if (le.y >= 0) {
                    specv[le.y] = acc;
                    mn = fminf(mn, acc);
                    mx = fmaxf(mx, acc);
                }
            }
            // Rows of more than 64 entries (a few "hub" channels that very many others were merged into): one
            // wavefront per row, 64 entries at a time by the same lane-by-lane addition; the sum so far enters the
            // next block as "sum + first product", which is the next step of the same left-to-right order.  Their
            // lists are read from global memory (they are short and rare).
            if (a.n_xl > 0) {
                for (int r = wave; r < a.n_xl; r += nt >> 6) {
                    const int4 hd = reinterpret_cast<const int4 *>(a.xlrows)[r];
                    const int first = __builtin_amdgcn_readfirstlane(hd.x), n = __builtin_amdgcn_readfirstlane(hd.y);
                    const int value_slot = __builtin_amdgcn_readfirstlane(hd.z);
                    const float keep = lane > 0 ? 1.0f : 0.0f;
                    float sum = 0.0f;
                    for (int e0 = 0; e0 < n; e0 += 256) { // four blocks' entries and staged values requested at once
                        int2 item[4];
                        Staged sv[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int e = e0 + 64 * u + lane;
                            item[u] = make_int2((int32_t)zero_at, 0);
                            if (e < n) item[u] = reinterpret_cast<const int2 *>(a.xlent)[first + e];
                        }
#pragma unroll
                        for (int u = 0; u < 4; ++u) sv[u] = staged_fetch((uint32_t)item[u].x);
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int b0 = e0 + 64 * u;
                            if (b0 < n) {
                                float p = __int_as_float(item[u].y) * staged_norm(sv[u]);
                                if (b0 > 0 && lane == 0) p = sum + p;
                                const int steps = n - b0 - 1 < 63 ? n - b0 - 1 : 63; // the block's last entry sits in this lane
                                float acc = p;
                                for (int t = 0; t < steps; ++t) acc = chain_step(acc, keep, p);
                                sum = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(acc), steps));
                            }
                        }
                    }
                    if (lane == 0) {
                        specv[value_slot] = sum;
                        mn = fminf(mn, sum);
                        mx = fmaxf(mx, sum);
                    }
                }
            }
        }

        // ---- per-token range (Eq. 2)
        wave_minmax(mn, mx);
        if (lane == 0) {
            red_f[wave] = mn;
            red_f[16 + wave] = -mx; // negated: one butterfly of minima then serves both
        }
        __syncthreads(); // also: the computed channels' values are complete

        // ================= phase 3
        if constexpr (!OUT_IN_PHASE_1) finish_rowsum(prev);
        const bool code0 = ltid < a.n_dest;
        const float spec_v0 = code0 ? specv[ltid] : 0.0f; // first pass of the computed channels' codes:
        const int32_t spec_d0 = code0 ? dest[ltid] : 0;    // requested now, used after the range is known
        {
            const float v = dpp_min_row16(red_f[lane & 31]);
            mn = lane_f32(v, 0);
            mx = -lane_f32(v, 16);
        }
        const float range = mx - mn;
        const float alpha = range > 0.0f ? range / (float)QMAX : 1.0f;
        const float inv = 1.0f / alpha;
        const int32_t fast = __builtin_amdgcn_readfirstlane(fabsf(mn * inv) < FAST_LIMIT && fabsf(mx * inv) < FAST_LIMIT); // a scalar: a branch, not a lane mask
        int32_t beta;
        if (fast) beta = -rne_product_fast(mn, inv);
        else beta = (int32_t)fmin(fmax(-rne_product_slow(mn, inv), -2147483647.0), 2147483647.0);

        if (tid == 0) { // early, so that the stores have retired when the next row is waited for
            a.alpha[row] = alpha;
            a.zero[row] = beta;
        }

        // ---- step a4, first half: codes of the lane's own chunks, packed in input order
        {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int i = ltid + it * nt;
                if (FULL || i < n_chunks) {
                    uint32_t w0, w1;
                    quant_pack<BITS>(y[it], 0xffu, fast, inv, beta, w0, w1);
                    if constexpr (W == 1) pk[i] = w0;
                    else reinterpret_cast<uint2 *>(pk)[i] = make_uint2(w0, w1);
                }
            }
        }
        // codes of the computed channels, straight into their place in their group's word
        {
            auto put_code = [&](float v, int32_t dj) {
                const uint32_t code = one_code(v, fast, inv, beta);
                if constexpr (W == 1) {
                    atomicOr(&ins[dj >> 3], code << (BITS * (dj & 7)));
                } else {
                    atomicOr(reinterpret_cast<unsigned long long *>(ins) + (dj >> 3), (unsigned long long)code << (BITS * (dj & 7)));
                }
            };
            if (code0) put_code(spec_v0, spec_d0);
            if (a.n_dest > nt)
                for (int j = ltid + nt; j < a.n_dest; j += nt) put_code(specv[j], dest[j]);
        }
        // no barrier here: what this phase wrote is read behind the first barrier of the next row and written
        // again behind its second
        if constexpr (OUT_IN_PHASE_1) __syncthreads(); // packed words and computed channels' codes complete
        prev = row;
    }
    // the last row's output groups
    {
        __syncthreads(); // packed words and computed channels' codes complete
        const int ltid = threadIdx.x;
        OutState o;
        out_read_work(o, ltid);
        out_read_codes(o);
        int32_t sum = out_store(o, prev, ltid);
        sum = wave_sum_i32(sum);
        if (lane == 0) red_i[wave] = sum;
        __syncthreads();
        finish_rowsum(prev);
    }
}

struct Shape {
    int iters, nt; // chunks per lane, lanes
};

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

// Chunks (or output groups) per lane and the workgroup size for N rows of `units` of them.  A workgroup's
// waves go to the CU's four SIMDs in turn, so the SIMD with the most of them, ceil(waves / 4), sets the pace:
// the cost of a row is that count times (chunks per lane + the fixed work of a wave and row, about one
// chunk's worth).  With fewer rows than CUs every workgroup has one row and the fewest chunks per lane win.
// The irregular part of the plan (long-row entries, computed channels, composite groups) is dealt out over the
// lanes, and every further pass over one of its lists is a chain of dependent LDS reads that nothing overlaps:
// if some shape has enough lanes for the longest of the three lists (`irregular`), only such shapes are
// considered; if none has, the one with the most lanes.  (Measured at the 5120- and 4096-channel shapes over maps
// from 1 % to 25 % of the channels merged: the best of the shapes in nine cases of ten, and up to 1.8 times
// faster than the shape the regular part alone would pick.)
Shape pick_shape(int units, int64_t N, bool layer_norm, int irregular)
{
    Shape best{0, 0};
    int best_cost = 0;
    bool best_covers = false;
    for (int iters = 1; iters <= (layer_norm ? 4 : 5); ++iters) { // LayerNorm at five chunks per lane spills
        const int nt = ((units + iters - 1) / iters + 63) / 64 * 64;
        if (nt > (iters == 5 ? 768 : 1024)) continue; // five chunks per lane need the registers of three waves per SIMD
        const int waves = nt / 64;
        const int cost = N <= cu_count() ? iters : (waves + 3) / 4 * (iters + 1);
        const bool covers = nt >= irregular;
        // a shape that covers beats one that does not; among equals the cheaper one; the first feasible shape has
        // the most lanes and stays if nothing covers
        const bool better = best.iters == 0 || (covers && !best_covers) || (covers == best_covers && covers && cost < best_cost);
        if (better) {
            best = {iters, nt};
            best_cost = cost;
            best_covers = covers;
        }
    }
    return best;
}

// What the runtime is asked once per kernel, workgroup size and LDS size and then remembered (no runtime
// query sits between a caller's stream capture and the launch): the raised LDS limit and the number of
// resident workgroups per CU.
constexpr int MAX_LDS = (int)qllm_detail::FUSED_MAX_LDS; // dynamic LDS a launch may ask for
struct LaunchFacts {
    const void *kernel;
    int nt;
    size_t lds;
    int per_cu;
};
std::mutex facts_lock;
std::vector<LaunchFacts> facts;

template <typename K>
int32_t launch(K kernel, const FusedArgs &a, const Shape &sh, size_t lds, hipStream_t stream)
{
    const void *fn = reinterpret_cast<const void *>(kernel);
    int per_cu = 0;
    {
        std::lock_guard<std::mutex> hold(facts_lock);
        for (const LaunchFacts &f : facts)
            if (f.kernel == fn && f.nt == sh.nt && f.lds == lds) per_cu = f.per_cu;
        if (per_cu == 0) {
            bool seen = false;
            for (const LaunchFacts &f : facts) seen = seen || f.kernel == fn;
            if (!seen) { // once per kernel, to the most this file ever asks for (see MAX_LDS below)
                const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
                if (e != hipSuccess) {
                    (void)hipGetLastError();
                    qllm_note_hip_error("planned fused kernel: raising the LDS limit", hipGetErrorName(e));
                    return QLLM_ERR_HIP;
                }
            }
            // resident workgroups per CU (registers, LDS, lanes): the grid is exactly what is resident at once
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, sh.nt, lds) != hipSuccess) {
                (void)hipGetLastError();
                per_cu = 1;
            }
            if (per_cu < 1) per_cu = 1;
            facts.push_back(LaunchFacts{fn, sh.nt, lds, per_cu});
        }
    }
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

template <typename XT, int BITS, int NORM, bool FULL>
int32_t dispatch(const FusedArgs &a, const Shape &sh, size_t lds, bool stream_lists, hipStream_t stream)
{
    // 4 chunks per lane: gamma fits in registers next to y and the prefetched row, except with LayerNorm
    if (stream_lists) return launch(fused_planned_kernel<XT, BITS, 4, 1024, NORM != QLLM_NORM_LAYER, NORM, FULL, true>, a, sh, lds, stream);
    if (sh.iters == 1) return launch(fused_planned_kernel<XT, BITS, 1, 1024, true, NORM, FULL>, a, sh, lds, stream);
    if (sh.iters == 2) return launch(fused_planned_kernel<XT, BITS, 2, 1024, true, NORM, FULL>, a, sh, lds, stream);
    if (sh.iters == 3) return launch(fused_planned_kernel<XT, BITS, 3, 1024, NORM != QLLM_NORM_LAYER, NORM, FULL>, a, sh, lds, stream);
    if constexpr (NORM != QLLM_NORM_LAYER) {
        if (sh.iters == 5) return launch(fused_planned_kernel<XT, BITS, 5, 768, true, NORM, FULL>, a, sh, lds, stream);
    }
    return launch(fused_planned_kernel<XT, BITS, 4, 1024, NORM != QLLM_NORM_LAYER, NORM, FULL>, a, sh, lds, stream);
}

template <typename XT, int BITS, int NORM>
int32_t dispatch_full(const FusedArgs &a, const Shape &sh, size_t lds, bool stream_lists, hipStream_t stream)
{
    // every lane has its chunks and every slot a group (the composite groups all fit in the last pass's slots;
    // otherwise the slots before that pass that the plain groups leave over stay empty)
    const bool full = a.n_chunks == sh.iters * sh.nt && a.n_work == a.n_chunks && a.n_comp <= sh.nt;
    return full ? dispatch<XT, BITS, NORM, true>(a, sh, lds, stream_lists, stream) : dispatch<XT, BITS, NORM, false>(a, sh, lds, stream_lists, stream);
}

template <typename XT, int BITS>
int32_t dispatch_norm(const FusedArgs &a, const Shape &sh, size_t lds, bool stream_lists, hipStream_t stream)
{
    if (a.norm == QLLM_NORM_LAYER) return dispatch_full<XT, BITS, QLLM_NORM_LAYER>(a, sh, lds, stream_lists, stream);
    if (a.norm == QLLM_NORM_RMS) return dispatch_full<XT, BITS, QLLM_NORM_RMS>(a, sh, lds, stream_lists, stream);
    return dispatch_full<XT, BITS, QLLM_NORM_NONE>(a, sh, lds, stream_lists, stream);
}

template <typename XT>
int32_t dispatch_bits(const FusedArgs &a, int bits, const Shape &sh, size_t lds, bool stream_lists, hipStream_t stream)
{
    if (bits == 4) return dispatch_norm<XT, 4>(a, sh, lds, stream_lists, stream);
    if (bits == 6) return dispatch_norm<XT, 6>(a, sh, lds, stream_lists, stream);
    return dispatch_norm<XT, 8>(a, sh, lds, stream_lists, stream);
}

// Which form of the kernel a map gets, with its launch shape and LDS size: the lists of the irregular part in
// LDS when they fit there next to the row's packed codes; else, if the plan stages every chunk, the lists
// streamed from global memory; else none (the caller then runs the kernel that walks the CSR map).
struct Choice {
    int kind; // QLLM_FUSED_WALKS_MAP / QLLM_FUSED_LISTS_IN_LDS / QLLM_FUSED_LISTS_STREAMED
    Shape sh;
    size_t lds;
};

Choice choose(const FusedArgs &a, int32_t x_dtype, int32_t bits)
{
    Choice c{QLLM_FUSED_WALKS_MAP, {0, 0}, 0};
    const int units = a.n_chunks > a.n_work ? a.n_chunks : a.n_work;
    if (!a.work || units > 4096 || !a.vec_ok || a.C % GROUP != 0) return c;
    const qllm_detail::PlanCounts p{a.n_comp, a.n_long, a.n_pub, a.n_chunks, a.n_spec, a.n_dest, a.n_segw};
    const int64_t w = bits == 4 ? 1 : 2;
    {
        const int irregular = std::max(a.n_long, std::max(a.n_spec, a.n_comp));
        const Shape sh = pick_shape(units, a.N, a.norm == QLLM_NORM_LAYER, irregular);
        // staged x, and gamma / beta at the same positions when there is a norm / a shift
        const int64_t stage_sets = 1 + (a.norm != QLLM_NORM_NONE ? 1 : 0) + (a.norm == QLLM_NORM_LAYER && a.beta ? 1 : 0);
        const int64_t lds = qllm_detail::fused_lists_lds_bytes(p, w, stage_sets, (int64_t)sh.iters * sh.nt);
        if (lds <= MAX_LDS) return Choice{QLLM_FUSED_LISTS_IN_LDS, sh, (size_t)lds};
    }
    if (a.n_pub != a.n_chunks) return c; // staged positions are not channel numbers
    const Shape sh{4, ((units + 3) / 4 + 63) / 64 * 64};
    const int64_t lds = qllm_detail::fused_streamed_lds_bytes(p, w, a.C, x_dtype == QLLM_BF16 ? 2 : 4, (int64_t)sh.iters * sh.nt);
    if (lds <= MAX_LDS) return Choice{QLLM_FUSED_LISTS_STREAMED, sh, (size_t)lds};
    return c;
}

} // namespace

int32_t qllm_choose_fused_planned(const FusedArgs &a, int32_t x_dtype, int32_t bits) { return choose(a, x_dtype, bits).kind; }

int32_t qllm_launch_fused_planned(const FusedArgs &a, int32_t x_dtype, int32_t bits, hipStream_t stream)
{
    const Choice c = choose(a, x_dtype, bits);
    if (c.kind == QLLM_FUSED_WALKS_MAP) return QLLM_ERR_WORKSPACE;
    const bool stream_lists = c.kind == QLLM_FUSED_LISTS_STREAMED;
    if (x_dtype == QLLM_BF16) return dispatch_bits<uint16_t>(a, bits, c.sh, c.lds, stream_lists, stream);
    return dispatch_bits<float>(a, bits, c.sh, c.lds, stream_lists, stream);
}
