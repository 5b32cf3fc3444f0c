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

#include <mutex>
#include <vector>

#include "qllm.h"
#include "fused_common.h"

using namespace qllm_detail;

namespace {

// work-list entries (see qllm_plan_map_host): kind << 28 | group << 15 | d
constexpr int KIND_PLAIN = 0, KIND_GENERAL = 1, KIND_PAD = 2, KIND_NONE = 3;
constexpr int32_t WORK_NONE = KIND_NONE << 28;
constexpr int32_t ITEM_LONG = -2; // first word of a plan item whose entries are in the table of long rows
constexpr int32_t ITEM_SKIP = 0x7fc00001; // second word the kernel gives such an item in LDS (as a scale: a NaN, never a real one)

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

// value of the lane below (lane 0: zero) + p, across the whole wavefront
__device__ __forceinline__ float below_plus(float acc, float p)
{
    float r;
    asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %2 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0" : "=v"(r) : "v"(acc), "v"(p));
    return r;
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
// The word after the last chunk exists (and is only ever shifted out).
template <int BITS>
__device__ __forceinline__ void funnel(const uint32_t *pk, int u, int v, uint32_t &w0, uint32_t &w1)
{
    if constexpr (BITS == 4) {
        const uint32_t lo = pk[u], hi = pk[u + 1];
        w0 = __builtin_amdgcn_alignbit(hi, lo, 4 * v); // ({hi, lo} >> 4v), low 32 bits
        w1 = 0;
    } else {
        const uint2 a = reinterpret_cast<const uint2 *>(pk)[u], b = reinterpret_cast<const uint2 *>(pk)[u + 1];
        const uint64_t A = (uint64_t)a.x | ((uint64_t)a.y << 32), B = (uint64_t)b.x | ((uint64_t)b.y << 32);
        uint64_t r;
        if constexpr (BITS == 6) {
            r = ((A >> (6 * v)) | (B << (48 - 6 * v))) & 0xffffffffffffull;
        } else {
            const uint64_t up = B << ((64 - 8 * v) & 63);
            r = (A >> (8 * v)) | (v ? up : 0ull);
        }
        w0 = (uint32_t)r;
        w1 = (uint32_t)(r >> 32);
    }
}

// GAM_REG: the lane's share of gamma stays in registers for the lifetime of the workgroup; otherwise it
// is re-read (from L2) for every row, which frees 8 registers per chunk.
template <typename XT, int BITS, int ITERS, int NT_MAX, bool GAM_REG, bool LAYER>
__global__ __launch_bounds__(NT_MAX) void fused_planned_kernel(const FusedArgs a)
{
    extern __shared__ __align__(16) float lds[];
    float *pub = lds;                         // [8 * n_pub]      y of the chunks that general groups read
    float *zero = pub + GROUP * a.n_pub;      // [4] a zero: the "second source" of single-entry items
    float *exc = zero + 4;                    // [8 * n_general]  reassembled channels of the general groups
    int4 *longs = reinterpret_cast<int4 *>(exc + GROUP * a.n_general); // [n_long] entries of the long rows
    int2 *items = reinterpret_cast<int2 *>(longs + a.n_long);          // [8 * n_general] entries of the general groups
    uint32_t *pk = reinterpret_cast<uint32_t *>(items + GROUP * a.n_general); // [(n_chunks + 1) * PKW] packed codes, input order
    uint32_t *masks = pk + (a.n_chunks + 1) * PKW<BITS>;               // [n_mask] chunks of which only some channels pass
    uint32_t *chunkw = masks + a.n_mask;                               // [n_chunks] pass bits | staging slot << 8
    int32_t *work = reinterpret_cast<int32_t *>(chunkw + a.n_chunks); // [n_work] work list of the output groups
    __shared__ double red_d[2][16];
    __shared__ float red_f[32];
    __shared__ int32_t red_i[16];
    // bf16 rows are prefetched one row ahead; fp32 rows would need twice the registers and are not
    constexpr bool PREFETCH = sizeof(XT) == 2;
    constexpr int ITEMS_REG = ITERS >= 4 ? ITERS : ITERS + 1; // general-group entries a lane keeps in registers
    constexpr int W = PKW<BITS>;
    constexpr uint32_t NOT_PUBLISHED = 0xffffffu;

    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6;
    const int n_chunks = a.n_chunks;
    const int n_items = a.n_general * GROUP;
    const float inf = __builtin_inff();

    // ---- per-lane state that outlives the rows
    float gam[GAM_REG ? ITERS : 1][GROUP];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int i = tid + it * nt;
        if constexpr (GAM_REG) load_gamma(gam[it], a.gamma, i * GROUP, a.C, a.norm != QLLM_NORM_NONE);
    }
    for (int j = tid; j < a.n_long; j += nt) longs[j] = reinterpret_cast<const int4 *>(a.longs)[j];
    for (int j = tid; j < a.n_mask; j += nt) masks[j] = (uint32_t)a.masks[j];
    for (int j = tid; j < n_chunks; j += nt) chunkw[j] = (uint32_t)a.chunks[j];
    for (int j = tid; j < a.n_work; j += nt) work[j] = a.work[j];
    if (tid < 4) zero[tid] = 0.0f;
    if (tid < W) pk[n_chunks * W + tid] = 0u;
    if (tid < 16) { // reduction slots of waves that do not exist hold the identity
        red_d[0][tid] = 0.0;
        red_d[1][tid] = 0.0;
        red_f[tid] = inf;
        red_f[16 + tid] = inf; // minus the maximum
        red_i[tid] = 0;
    }
    // general-group entries {staged position of source 0 | of source 1 << 16, scale}: kept in LDS (a
    // register pair per entry and lane would be too many); long rows are marked and read the zero
    const uint32_t zero_at = (uint32_t)(GROUP * a.n_pub);
    for (int j = tid; j < n_items; j += nt) {
        int2 e = reinterpret_cast<const int2 *>(a.items)[j];
        if (e.x == ITEM_LONG) e = make_int2((int32_t)(zero_at | (zero_at << 16)), ITEM_SKIP);
        items[j] = e;
    }

    // gamma has to have arrived before the row loop is entered: a load still pending there would make
    // every pass of the loop wait for whatever was requested last, the next row's prefetch included.
    if constexpr (GAM_REG) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
#pragma unroll
            for (int j = 0; j < GROUP; ++j) asm volatile("" : "+v"(gam[it][j]));
        }
    }

    // The reduction slots were set by the first lanes of wave 0; the other waves write theirs before
    // the first barrier of the first row, so the set-up has to be over for everybody first.
    __syncthreads();

    const XT *xbase = reinterpret_cast<const XT *>(a.x);
    Raw<XT> raw[ITERS], ahead[PREFETCH ? ITERS : 1];
    int64_t row = blockIdx.x, done_row = -1;
    if (PREFETCH && row < a.N) { // the first row
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = tid + it * nt;
            if (i < n_chunks) load_raw(raw[it], xbase + row * a.ldx, i * GROUP);
        }
    }

    // rowsum of a finished row: the waves' partial sums are complete once a barrier has passed
    auto finish_rowsum = [&]() {
        if (wave == 0 && done_row >= 0) {
            const int32_t s = dpp_add_row16(red_i[lane & 15]);
            if (lane == 0) a.rowsum[done_row] = s;
        }
    };

    for (; row < a.N; row += gridDim.x) {
        // Addresses derived from the lane's number cost an instruction or two per row to recompute, but a
        // register each to keep: hide from the optimiser that the number does not change from row to row.
        int ltid = threadIdx.x;
        asm volatile("" : "+v"(ltid));
        // ---- step a1.  A bf16 row is already here (it was requested while the row before it was worked
        //      on); request the next one.  Its registers move up further down, before this row's stores.
        if constexpr (PREFETCH) {
            const int64_t next = row + gridDim.x;
            if (next < a.N) {
#pragma unroll
                for (int it = 0; it < ITERS; ++it) {
                    const int i = ltid + it * nt;
                    if (i < n_chunks) load_raw(ahead[it], xbase + next * a.ldx, i * GROUP);
                }
            }
        } else {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int i = ltid + it * nt;
                if (i < n_chunks) load_raw(raw[it], xbase + row * a.ldx, i * GROUP);
            }
        }

        // row statistics in fp64 (two interleaved partial sums per lane: the additions do not wait for
        // one another; the order is fixed, so the result is reproducible)
        float mu = 0.0f, rstd = 1.0f;
        if (!LAYER && a.norm == QLLM_NORM_RMS) {
            double q0 = 0.0, q1 = 0.0;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                if (ltid + it * nt < n_chunks) {
                    float v[GROUP];
                    widen(raw[it], v);
#pragma unroll
                    for (int j = 0; j < GROUP; j += 2) {
                        const double d0 = (double)v[j], d1 = (double)v[j + 1];
                        q0 = __builtin_fma(d0, d0, q0);
                        q1 = __builtin_fma(d1, d1, q1);
                    }
                }
            }
            const double q = wave_sum(q0 + q1);
            if (lane == 0) red_d[0][wave] = q;
            __syncthreads(); // also: the previous row's last LDS reads are over
            finish_rowsum();
            rstd = rsqrt_to_f32(total16(red_d[0], lane) * a.inv_C + (double)a.eps);
        } else if constexpr (LAYER) {
            double s0 = 0.0, s1 = 0.0;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                if (ltid + it * nt < n_chunks) {
                    float v[GROUP];
                    widen(raw[it], v);
#pragma unroll
                    for (int j = 0; j < GROUP; j += 2) {
                        s0 += (double)v[j];
                        s1 += (double)v[j + 1];
                    }
                }
            }
            const double s = wave_sum(s0 + s1);
            if (lane == 0) red_d[0][wave] = s;
            __syncthreads(); // also: the previous row's last LDS reads are over
            finish_rowsum();
            const double mu64 = total16(red_d[0], lane) * a.inv_C;
            double q0 = 0.0, q1 = 0.0;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                if (ltid + it * nt < n_chunks) {
                    float v[GROUP];
                    widen(raw[it], v);
#pragma unroll
                    for (int j = 0; j < GROUP; j += 2) {
                        const double d0 = (double)v[j] - mu64, d1 = (double)v[j + 1] - mu64;
                        q0 = __builtin_fma(d0, d0, q0);
                        q1 = __builtin_fma(d1, d1, q1);
                    }
                }
            }
            const double q = wave_sum(q0 + q1);
            if (lane == 0) red_d[1][wave] = q;
            __syncthreads();
            mu = (float)mu64;
            rstd = rsqrt_to_f32(total16(red_d[1], lane) * a.inv_C + (double)a.eps);
        } else {
            __syncthreads(); // the previous row's last LDS reads are over
            finish_rowsum();
        }

        // ---- y, kept in registers; staged in LDS where a general group reads it; min/max over the
        //      channels that pass unscaled
        float y[ITERS][GROUP];
        float mn = inf, mx = -inf;
        const float *gamma_row = a.gamma, *beta_row = a.beta; // opaque, so that per-row loads stay per row
        asm volatile("" : "+s"(gamma_row), "+s"(beta_row));
        const bool shift = LAYER && a.beta != nullptr;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = ltid + it * nt;
            float gjit[GROUP];
            if constexpr (!GAM_REG) load_gamma(gjit, gamma_row, i * GROUP, a.C, a.norm != QLLM_NORM_NONE);
            const float *g8 = GAM_REG ? gam[GAM_REG ? it : 0] : gjit;
            if (i < n_chunks) {
                forget(raw[it]);
                widen(raw[it], y[it]);
                float bj[GROUP];
                if constexpr (LAYER) load_gamma(bj, beta_row, i * GROUP, a.C, shift); // beta: re-read (from L2) for every row
#pragma unroll
                for (int j = 0; j < GROUP; ++j) {
                    float t = y[it][j];
                    if constexpr (LAYER) t = t - mu;
                    t = t * rstd;
                    t = t * g8[j];
                    if constexpr (LAYER) {
                        if (shift) t = t + bj[j];
                    }
                    y[it][j] = t;
                }
                const uint32_t cw = chunkw[i], slot = cw >> 8;
                if (slot != NOT_PUBLISHED) {
                    float4 *dst = reinterpret_cast<float4 *>(pub + slot * GROUP);
                    dst[0] = make_float4(y[it][0], y[it][1], y[it][2], y[it][3]);
                    dst[1] = make_float4(y[it][4], y[it][5], y[it][6], y[it][7]);
                }
                if ((cw & 0xffu) == 0xffu) {
#pragma unroll
                    for (int j = 0; j < GROUP; j += 2) {
                        mn = fminf(fminf(mn, y[it][j]), y[it][j + 1]);
                        mx = fmaxf(fmaxf(mx, y[it][j]), y[it][j + 1]);
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < GROUP; ++j) y[it][j] = 0.0f;
            }
        }
        __syncthreads(); // staged y complete

        // ---- steps a2 + a3 for the general groups: sub-channels (scale 1/T), merged channels
        //      (scale 1/g each) and the plain channels that share a group of 8 with them.
        //      All LDS reads are issued before any of them is used.
        {
            int2 item[ITEMS_REG];
            float y0[ITEMS_REG], y1[ITEMS_REG];
#pragma unroll
            for (int m = 0; m < ITEMS_REG; ++m) {
                const int j = ltid + m * nt;
                item[m] = j < n_items ? items[j] : make_int2((int32_t)(zero_at | (zero_at << 16)), ITEM_SKIP);
            }
#pragma unroll
            for (int m = 0; m < ITEMS_REG; ++m) {
                const uint32_t p = (uint32_t)item[m].x;
                y0[m] = lds[p & 0xffffu];
                y1[m] = lds[p >> 16];
            }
#pragma unroll
            for (int m = 0; m < ITEMS_REG; ++m) {
                const float sc = __int_as_float(item[m].y);
                float xv = sc * y0[m];
                xv = xv + sc * y1[m];
                const bool real = item[m].y != ITEM_SKIP;
                mn = fminf(mn, real ? xv : inf);
                mx = fmaxf(mx, real ? xv : -inf);
                if (real) exc[ltid + m * nt] = xv;
            }
            // Chunks of which only some channels pass (the others are split or merged away) enter min/max
            // here, from their staged copy, one chunk per lane: there are few of them, but every wavefront
            // owns some, so taking them where y is produced would cost every wavefront a masked pass per
            // chunk.  Dealt out from the last lane down; the long rows below start at the first lane.
            for (int base = 0; base < a.n_mask; base += nt) {
                const int j = base + (nt - 1 - ltid);
                const uint32_t cw = j < a.n_mask ? masks[j] : 0u;
                if (cw & 0xffu) {
                    const float4 *c4 = reinterpret_cast<const float4 *>(pub + (cw >> 8) * GROUP);
                    const float4 lo = c4[0], hi = c4[1];
                    const float yv[GROUP] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                    for (int k = 0; k < GROUP; k += 2) {
                        const bool in0 = cw >> k & 1u, in1 = cw >> (k + 1) & 1u;
                        mn = fminf(fminf(mn, in0 ? yv[k] : inf), in1 ? yv[k + 1] : inf);
                        mx = fmaxf(fmaxf(mx, in0 ? yv[k] : -inf), in1 ? yv[k + 1] : -inf);
                    }
                }
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
                const float p = __int_as_float(le.z) * lds[le.x];
                const int pos = le.w & 0xff, steps = __builtin_amdgcn_readfirstlane(le.w >> 8);
                float acc = p;
                for (int t = 0; t < steps; ++t) {
                    const float sum = below_plus(acc, p);
                    acc = pos > 0 ? sum : p;
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
            red_f[16 + wave] = -mx; // negated: one butterfly of minima then serves both
        }
        __syncthreads(); // also: the general groups' values are complete
        {
            const float v = dpp_min_row16(red_f[lane & 31]);
            mn = lane_f32(v, 0);
            mx = -lane_f32(v, 16);
        }
        constexpr int QMAX = (1 << BITS) - 1;
        const float range = mx - mn;
        const float alpha = range > 0.0f ? range / (float)QMAX : 1.0f;
        const float inv = 1.0f / alpha;
        const int32_t fast = fabsf(mn * inv) < FAST_LIMIT && fabsf(mx * inv) < FAST_LIMIT;
        int32_t beta;
        if (fast) beta = -rne_product_fast(mn, inv);
        else beta = (int32_t)fmin(fmax(-rne_product_slow(mn, inv), -2147483647.0), 2147483647.0);

        // ---- step a4, first half: codes of the lane's own chunks, packed in input order
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = ltid + it * nt;
            if (i < n_chunks) {
                uint32_t w0, w1;
                quant_pack<BITS>(y[it], 0xffu, fast, inv, beta, w0, w1);
                if constexpr (W == 1) pk[i] = w0;
                else reinterpret_cast<uint2 *>(pk)[i] = make_uint2(w0, w1);
            }
        }
        __syncthreads(); // packed words complete

        // The next row moves up BEFORE this row's stores are issued: loads and stores retire in order
        // through one counter, so a wait for the loads placed after the stores would wait for the
        // stores too.
        if constexpr (PREFETCH) {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) move_up(raw[it], ahead[it]);
        }

        // ---- step a4, second half: the lane's output groups
        int32_t sum = 0;
        uint8_t *out_row = a.codes + row * a.row_bytes;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = ltid + it * nt;
            const int32_t e = i < a.n_work ? work[i] : WORK_NONE;
            const int kind = (uint32_t)e >> 28;
            if (kind != KIND_NONE) {
                const int g = (e >> 15) & 0x1fff, d = e & 0x7fff;
                uint32_t w0 = 0, w1 = 0;
                if (kind == KIND_PLAIN) {
                    funnel<BITS>(pk, d >> 3, d & 7, w0, w1);
                } else if (kind == KIND_GENERAL) {
                    const float4 e0 = *reinterpret_cast<const float4 *>(exc + d * GROUP);
                    const float4 e1 = *reinterpret_cast<const float4 *>(exc + d * GROUP + 4);
                    const float val[GROUP] = {e0.x, e0.y, e0.z, e0.w, e1.x, e1.y, e1.z, e1.w};
                    const int left = a.C_out - g * GROUP;
                    quant_pack<BITS>(val, left < GROUP ? (1u << left) - 1u : 0xffu, fast, inv, beta, w0, w1);
                }
                store_group<BITS>(out_row, g, w0, w1);
                sum += code_sum<BITS>(w0, w1);
            }
        }
        sum = wave_sum_i32(sum);
        if (lane == 0) red_i[wave] = sum; // read after the next barrier
        if (tid == 0) {
            a.alpha[row] = alpha;
            a.zero[row] = beta;
        }
        done_row = row;
    }
    __syncthreads();
    finish_rowsum();
}

struct Shape {
    int iters, nt;
};

// Chunks (or output groups) per lane and the workgroup size for a row of `units` of them.
Shape pick_shape(int units)
{
    Shape s;
    if (units <= 256) s = {1, 0};
    else if (units <= 2048) s = {2, 0};
    else s = {4, 0};
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

// What the runtime is asked once per kernel, workgroup size and LDS size and then remembered (no runtime
// query sits between a caller's stream capture and the launch): the raised LDS limit and the number of
// resident workgroups per CU.
constexpr int MAX_LDS = 159 * 1024; // dynamic LDS a launch may ask for (160 KB per CU, less the static arrays)
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

template <typename XT, int BITS, bool LAYER>
int32_t dispatch(const FusedArgs &a, const Shape &sh, size_t lds, hipStream_t stream)
{
    if (sh.iters == 1) return launch(fused_planned_kernel<XT, BITS, 1, 256, true, LAYER>, a, sh, lds, stream);
    if (sh.iters == 2) return launch(fused_planned_kernel<XT, BITS, 2, 1024, true, LAYER>, a, sh, lds, stream);
    // 16 waves x 4 chunks: gamma fits in registers next to y and the prefetched row, except with LayerNorm
    return launch(fused_planned_kernel<XT, BITS, 4, 1024, !LAYER, LAYER>, a, sh, lds, stream);
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
    const int units = a.n_chunks > a.n_work ? a.n_chunks : a.n_work;
    if (units > 4096 || !a.vec_ok || a.C % GROUP != 0) return QLLM_ERR_WORKSPACE;
    const Shape sh = pick_shape(units);
    const size_t lds = ((size_t)a.n_pub + (size_t)a.n_general) * GROUP * sizeof(float) + 16 + (size_t)a.n_long * 16 +
                       (size_t)a.n_general * GROUP * 8 + ((size_t)a.n_chunks + 1) * (bits == 4 ? 4 : 8) +
                       ((size_t)a.n_mask + (size_t)a.n_chunks + (size_t)a.n_work) * 4;
    if (lds > (size_t)MAX_LDS) return QLLM_ERR_WORKSPACE;
    const int items_reg = sh.iters >= 4 ? sh.iters : sh.iters + 1;
    if ((int64_t)a.n_general * GROUP > (int64_t)items_reg * sh.nt) return QLLM_ERR_WORKSPACE; // a lane takes at most that many general-group entries
    if (x_dtype == QLLM_BF16) return dispatch_bits<uint16_t>(a, bits, sh, lds, stream);
    return dispatch_bits<float>(a, bits, sh, lds, stream);
}
