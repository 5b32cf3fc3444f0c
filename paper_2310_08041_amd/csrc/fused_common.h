// Internal to libqllm: what the two fused-kernel translation units share.
#ifndef QLLM_FUSED_COMMON_H
#define QLLM_FUSED_COMMON_H

#include <hip/hip_runtime.h>

#include <stdint.h>

#include "qllm.h"

extern "C" void qllm_note_hip_error(const char *step, const char *name);

namespace qllm_detail {

constexpr int GROUP = QLLM_MAP_GROUP; // 8 channels per lane and step
constexpr float MAGIC = 12582912.0f;  // 1.5 * 2^23: x + MAGIC rounds x to an integer, ties to even
constexpr int32_t MAGIC_BITS = 0x4B400000;
constexpr float FAST_LIMIT = 2097152.0f; // 2^21: below it the MAGIC trick is exact

struct FusedArgs {
    const void *x;
    int64_t ldx;
    int32_t N, C, norm, vec_ok;
    const float *gamma, *beta;
    float eps;
    double inv_C; // 1 / C
    const int32_t *row_ptr, *src, *desc;
    const float *scale;
    const int32_t *work, *chunks, *spec, *dest, *longs, *segs, *recs, *xlrows, *xlent; // the parts of the plan (see qllm_plan_map_host)
    int32_t n_comp, n_long, n_pub, n_work, n_chunks, n_spec, n_dest, n_segw, n_xl;
    int32_t C_out, n_groups, n_groups_pad, S;
    uint8_t *codes;
    int64_t row_bytes;
    float *alpha;
    int32_t *zero, *rowsum;
    // calibration variant
    float *absmax, *y_dump;
    int32_t n_dump;
};

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// ---- Eq. (2) for one value; the row's parameters are uniform over the workgroup
// rne(x*inv) on the exact product.  Fast form: one fused multiply-add against MAGIC, whose single
// rounding lands on the integer grid.  Slow form (huge quotients): the product is exact in fp64.
__device__ __forceinline__ int32_t rne_product_fast(float x, float inv)
{
    return __float_as_int(__builtin_fmaf(x, inv, MAGIC)) - MAGIC_BITS;
}

__device__ __forceinline__ double rne_product_slow(float x, float inv)
{
    return rint((double)x * (double)inv);
}

template <int QMAX>
__device__ __forceinline__ int32_t quant_code(float x, float inv, int32_t beta, int32_t fast)
{
    if (fast) {
        const int32_t q = rne_product_fast(x, inv) + beta; // both below 2^22 in magnitude
        return q < 0 ? 0 : (q > QMAX ? QMAX : q);
    }
    const double q = rne_product_slow(x, inv) + (double)beta;
    return (int32_t)fmin(fmax(q, 0.0), (double)QMAX);
}

} // namespace qllm_detail

// Launches the planned kernel (fused_planned.hip).  Returns QLLM_ERR_WORKSPACE if the shape or the
// general groups are more than it holds on chip: the caller then takes the plain kernel.
int32_t qllm_launch_fused_planned(const qllm_detail::FusedArgs &a, int32_t x_dtype, int32_t bits, hipStream_t stream);
// QLLM_FUSED_*: the form of the fused kernel that qllm_launch_fused_planned would run for these arguments
int32_t qllm_choose_fused_planned(const qllm_detail::FusedArgs &a, int32_t x_dtype, int32_t bits);

#endif
