// The gated activation that feeds a down projection in the models of Sec. 5: x = silu(gate) * up,
// silu(g) = g / (1 + e^-g), bfloat16 in and out.  The producer of the activations that the headline shape
// (a down projection) reassembles; element-wise and bound by HBM (6 bytes per element).
//
// The paper fixes none of its arithmetic.  Here it is a fixed sequence of fp32 operations, each rounded once,
// with nothing left to the hardware's estimate instructions, so that a CPU can state the same sequence and get
// the same bits:
//     z = min(max(-g, -86), 88);  n = rint(z * log2 e);  r = fma(n, -ln2_hi, z);  r = fma(n, -ln2_lo, r)
//     p = degree-5 polynomial of the Cephes expf in r (Horner, fma);  e = (fma(p, r * r, r) + 1) * 2^n
//     s = g / (1 + e), correctly rounded;  s = -0 where g < -88;  x = bf16(s * up), nearest even
// Within 2 ulp of the real-number silu before the product (every finite bfloat16 gate checked on the CPU side).
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "qllm.h"

extern "C" void qllm_note_hip_error(const char *step, const char *name);

namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float silu_times_up(float g, float up)
{
    const float LOG2E = 1.44269504088896341f, LN2_HI = 0.693359375f, LN2_LO = -2.12194440e-4f;
    float z = -g;
    z = fminf(fmaxf(z, -86.0f), 88.0f);
    const float n = __builtin_rintf(z * LOG2E);
    float r = __builtin_fmaf(n, -LN2_HI, z);
    r = __builtin_fmaf(n, -LN2_LO, r);
    float p = 1.9875691500e-4f;
    p = __builtin_fmaf(p, r, 1.3981999507e-3f);
    p = __builtin_fmaf(p, r, 8.3334519073e-3f);
    p = __builtin_fmaf(p, r, 4.1665795894e-2f);
    p = __builtin_fmaf(p, r, 1.6666665459e-1f);
    p = __builtin_fmaf(p, r, 5.0000001201e-1f);
    float e = __builtin_fmaf(p, r * r, r);
    e = e + 1.0f;
    e = e * __uint_as_float((uint32_t)((int32_t)n + 127) << 23); // 2^n, n in [-124, 127]
    const float d = 1.0f + e;
    float s = g / d; // IEEE division (the compiler's correctly rounded sequence)
    if (g < -88.0f) s = -0.0f;
    return s * up;
}

// 8 elements (16 bytes of gate, 16 of up, 16 of x) per lane and step; rows whose start or stride is not a
// multiple of 8 elements, and row tails, go element by element.
__global__ __launch_bounds__(256) void swiglu_kernel(const uint16_t *gate, int64_t ld_gate, const uint16_t *up, int64_t ld_up,
                                                    int64_t N, int64_t C, uint16_t *x, int64_t ldx, int vec)
{
    const int64_t chunks = vec ? C / 8 : 0;
    const int64_t per_row = chunks + (C - chunks * 8); // whole chunks, then single elements
    const int64_t total = N * per_row, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int64_t n = i / per_row, k = i - n * per_row;
        if (k < chunks) {
            const uint4 gq = *reinterpret_cast<const uint4 *>(gate + n * ld_gate + 8 * k);
            const uint4 uq = *reinterpret_cast<const uint4 *>(up + n * ld_up + 8 * k);
            const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w}, uw[4] = {uq.x, uq.y, uq.z, uq.w};
            uint32_t out[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const float lo = silu_times_up(__uint_as_float(gw[h] << 16), __uint_as_float(uw[h] << 16));
                const float hi = silu_times_up(__uint_as_float(gw[h] & 0xffff0000u), __uint_as_float(uw[h] & 0xffff0000u));
                out[h] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
            }
            *reinterpret_cast<uint4 *>(x + n * ldx + 8 * k) = make_uint4(out[0], out[1], out[2], out[3]);
        } else {
            const int64_t c = chunks * 8 + (k - chunks);
            const float v = silu_times_up(__uint_as_float((uint32_t)gate[n * ld_gate + c] << 16), __uint_as_float((uint32_t)up[n * ld_up + c] << 16));
            const uint32_t pair = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{v, 0.0f}, bf16x2));
            x[n * ldx + c] = (uint16_t)pair;
        }
    }
}

} // namespace

extern "C" int32_t qllm_swiglu(const void *gate, int64_t ld_gate, const void *up, int64_t ld_up, int64_t N, int64_t C, void *x,
                               int64_t ldx, void *hip_stream)
{
    if (!gate || !up || !x) return QLLM_ERR_NULL;
    if (N < 0 || C <= 0 || ld_gate < C || ld_up < C || ldx < C) return QLLM_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(gate) | reinterpret_cast<uintptr_t>(up) | reinterpret_cast<uintptr_t>(x)) & 1u) return QLLM_ERR_ALIGN;
    if (N == 0) return QLLM_OK;
    const bool vec = ((reinterpret_cast<uintptr_t>(gate) | reinterpret_cast<uintptr_t>(up) | reinterpret_cast<uintptr_t>(x)) & 15u) == 0 &&
                     ((ld_gate | ld_up | ldx) & 7) == 0;
    const int64_t items = N * (vec ? C / 8 + C % 8 : C);
    const int64_t blocks = (items + 255) / 256;
    (void)hipGetLastError();
    hipLaunchKernelGGL(swiglu_kernel, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       static_cast<const uint16_t *>(gate), ld_gate, static_cast<const uint16_t *>(up), ld_up, N, C,
                       static_cast<uint16_t *>(x), ldx, vec ? 1 : 0);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error("swiglu: launch", hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}
