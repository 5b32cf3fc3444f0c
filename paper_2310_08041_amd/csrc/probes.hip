// Measurement probes: what the machine delivers on the two resources the hot path is priced against,
// with none of the path's own work in the way.  They compute nothing of the method; bench.py runs
// them next to the real kernels and reports both fractions (of the published peak, of the probe).
//   qllm_probe_mfma    every wave issues nothing but v_mfma_i32_16x16x64_i8 on register operands
//                      that look like 4-bit codes (the matrix cores clock with operand activity)
//   qllm_probe_mfma_fp6  the same with v_mfma_f32_16x16x128_f8f6f4 on E2M3 operands that hold 4-bit codes
//   qllm_probe_stream  reads 16 bytes per lane and writes 4, the 4 : 1 mix of the fused kernel
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "qllm.h"
#include "qllm_probes.h"

extern "C" void qllm_note_hip_error(const char *step, const char *name);

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(512) void probe_mfma_kernel(int32_t iters, int32_t *sink)
{
    const uint32_t seed = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
    v4i fa[8], fw[4], acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t h = seed * (2 * i + 3);
        fa[i] = v4i{(int)(h & 0x0f0f0f0fu), (int)((h >> 1) & 0x0f0f0f0fu), (int)((h >> 2) & 0x0f0f0f0fu), (int)((h >> 3) & 0x0f0f0f0fu)};
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t h = seed * (2 * j + 17);
        fw[j] = v4i{(int)(h & 0x0f0f0f0fu), (int)((h >> 1) & 0x0f0f0f0fu), (int)((h >> 2) & 0x0f0f0f0fu), (int)((h >> 3) & 0x0f0f0f0fu)};
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[j], fa[i], acc[i][j], 0, 0, 0);
        // new operands every turn (a rotate), as in a real product; keeps them nibble-shaped
#pragma unroll
        for (int i = 0; i < 8; ++i) fa[i].x = (int)__builtin_amdgcn_alignbit((uint32_t)fa[i].x, (uint32_t)fa[i].x, 8);
    }
    int32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s += acc[i][j].x + acc[i][j].y + acc[i][j].z + acc[i][j].w;
    if (s == 0x7fffffff) sink[0] = s; // keeps the work alive; practically never taken
}

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// 32 four-bit codes drawn from h, each in a 6-bit field (the E2M3 number code / 8)
__device__ v8i codes_in_fields(uint32_t h)
{
    uint32_t a[7] = {0, 0, 0, 0, 0, 0, 0};
    for (int e = 0; e < 32; ++e) {
        h = h * 1664525u + 1013904223u;
        const uint64_t c = (h >> 20) & 15u;
        const int bit = 6 * e, w = bit >> 5, sh = bit & 31;
        a[w] |= (uint32_t)(c << sh);
        if (sh > 26) a[w + 1] |= (uint32_t)(c >> (32 - sh));
    }
    return v8i{(int)a[0], (int)a[1], (int)a[2], (int)a[3], (int)a[4], (int)a[5], 0, 0};
}

__global__ __launch_bounds__(512) void probe_mfma_fp6_kernel(int32_t iters, float *sink)
{
    const uint32_t seed = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
    v8i fa[8], fw[4];
    v4f acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) fa[i] = codes_in_fields(seed * (2 * i + 3));
#pragma unroll
    for (int j = 0; j < 4; ++j) fw[j] = codes_in_fields(seed * (2 * j + 17));
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fw[j], fa[i], acc[i][j], 2, 2, 0, 0, 0, 0);
        // new operands every turn (a rotate by two fields); the mask keeps every field a code
#pragma unroll
        for (int i = 0; i < 8; ++i) fa[i][1] = (int)(__builtin_amdgcn_alignbit((uint32_t)fa[i][1], (uint32_t)fa[i][1], 12) & 0x3cf3cf3cu);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    if (s == 123.456f) sink[0] = s; // keeps the work alive; never taken (the sums are multiples of 1/64)
}

__global__ __launch_bounds__(256) void probe_stream_kernel(const uint4 *src, uint32_t *dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        dst[i] = v.x ^ v.y ^ v.z ^ v.w;
    }
}

int32_t after_launch(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error(what, hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}

} // namespace

extern "C" int32_t qllm_probe_mfma(int32_t workgroups, int32_t iters, int32_t *sink, void *hip_stream)
{
    if (!sink) return QLLM_ERR_NULL;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return QLLM_ERR_SHAPE;
    (void)hipGetLastError();
    hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)workgroups), dim3(512), 0, reinterpret_cast<hipStream_t>(hip_stream), iters, sink);
    return after_launch("mfma probe: launch");
}

extern "C" int32_t qllm_probe_mfma_fp6(int32_t workgroups, int32_t iters, float *sink, void *hip_stream)
{
    if (!sink) return QLLM_ERR_NULL;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return QLLM_ERR_SHAPE;
    (void)hipGetLastError();
    hipLaunchKernelGGL(probe_mfma_fp6_kernel, dim3((unsigned)workgroups), dim3(512), 0, reinterpret_cast<hipStream_t>(hip_stream), iters, sink);
    return after_launch("fp6 mfma probe: launch");
}

extern "C" int32_t qllm_probe_stream(const void *src, void *dst, int64_t bytes, int32_t workgroups, void *hip_stream)
{
    if (!src || !dst) return QLLM_ERR_NULL;
    if (bytes <= 0 || bytes % 16 != 0 || workgroups <= 0 || workgroups > (1 << 20)) return QLLM_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 3u)) return QLLM_ERR_ALIGN;
    (void)hipGetLastError();
    hipLaunchKernelGGL(probe_stream_kernel, dim3((unsigned)workgroups), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const uint4 *>(src), reinterpret_cast<uint32_t *>(dst), bytes / 16);
    return after_launch("stream probe: launch");
}
