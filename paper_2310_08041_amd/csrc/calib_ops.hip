// Two small device operations of the offline search for theta (Algorithm 1): the full-precision output
// of the layer that the quantized layer is scored against, and the squared error between the two.
// Neither is on the hot path; both are plain, deterministic fp64 kernels.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "qllm.h"

extern "C" void qllm_note_hip_error(const char *step, const char *name);

namespace {

constexpr int TM = 64, TN = 64, TK = 16, THREADS = 256;

// out[n, o] = sum_c y[n, c] * W[c, o], every product and sum in double (fp32 inputs widened exactly), c ascending.
// A workgroup owns a 64 x 64 tile of the output, a lane 4 x 4 of it.
__global__ __launch_bounds__(THREADS) void linear_f64_kernel(const float *y, int64_t N, int64_t C, int64_t ldy, const float *W,
                                                             int64_t O, int64_t ldw, double *out, int64_t ldo)
{
    __shared__ double ys[TK][TM + 1], ws[TK][TN + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int64_t n0 = (int64_t)blockIdx.y * TM, o0 = (int64_t)blockIdx.x * TN;
    double acc[4][4] = {};
    for (int64_t c0 = 0; c0 < C; c0 += TK) {
        for (int e = tid; e < TM * TK; e += THREADS) { // y tile: consecutive lanes along c
            const int k = e % TK, r = e / TK;
            const int64_t n = n0 + r, c = c0 + k;
            ys[k][r] = (n < N && c < C) ? (double)y[n * ldy + c] : 0.0;
        }
        for (int e = tid; e < TN * TK; e += THREADS) { // W tile: consecutive lanes along o
            const int j = e % TN, k = e / TN;
            const int64_t c = c0 + k, o = o0 + j;
            ws[k][j] = (c < C && o < O) ? (double)W[c * ldw + o] : 0.0;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < TK; ++k) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = ys[k][ty * 4 + i];
                b[i] = ws[k][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fma(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + ty * 4 + i, o = o0 + tx * 4 + j;
            if (n < N && o < O) out[n * ldo + o] = acc[i][j];
        }
}

__device__ __forceinline__ double widen_out(const void *p, int32_t dtype, int64_t at)
{
    if (dtype == QLLM_BF16) return (double)__uint_as_float((uint32_t)static_cast<const uint16_t *>(p)[at] << 16);
    return (double)static_cast<const float *>(p)[at];
}

// One partial sum per row: sum_o (got[n, o] - ref[n, o])^2 in double, o ascending within a lane, lanes and waves
// combined in a fixed order.
__global__ __launch_bounds__(THREADS) void sq_error_rows_kernel(const void *got, int32_t dtype, int64_t O, int64_t ldg,
                                                                const double *ref, int64_t ldr, double *partial)
{
    __shared__ double red[THREADS / 64];
    const int64_t n = blockIdx.x;
    double s = 0.0;
    for (int64_t o = threadIdx.x; o < O; o += THREADS) {
        const double d = widen_out(got, dtype, n * ldg + o) - ref[n * ldr + o];
        s = __builtin_fma(d, d, s);
    }
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) partial[n] = (red[0] + red[1]) + (red[2] + red[3]);
}

// The rows' partial sums added up by one workgroup, in a fixed order.
__global__ __launch_bounds__(THREADS) void sq_error_total_kernel(const double *partial, int64_t N, double *result)
{
    __shared__ double red[THREADS];
    double s = 0.0;
    for (int64_t n = threadIdx.x; n < N; n += THREADS) s += partial[n];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int off = THREADS / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *result = red[0];
}

int32_t launched(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error(what, hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}

} // namespace

extern "C" int32_t qllm_linear_f64(const float *y, int64_t N, int64_t C, int64_t ldy, const float *W, int64_t O, int64_t ldw,
                                   double *out, int64_t ldo, void *hip_stream)
{
    if (!y || !W || !out) return QLLM_ERR_NULL;
    if (N < 0 || C <= 0 || O <= 0 || ldy < C || ldw < O || ldo < O) return QLLM_ERR_SHAPE;
    if ((N + TM - 1) / TM > 65535) return QLLM_ERR_SHAPE;
    if (N == 0) return QLLM_OK;
    (void)hipGetLastError();
    hipLaunchKernelGGL(linear_f64_kernel, dim3((unsigned)((O + TN - 1) / TN), (unsigned)((N + TM - 1) / TM)), dim3(THREADS), 0,
                       reinterpret_cast<hipStream_t>(hip_stream), y, N, C, ldy, W, O, ldw, out, ldo);
    return launched("full-precision layer output: launch");
}

extern "C" int64_t qllm_sq_error_workspace_bytes(int64_t N)
{
    return N < 0 ? (int64_t)QLLM_ERR_SHAPE : N * (int64_t)sizeof(double);
}

extern "C" int32_t qllm_sq_error(const void *got, int32_t got_dtype, int64_t N, int64_t O, int64_t ldg, const double *ref,
                                 int64_t ldr, double *result, void *workspace, int64_t workspace_bytes, void *hip_stream)
{
    if (!got || !ref || !result) return QLLM_ERR_NULL;
    if (got_dtype != QLLM_F32 && got_dtype != QLLM_BF16) return QLLM_ERR_DTYPE;
    if (N <= 0 || O <= 0 || ldg < O || ldr < O || N > INT32_MAX) return QLLM_ERR_SHAPE;
    if (!workspace || workspace_bytes < qllm_sq_error_workspace_bytes(N)) return QLLM_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 7u) return QLLM_ERR_ALIGN;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    double *partial = static_cast<double *>(workspace);
    (void)hipGetLastError();
    hipLaunchKernelGGL(sq_error_rows_kernel, dim3((unsigned)N), dim3(THREADS), 0, stream, got, got_dtype, O, ldg, ref, ldr, partial);
    int32_t rc = launched("squared output error: rows");
    if (rc != QLLM_OK) return rc;
    hipLaunchKernelGGL(sq_error_total_kernel, dim3(1), dim3(THREADS), 0, stream, partial, N, result);
    return launched("squared output error: total");
}
