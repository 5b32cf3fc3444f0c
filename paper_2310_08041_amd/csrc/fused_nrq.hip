// Fused norm + channel disassembly + channel assembly + per-token quantization for gfx950.
//
// One workgroup owns one token row at a time.  The row is read from HBM once (16-byte loads,
// consecutive lanes on consecutive addresses), its statistics are reduced with wavefront shuffles
// (fp64), the normalised row y is staged in LDS in fp32, the reassembly map is applied as a gather
// from LDS (Eq. 3 and Eq. 4 composed), min/max are reduced with shuffles, and the codes of Eq. (2)
// are packed in registers and written with one coalesced store per lane.  Neither y nor the
// reassembled row ever goes to HBM.
//
// LDS layout of y ("transposed by 8"): channel c lives at float index (c & 7) * S + (c >> 3),
// S = ceil(C / 8).  A lane that owns 8 consecutive channels therefore touches, for each of the 8
// LDS rows, the dword next to its neighbour lane's: reads and writes are bank-conflict free also
// when the map shifts the source channels by an amount that is not a multiple of 8.
//
// Two kernels.  fused_planned_kernel (fused_planned.hip) is the fast one: persistent workgroups (each keeps
// its share of gamma in registers and the map's plan in LDS across the rows it processes, or, for maps too
// big for that, reads the plan's lists from L2), the next row's loads in flight while the current row is
// worked on.  It needs the plan of qllm_plan_map_host.  fused_nrq_kernel is the plain one that walks the
// CSR; it serves maps without a plan, rows that are not 16-byte aligned or whole chunks long, and the few
// shapes whose row does not fit on chip next to its codes.  qllm_fused_kernel_choice tells which runs.
//
// Compiled with -ffp-contract=off: every fp32 product and sum is rounded on its own; the only fused
// multiply-adds are the explicit ones of the quantizer, whose single rounding is the definition.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "qllm.h"
#include "fused_common.h"

using namespace qllm_detail;

namespace {

// ---- block-wide reductions: shuffles inside a wavefront, then a fixed-order sum over the waves
template <int THREADS>
__device__ __forceinline__ double block_sum_f64(double v, double *red)
{
    constexpr int WAVES = THREADS / 64;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads(); // red may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = red[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) s += red[w];
    return s;
}

template <int THREADS>
__device__ __forceinline__ void block_minmax_f32(float &mn, float &mx, float *red)
{
    constexpr int WAVES = THREADS / 64;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, o, 64));
        mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6] = mn;
        red[WAVES + (threadIdx.x >> 6)] = mx;
    }
    __syncthreads();
    mn = red[0];
    mx = red[WAVES];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) {
        mn = fminf(mn, red[w]);
        mx = fmaxf(mx, red[WAVES + w]);
    }
}

template <int THREADS>
__device__ __forceinline__ int32_t block_sum_i32(int32_t v, int32_t *red)
{
    constexpr int WAVES = THREADS / 64;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    int32_t s = red[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) s += red[w];
    return s;
}

// ---- step a1: load one row, normalise it, leave y in LDS (transposed-by-8 layout)
template <typename XT, int THREADS, int ITERS>
__device__ __forceinline__ void load_norm_stage(const FusedArgs &a, int64_t row, float *ylds, double *red_d)
{
    const int tid = threadIdx.x;
    const int n_chunks = (a.C + GROUP - 1) / GROUP;
    const XT *xr = reinterpret_cast<const XT *>(a.x) + row * a.ldx;
    float v[ITERS][GROUP];

#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int i = tid + it * THREADS;
        const int c0 = i * GROUP;
#pragma unroll
        for (int j = 0; j < GROUP; ++j) v[it][j] = 0.0f;
        if (i < n_chunks) {
            if (a.vec_ok && c0 + GROUP <= a.C) {
                if constexpr (sizeof(XT) == 2) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(xr + c0);
                    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        v[it][2 * p] = __uint_as_float(w[p] << 16);
                        v[it][2 * p + 1] = __uint_as_float(w[p] & 0xffff0000u);
                    }
                } else {
                    const float4 lo = *reinterpret_cast<const float4 *>(xr + c0);
                    const float4 hi = *reinterpret_cast<const float4 *>(xr + c0 + 4);
                    v[it][0] = lo.x; v[it][1] = lo.y; v[it][2] = lo.z; v[it][3] = lo.w;
                    v[it][4] = hi.x; v[it][5] = hi.y; v[it][6] = hi.z; v[it][7] = hi.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < GROUP; ++j)
                    if (c0 + j < a.C) {
                        if constexpr (sizeof(XT) == 2) v[it][j] = bf16_to_f32(xr[c0 + j]);
                        else v[it][j] = xr[c0 + j];
                    }
            }
        }
    }

    float mu = 0.0f, rstd = 1.0f;
    if (a.norm == QLLM_NORM_RMS) {
        double q = 0.0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it)
#pragma unroll
            for (int j = 0; j < GROUP; ++j) {
                const double d = (double)v[it][j]; // slots past C hold 0 and add nothing
                q = __builtin_fma(d, d, q);
            }
        q = block_sum_f64<THREADS>(q, red_d);
        rstd = (float)(1.0 / sqrt(q / (double)a.C + (double)a.eps));
    } else if (a.norm == QLLM_NORM_LAYER) {
        double s = 0.0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it)
#pragma unroll
            for (int j = 0; j < GROUP; ++j) s += (double)v[it][j];
        s = block_sum_f64<THREADS>(s, red_d);
        const double mu64 = s / (double)a.C;
        double q = 0.0;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int c0 = (tid + it * THREADS) * GROUP;
#pragma unroll
            for (int j = 0; j < GROUP; ++j)
                if (c0 + j < a.C) {
                    const double d = (double)v[it][j] - mu64;
                    q = __builtin_fma(d, d, q);
                }
        }
        q = block_sum_f64<THREADS>(q, red_d);
        mu = (float)mu64;
        rstd = (float)(1.0 / sqrt(q / (double)a.C + (double)a.eps));
    }

#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int i = tid + it * THREADS;
        const int c0 = i * GROUP;
        if (i < n_chunks) {
            float g[GROUP], b[GROUP];
            const bool full = c0 + GROUP <= a.C;
            if (a.norm != QLLM_NORM_NONE) {
                if (full) {
                    const float4 g0 = *reinterpret_cast<const float4 *>(a.gamma + c0);
                    const float4 g1 = *reinterpret_cast<const float4 *>(a.gamma + c0 + 4);
                    g[0] = g0.x; g[1] = g0.y; g[2] = g0.z; g[3] = g0.w;
                    g[4] = g1.x; g[5] = g1.y; g[6] = g1.z; g[7] = g1.w;
                } else {
#pragma unroll
                    for (int j = 0; j < GROUP; ++j) g[j] = c0 + j < a.C ? a.gamma[c0 + j] : 0.0f;
                }
            }
            const bool shift = a.norm == QLLM_NORM_LAYER && a.beta != nullptr;
            if (shift) {
#pragma unroll
                for (int j = 0; j < GROUP; ++j) b[j] = c0 + j < a.C ? a.beta[c0 + j] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < GROUP; ++j) {
                float t = v[it][j];
                if (a.norm == QLLM_NORM_LAYER) {
                    t = t - mu;
                    t = t * rstd;
                    t = t * g[j];
                    if (shift) t = t + b[j];
                } else if (a.norm == QLLM_NORM_RMS) {
                    t = t * rstd;
                    t = t * g[j];
                }
                ylds[j * a.S + i] = t;
            }
        }
    }
}

template <typename XT, int BITS, int THREADS, int ITERS>
__global__ __launch_bounds__(THREADS) void fused_nrq_kernel(const FusedArgs a)
{
    extern __shared__ float ylds[];
    __shared__ double red_d[THREADS / 64];
    __shared__ float red_f[2 * (THREADS / 64)];
    __shared__ int32_t red_i[THREADS / 64];
    constexpr int QMAX = (1 << BITS) - 1;
    const int tid = threadIdx.x;

    for (int64_t row = blockIdx.x; row < a.N; row += gridDim.x) {
        load_norm_stage<XT, THREADS, ITERS>(a, row, ylds, red_d);
        __syncthreads();

        // ---- steps a2 + a3: gather through the map; 8 reassembled channels per lane and step
        float val[ITERS][GROUP];
        int32_t rot[ITERS];  // slot k of val holds reassembled channel 8g + ((k - rot) & 7)
        uint32_t live[ITERS]; // bit k: slot k is a real channel (not padding)
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int g = tid + it * THREADS;
            rot[it] = 0;
            live[it] = 0;
#pragma unroll
            for (int k = 0; k < GROUP; ++k) val[it][k] = 0.0f;
            if (g < a.n_groups) {
                const int32_t d = a.desc ? a.desc[g] : -1;
                if (d >= 0) { // eight single-source channels with scale 1 and consecutive sources
                    const int v = d & 7, u = d >> 3;
                    rot[it] = v;
                    live[it] = 0xffu;
#pragma unroll
                    for (int k = 0; k < GROUP; ++k) val[it][k] = ylds[k * a.S + u + (k < v ? 1 : 0)];
                } else {
#pragma unroll
                    for (int k = 0; k < GROUP; ++k) {
                        const int ch = g * GROUP + k;
                        if (ch < a.C_out) {
                            int32_t e = a.row_ptr[ch];
                            const int32_t e1 = a.row_ptr[ch + 1];
                            int32_t s = a.src[e];
                            float acc = a.scale[e] * ylds[(s & 7) * a.S + (s >> 3)];
                            for (++e; e < e1; ++e) {
                                s = a.src[e];
                                acc = acc + a.scale[e] * ylds[(s & 7) * a.S + (s >> 3)];
                            }
                            val[it][k] = acc;
                            live[it] |= 1u << k;
                        }
                    }
                }
#pragma unroll
                for (int k = 0; k < GROUP; ++k)
                    if (live[it] >> k & 1u) {
                        mn = fminf(mn, val[it][k]);
                        mx = fmaxf(mx, val[it][k]);
                    }
            }
        }
        block_minmax_f32<THREADS>(mn, mx, red_f);

        // ---- step a4: Eq. (2)
        const float range = mx - mn;
        const float alpha = range > 0.0f ? range / (float)QMAX : 1.0f;
        const float inv = 1.0f / alpha;
        const int32_t fast = fabsf(mn * inv) < FAST_LIMIT && fabsf(mx * inv) < FAST_LIMIT;
        int32_t beta;
        if (fast) beta = -rne_product_fast(mn, inv);
        else beta = (int32_t)fmin(fmax(-rne_product_slow(mn, inv), -2147483647.0), 2147483647.0);

        int32_t sum = 0;
        uint8_t *out_row = a.codes + row * a.row_bytes;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int g = tid + it * THREADS;
            if (g < a.n_groups_pad) {
                uint64_t packed = 0;
#pragma unroll
                for (int k = GROUP - 1; k >= 0; --k) {
                    int32_t q = quant_code<QMAX>(val[it][k], inv, beta, fast);
                    q = (live[it] >> k & 1u) ? q : 0;
                    sum += q;
                    packed = (packed << BITS) | (uint64_t)q;
                }
                // slot k -> channel (k - rot) & 7: rotate the 8*BITS-bit word right by rot*BITS
                const int sh = rot[it] * BITS;
                if constexpr (BITS == 4) {
                    const uint32_t p = (uint32_t)packed;
                    reinterpret_cast<uint32_t *>(out_row)[g] = (p >> sh) | (p << ((32 - sh) & 31));
                } else if constexpr (BITS == 8) {
                    reinterpret_cast<uint64_t *>(out_row)[g] = (packed >> sh) | (packed << ((64 - sh) & 63));
                } else {
                    const uint64_t p = ((packed >> sh) | (packed << (48 - sh))) & 0xffffffffffffull;
                    uint16_t *o16 = reinterpret_cast<uint16_t *>(out_row + (int64_t)g * 6);
                    o16[0] = (uint16_t)p;
                    o16[1] = (uint16_t)(p >> 16);
                    o16[2] = (uint16_t)(p >> 32);
                }
            }
        }
        sum = block_sum_i32<THREADS>(sum, red_i);
        if (tid == 0) {
            a.alpha[row] = alpha;
            a.zero[row] = beta;
            a.rowsum[row] = sum;
        }
        __syncthreads(); // ylds is overwritten by the next row
    }
}

// ---- calibration statistic: per-channel max |y| (Sec. 4.1.1; vector m of Algorithm 1)
template <typename XT, int THREADS, int ITERS>
__global__ __launch_bounds__(THREADS) void norm_absmax_kernel(const FusedArgs a)
{
    extern __shared__ float ylds[];
    __shared__ double red_d[THREADS / 64];
    const int tid = threadIdx.x;
    const int n_chunks = (a.C + GROUP - 1) / GROUP;
    float best[ITERS][GROUP];
#pragma unroll
    for (int it = 0; it < ITERS; ++it)
#pragma unroll
        for (int j = 0; j < GROUP; ++j) best[it][j] = 0.0f;

    for (int64_t row = blockIdx.x; row < a.N; row += gridDim.x) {
        load_norm_stage<XT, THREADS, ITERS>(a, row, ylds, red_d);
        // every lane re-reads only what it wrote itself: no barrier needed before the read
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int i = tid + it * THREADS;
            if (i < n_chunks) {
#pragma unroll
                for (int j = 0; j < GROUP; ++j) {
                    const float y = ylds[j * a.S + i];
                    best[it][j] = fmaxf(best[it][j], fabsf(y));
                    if (a.y_dump && row < a.n_dump && i * GROUP + j < a.C)
                        a.y_dump[row * a.C + i * GROUP + j] = y;
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int i = tid + it * THREADS;
#pragma unroll
        for (int j = 0; j < GROUP; ++j)
            if (i < n_chunks && i * GROUP + j < a.C) // |y| >= 0: its bit pattern orders like an unsigned integer
                atomicMax(reinterpret_cast<unsigned int *>(a.absmax) + i * GROUP + j, __float_as_uint(best[it][j]));
    }
}

template <typename K>
int32_t launch_with_lds(K kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, const FusedArgs &args)
{
    if (lds_bytes > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            qllm_note_hip_error("fused kernel: raising the LDS limit", hipGetErrorName(e));
            return QLLM_ERR_HIP;
        }
    }
    (void)hipGetLastError(); // drop any stale error of the calling thread: only this launch is judged
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error("fused kernel: launch", hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}

template <typename XT, int BITS>
int32_t dispatch_size(const FusedArgs &a, int max_units, hipStream_t stream)
{
    const size_t lds = (size_t)a.S * GROUP * sizeof(float);
    const dim3 grid((unsigned)(a.N < 1048576 ? a.N : 1048576));
    if (max_units <= 256) return launch_with_lds(fused_nrq_kernel<XT, BITS, 256, 1>, grid, dim3(256), lds, stream, a);
    if (max_units <= 1024) return launch_with_lds(fused_nrq_kernel<XT, BITS, 256, 4>, grid, dim3(256), lds, stream, a);
    if (max_units <= 2048) return launch_with_lds(fused_nrq_kernel<XT, BITS, 1024, 2>, grid, dim3(1024), lds, stream, a);
    return launch_with_lds(fused_nrq_kernel<XT, BITS, 1024, 4>, grid, dim3(1024), lds, stream, a);
}

template <typename XT>
int32_t dispatch_bits(const FusedArgs &a, int bits, int max_units, hipStream_t stream)
{
    if (bits == 4) return dispatch_size<XT, 4>(a, max_units, stream);
    if (bits == 6) return dispatch_size<XT, 6>(a, max_units, stream);
    return dispatch_size<XT, 8>(a, max_units, stream);
}

int32_t check_common(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx, int32_t norm,
                     const float *gamma)
{
    if (!x) return QLLM_ERR_NULL;
    if (x_dtype != QLLM_F32 && x_dtype != QLLM_BF16) return QLLM_ERR_DTYPE;
    if (norm != QLLM_NORM_NONE && norm != QLLM_NORM_LAYER && norm != QLLM_NORM_RMS) return QLLM_ERR_DTYPE;
    if (N < 0 || N > INT32_MAX || C <= 0 || C > QLLM_MAX_CHANNELS || ldx < C) return QLLM_ERR_SHAPE;
    if (norm != QLLM_NORM_NONE && !gamma) return QLLM_ERR_NULL;
    if (norm != QLLM_NORM_NONE && (reinterpret_cast<uintptr_t>(gamma) & 15u)) return QLLM_ERR_ALIGN;
    return QLLM_OK;
}

void fill_input(FusedArgs &a, const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx, int32_t norm,
                const float *gamma, const float *beta, float eps)
{
    const size_t esz = x_dtype == QLLM_BF16 ? 2 : 4;
    a.x = x;
    a.ldx = ldx;
    a.N = (int32_t)N;
    a.C = (int32_t)C;
    a.norm = norm;
    a.vec_ok = ((reinterpret_cast<uintptr_t>(x) & 15u) == 0 && (ldx * esz) % 16 == 0) ? 1 : 0;
    a.gamma = gamma;
    a.beta = beta;
    a.eps = eps;
    a.inv_C = 1.0 / (double)C;
    a.S = (int32_t)((C + GROUP - 1) / GROUP);
}

// The parts of a map's plan: the host copy of its header says where they are (see qllm_plan_map_host).
int32_t fill_plan(FusedArgs &a, const qllm_map *map, int64_t C)
{
    if (!map->plan) return QLLM_OK;
    const int32_t *h = map->plan_head;
    if (reinterpret_cast<uintptr_t>(map->plan) & 15u) return QLLM_ERR_ALIGN;
    if (h[0] != 0x514c4d50 || h[1] != 8 || h[2] != C || h[3] != map->C_out) return QLLM_ERR_MAP;
    const int64_t n_chunks = (C + GROUP - 1) / GROUP, n_work = (map->C_out + QLLM_K_PAD - 1) / QLLM_K_PAD * QLLM_K_PAD / GROUP;
    auto round4 = [](int64_t v) { return (v + 3) / 4 * 4; };
    if (h[4] != n_work || h[6] != n_chunks || h[5] < 0 || h[5] > n_work || h[7] < 0 || h[8] < 0 || h[8] > n_chunks ||
        h[9] < 0 || h[10] < h[9] || h[11] < h[5] || h[14] < 0 || h[14] > h[10] - h[9] || h[15] < 64 * (int64_t)h[14])
        return QLLM_ERR_MAP;
    const int64_t off_work = QLLM_PLAN_HEAD, off_chunks = round4(off_work + n_work), off_spec = round4(off_chunks + n_chunks);
    const int64_t off_dest = round4(off_spec + 2 * (int64_t)h[9]), off_longs = round4(off_dest + h[10]);
    const int64_t off_segs = off_longs + 4 * (int64_t)h[7];
    const int64_t off_recs = round4(off_segs + h[11]);
    const int64_t off_xlrows = off_recs + 8 * (int64_t)h[5], off_xlent = off_xlrows + 4 * (int64_t)h[14];
    if (h[12] != off_chunks || h[13] != off_xlent + 2 * (int64_t)h[15]) return QLLM_ERR_MAP;
    a.work = map->plan + off_work;
    a.chunks = map->plan + off_chunks;
    a.spec = map->plan + off_spec;
    a.dest = map->plan + off_dest;
    a.longs = map->plan + off_longs;
    a.segs = map->plan + off_segs;
    a.recs = map->plan + off_recs;
    a.xlrows = map->plan + off_xlrows;
    a.xlent = map->plan + off_xlent;
    a.n_xl = h[14];
    a.n_work = h[4];
    a.n_comp = h[5];
    a.n_chunks = h[6];
    a.n_long = h[7];
    a.n_pub = h[8];
    a.n_spec = h[9];
    a.n_dest = h[10];
    a.n_segw = h[11];
    return QLLM_OK;
}

} // namespace

extern "C" int32_t qllm_norm_reassemble_quant(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                              int32_t norm, const float *gamma, const float *beta, float eps,
                                              const qllm_map *map, int32_t bits, const qllm_qact *out,
                                              void *hip_stream)
{
    int32_t rc = check_common(x, x_dtype, N, C, ldx, norm, gamma);
    if (rc != QLLM_OK) return rc;
    if (!map || !out) return QLLM_ERR_NULL;
    if (!map->row_ptr || !map->src || !map->scale) return QLLM_ERR_NULL;
    if (!out->codes || !out->scale || !out->zero || !out->rowsum) return QLLM_ERR_NULL;
    if (bits != 4 && bits != 6 && bits != 8) return QLLM_ERR_BITS;
    if (map->C_in != C || map->C_out <= 0 || map->C_out > QLLM_MAX_CHANNELS || map->nnz < map->C_out)
        return QLLM_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(out->codes) & 15u) return QLLM_ERR_ALIGN;
    if (N == 0) return QLLM_OK;

    FusedArgs a{};
    fill_input(a, x, x_dtype, N, C, ldx, norm, gamma, beta, eps);
    a.row_ptr = map->row_ptr;
    a.src = map->src;
    a.scale = map->scale;
    rc = fill_plan(a, map, C);
    if (rc != QLLM_OK) return rc;
    a.C_out = (int32_t)map->C_out;
    a.n_groups = (int32_t)((map->C_out + GROUP - 1) / GROUP);
    a.row_bytes = qllm_packed_row_bytes(map->C_out, bits);
    a.n_groups_pad = (int32_t)(a.row_bytes * 8 / bits / GROUP);
    a.codes = out->codes;
    a.alpha = out->scale;
    a.zero = out->zero;
    a.rowsum = out->rowsum;
    const int max_units = a.S > a.n_groups_pad ? a.S : a.n_groups_pad;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (map->plan) {
        rc = qllm_launch_fused_planned(a, x_dtype, bits, stream);
        if (rc != QLLM_ERR_WORKSPACE) return rc; // does not fit on chip: the plain kernel below handles it
    }
    if (x_dtype == QLLM_BF16) return dispatch_bits<uint16_t>(a, bits, max_units, stream);
    return dispatch_bits<float>(a, bits, max_units, stream);
}

extern "C" int32_t qllm_fused_kernel_choice(const qllm_map *map, int32_t x_dtype, int64_t N, int64_t ldx, int32_t norm,
                                            int32_t has_beta, int32_t bits)
{
    if (!map) return QLLM_ERR_NULL;
    if (x_dtype != QLLM_F32 && x_dtype != QLLM_BF16) return QLLM_ERR_DTYPE;
    if (norm != QLLM_NORM_NONE && norm != QLLM_NORM_LAYER && norm != QLLM_NORM_RMS) return QLLM_ERR_DTYPE;
    if (bits != 4 && bits != 6 && bits != 8) return QLLM_ERR_BITS;
    const int64_t C = map->C_in;
    if (N < 0 || N > INT32_MAX || C <= 0 || C > QLLM_MAX_CHANNELS || ldx < C || map->C_out <= 0 || map->C_out > QLLM_MAX_CHANNELS)
        return QLLM_ERR_SHAPE;
    FusedArgs a{};
    // stand-ins for the buffers: 16-byte aligned, and only their being there or not matters here
    static const float present[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    fill_input(a, nullptr, x_dtype, N, C, ldx, norm, present, has_beta ? present : nullptr, 0.0f);
    const int32_t rc = fill_plan(a, map, C);
    if (rc != QLLM_OK) return rc;
    return qllm_choose_fused_planned(a, x_dtype, bits);
}

extern "C" int32_t qllm_norm_channel_absmax(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                            int32_t norm, const float *gamma, const float *beta, float eps,
                                            float *absmax, float *y_dump, int64_t n_dump, void *hip_stream)
{
    int32_t rc = check_common(x, x_dtype, N, C, ldx, norm, gamma);
    if (rc != QLLM_OK) return rc;
    if (!absmax) return QLLM_ERR_NULL;
    if (n_dump < 0 || n_dump > N) return QLLM_ERR_SHAPE;
    if (N == 0) return QLLM_OK;
    FusedArgs a{};
    fill_input(a, x, x_dtype, N, C, ldx, norm, gamma, beta, eps);
    a.absmax = absmax;
    a.y_dump = n_dump > 0 ? y_dump : nullptr;
    a.n_dump = (int32_t)n_dump;
    if (n_dump > 0 && !y_dump) return QLLM_ERR_NULL;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    const size_t lds = (size_t)a.S * GROUP * sizeof(float);
    const dim3 grid((unsigned)(N < 1024 ? N : 1024));
    const bool big = a.S > 1024;
    if (x_dtype == QLLM_BF16) {
        if (big) return launch_with_lds(norm_absmax_kernel<uint16_t, 1024, 4>, grid, dim3(1024), lds, stream, a);
        return launch_with_lds(norm_absmax_kernel<uint16_t, 256, 4>, grid, dim3(256), lds, stream, a);
    }
    if (big) return launch_with_lds(norm_absmax_kernel<float, 1024, 4>, grid, dim3(1024), lds, stream, a);
    return launch_with_lds(norm_absmax_kernel<float, 256, 4>, grid, dim3(256), lds, stream, a);
}
