// Integer GEMM on the gfx950 int8 matrix cores with a dequantising epilogue.
//
//   acc[n, o] = sum_k a[n, k] * w[o, k]          (Eq. 1 on the codes of Eq. 2; exact int32)
//   Y[n, o]   = ((float)(acc - bx[n]*cs[o] - bw[o]*rs[n] + K*bx[n]*bw[o]) * ax[n]) * aw[o]
//
// Both operands arrive as packed 4/6/8-bit codes, K contiguous.  A workgroup of 256 lanes (4 waves,
// 2 x 2) owns a 128 x 128 tile of Y.  Per K-tile of 256 codes every lane fetches 64-code units of
// the packed rows from HBM into registers (16-byte loads), expands them to one byte per code and
// stores them into LDS (16-byte chunks, XOR-swizzled by row so that the matrix-core operand reads
// are bank-conflict free); the loads of the next K-tile are in flight while the current one is
// multiplied.  Each wave multiplies 64 x 64 with v_mfma_i32_16x16x64_i8 (16 accumulator tiles).
//
// 8-bit codes do not fit a signed byte: they are stored as code-128 and the accumulator is corrected
// with the row / column sums the epilogue already has.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include <mutex>
#include <type_traits>
#include <vector>

#include "qllm.h"

extern "C" void qllm_note_hip_error(const char *step, const char *name);

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, KT = 256; // block tile; KT codes per LDS stage
constexpr int THREADS = 256;
constexpr int UNIT = 64;                    // codes per fetch unit = K of one MFMA
constexpr int ROW_LDS = KT;                 // bytes per tile row in LDS (one byte per code)

struct GemmArgs {
    const uint8_t *a_codes, *w_codes;
    int64_t a_row_bytes, w_row_bytes;
    const float *ax, *aw;
    const int32_t *bx, *bw, *rs, *cs;
    int32_t N, O, K, Kpad;
    int32_t small_zero; // zero-points below this (in magnitude) keep every epilogue term inside 24 / 32 bits; 0: never
    void *y;
    int64_t ldy;
    int32_t *acc_dump;
    int32_t *partial; // [splits][N][O] raw accumulators when K is split over workgroups, else unused
    int32_t splits;
    const uint8_t *a_tiles, *w_tiles; // both operands as 6-bit fields in matrix-core order (see TILES6 below), or null
    const uint8_t *a_tiles8, *w_tiles8; // both operands as bytes in matrix-core order (see TILES8 below), or null
    // A launch of the FP6 or the byte-operand kernel may cover the output features o_first .. O - 1 only (the call is
    // then two launches with different tiles, each with its own O); never together with acc_dump, whose rows are O long.
    int32_t o_first;
};

template <int BITS>
struct Unit {
    uint4 r[BITS / 2]; // 64 codes: 32 / 48 / 64 bytes
};

// unit number `unit` (64 codes each) of a packed row
template <int BITS>
__device__ __forceinline__ void load_unit(Unit<BITS> &u, const uint8_t *row, int unit)
{
    const uint4 *p = reinterpret_cast<const uint4 *>(row + (int64_t)unit * (UNIT * BITS / 8));
#pragma unroll
    for (int i = 0; i < BITS / 2; ++i) u.r[i] = p[i];
}

// 8 nibbles of w -> 8 bytes in channel order
__device__ __forceinline__ void expand4(uint32_t w, uint32_t &d0, uint32_t &d1)
{
    const uint32_t lo = w & 0x0f0f0f0fu;        // codes 0 2 4 6
    const uint32_t hi = (w >> 4) & 0x0f0f0f0fu; // codes 1 3 5 7
    d0 = __builtin_amdgcn_perm(hi, lo, 0x05010400u); // lo.b0 hi.b0 lo.b1 hi.b1
    d1 = __builtin_amdgcn_perm(hi, lo, 0x07030602u); // lo.b2 hi.b2 lo.b3 hi.b3
}

// four 6-bit codes in the low 24 bits of t (higher bits are ignored) -> four bytes
__device__ __forceinline__ uint32_t spread6(uint32_t t)
{
    const uint32_t x = (t & 0xfffu) | ((t << 4) & 0x0fff0000u);      // codes 0,1 in the low half, 2,3 in the high half
    return (x & 0x003f003fu) | ((x << 2) & 0x3f003f00u);
}

// One unit (64 packed codes) -> 64 bytes, as 16 dwords.  PERM: both operands are 4-bit, so the order of
// the codes inside a unit is free as long as both sides use the same one; even codes then odd codes of
// each dword is the cheapest (two masks and a shift instead of two more byte permutes).  8-bit codes
// become code - 128, a signed byte (the epilogue adds the difference back).
template <int BITS, bool PERM>
__device__ __forceinline__ void expand_unit(const Unit<BITS> &u, uint32_t (&d)[16])
{
    if constexpr (BITS == 4) {
        const uint32_t w[8] = {u.r[0].x, u.r[0].y, u.r[0].z, u.r[0].w, u.r[1].x, u.r[1].y, u.r[1].z, u.r[1].w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (PERM) {
                d[2 * i] = w[i] & 0x0f0f0f0fu;
                d[2 * i + 1] = (w[i] >> 4) & 0x0f0f0f0fu;
            } else {
                expand4(w[i], d[2 * i], d[2 * i + 1]);
            }
        }
    } else if constexpr (BITS == 6) {
        const uint32_t w[12] = {u.r[0].x, u.r[0].y, u.r[0].z, u.r[0].w, u.r[1].x, u.r[1].y,
                                u.r[1].z, u.r[1].w, u.r[2].x, u.r[2].y, u.r[2].z, u.r[2].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { // 3 dwords = 4 groups of 24 bits
            const uint32_t w0 = w[3 * i], w1 = w[3 * i + 1], w2 = w[3 * i + 2];
            d[4 * i + 0] = spread6(w0);
            d[4 * i + 1] = spread6(__builtin_amdgcn_alignbit(w1, w0, 24));
            d[4 * i + 2] = spread6(__builtin_amdgcn_alignbit(w2, w1, 16));
            d[4 * i + 3] = spread6(w2 >> 8);
        }
    } else {
        const uint32_t w[16] = {u.r[0].x, u.r[0].y, u.r[0].z, u.r[0].w, u.r[1].x, u.r[1].y, u.r[1].z, u.r[1].w,
                                u.r[2].x, u.r[2].y, u.r[2].z, u.r[2].w, u.r[3].x, u.r[3].y, u.r[3].z, u.r[3].w};
#pragma unroll
        for (int i = 0; i < 16; ++i) d[i] = w[i] ^ 0x80808080u; // code - 128 as a signed byte
    }
}

// Expands one unit and stores it as four 16-byte chunks of LDS row `row` (ROWB bytes per row, chunks
// XOR-swizzled by row).
template <int BITS, int ROWB, bool PERM>
__device__ __forceinline__ void store_unit(const Unit<BITS> &u, uint8_t *tile, int row, int ku)
{
    uint32_t d[16];
    expand_unit<BITS, PERM>(u, d);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int chunk = (ku * 4 + c) ^ (row & 7);
        *reinterpret_cast<uint4 *>(tile + row * ROWB + chunk * 16) =
            make_uint4(d[4 * c], d[4 * c + 1], d[4 * c + 2], d[4 * c + 3]);
    }
}

// Chunk c (16 codes -> 16 bytes) of one unit, expanded and stored; c is a constant where this is
// called, so only that chunk's share of the expansion is left of expand_unit.
template <int BITS, int ROWB, bool PERM>
__device__ __forceinline__ void store_chunk(const Unit<BITS> &u, uint8_t *tile, int row, int ku, int c)
{
    uint32_t d[16];
    expand_unit<BITS, PERM>(u, d);
    const int chunk = (ku * 4 + c) ^ (row & 7);
    *reinterpret_cast<uint4 *>(tile + row * ROWB + chunk * 16) = make_uint4(d[4 * c], d[4 * c + 1], d[4 * c + 2], d[4 * c + 3]);
}

template <int ROWB>
__device__ __forceinline__ v4i load_frag(const uint8_t *tile, int row, int chunk)
{
    return *reinterpret_cast<const v4i *>(tile + row * ROWB + ((chunk ^ (row & 7)) * 16));
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Two floats -> two bfloat16 in one dword, round to nearest even: the hardware's packed conversion
// (v_cvt_pk_bf16_f32), one instruction where the integer form above takes about ten for the pair.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_rne(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// Stores 4 consecutive output features of one token (16 bytes per lane for fp32, 8 for bf16) and,
// if asked for, the raw accumulators.
template <typename YT>
__device__ __forceinline__ void store4(const GemmArgs &g, const float *out, const int32_t *raw, int n, int ob)
{
    if (ob + 3 < g.O) {
        if constexpr (sizeof(YT) == 4) {
            float *yp = reinterpret_cast<float *>(g.y) + (int64_t)n * g.ldy + ob;
            if ((reinterpret_cast<uintptr_t>(yp) & 15u) == 0) {
                *reinterpret_cast<float4 *>(yp) = make_float4(out[0], out[1], out[2], out[3]);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) yp[r] = out[r];
            }
        } else {
            uint16_t *yp = reinterpret_cast<uint16_t *>(g.y) + (int64_t)n * g.ldy + ob;
            const uint32_t p0 = f32x2_to_bf16x2_rne(out[0], out[1]), p1 = f32x2_to_bf16x2_rne(out[2], out[3]);
            if ((reinterpret_cast<uintptr_t>(yp) & 7u) == 0) {
                *reinterpret_cast<uint2 *>(yp) = make_uint2(p0, p1);
            } else {
                yp[0] = (uint16_t)p0; yp[1] = (uint16_t)(p0 >> 16);
                yp[2] = (uint16_t)p1; yp[3] = (uint16_t)(p1 >> 16);
            }
        }
        if (g.acc_dump) {
#pragma unroll
            for (int r = 0; r < 4; ++r) g.acc_dump[(int64_t)n * g.O + ob + r] = raw[r];
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (ob + r < g.O) {
                if constexpr (sizeof(YT) == 4)
                    reinterpret_cast<float *>(g.y)[(int64_t)n * g.ldy + ob + r] = out[r];
                else
                    reinterpret_cast<uint16_t *>(g.y)[(int64_t)n * g.ldy + ob + r] = f32_to_bf16_rne(out[r]);
                if (g.acc_dump) g.acc_dump[(int64_t)n * g.O + ob + r] = raw[r];
            }
    }
}

// Dequantising epilogue of one wave tile: NI x NJ matrix-core tiles of 16 x 16; the lane holds, for
// tile (i, j), token n_base + 16 i + (lane & 15) and features o_base + 16 j + 4 (lane >> 4) + 0..3.
//   bracket = acc - bx*cs - bw*rs + K*bx*bw       (exact integer)
//   Y       = ((float)bracket * ax) * aw
// When both zero-points are small (the usual case: |beta| < g.small_zero, a bound the launcher derives
// from K and the bit widths) every factor fits 24 bits and every sum 32 bits, and the bracket costs
// three full-rate multiply-adds; otherwise it is formed in 64-bit arithmetic.
// An accumulator as the integer it stands for: the int8 matrix cores' own, or 64 x the FP6 path's float (exact).
typedef float v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int32_t acc_int(const v4i &a, int r) { return a[r]; }
__device__ __forceinline__ int32_t acc_int(const v4f &a, int r) { return (int32_t)(a[r] * 64.0f); }

template <int ABITS, int WBITS, typename YT, int NI, int NJ, typename ACC>
__device__ __forceinline__ void finish_wave_tile(const GemmArgs &g, const ACC (&acc)[NI][NJ], int n_base, int o_base,
                                                 int lane, int32_t k_biased = -1)
{
    constexpr int SA = ABITS == 8 ? 1 : 0, SW = WBITS == 8 ? 1 : 0;
    int32_t cs[NJ][4], bw[NJ][4];
    float aw[NJ][4];
    bool cols_small = true;
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int o = min(o_base + j * 16 + 4 * (lane >> 4) + r, g.O - 1);
            cs[j][r] = g.cs[o];
            bw[j][r] = g.bw[o];
            aw[j][r] = g.aw[o];
            cols_small = cols_small && abs(bw[j][r]) < g.small_zero;
        }
    // 8-bit codes went into the matrix cores as code - 128; where both sides did, every place of K that held such a
    // pair adds 128 * 128: the padded row length, unless the kernel says how many places it summed that way
    const int32_t k_off = 16384 * SA * SW * (k_biased >= 0 ? k_biased : g.Kpad);

    // The usual case, decided once for the wave: the tile lies inside Y, Y's rows are aligned for whole stores, nobody
    // asked for the raw accumulators, and every zero-point of the tile is small.  Then the tile is straight-line
    // code: three 24-bit multiply-adds, a conversion and two multiplications per output, one store per four.
    {
        const bool inside = n_base + 16 * NI <= g.N && o_base + 16 * NJ <= g.O;
        const bool aligned = (reinterpret_cast<uintptr_t>(g.y) & (sizeof(YT) == 4 ? 15u : 7u)) == 0 && (g.ldy & 3) == 0;
        if (inside && aligned && !g.acc_dump) { // wave-uniform so far: the loads below are in bounds
            int32_t bxs[NI], rss[NI];
            float axs[NI];
            bool small = cols_small;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int n = n_base + i * 16 + (lane & 15);
                bxs[i] = g.bx[n];
                rss[i] = g.rs[n];
                axs[i] = g.ax[n];
                small = small && abs(bxs[i]) < g.small_zero;
            }
            if (__all(small)) {
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const int n = n_base + i * 16 + (lane & 15);
                    const int32_t kbx = g.K * bxs[i];
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        float out[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            int32_t t = acc_int(acc[i][j], r) + 128 * SW * rss[i] + 128 * SA * cs[j][r] - k_off;
                            t -= __mul24(bxs[i], cs[j][r]);
                            t -= __mul24(bw[j][r], rss[i]);
                            t += __mul24(kbx, bw[j][r]);
                            float v = (float)t;
                            v = v * axs[i];
                            v = v * aw[j][r];
                            out[r] = v;
                        }
                        const int64_t at = (int64_t)n * g.ldy + o_base + j * 16 + 4 * (lane >> 4);
                        if constexpr (sizeof(YT) == 4)
                            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(g.y) + at) = make_float4(out[0], out[1], out[2], out[3]);
                        else
                            *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(g.y) + at) =
                                make_uint2(f32x2_to_bf16x2_rne(out[0], out[1]), f32x2_to_bf16x2_rne(out[2], out[3]));
                    }
                }
                return;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int n = n_base + i * 16 + (lane & 15);
        if (n >= g.N) continue;
        const int32_t bx = g.bx[n], rs = g.rs[n];
        const float ax = g.ax[n];
        const bool small = cols_small && abs(bx) < g.small_zero;
        const int32_t kbx = g.K * bx; // only used when small
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float out[4];
            int32_t raw[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // the true accumulator fits int32 (checked by the launcher), so wrapping sums are exact
                raw[r] = acc_int(acc[i][j], r) + 128 * SW * rs + 128 * SA * cs[j][r] - k_off;
                float v;
                if (small) {
                    int32_t t = raw[r] - __mul24(bx, cs[j][r]);
                    t -= __mul24(bw[j][r], rs);
                    t += __mul24(kbx, bw[j][r]);
                    v = (float)t;
                } else {
                    const int64_t t = (int64_t)raw[r] - (int64_t)bx * cs[j][r] - (int64_t)bw[j][r] * rs +
                                      (int64_t)g.K * bx * bw[j][r];
                    v = (float)t;
                }
                v = v * ax;
                v = v * aw[j][r];
                out[r] = v;
            }
            store4<YT>(g, out, raw, n, o_base + j * 16 + 4 * (lane >> 4));
        }
    }
}

template <int ABITS, int WBITS, typename YT>
__global__ __launch_bounds__(THREADS) void int_gemm_kernel(const GemmArgs g)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds_a[BM * ROW_LDS];
    __shared__ __attribute__((aligned(16))) uint8_t lds_w[BN * ROW_LDS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1; // wave position in the 2 x 2 arrangement
    const int n0 = blockIdx.y * BM, o0 = blockIdx.x * BN;

    // fetch assignment: units tid and tid + 256 of each operand tile (unit = row * 4 + ku)
    const int f_row = tid >> 2, f_ku = tid & 3;
    const uint8_t *a_row[2], *w_row[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int rn = min(n0 + f_row + 64 * h, g.N - 1); // rows past the edge re-read the last row
        const int ro = min(o0 + f_row + 64 * h, g.O - 1);
        a_row[h] = g.a_codes + (int64_t)rn * g.a_row_bytes;
        w_row[h] = g.w_codes + (int64_t)ro * g.w_row_bytes;
    }

    v4i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    Unit<ABITS> ua[2];
    Unit<WBITS> uw[2];
    const int n_kt = g.Kpad / KT;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        load_unit<ABITS>(ua[h], a_row[h], f_ku);
        load_unit<WBITS>(uw[h], w_row[h], f_ku);
    }

    for (int kt = 0; kt < n_kt; ++kt) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            store_unit<ABITS, ROW_LDS, ABITS == 4 && WBITS == 4>(ua[h], lds_a, f_row + 64 * h, f_ku);
            store_unit<WBITS, ROW_LDS, ABITS == 4 && WBITS == 4>(uw[h], lds_w, f_row + 64 * h, f_ku);
        }
        __syncthreads();
        if (kt + 1 < n_kt) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                load_unit<ABITS>(ua[h], a_row[h], (kt + 1) * (KT / UNIT) + f_ku);
                load_unit<WBITS>(uw[h], w_row[h], (kt + 1) * (KT / UNIT) + f_ku);
            }
        }
#pragma unroll
        for (int ks = 0; ks < KT / UNIT; ++ks) {
            const int chunk = ks * 4 + (lane >> 4);
            v4i fa[4], fw[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) fa[i] = load_frag<ROW_LDS>(lds_a, wm * 64 + i * 16 + (lane & 15), chunk);
#pragma unroll
            for (int j = 0; j < 4; ++j) fw[j] = load_frag<ROW_LDS>(lds_w, wn * 64 + j * 16 + (lane & 15), chunk);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    // operand order (w, a): the lane then holds 4 consecutive OUTPUT features of one
                    // token, so the stores below write 16 bytes per lane
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[j], fa[i], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // ---- epilogue.  acc[i][j][r]: token n0 + wm*64 + i*16 + (lane & 15),
    //                               feature o0 + wn*64 + j*16 + 4*(lane >> 4) + r
    finish_wave_tile<ABITS, WBITS, YT, 4, 4>(g, acc, n0 + wm * 64, o0 + wn * 64, lane);
}

// ---- the large-tile kernel for bit pairs other than 4/4: 512 lanes (8 waves, 2 x 4), a 256 x 256 tile
// of Y, K-tiles of 128 codes, one byte per code in two LDS buffers.  While the matrix cores work
// through buffer `cur`, the lanes expand the next K-tile (fetched one iteration earlier) into the other
// buffer, one 16-byte chunk per group of four matrix-core operations, and fetch the one after it: one
// barrier per K-tile.
constexpr int LBM = 256, LBN = 256, LKT = 128, LTHREADS = 512, LROWB = LKT; // one byte per code in LDS
constexpr int LBUF = (LBM + LBN) * LROWB;                                   // 64 KB per buffer

template <int ABITS, int WBITS, typename YT>
__global__ __launch_bounds__(LTHREADS) void int_gemm_big_kernel(const GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr bool PERM = ABITS == 4 && WBITS == 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3; // wave tile: 128 tokens x 64 features
    const int n0 = blockIdx.y * LBM, o0 = blockIdx.x * LBN;

    // fetch assignment: one unit of each operand per lane and K-tile (unit = row * 2 + ku)
    const int f_row = tid >> 1, f_ku = tid & 1;
    const uint8_t *a_row = g.a_codes + (int64_t)min(n0 + f_row, g.N - 1) * g.a_row_bytes; // past the edge:
    const uint8_t *w_row = g.w_codes + (int64_t)min(o0 + f_row, g.O - 1) * g.w_row_bytes; // re-read the last row

    v4i acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    Unit<ABITS> ua;
    Unit<WBITS> uw;
    const int n_kt = g.Kpad / LKT;
    load_unit<ABITS>(ua, a_row, f_ku);
    load_unit<WBITS>(uw, w_row, f_ku);
    store_unit<ABITS, LROWB, PERM>(ua, lds, f_row, f_ku);
    store_unit<WBITS, LROWB, PERM>(uw, lds + LBM * LROWB, f_row, f_ku);
    load_unit<ABITS>(ua, a_row, min(1, n_kt - 1) * 2 + f_ku);
    load_unit<WBITS>(uw, w_row, min(1, n_kt - 1) * 2 + f_ku);
    __syncthreads();

    // One K-tile = 16 groups of four matrix-core operations: group s multiplies the token-side
    // fragment s (rows 16 (s & 7) .. of the wave's 128, half s >> 3 of the K-tile) with the four
    // feature-side fragments of that half.  Everything else is spread over the groups, in an order
    // fixed by scheduling fences, so that the matrix cores never wait for it:
    //   * token-side fragment s + DIST is requested in group s (a ring of RING registers), also
    //     across the K-tile boundary; the feature-side fragments of the second half in groups 0..3,
    //     those of the next K-tile's first half in the last two groups;
    //   * the refill of the other buffer (expand one 16-byte chunk of the unit fetched a K-tile
    //     ago, store it) takes groups 4..11, one chunk each; the fetch of the K-tile after that
    //     follows in group 12;
    //   * the one barrier per K-tile sits after group 15 - DIST: every refill store precedes it and
    //     every read of the next K-tile follows it; every read of this K-tile precedes it and the
    //     stores that will overwrite this buffer follow the next one.
    // The last K-tile refills and prefetches like the others (a re-read of the last K-tile into the
    // buffer nobody reads any more), which keeps the loop body free of branches.
    constexpr int DIST = 2, RING = 4, GROUPS = 8 * (LKT / UNIT), REFILL0 = 4;
    static_assert(GROUPS == 16 && GROUPS % RING == 0 && DIST < RING && REFILL0 + 8 < GROUPS - DIST, "group plan");
    // The loop is rotated by DIST groups: an iteration starts, right after the barrier, with the last
    // DIST groups of the previous K-tile (which request the first fragments of this one) and ends
    // with the barrier, so that no LDS request is pending across the loop's back edge.  Before the
    // first K-tile those groups multiply zeros; after the last one they run once more on their own.
    v4i fw[2][4], fa[RING];
#pragma unroll
    for (int j = 0; j < 4; ++j) fw[1][j] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int s = GROUPS - DIST; s < GROUPS; ++s) fa[s % RING] = v4i{0, 0, 0, 0};
    const int frow = lane & 15, fchunk = lane >> 4;

    for (int kt = 0; kt < n_kt; ++kt) {
        uint8_t *cur = lds + (kt & 1) * LBUF, *nxt = lds + ((kt + 1) & 1) * LBUF;
        const int kt2 = min(kt + 2, n_kt - 1);
#pragma unroll
        for (int u = 0; u < GROUPS; ++u) {
            const int s = (u + GROUPS - DIST) % GROUPS, ks = s >> 3, t = (s + DIST) % GROUPS;
            auto multiply = [&] {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[s & 7][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[ks][j], fa[s % RING], acc[s & 7][j], 0, 0, 0);
            };
            // group 0 is the first to use what the two groups before it asked for: its own requests
            // come after its operations, so that it waits for nothing newer than it needs
            if (s == 0) {
                multiply();
                __builtin_amdgcn_sched_barrier(0);
            }
            // fragment requests (all from this iteration's K-tile)
            fa[t % RING] = load_frag<LROWB>(cur, wm * 128 + (t & 7) * 16 + frow, (t >> 3) * 4 + fchunk);
            if (s < 4) fw[1][s] = load_frag<LROWB>(cur + LBM * LROWB, wn * 64 + s * 16 + frow, 4 + fchunk);
            if (s >= GROUPS - 2) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int j = (s - (GROUPS - 2)) * 2 + h;
                    fw[0][j] = load_frag<LROWB>(cur + LBM * LROWB, wn * 64 + j * 16 + frow, fchunk);
                }
            }
            // refill of the other buffer, fetch of the K-tile after it
            if (s >= REFILL0 && s < REFILL0 + 4) store_chunk<ABITS, LROWB, PERM>(ua, nxt, f_row, f_ku, s - REFILL0);
            if (s >= REFILL0 + 4 && s < REFILL0 + 8) store_chunk<WBITS, LROWB, PERM>(uw, nxt + LBM * LROWB, f_row, f_ku, s - REFILL0 - 4);
            if (s == REFILL0 + 8) {
                load_unit<ABITS>(ua, a_row, kt2 * 2 + f_ku);
                load_unit<WBITS>(uw, w_row, kt2 * 2 + f_ku);
            }
            if (s != 0) multiply();
            if (u == GROUPS - 1) __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int s = GROUPS - DIST; s < GROUPS; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[s & 7][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[1][j], fa[s % RING], acc[s & 7][j], 0, 0, 0);

    finish_wave_tile<ABITS, WBITS, YT, 8, 4>(g, acc, n0 + wm * 128, o0 + wn * 64, lane);
}

// ---- 4-bit codes on both sides, many tokens: the same 256 x 256 tile and 2 x 4 waves, but the codes
// stay packed (two per byte) in LDS and are split into bytes in registers, after the operand read.
// That halves the LDS traffic of the kernel above, which was what held it back: per K-tile of 128
// codes its expanded stores and operand reads kept LDS busy as long as the matrix cores were.
//   * LDS row = the 64 packed bytes of a K-tile; a lane (r, q) of an operand read takes the 16 bytes
//     q of row r: the low nibbles are its 16 codes for one matrix-core operation (m = 0), the high
//     nibbles those for a second one (m = 1).  Which 64 codes of the K-tile an operation sums is free
//     as long as both operands agree, and they do: same read, same split.
//   * Where a row's four 16-byte pieces sit in LDS is chosen for the banks.  Within a block of 16
//     rows, row r is stored as row place16(r) and its piece q at position q ^ (r & 3): a read by
//     lanes (r, q) then covers the block's 1 KB exactly once and each lane falls on the same banks
//     as in the byte-per-code layout of the kernel above (measured free of conflicts; rows kept in
//     order with any XOR of the piece index cost two passes per read).  The stores go the other way
//     round: lane t writes the t-th 16 bytes of the buffer half and fetches whichever row and piece
//     belong there, still four lanes per row.
//   * One K-tile = 16 groups of four matrix-core operations, (i, m) = (s >> 1, s & 1): token rows
//     16 i .. of the wave's 128, nibble m, times the wave's four feature-side operands of nibble m.
//     The eight feature-side operands of a K-tile stay split in registers; the token side streams:
//     packed read two row blocks ahead (a ring of four), split one group ahead.
//   * As above the order is fixed by scheduling fences, the loop is rotated by four groups (it
//     starts, after the barrier, with the last four groups of the previous K-tile, which request
//     the first operands of this one and multiply zeros the first time round) and refills without
//     branches.
constexpr int PROWB = 64;                       // packed bytes per LDS row and K-tile
constexpr int PBUF = (LBM + LBN) * PROWB;       // 32 KB per buffer
constexpr int PKT = 128;                        // codes per K-tile
constexpr int NBUF = 4;                         // ring of LDS buffers
constexpr int WAIT_VM8 = 8 | (7 << 4) | (15 << 8);       // s_waitcnt vmcnt(8) and nothing else
constexpr int WAIT_VM0 = 0 | (7 << 4) | (15 << 8);       // s_waitcnt vmcnt(0) and nothing else
constexpr int WAIT_VM8_LGKM0 = 8 | (7 << 4) | (0 << 8);  // s_waitcnt vmcnt(8) lgkmcnt(0)

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ v4i nib_lo(v4u p) { return (v4i)(p & 0x0f0f0f0fu); }
__device__ __forceinline__ v4i nib_hi(v4u p) { return (v4i)((p >> 4) & 0x0f0f0f0fu); }
// place of row r (0..15) inside its block of 16 rows, and the row stored at place p
__device__ __forceinline__ int place16(int r) { return ((r & 2) << 2) | ((r & 8) >> 1) | ((r & 1) << 1) | ((r & 4) >> 2); }
__device__ __forceinline__ int row_at16(int p) { return ((p & 2) >> 1) | ((p & 8) >> 2) | ((p & 1) << 2) | ((p & 4) << 1); }

// MI x NJ matrix-core tiles per wave: 8 x 4 (a 256 x 256 tile of Y per workgroup, the shape for many
// tokens) or 4 x 2 (128 x 128: four times as many workgroups, two of which share a CU, for shapes
// whose 256 x 256 tiles would leave most of the chip idle).
// SPLIT: K is dealt out to gridDim.z workgroups per tile of Y (shapes with so few tiles that most CUs
// would idle through a long K loop); each writes its raw accumulators to g.partial and
// splitk_finish_kernel adds them up and does the epilogue.
template <typename YT, int MI, int NJ, bool SPLIT = false>
__global__ __launch_bounds__(LTHREADS, MI == 8 ? 1 : 2) void int_gemm_w4a4_kernel(const GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int TM = 2 * MI * 16, TN = 4 * NJ * 16;     // the workgroup's tile of Y: 2 x 4 waves
    constexpr int STAGE = (TM + TN) * PROWB;              // bytes of one buffer of the ring
    constexpr int BLOCKS = (TM + TN) / 16, NLOAD = BLOCKS / 8; // 16-row blocks per K-tile; loads per wave and K-tile
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3; // wave tile: 16 MI tokens x 16 NJ features
    const int n0 = blockIdx.y * TM, o0 = blockIdx.x * TN;

    // fetch assignment: wave w brings in the 16-row blocks w, w + 8, .. of the buffer (the tile's token
    // rows first, then its feature rows); lane l fills the l-th 16 bytes of a block, that is piece
    // f_piece of the block's row f_row
    const int f_row = row_at16(lane >> 2), f_piece = (lane & 3) ^ (f_row & 3);
    const uint8_t *src[NLOAD];
#pragma unroll
    for (int t = 0; t < NLOAD; ++t) { // past the edge: re-read the last row
        const int blk = wave + 8 * t;
        src[t] = blk < TM / 16
                     ? g.a_codes + (int64_t)min(n0 + blk * 16 + f_row, g.N - 1) * g.a_row_bytes + f_piece * 16
                     : g.w_codes + (int64_t)min(o0 + (blk - TM / 16) * 16 + f_row, g.O - 1) * g.w_row_bytes + f_piece * 16;
    }

    // operand reads: lane (r, q) takes piece q of row r of a block of 16 rows
    const int r = lane & 15, q = lane >> 4;
    const int a_off = (wm * 16 * MI + place16(r)) * PROWB + ((q ^ (r & 3)) << 4);      // + i * 16 rows
    const int w_off = (TM + wn * 16 * NJ + place16(r)) * PROWB + ((q ^ (r & 3)) << 4); // + j * 16 rows

    v4i acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    // Refill: 16-byte global loads that write LDS directly (lane l of a wave lands at the wave's LDS
    // base + 16 l, which is why a block's order above is the lanes' order): no staging registers, no
    // LDS store instructions; NLOAD loads per wave and K-tile, issued three K-tiles ahead into a ring
    // of four buffers.  Loads complete in order, so "at most 2 NLOAD outstanding" before the barrier
    // means the next K-tile has landed.
    constexpr int WAIT_LANDED = 2 * NLOAD | (7 << 4) | (15 << 8);    // s_waitcnt vmcnt(2 NLOAD)
    constexpr int WAIT_LANDED_LGKM0 = 2 * NLOAD | (7 << 4) | (0 << 8); // ... and lgkmcnt(0)
    const int all_kt = g.Kpad / PKT;
    const int kt_first = SPLIT ? (int)((int64_t)all_kt * blockIdx.z / gridDim.z) : 0;
    const int n_kt = (SPLIT ? (int)((int64_t)all_kt * (blockIdx.z + 1) / gridDim.z) : all_kt) - kt_first; // this workgroup's K-tiles
    auto fetch = [&](int kt) { // its K-tile kt (clamped to the last one) -> buffer kt & 3
        const int ktc = kt_first + min(kt, n_kt - 1);
        uint8_t *dst = lds + (kt & (NBUF - 1)) * STAGE + wave * 16 * PROWB;
#pragma unroll
        for (int t = 0; t < NLOAD; ++t)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[t] + (int64_t)ktc * PROWB),
                                             (__attribute__((address_space(3))) void *)(dst + t * 8 * 16 * PROWB), 16, 0, 0);
    };
    fetch(0);
    fetch(1);
    fetch(2);
    __builtin_amdgcn_s_waitcnt(WAIT_LANDED);
    __syncthreads();

    constexpr int GROUPS = 2 * MI, ROT = 5, RING = 4, AHEAD = 3;
    static_assert(MI % RING == 0 && ROT == 2 * AHEAD - 1 && ROT < GROUPS && NJ % 2 == 0, "group plan");
    v4u ap[RING], wp[NJ];
    v4i fa[2], fw[2][NJ];
#pragma unroll
    for (int k = 0; k < RING; ++k) ap[k] = v4u{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < NJ; ++j) fw[0][j] = fw[1][j] = v4i{0, 0, 0, 0};
    fa[0] = fa[1] = v4i{0, 0, 0, 0};

    for (int kt = 0; kt < n_kt; ++kt) {
        const uint8_t *cur = lds + (kt & (NBUF - 1)) * STAGE;
#pragma unroll
        for (int u = 0; u < GROUPS; ++u) {
            const int s = (u + GROUPS - ROT) % GROUPS, i = s >> 1, m = s & 1;
            // the K-tile three ahead, into the buffer whose last reader passed the previous barrier
            if (s == 0) fetch(kt + 3);
            // the group's operations
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[m][j], fa[m], acc[i][j], 0, 0, 0);
            // splits for the next group: the other nibble of this row block, or the next block's low one
            if (m == 0) fa[1] = nib_hi(ap[i % RING]);
            else fa[0] = nib_lo(ap[(i + 1) % RING]);
            // feature side of the new K-tile: low nibbles once the last low group of the old one is
            // through (the last but one), high nibbles after its last high group (the last)
            if (s == GROUPS - 1) {
#pragma unroll
                for (int j = 0; j < NJ; ++j) fw[0][j] = nib_lo(wp[j]);
            }
            if (s == 0) {
#pragma unroll
                for (int j = 0; j < NJ; ++j) fw[1][j] = nib_hi(wp[j]);
            }
            if (u == GROUPS - 1) {
                // next K-tile landed (this wave's share; the barrier adds the others'), own reads done
                __builtin_amdgcn_s_waitcnt(WAIT_LANDED_LGKM0);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            // requests come after the split that had to wait for an earlier one, so that the wait
            // does not cover them: token rows three blocks ahead (after a high-nibble group), the
            // feature rows of this iteration's K-tile in its first two groups.  All of them read
            // this iteration's K-tile: the first group of the iteration is the first to look ahead.
            __builtin_amdgcn_sched_barrier(0);
            if (m == 1) ap[(i + AHEAD) % RING] = *reinterpret_cast<const v4u *>(cur + a_off + ((i + AHEAD) % MI) * 16 * PROWB);
            if (u < 2) {
#pragma unroll
                for (int h = 0; h < NJ / 2; ++h)
                    wp[(NJ / 2) * u + h] = *reinterpret_cast<const v4u *>(cur + w_off + ((NJ / 2) * u + h) * 16 * PROWB);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // the loads past the last K-tile went to buffers nobody reads; they must not outlive the workgroup
    __builtin_amdgcn_s_waitcnt(WAIT_VM0);
    // the last groups of the last K-tile
#pragma unroll
    for (int s = GROUPS - ROT; s < GROUPS; ++s) {
        const int i = s >> 1, m = s & 1;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw[m][j], fa[m], acc[i][j], 0, 0, 0);
        if (m == 0) fa[1] = nib_hi(ap[i % RING]);
        else if (i < MI - 1) fa[0] = nib_lo(ap[(i + 1) % RING]);
    }

    if constexpr (SPLIT) {
        // raw accumulators of this part of K: token n, four consecutive features per lane and tile
        int32_t *part = g.partial + (int64_t)blockIdx.z * g.N * g.O;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int n = n0 + wm * 16 * MI + i * 16 + (lane & 15);
            if (n >= g.N) continue;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int o = o0 + wn * 16 * NJ + j * 16 + 4 * (lane >> 4);
                int32_t *p = part + (int64_t)n * g.O + o;
                if (o + 3 < g.O && (g.O & 3) == 0) {
                    *reinterpret_cast<v4i *>(p) = acc[i][j];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (o + e < g.O) p[e] = acc[i][j][e];
                }
            }
        }
    } else {
        finish_wave_tile<4, 4, YT, MI, NJ>(g, acc, n0 + wm * 16 * MI, o0 + wn * 16 * NJ, lane);
    }
}

// ---- 4-bit codes on both sides on the FP6 matrix cores.
// gfx950 multiplies 6-bit floating-point operands (E2M3: sign, 2 exponent bits, 3 mantissa bits, no
// infinities or NaNs) at twice the rate of int8, 128 values of K per operation.  The 6-bit pattern
// 00cccc, a 4-bit code c zero-extended, IS the E2M3 number c / 8 (exponent field 0: c / 8 for c < 8;
// exponent field 1: (8 + (c - 8)) / 8), so the product of two codes is a * w / 64 exactly, and the
// fp32 accumulation is exact as well: every partial sum, whatever the order and grouping the hardware
// adds in, is a multiple of 1/64 below 225 K / 64 < 2^24 / 64 (K < 74565; the entry point allows
// 32768), hence a representable fp32 number, so no addition ever rounds.  64 acc is the int32
// accumulator of Eq. (1), bit for bit.
//
// TILES6, the operand format (made once per weight by qllm_pack_tiles6, per call for the activations):
// rows in blocks of 16, K in tiles of 128 codes; block b, K-tile t is the 1536 bytes at
// (b * tiles + t) * 1536 and holds what the 64 lanes of one operand read need, lane l = 16 q + r having
// row 16 b + r and codes 128 t + 32 q + e, e = 0..31, code e in bits 6 e .. 6 e + 3 of a 192-bit
// little-endian number: its first 16 bytes at 16 l, its last 8 at 1024 + 8 l.  Rows past the matrix
// are zero codes.  A stage of LDS is such blocks one after the other exactly as they lie in memory,
// so the refill is a plain copy (16-byte loads that write LDS directly) and both operand reads
// (ds_read_b128 of 1 KB, ds_read_b64 of 512 bytes per wave) are contiguous: no bank conflicts, and no
// vector instruction between LDS and the matrix cores.
//
// Same tiling as the int8 kernel above (2 x 4 waves, MI x NJ operations of 16 x 16 per wave and
// K-tile), a ring of three stages (48 KB each for the 256 x 256 tile), fetches two K-tiles ahead.
// One K-tile = MI groups of NJ operations (group i: token rows 16 i ..); token-side operands are
// requested AHEAD groups before their use into a ring of four, the feature side at the start of the
// iteration into the register set the previous K-tile does not use; the loop is rotated by AHEAD
// groups (an iteration starts with the last groups of the K-tile before, zeros the first time), and
// unrolled by two so that the alternation of the feature-side register sets is static.
typedef int v8i __attribute__((ext_vector_type(8)));
constexpr int T6_BLOCK = 1536, T6_X = 1024, T6_KT = 128, T6_STAGES = 3;

typedef int v2i __attribute__((ext_vector_type(2)));
struct Frag6 {
    v4i x;
    v2i y;
};
__device__ __forceinline__ v8i operand6(const Frag6 &f) { return v8i{f.x[0], f.x[1], f.x[2], f.x[3], f.y[0], f.y[1], 0, 0}; }
__device__ __forceinline__ Frag6 read6(const uint8_t *block, int lane)
{
    Frag6 f;
    f.x = *reinterpret_cast<const v4i *>(block + 16 * lane);
    f.y = *reinterpret_cast<const v2i *>(block + T6_X + 8 * lane);
    return f;
}

// SPLIT: K is dealt out to gridDim.z workgroups per tile of Y, as in int_gemm_w4a4_kernel; the parts' sums leave as
// the integers they stand for.
template <typename YT, int MI, int NJ, bool SPLIT = false>
__global__ __launch_bounds__(LTHREADS, MI == 8 ? 1 : 2) void gemm_w4a4_fp6_kernel(const GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int TM = 2 * MI * 16, TN = 4 * NJ * 16;
    constexpr int BLOCKS = (TM + TN) / 16, STAGE = BLOCKS * T6_BLOCK, NLOAD = STAGE / (8 * 1024);
    static_assert(STAGE % (8 * 1024) == 0, "a stage is a whole number of 1 KB loads per wave");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int n0 = blockIdx.y * TM, o0 = g.o_first + blockIdx.x * TN;
    const int all_kt = g.Kpad / T6_KT;
    const int a_blocks = (g.N + 15) / 16, w_blocks = (g.O + 15) / 16;

    // fetch assignment: load t of wave w fills bytes 1024 (NLOAD w + t) .. of the stage, lane l its l-th 16.  The
    // token side of a stage is a whole number of such loads, so a load is all token side or all feature side: one
    // base for the wave, a 32-bit offset per lane that never changes (the K-tile moves the base).
    uint32_t src_off[NLOAD];
#pragma unroll
    for (int t = 0; t < NLOAD; ++t) {
        const int off = (wave * NLOAD + t) * 1024 + lane * 16, blk = off / T6_BLOCK, within = off % T6_BLOCK;
        const bool token = blk < TM / 16; // past the edge: the last block again (its results are not stored)
        const int rb = token ? min(n0 / 16 + blk, a_blocks - 1) : min(o0 / 16 + blk - TM / 16, w_blocks - 1);
        src_off[t] = (uint32_t)rb * (uint32_t)all_kt * T6_BLOCK + within;
    }
    static_assert((TM / 16 * T6_BLOCK) % 1024 == 0, "token side = whole loads");
    // load t of K-tile kt (clamped to the last one) -> that stage of the ring
    auto fetch_one = [&](int kt, int stage, int t) {
        const int ktc = min(kt, all_kt - 1);
        const bool token = (wave * NLOAD + t) * 1024 < TM / 16 * T6_BLOCK;
        const uint8_t *base = (token ? g.a_tiles : g.w_tiles) + (int64_t)ktc * T6_BLOCK;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + src_off[t]),
                                         (__attribute__((address_space(3))) void *)(lds + stage * STAGE + (wave * NLOAD + t) * 1024), 16, 0,
                                         0);
    };
    auto fetch = [&](int kt, int stage) {
#pragma unroll
        for (int t = 0; t < NLOAD; ++t) fetch_one(kt, stage, t);
    };
    constexpr int WAIT_LANDED = NLOAD | (7 << 4) | (15 << 8);       // s_waitcnt vmcnt(NLOAD): all but the newest fetch
    constexpr int WAIT_LANDED_LGKM0 = NLOAD | (7 << 4) | (0 << 8);  // ... and lgkmcnt(0)

    v4f acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    // this workgroup's K-tiles (fetches past them, up to the last K-tile of the row, go to stages nobody reads)
    const int kt_first = SPLIT ? (int)((int64_t)all_kt * blockIdx.z / gridDim.z) : 0;
    const int kt_end = SPLIT ? (int)((int64_t)all_kt * (blockIdx.z + 1) / gridDim.z) : all_kt;
    fetch(kt_first, 0);
    fetch(kt_first + 1, 1);
    __builtin_amdgcn_s_waitcnt(WAIT_LANDED);
    __syncthreads();

    // Token-side operands: all MI blocks of a K-tile have registers of their own; the large tile requests them two
    // per group in the first MI / 2 groups of the iteration, so that the wait for "own reads done" before the
    // barrier finds them long back.
    constexpr int RING = MI, AHEAD = 2, PER_STEP = MI == 8 ? 2 : 1;
    // block b is requested in step b / PER_STEP, after the group of the K-tile before that used its registers (step b + AHEAD - MI)
    static_assert(MI % PER_STEP == 0 && (MI - 1) / PER_STEP > AHEAD - 1 && (MI - AHEAD) / PER_STEP > 0, "group plan");
    Frag6 ar[RING], wr[2][NJ];
#pragma unroll
    for (int k = 0; k < RING; ++k) ar[k] = Frag6{v4i{0, 0, 0, 0}, v2i{0, 0}};
#pragma unroll
    for (int j = 0; j < NJ; ++j) wr[0][j] = wr[1][j] = Frag6{v4i{0, 0, 0, 0}, v2i{0, 0}};

    const int a_blk0 = wm * MI, w_blk0 = TM / 16 + wn * NJ; // the wave's first token-side and feature-side block of a stage
    int stage = 0, fetch_stage = 2;
    // one K-tile, P = which feature-side register set it reads into (the other one still serves the
    // AHEAD groups left of the K-tile before)
    auto k_tile = [&](auto parity, int kt) {
        constexpr int P = decltype(parity)::value;
        const uint8_t *cur = lds + stage * STAGE;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            wr[P][j] = read6(cur + (w_blk0 + j) * T6_BLOCK, lane);
            __builtin_amdgcn_sched_barrier(0); // also keeps the 8-byte reads of neighbouring blocks from being merged
        }
#pragma unroll
        for (int u = 0; u < MI; ++u) {
            const bool old = u < AHEAD;
            const int i = old ? MI - AHEAD + u : u - AHEAD;
            // The K-tile two ahead, into the stage whose last reader passed the previous barrier: one load per group,
            // not all at once (the eight waves' loads of a K-tile keep the CU's address unit busy for three quarters of
            // a K-tile's matrix-core time; a wave whose load is not accepted yet issues nothing else either).
            if (u < NLOAD) fetch_one(kt + 2, fetch_stage, u);
            if (PER_STEP * u < MI) {
#pragma unroll
                for (int h = 0; h < PER_STEP; ++h) {
                    ar[PER_STEP * u + h] = read6(cur + (a_blk0 + PER_STEP * u + h) * T6_BLOCK, lane);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(operand6(wr[old ? 1 - P : P][j]), operand6(ar[i]),
                                                                             acc[i][j], 2, 2, 0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the next K-tile has landed (this wave's share; the barrier adds the others'), own reads done
        __builtin_amdgcn_s_waitcnt(WAIT_LANDED_LGKM0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        fetch_stage = stage;
        stage = stage == T6_STAGES - 1 ? 0 : stage + 1;
    };
    int kt = kt_first;
    for (; kt + 1 < kt_end; kt += 2) {
        k_tile(std::integral_constant<int, 0>{}, kt);
        k_tile(std::integral_constant<int, 1>{}, kt + 1);
    }
    if (kt < kt_end) k_tile(std::integral_constant<int, 0>{}, kt);
    // the loads past the last K-tile went to stages nobody reads; they must not outlive the workgroup
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
    // the last groups of the last K-tile
    auto last_groups = [&](auto parity) {
        constexpr int P = decltype(parity)::value;
#pragma unroll
        for (int i = MI - AHEAD; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(operand6(wr[P][j]), operand6(ar[i]), acc[i][j], 2, 2,
                                                                             0, 0, 0, 0);
    };
    if ((kt_end - kt_first) & 1) last_groups(std::integral_constant<int, 0>{});
    else last_groups(std::integral_constant<int, 1>{});

    if constexpr (SPLIT) {
        // this part's sums as integers (64 acc, exactly): token n, four consecutive features per lane and tile
        int32_t *part = g.partial + (int64_t)blockIdx.z * g.N * g.O;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int n = n0 + wm * 16 * MI + i * 16 + (lane & 15);
            if (n >= g.N) continue;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int o = o0 + wn * 16 * NJ + j * 16 + 4 * (lane >> 4);
                int32_t *p = part + (int64_t)n * g.O + o;
                const v4i v{acc_int(acc[i][j], 0), acc_int(acc[i][j], 1), acc_int(acc[i][j], 2), acc_int(acc[i][j], 3)};
                if (o + 3 < g.O && (g.O & 3) == 0) {
                    *reinterpret_cast<v4i *>(p) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (o + e < g.O) p[e] = v[e];
                }
            }
        }
    } else {
        finish_wave_tile<4, 4, YT, MI, NJ>(g, acc, n0 + wm * 16 * MI, o0 + wn * 16 * NJ, lane); // 64 acc: the integer accumulators, exactly
    }
}

// 4 nibbles in bits 0..15 -> four 6-bit fields in bits 0..23
__device__ __forceinline__ uint32_t spread4(uint32_t x)
{
    const uint32_t y = (x & 0xffu) | ((x & 0xff00u) << 4); // nibbles 0, 1 in bits 0..7; 2, 3 in bits 12..19
    return (y & 0x00f00fu) | ((y & 0x0f00f0u) << 2);       // nibble k in bits 6 k .. 6 k + 3
}

// Packed 4-bit rows -> TILES6; one lane per (block, K-tile, lane of the operand read).
__global__ __launch_bounds__(256) void tiles6_kernel(const uint8_t *codes, int64_t row_bytes, int32_t rows, int32_t n_kt,
                                                    uint8_t *tiles, int64_t n_items)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_items) return;
    const int l = (int)(idx & 63), r = l & 15, q = l >> 4;
    const int64_t bk = idx >> 6, b = bk / n_kt;
    const int kt = (int)(bk - b * n_kt);
    const int64_t row = b * 16 + r;
    uint4 p = make_uint4(0u, 0u, 0u, 0u);
    if (row < rows) p = *reinterpret_cast<const uint4 *>(codes + row * row_bytes + kt * (T6_KT / 2) + q * 16);
    const uint32_t w[4] = {p.x, p.y, p.z, p.w};
    uint32_t s[8]; // eight pieces of 24 bits
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s[2 * i] = spread4(w[i] & 0xffffu);
        s[2 * i + 1] = spread4(w[i] >> 16);
    }
    uint8_t *blk = tiles + bk * T6_BLOCK;
    *reinterpret_cast<uint4 *>(blk + 16 * l) =
        make_uint4(s[0] | (s[1] << 24), (s[1] >> 8) | (s[2] << 16), (s[2] >> 16) | (s[3] << 8), s[4] | (s[5] << 24));
    *reinterpret_cast<uint2 *>(blk + T6_X + 8 * l) = make_uint2((s[5] >> 8) | (s[6] << 16), (s[6] >> 16) | (s[7] << 8));
}

// ---- 6- and 8-bit codes (and 8-bit activations on 4-bit weights) straight from LDS into the int8 matrix cores.
// TILES8, the operand format (made once per weight by qllm_pack_tiles8, per call for the activations): one byte
// per code, rows in blocks of 16, K in tiles of 64 codes; block b, K-tile t is the 1024 bytes at
// (b * tiles + t) * 1024 and holds what the 64 lanes of one operand read need: lane l = 16 q + r has row
// 16 b + r and codes 64 t + 16 q + e, e = 0..15, at byte 16 l + e.  A 4- or 6-bit code is its own value; an 8-bit
// code c is stored as c ^ 0x80, the signed byte c - 128 (the epilogue adds the difference back).  Rows past the
// matrix and places past K are zero bytes: they add nothing.  As with TILES6 a stage of LDS is such blocks as
// they lie in memory, the refill a plain copy by 16-byte loads that write LDS directly, an operand read one
// contiguous ds_read_b128 per wave, and there is no vector instruction between LDS and the matrix cores (the
// kernels that expand packed codes at refill time spend most of their issue slots on that).
// Tiling, ring, group plan and loop rotation are those of gemm_w4a4_fp6_kernel; one K-tile here is 64 codes,
// which takes the int8 matrix cores as long as 128 codes take the FP6 ones.
constexpr int T8_BLOCK = 1024, T8_KT = 64, T8_STAGES = 3;

// SPLIT: K is dealt out to gridDim.z workgroups per tile of Y (so few tiles that most CUs would idle); each writes
// its raw accumulators to g.partial and splitk_finish_kernel adds them up and does the epilogue.
template <int ABITS, int WBITS, typename YT, int MI, int NJ, bool SPLIT = false>
__global__ __launch_bounds__(LTHREADS, MI == 8 ? 1 : 2) void gemm_tiles8_kernel(const GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int TM = 2 * MI * 16, TN = 4 * NJ * 16;
    constexpr int BLOCKS = (TM + TN) / 16, STAGE = BLOCKS * T8_BLOCK, NLOAD = STAGE / (8 * 1024);
    static_assert(STAGE % (8 * 1024) == 0 && NLOAD <= MI, "a stage is a whole number of 1 KB loads per wave, one per group");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int n0 = blockIdx.y * TM, o0 = g.o_first + blockIdx.x * TN;
    const int all_kt = (g.K + T8_KT - 1) / T8_KT;
    const int a_blocks = (g.N + 15) / 16, w_blocks = (g.O + 15) / 16;

    // fetch assignment: load t of wave w fills block NLOAD w + t of the stage, lane l its l-th 16 bytes; a load is
    // all token side or all feature side: one base for the wave, a 32-bit offset per lane that never changes
    uint32_t src_off[NLOAD];
#pragma unroll
    for (int t = 0; t < NLOAD; ++t) {
        const int blk = wave * NLOAD + t;
        const bool token = blk < TM / 16; // past the edge: the last block again (its results are not stored)
        const int rb = token ? min(n0 / 16 + blk, a_blocks - 1) : min(o0 / 16 + blk - TM / 16, w_blocks - 1);
        src_off[t] = (uint32_t)rb * (uint32_t)all_kt * T8_BLOCK + lane * 16;
    }
    auto fetch_one = [&](int kt, int stage, int t) { // load t of K-tile kt (clamped to the last one) -> that stage
        const int ktc = min(kt, all_kt - 1);
        const bool token = wave * NLOAD + t < TM / 16;
        const uint8_t *base = (token ? g.a_tiles8 : g.w_tiles8) + (int64_t)ktc * T8_BLOCK;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + src_off[t]),
                                         (__attribute__((address_space(3))) void *)(lds + stage * STAGE + (wave * NLOAD + t) * 1024), 16, 0,
                                         0);
    };
    auto fetch = [&](int kt, int stage) {
#pragma unroll
        for (int t = 0; t < NLOAD; ++t) fetch_one(kt, stage, t);
    };
    constexpr int WAIT_LANDED = NLOAD | (7 << 4) | (15 << 8);       // s_waitcnt vmcnt(NLOAD): all but the newest fetch
    constexpr int WAIT_LANDED_LGKM0 = NLOAD | (7 << 4) | (0 << 8);  // ... and lgkmcnt(0)

    v4i acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    // this workgroup's K-tiles (fetches past them, up to the last K-tile of the row, go to stages nobody reads)
    const int kt_first = SPLIT ? (int)((int64_t)all_kt * blockIdx.z / gridDim.z) : 0;
    const int kt_end = SPLIT ? (int)((int64_t)all_kt * (blockIdx.z + 1) / gridDim.z) : all_kt;
    fetch(kt_first, 0);
    fetch(kt_first + 1, 1);
    __builtin_amdgcn_s_waitcnt(WAIT_LANDED);
    __syncthreads();

    constexpr int RING = MI, AHEAD = 2, PER_STEP = MI == 8 ? 2 : 1;
    static_assert(MI % PER_STEP == 0 && (MI - 1) / PER_STEP > AHEAD - 1 && (MI - AHEAD) / PER_STEP > 0, "group plan");
    v4i ar[RING], wr[2][NJ];
#pragma unroll
    for (int k = 0; k < RING; ++k) ar[k] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < NJ; ++j) wr[0][j] = wr[1][j] = v4i{0, 0, 0, 0};

    const int a_blk0 = wm * MI, w_blk0 = TM / 16 + wn * NJ; // the wave's first token-side and feature-side block of a stage
    int stage = 0, fetch_stage = 2;
    auto k_tile = [&](auto parity, int kt) {
        constexpr int P = decltype(parity)::value;
        const uint8_t *cur = lds + stage * STAGE;
#pragma unroll
        for (int j = 0; j < NJ; ++j) wr[P][j] = *reinterpret_cast<const v4i *>(cur + (w_blk0 + j) * T8_BLOCK + 16 * lane);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < MI; ++u) {
            const bool old = u < AHEAD;
            const int i = old ? MI - AHEAD + u : u - AHEAD;
            if (u < NLOAD) fetch_one(kt + 2, fetch_stage, u); // one load per group, not all at once
            if (PER_STEP * u < MI) {
#pragma unroll
                for (int h = 0; h < PER_STEP; ++h)
                    ar[PER_STEP * u + h] = *reinterpret_cast<const v4i *>(cur + (a_blk0 + PER_STEP * u + h) * T8_BLOCK + 16 * lane);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wr[old ? 1 - P : P][j], ar[i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the next K-tile has landed (this wave's share; the barrier adds the others'), own reads done
        __builtin_amdgcn_s_waitcnt(WAIT_LANDED_LGKM0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        fetch_stage = stage;
        stage = stage == T8_STAGES - 1 ? 0 : stage + 1;
    };
    int kt = kt_first;
    for (; kt + 1 < kt_end; kt += 2) {
        k_tile(std::integral_constant<int, 0>{}, kt);
        k_tile(std::integral_constant<int, 1>{}, kt + 1);
    }
    if (kt < kt_end) k_tile(std::integral_constant<int, 0>{}, kt);
    // the loads past the last K-tile went to stages nobody reads; they must not outlive the workgroup
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
    auto last_groups = [&](auto parity) { // the last groups of the last K-tile
        constexpr int P = decltype(parity)::value;
#pragma unroll
        for (int i = MI - AHEAD; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wr[P][j], ar[i], acc[i][j], 0, 0, 0);
    };
    if ((kt_end - kt_first) & 1) last_groups(std::integral_constant<int, 0>{});
    else last_groups(std::integral_constant<int, 1>{});

    if constexpr (SPLIT) {
        // raw accumulators of this part of K: token n, four consecutive features per lane and tile
        int32_t *part = g.partial + (int64_t)blockIdx.z * g.N * g.O;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int n = n0 + wm * 16 * MI + i * 16 + (lane & 15);
            if (n >= g.N) continue;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int o = o0 + wn * 16 * NJ + j * 16 + 4 * (lane >> 4);
                int32_t *p = part + (int64_t)n * g.O + o;
                if (o + 3 < g.O && (g.O & 3) == 0) {
                    *reinterpret_cast<v4i *>(p) = acc[i][j];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (o + e < g.O) p[e] = acc[i][j][e];
                }
            }
        }
    } else {
        // places past K are zero bytes on both sides, so only the K real places carry the two offsets of 128
        finish_wave_tile<ABITS, WBITS, YT, MI, NJ>(g, acc, n0 + wm * 16 * MI, o0 + wn * 16 * NJ, lane, g.K);
    }
}

// Packed rows -> TILES8; one lane per (block, K-tile, lane of the operand read): 16 codes of one row.
template <int BITS>
__global__ __launch_bounds__(256) void tiles8_kernel(const uint8_t *codes, int64_t row_bytes, int32_t rows, int32_t K, int32_t n_kt,
                                                    uint8_t *tiles, int64_t n_items)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_items) return;
    const int l = (int)(idx & 63), r = l & 15, q = l >> 4;
    const int64_t bk = idx >> 6, b = bk / n_kt;
    const int kt = (int)(bk - b * n_kt);
    const int64_t row = b * 16 + r;
    const int k0 = kt * T8_KT + 16 * q; // the lane's first code
    uint32_t d[4] = {0u, 0u, 0u, 0u};
    if (row < rows && k0 < K) {
        // the lane's 2 * BITS bytes of the packed row, dword by dword; what lies past the row's end reads as zero codes
        const int64_t at = (int64_t)k0 * BITS / 8; // a multiple of 4
        const uint8_t *src = codes + row * row_bytes + at;
        uint32_t w[BITS / 2];
#pragma unroll
        for (int i = 0; i < BITS / 2; ++i) w[i] = at + 4 * i < row_bytes ? reinterpret_cast<const uint32_t *>(src)[i] : 0u;
        if constexpr (BITS == 4) {
            expand4(w[0], d[0], d[1]);
            expand4(w[1], d[2], d[3]);
        } else if constexpr (BITS == 6) {
            d[0] = spread6(w[0]);
            d[1] = spread6(__builtin_amdgcn_alignbit(w[1], w[0], 24));
            d[2] = spread6(__builtin_amdgcn_alignbit(w[2], w[1], 16));
            d[3] = spread6(w[2] >> 8);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // code - 128 as a signed byte, in the places that hold a code
                const int left = K - (k0 + 4 * i);
                const uint32_t live = left >= 4 ? 0xffffffffu : left <= 0 ? 0u : (1u << (8 * left)) - 1u;
                d[i] = (w[i] ^ 0x80808080u) & live;
            }
        }
    }
    *reinterpret_cast<uint4 *>(tiles + bk * T8_BLOCK + 16 * l) = make_uint4(d[0], d[1], d[2], d[3]);
}

// Sum of the parts of a split K and the dequantising epilogue, one output per lane; the bracket in 64-bit
// arithmetic, which gives the same float as the narrow form.  SA / SW: that side's codes are 8-bit and went into
// the matrix cores as code - 128 in every one of the K places (the byte-operand path), which is added back here.
template <typename YT, int SA = 0, int SW = 0>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const GemmArgs g)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)g.N * g.O) return;
    const int n = (int)(idx / g.O), o = (int)(idx % g.O);
    int32_t raw = 0; // the true accumulator fits int32 (checked by the launcher), so wrapping sums are exact
    for (int z = 0; z < g.splits; ++z) raw += g.partial[(int64_t)z * g.N * g.O + idx];
    raw += 128 * SW * g.rs[n] + 128 * SA * g.cs[o] - 16384 * SA * SW * g.K;
    const int64_t bx = g.bx[n], bw = g.bw[o];
    const int64_t t = (int64_t)raw - bx * g.cs[o] - bw * g.rs[n] + (int64_t)g.K * bx * bw;
    float v = (float)t;
    v = v * g.ax[n];
    v = v * g.aw[o];
    if constexpr (sizeof(YT) == 4) reinterpret_cast<float *>(g.y)[(int64_t)n * g.ldy + o] = v;
    else reinterpret_cast<uint16_t *>(g.y)[(int64_t)n * g.ldy + o] = f32_to_bf16_rne(v);
    if (g.acc_dump) g.acc_dump[idx] = raw;
}

// ---- few tokens (decode): the weights are read once from HBM and that is the whole cost.  A
// workgroup owns 32 output features (two matrix-core row tiles) and all N <= 16 NT tokens (NT 1 or 2);
// its 8 waves split K: wave w takes the 256-code steps w, w + 8, ... and works on its own, without
// barriers, until the partial tiles are added up at the end.
//   * Global loads are laid out for the memory pipeline, not for the matrix cores: consecutive lanes
//     take consecutive 16-byte pieces of a row's 256 codes, so one load instruction touches whole
//     cache lines (a lane per matrix-core operand row would touch three to four times as many lines,
//     and the address unit, one line per cycle, would be the limit).  Two steps' loads are in flight.
//   * The pieces pass through a wave-private strip of LDS, still packed, and come back as the 64 codes
//     256 s + 64 c .. + 63 of row r for lane (r, c), are expanded in registers and feed four
//     matrix-core operations, the m-th on codes 16 m .. 16 m + 15 of every lane's 64: which 64 codes
//     of the step one operation sums is free as long as both operands agree.
constexpr int SK_THREADS = 512, SK_WAVES = 8, SK_RT = 2, SK_STEP = 256;

template <int BITS>
constexpr int SK_ROW = SK_STEP * BITS / 8 + 16; // bytes of LDS per row and step: the packed codes and a pad against bank conflicts

template <int ABITS, int WBITS, int NT>
constexpr int SK_STRIP = 16 * SK_RT * SK_ROW<WBITS> + 16 * NT * SK_ROW<ABITS>; // LDS bytes per wave

template <int ABITS, int WBITS, typename YT, int NT>
__global__ __launch_bounds__(SK_THREADS) void int_gemm_skinny_kernel(const GemmArgs g)
{
    // [SK_WAVES] strips; afterwards reused as [SK_WAVES][NT * SK_RT][64] v4i for the final sum
    extern __shared__ __align__(16) uint8_t sk_lds[];
    constexpr bool PERM = ABITS == 4 && WBITS == 4;
    constexpr int WPIECES = SK_STEP * WBITS / 8 / 16, APIECES = SK_STEP * ABITS / 8 / 16; // 16-byte pieces per row and step
    constexpr int WLOADS = 16 * SK_RT * WPIECES / 64, ALOADS = 16 * NT * APIECES / 64;     // load instructions per step
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, c = lane >> 4;
    const int o0 = blockIdx.x * (16 * SK_RT);
    uint8_t *w_strip = sk_lds + wave * SK_STRIP<ABITS, WBITS, NT>, *a_strip = w_strip + 16 * SK_RT * SK_ROW<WBITS>;

    // piece lane + 64 t of a step: where it comes from (without the step's offset) and where it goes
    const uint8_t *w_src[WLOADS], *a_src[ALOADS];
    int w_dst[WLOADS], a_dst[ALOADS];
#pragma unroll
    for (int t = 0; t < WLOADS; ++t) {
        const int q = lane + 64 * t, row = q / WPIECES, piece = q % WPIECES;
        w_src[t] = g.w_codes + (int64_t)min(o0 + row, g.O - 1) * g.w_row_bytes + 16 * piece;
        w_dst[t] = row * SK_ROW<WBITS> + 16 * piece;
    }
#pragma unroll
    for (int t = 0; t < ALOADS; ++t) {
        const int q = lane + 64 * t, row = q / APIECES, piece = q % APIECES;
        a_src[t] = g.a_codes + (int64_t)min(row, g.N - 1) * g.a_row_bytes + 16 * piece;
        a_dst[t] = row * SK_ROW<ABITS> + 16 * piece;
    }

    v4i acc[NT][SK_RT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < SK_RT; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    v4i w0[WLOADS], a0[ALOADS], w1[WLOADS], a1[ALOADS]; // two register stages
    auto fetch = [&](v4i (&tw)[WLOADS], v4i (&ta)[ALOADS], int s) {
#pragma unroll
        for (int k = 0; k < WLOADS; ++k) tw[k] = *reinterpret_cast<const v4i *>(w_src[k] + (int64_t)s * (SK_STEP * WBITS / 8));
#pragma unroll
        for (int k = 0; k < ALOADS; ++k) ta[k] = *reinterpret_cast<const v4i *>(a_src[k] + (int64_t)s * (SK_STEP * ABITS / 8));
    };
    auto work = [&](const v4i (&tw)[WLOADS], const v4i (&ta)[ALOADS]) {
        // a wave's LDS operations complete in order: these writes follow the previous step's reads
#pragma unroll
        for (int k = 0; k < WLOADS; ++k) *reinterpret_cast<v4i *>(w_strip + w_dst[k]) = tw[k];
#pragma unroll
        for (int k = 0; k < ALOADS; ++k) *reinterpret_cast<v4i *>(a_strip + a_dst[k]) = ta[k];
        uint32_t da[NT][16];
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            Unit<ABITS> u;
            const uint4 *p = reinterpret_cast<const uint4 *>(a_strip + (16 * i + r) * SK_ROW<ABITS> + c * (SK_STEP * ABITS / 8 / 4));
#pragma unroll
            for (int k = 0; k < ABITS / 2; ++k) u.r[k] = p[k];
            expand_unit<ABITS, PERM>(u, da[i]);
        }
#pragma unroll
        for (int j = 0; j < SK_RT; ++j) {
            Unit<WBITS> u;
            const uint4 *p = reinterpret_cast<const uint4 *>(w_strip + (16 * j + r) * SK_ROW<WBITS> + c * (SK_STEP * WBITS / 8 / 4));
#pragma unroll
            for (int k = 0; k < WBITS / 2; ++k) u.r[k] = p[k];
            uint32_t dw[16];
            expand_unit<WBITS, PERM>(u, dw);
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int i = 0; i < NT; ++i) {
                    const v4i fw = {(int)dw[4 * m], (int)dw[4 * m + 1], (int)dw[4 * m + 2], (int)dw[4 * m + 3]};
                    const v4i fa = {(int)da[i][4 * m], (int)da[i][4 * m + 1], (int)da[i][4 * m + 2], (int)da[i][4 * m + 3]};
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fw, fa, acc[i][j], 0, 0, 0);
                }
        }
    };

    // Every fetch is unconditional (past the end a wave re-reads its first step, from cache), so that
    // the number of loads in flight at each wait is known when the code is compiled.
    const int n_steps = g.Kpad / SK_STEP; // rows are padded to a multiple of 256 codes
    int s = wave;
    if (s < n_steps) {
        fetch(w0, a0, s);
        fetch(w1, a1, s + SK_WAVES < n_steps ? s + SK_WAVES : wave);
        while (true) { // two steps per turn: the register stages alternate without being indexed
            work(w0, a0);
            fetch(w0, a0, s + 2 * SK_WAVES < n_steps ? s + 2 * SK_WAVES : wave);
            s += SK_WAVES;
            if (s >= n_steps) break;
            work(w1, a1);
            fetch(w1, a1, s + 2 * SK_WAVES < n_steps ? s + 2 * SK_WAVES : wave);
            s += SK_WAVES;
            if (s >= n_steps) break;
        }
    }

    // ---- add the 8 partial tiles up; wave t finishes tile t
    __syncthreads(); // the strips are no longer read
    v4i *red = reinterpret_cast<v4i *>(sk_lds);
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < SK_RT; ++j) red[(wave * (NT * SK_RT) + i * SK_RT + j) * 64 + lane] = acc[i][j];
    __syncthreads();
    if (wave < NT * SK_RT) {
        v4i sum[1][1] = {{red[wave * 64 + lane]}};
#pragma unroll
        for (int w = 1; w < SK_WAVES; ++w) sum[0][0] += red[(w * (NT * SK_RT) + wave) * 64 + lane];
        finish_wave_tile<ABITS, WBITS, YT, 1, 1>(g, sum, 16 * (wave / SK_RT), o0 + 16 * (wave % SK_RT), lane);
    }
}

template <int ABITS, int WBITS>
constexpr size_t skinny_lds(int nt)
{
    const size_t strips = (size_t)SK_WAVES * (nt == 1 ? SK_STRIP<ABITS, WBITS, 1> : nt == 2 ? SK_STRIP<ABITS, WBITS, 2> : SK_STRIP<ABITS, WBITS, 4>);
    const size_t red = (size_t)SK_WAVES * nt * SK_RT * 64 * sizeof(v4i);
    return strips > red ? strips : red;
}

// kernels whose LDS limit has been raised (once each: every kernel here always asks for the same amount,
// and no runtime call then sits between a caller's stream capture and the launch)
std::mutex raised_lock;
std::vector<const void *> raised;

template <typename K>
int32_t launch_kernel(K kernel, dim3 grid, dim3 block, size_t lds, const GemmArgs &g, hipStream_t stream)
{
    if (lds > 48 * 1024) {
        const void *fn = reinterpret_cast<const void *>(kernel);
        std::lock_guard<std::mutex> hold(raised_lock);
        bool done = false;
        for (const void *k : raised) done = done || k == fn;
        if (!done) {
            const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                qllm_note_hip_error("int gemm: raising the LDS limit", hipGetErrorName(e));
                return QLLM_ERR_HIP;
            }
            raised.push_back(fn);
        }
    }
    (void)hipGetLastError(); // drop any stale error of the calling thread: only this launch is judged
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, g);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error("int gemm: launch", hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}

// How a product with 256 x 256 or 128 x 128 tiles is laid over the chip.  A round of 256 large tiles (one per CU)
// takes one unit of time, a round of 512 small ones (two per CU; half the outputs at about three quarters of the
// rate) 0.65.  Large tiles throughout, small tiles throughout, or -- when the large tiles fill whole rounds and
// leave a rest -- large tiles for the output features of the whole rounds and small tiles for the others, as two
// launches (7B q/k/v: 384 large tiles are two rounds, 1536 small ones three; 256 large + 512 small are 1.65).
struct TilePlan {
    bool small;      // 128 x 128 tiles for everything (or for everything from o_split on)
    int32_t o_split; // > 0: large tiles for features below o_split, small tiles from there on
};
TilePlan plan_tiles(int64_t N, int64_t O, bool may_split_launch)
{
    const int64_t nb = (N + LBM - 1) / LBM, ob = (O + LBN - 1) / LBN, big_tiles = nb * ob;
    const int64_t small_tiles = ((O + 127) / 128) * ((N + 127) / 128);
    const double cost_big = (double)((big_tiles + 255) / 256), cost_small = 0.65 * (double)((small_tiles + 511) / 512);
    if (N <= 128) return TilePlan{true, 0};
    TilePlan best{cost_small < cost_big, 0};
    double best_cost = cost_small < cost_big ? cost_small : cost_big;
    const int64_t whole = big_tiles / 256, ca = whole * 256 / nb; // feature blocks that whole rounds of large tiles cover
    if (may_split_launch && whole >= 1 && ca > 0 && ca < ob) {
        const int64_t rest_small = ((O - ca * LBN + 127) / 128) * ((N + 127) / 128);
        const double cost = (double)((ca * nb + 255) / 256) + 0.65 * (double)((rest_small + 511) / 512);
        if (cost < best_cost - 0.05) best = TilePlan{false, (int32_t)(ca * LBN)};
    }
    return best;
}

// Packed 4-bit rows (device) -> TILES6 (device).
int32_t launch_tiles6(const uint8_t *codes, int64_t row_bytes, int64_t rows, int64_t Kpad, uint8_t *tiles, hipStream_t stream)
{
    const int64_t n_kt = Kpad / T6_KT, n_items = (rows + 15) / 16 * n_kt * 64;
    (void)hipGetLastError();
    hipLaunchKernelGGL(tiles6_kernel, dim3((unsigned)((n_items + 255) / 256)), dim3(256), 0, stream, codes, row_bytes, (int32_t)rows,
                       (int32_t)n_kt, tiles, n_items);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error("tiles6: launch", hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}

// 4-bit codes on both sides, more than 32 tokens, on the FP6 matrix cores: the activations are re-laid
// into g.a_tiles first; then the same choice between 256 x 256 and 128 x 128 tiles as on the int8 path.
int32_t launch_fp6(const GemmArgs &g, int32_t y_dtype, hipStream_t stream)
{
    const int32_t st = launch_tiles6(g.a_codes, g.a_row_bytes, g.N, g.Kpad, const_cast<uint8_t *>(g.a_tiles), stream);
    if (st != QLLM_OK) return st;
    const TilePlan plan = plan_tiles(g.N, g.O, g.splits == 1 && !g.acc_dump);
    auto launch_small = [&](const GemmArgs &ga) -> int32_t {
        const dim3 grid((unsigned)((ga.O - ga.o_first + 127) / 128), (unsigned)((ga.N + 127) / 128), (unsigned)(ga.splits > 1 ? ga.splits : 1));
        constexpr size_t lds = (size_t)T6_STAGES * 16 * T6_BLOCK;
        if (ga.splits > 1) {
            const int32_t sp = launch_kernel(gemm_w4a4_fp6_kernel<float, 4, 2, true>, grid, dim3(LTHREADS), lds, ga, stream);
            if (sp != QLLM_OK) return sp;
            const dim3 fgrid((unsigned)(((int64_t)ga.N * ga.O + 255) / 256));
            if (y_dtype == QLLM_F32) return launch_kernel(splitk_finish_kernel<float>, fgrid, dim3(256), 0, ga, stream);
            return launch_kernel(splitk_finish_kernel<uint16_t>, fgrid, dim3(256), 0, ga, stream);
        }
        if (y_dtype == QLLM_F32) return launch_kernel(gemm_w4a4_fp6_kernel<float, 4, 2>, grid, dim3(LTHREADS), lds, ga, stream);
        return launch_kernel(gemm_w4a4_fp6_kernel<uint16_t, 4, 2>, grid, dim3(LTHREADS), lds, ga, stream);
    };
    auto launch_big = [&](const GemmArgs &ga) -> int32_t {
        const dim3 grid((unsigned)((ga.O - ga.o_first + LBN - 1) / LBN), (unsigned)((ga.N + LBM - 1) / LBM));
        constexpr size_t lds = (size_t)T6_STAGES * 32 * T6_BLOCK;
        if (y_dtype == QLLM_F32) return launch_kernel(gemm_w4a4_fp6_kernel<float, 8, 4>, grid, dim3(LTHREADS), lds, ga, stream);
        return launch_kernel(gemm_w4a4_fp6_kernel<uint16_t, 8, 4>, grid, dim3(LTHREADS), lds, ga, stream);
    };
    if (g.splits > 1) return launch_small(g); // K is only split where the small tile is the choice
    if (plan.o_split > 0) { // whole rounds of large tiles, then the other output features with small ones
        GemmArgs first = g, rest = g;
        first.O = plan.o_split;
        rest.o_first = plan.o_split;
        const int32_t rc = launch_big(first);
        return rc != QLLM_OK ? rc : launch_small(rest);
    }
    return plan.small ? launch_small(g) : launch_big(g);
}

// Packed rows (device) -> TILES8 (device).
int32_t launch_tiles8(const uint8_t *codes, int32_t bits, int64_t rows, int64_t K, uint8_t *tiles, hipStream_t stream)
{
    const int64_t n_kt = (K + T8_KT - 1) / T8_KT, n_items = (rows + 15) / 16 * n_kt * 64;
    const dim3 grid((unsigned)((n_items + 255) / 256));
    const int64_t row_bytes = qllm_packed_row_bytes(K, bits);
    (void)hipGetLastError();
    if (bits == 4) hipLaunchKernelGGL(tiles8_kernel<4>, grid, dim3(256), 0, stream, codes, row_bytes, (int32_t)rows, (int32_t)K, (int32_t)n_kt, tiles, n_items);
    else if (bits == 6) hipLaunchKernelGGL(tiles8_kernel<6>, grid, dim3(256), 0, stream, codes, row_bytes, (int32_t)rows, (int32_t)K, (int32_t)n_kt, tiles, n_items);
    else hipLaunchKernelGGL(tiles8_kernel<8>, grid, dim3(256), 0, stream, codes, row_bytes, (int32_t)rows, (int32_t)K, (int32_t)n_kt, tiles, n_items);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error("tiles8: launch", hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}

// The byte-operand path's tile where K may be split: 128 x 128 (two workgroups per CU) where that is the plan
// for the whole product, as on the FP6 path, and for up to 128 tokens.
bool t8_small_tile(int64_t N, int64_t O) { return plan_tiles(N, O, false).small; }

// Into how many parts the byte-operand path splits K when it has room for the parts' accumulators: as on the
// 4-bit path, only where 128 x 128 tiles leave most CUs without a workgroup, every part at least eight K-tiles.
int32_t t8_splits(int64_t N, int64_t K, int64_t O)
{
    if (N <= 32 || !t8_small_tile(N, O)) return 1;
    const int64_t tiles = ((O + 127) / 128) * ((N + 127) / 128), n_kt = (K + T8_KT - 1) / T8_KT;
    if (tiles > 128) return 1;
    int64_t s = 256 / tiles;
    if (s > 4) s = 4;
    if (s > n_kt / 8) s = n_kt / 8;
    return s < 2 ? 1 : (int32_t)s;
}

// 6- or 8-bit activations, more than 32 tokens, byte operands straight into the int8 matrix cores: the
// activations are re-laid into the workspace, then the product, laid over the chip as on the FP6 path.
template <int ABITS, int WBITS>
int32_t launch_t8(const GemmArgs &g, int32_t y_dtype, hipStream_t stream)
{
    const int32_t st = launch_tiles8(g.a_codes, ABITS, g.N, g.K, const_cast<uint8_t *>(g.a_tiles8), stream);
    if (st != QLLM_OK) return st;
    const TilePlan plan = plan_tiles(g.N, g.O, g.splits == 1 && !g.acc_dump);
    auto launch_small = [&](const GemmArgs &ga) -> int32_t {
        const dim3 grid((unsigned)((ga.O - ga.o_first + 127) / 128), (unsigned)((ga.N + 127) / 128), (unsigned)(ga.splits > 1 ? ga.splits : 1));
        constexpr size_t lds = (size_t)T8_STAGES * 16 * T8_BLOCK;
        if (ga.splits > 1) {
            const int32_t sp = launch_kernel(gemm_tiles8_kernel<ABITS, WBITS, float, 4, 2, true>, grid, dim3(LTHREADS), lds, ga, stream);
            if (sp != QLLM_OK) return sp;
            constexpr int SA = ABITS == 8 ? 1 : 0, SW = WBITS == 8 ? 1 : 0;
            const dim3 fgrid((unsigned)(((int64_t)ga.N * ga.O + 255) / 256));
            if (y_dtype == QLLM_F32) return launch_kernel(splitk_finish_kernel<float, SA, SW>, fgrid, dim3(256), 0, ga, stream);
            return launch_kernel(splitk_finish_kernel<uint16_t, SA, SW>, fgrid, dim3(256), 0, ga, stream);
        }
        if (y_dtype == QLLM_F32) return launch_kernel(gemm_tiles8_kernel<ABITS, WBITS, float, 4, 2>, grid, dim3(LTHREADS), lds, ga, stream);
        return launch_kernel(gemm_tiles8_kernel<ABITS, WBITS, uint16_t, 4, 2>, grid, dim3(LTHREADS), lds, ga, stream);
    };
    auto launch_big = [&](const GemmArgs &ga) -> int32_t {
        const dim3 grid((unsigned)((ga.O - ga.o_first + LBN - 1) / LBN), (unsigned)((ga.N + LBM - 1) / LBM));
        constexpr size_t lds = (size_t)T8_STAGES * 32 * T8_BLOCK;
        if (y_dtype == QLLM_F32) return launch_kernel(gemm_tiles8_kernel<ABITS, WBITS, float, 8, 4>, grid, dim3(LTHREADS), lds, ga, stream);
        return launch_kernel(gemm_tiles8_kernel<ABITS, WBITS, uint16_t, 8, 4>, grid, dim3(LTHREADS), lds, ga, stream);
    };
    if (g.splits > 1) return launch_small(g); // K is only split where the small tile is the choice
    if (plan.o_split > 0) { // whole rounds of large tiles, then the other output features with small ones
        GemmArgs first = g, rest = g;
        first.O = plan.o_split;
        rest.o_first = plan.o_split;
        const int32_t rc = launch_big(first);
        return rc != QLLM_OK ? rc : launch_small(rest);
    }
    return plan.small ? launch_small(g) : launch_big(g);
}

// Up to this many tokens the weight-streaming kernel takes 4-bit codes on both sides (four token tiles per
// workgroup: its LDS strips hold no more, and none of the wider codes at that count).
constexpr int SK4_TOKENS = 64;

template <int ABITS, int WBITS>
int32_t launch(const GemmArgs &g, int32_t y_dtype, hipStream_t stream)
{
    if constexpr (ABITS == 4 && WBITS == 4) {
        if (g.N > 32 && g.N <= SK4_TOKENS) {
            const dim3 grid((unsigned)((g.O + 16 * SK_RT - 1) / (16 * SK_RT)));
            const size_t lds = skinny_lds<4, 4>(4);
            if (y_dtype == QLLM_F32) return launch_kernel(int_gemm_skinny_kernel<4, 4, float, 4>, grid, dim3(SK_THREADS), lds, g, stream);
            return launch_kernel(int_gemm_skinny_kernel<4, 4, uint16_t, 4>, grid, dim3(SK_THREADS), lds, g, stream);
        }
        if (g.a_tiles && g.w_tiles) return launch_fp6(g, y_dtype, stream);
        // 4-bit codes on both sides, more than 32 tokens.  256 x 256 tiles run one workgroup per CU, 128 x 128
        // tiles two, at about three quarters of the large tile's rate per matrix-core operation: the
        // small tile is taken where it fills the chip's rounds that much better (few tiles, or a last
        // round that is mostly empty: 384 large tiles are 1.5 rounds, 1536 small ones 3).
        const int64_t big_tiles = (int64_t)((g.O + LBN - 1) / LBN) * ((g.N + LBM - 1) / LBM);
        const int64_t small_tiles = (int64_t)((g.O + 127) / 128) * ((g.N + 127) / 128);
        const double big_fill = (double)big_tiles / (double)(256 * ((big_tiles + 255) / 256));
        const double small_fill = (double)small_tiles / (double)(512 * ((small_tiles + 511) / 512));
        if (g.N > 32 && (g.N <= 128 || big_fill < 0.78 * small_fill)) {
            const dim3 grid((unsigned)((g.O + 127) / 128), (unsigned)((g.N + 127) / 128), (unsigned)(g.splits > 1 ? g.splits : 1));
            constexpr size_t lds = (size_t)NBUF * 256 * PROWB;
            if (g.splits > 1) {
                const int32_t st = launch_kernel(int_gemm_w4a4_kernel<float, 4, 2, true>, grid, dim3(LTHREADS), lds, g, stream);
                if (st != QLLM_OK) return st;
                const dim3 fgrid((unsigned)(((int64_t)g.N * g.O + 255) / 256));
                if (y_dtype == QLLM_F32) return launch_kernel(splitk_finish_kernel<float>, fgrid, dim3(256), 0, g, stream);
                return launch_kernel(splitk_finish_kernel<uint16_t>, fgrid, dim3(256), 0, g, stream);
            }
            if (y_dtype == QLLM_F32)
                return launch_kernel(int_gemm_w4a4_kernel<float, 4, 2>, grid, dim3(LTHREADS), lds, g, stream);
            return launch_kernel(int_gemm_w4a4_kernel<uint16_t, 4, 2>, grid, dim3(LTHREADS), lds, g, stream);
        }
    } else {
        if (g.a_tiles8 && g.w_tiles8) return launch_t8<ABITS, WBITS>(g, y_dtype, stream);
    }
    if (g.N > 128) { // enough tokens to fill 256-row tiles
        const dim3 grid((unsigned)((g.O + LBN - 1) / LBN), (unsigned)((g.N + LBM - 1) / LBM));
        if constexpr (ABITS == 4 && WBITS == 4) {
            if (y_dtype == QLLM_F32)
                return launch_kernel(int_gemm_w4a4_kernel<float, 8, 4>, grid, dim3(LTHREADS), NBUF * PBUF, g, stream);
            return launch_kernel(int_gemm_w4a4_kernel<uint16_t, 8, 4>, grid, dim3(LTHREADS), NBUF * PBUF, g, stream);
        } else {
            if (y_dtype == QLLM_F32)
                return launch_kernel(int_gemm_big_kernel<ABITS, WBITS, float>, grid, dim3(LTHREADS), 2 * LBUF, g, stream);
            return launch_kernel(int_gemm_big_kernel<ABITS, WBITS, uint16_t>, grid, dim3(LTHREADS), 2 * LBUF, g, stream);
        }
    }
    if (g.N <= 32) { // decode: stream the weights once
        const dim3 grid((unsigned)((g.O + 16 * SK_RT - 1) / (16 * SK_RT)));
        const int nt = g.N <= 16 ? 1 : 2;
        const size_t lds = skinny_lds<ABITS, WBITS>(nt);
        if (y_dtype == QLLM_F32) {
            if (nt == 1) return launch_kernel(int_gemm_skinny_kernel<ABITS, WBITS, float, 1>, grid, dim3(SK_THREADS), lds, g, stream);
            return launch_kernel(int_gemm_skinny_kernel<ABITS, WBITS, float, 2>, grid, dim3(SK_THREADS), lds, g, stream);
        }
        if (nt == 1) return launch_kernel(int_gemm_skinny_kernel<ABITS, WBITS, uint16_t, 1>, grid, dim3(SK_THREADS), lds, g, stream);
        return launch_kernel(int_gemm_skinny_kernel<ABITS, WBITS, uint16_t, 2>, grid, dim3(SK_THREADS), lds, g, stream);
    }
    if constexpr (ABITS == 4 && WBITS == 4) {
        return QLLM_ERR_SHAPE; // not reached: every 4-bit shape was placed above
    } else { // 33..128 tokens, 6- or 8-bit codes
        const dim3 grid((unsigned)((g.O + BN - 1) / BN), (unsigned)((g.N + BM - 1) / BM));
        if (y_dtype == QLLM_F32) return launch_kernel(int_gemm_kernel<ABITS, WBITS, float>, grid, dim3(THREADS), 0, g, stream);
        return launch_kernel(int_gemm_kernel<ABITS, WBITS, uint16_t>, grid, dim3(THREADS), 0, g, stream);
    }
}

// Largest L such that |beta_x| < L and |beta_w| < L keep the epilogue inside narrow integers: row and column
// sums and K * beta_x below 2^23 (24-bit multiplies), and the accumulator together with the three correction
// terms -- in whatever order they are added -- below 2^31 in magnitude:
//     K * (qa * qw + (qa + qw) * L + L * L)  <  2^31,
// the largest value sum((a - beta_x) * (w - beta_w)) and each of its partial sums can take.
int32_t small_zero_bound(int64_t K, int32_t a_bits, int32_t w_bits)
{
    const int64_t qa = (1 << a_bits) - 1, qw = (1 << w_bits) - 1, qm = qa > qw ? qa : qw;
    if (qm * K >= (1 << 23) || qa * qw * K >= (1ll << 31)) return 0;
    int64_t L = 1 << 20;
    while (L > 0 && (K * L >= (1 << 23) || K * (qa * qw + (qa + qw) * L + L * L) >= (1ll << 31))) L /= 2;
    return (int32_t)L;
}

// Into how many parts K is split (1: not at all).  Only 4-bit codes with 128 x 128 tiles that leave
// most CUs without a workgroup (up to 64 tiles: four parts, up to 128: two; beyond that the parts'
// accumulators, written and read back, cost what the shorter K loop gains); every part keeps at least
// eight K-tiles.
int32_t k_splits(int64_t N, int64_t K, int64_t O, int32_t a_bits)
{
    if (a_bits != 4 || N <= 64) return 1; // up to 64 tokens the weight-streaming kernel runs (SK4_TOKENS)
    const int64_t tiles = ((O + 127) / 128) * ((N + 127) / 128);
    const int64_t n_kt = (K + QLLM_K_PAD - 1) / QLLM_K_PAD * QLLM_K_PAD / PKT;
    if (tiles > 128) return 1;
    int64_t s = 256 / tiles;
    if (s > 4) s = 4;
    if (s > n_kt / 8) s = n_kt / 8;
    return s < 2 ? 1 : (int32_t)s;
}

} // namespace

extern "C" int64_t qllm_gemm_workspace_floor_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits)
{
    if (a_bits != 4 && a_bits != 6 && a_bits != 8) return QLLM_ERR_BITS;
    if (N < 0 || K <= 0 || O <= 0) return QLLM_ERR_SHAPE;
    const int32_t s = k_splits(N, K, O, a_bits);
    return s > 1 ? (int64_t)s * N * O * (int64_t)sizeof(int32_t) : 0;
}

extern "C" int64_t qllm_gemm_workspace_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits)
{
    const int64_t floor_bytes = qllm_gemm_workspace_floor_bytes(N, K, O, a_bits);
    if (floor_bytes < 0) return floor_bytes;
    if (N <= 32 || (a_bits == 4 && N <= 64)) return floor_bytes; // the weight-streaming kernel needs none
    // 4-bit codes: the parts' accumulators where K is split (the floor), then the activations' tiles for the FP6 path
    if (a_bits == 4) return 225 * K < (1 << 24) ? (floor_bytes + 255) / 256 * 256 + qllm_tiles6_bytes(N, K) : floor_bytes;
    // the byte-operand path: the activations' bytes, then the parts' accumulators where it splits K
    const int32_t s8 = t8_splits(N, K, O);
    return (qllm_tiles8_bytes(N, K) + 255) / 256 * 256 + (s8 > 1 ? (int64_t)s8 * N * O * (int64_t)sizeof(int32_t) : 0);
}

extern "C" int32_t qllm_int_gemm(const qllm_qact *a, int32_t a_bits, int64_t N, const qllm_weight *w, void *y,
                                 int32_t y_dtype, int64_t ldy, int32_t *acc_dump, void *workspace,
                                 int64_t workspace_bytes, void *hip_stream)
{
    if (!a || !w || !y) return QLLM_ERR_NULL;
    if (!a->codes || !a->scale || !a->zero || !a->rowsum) return QLLM_ERR_NULL;
    if (!w->codes || !w->scale || !w->zero || !w->colsum) return QLLM_ERR_NULL;
    if (y_dtype != QLLM_F32 && y_dtype != QLLM_BF16) return QLLM_ERR_DTYPE;
    const int32_t wb = w->bits;
    const bool pair_ok = (a_bits == wb && (wb == 4 || wb == 6 || wb == 8)) || (a_bits == 8 && wb == 4);
    if (!pair_ok) return QLLM_ERR_BITS;
    if (N < 0 || N > INT32_MAX || w->O <= 0 || w->O > INT32_MAX || w->K <= 0 || w->K > (1 << 24) || ldy < w->O)
        return QLLM_ERR_SHAPE;
    // the largest possible sum of products must stay inside int32
    const int64_t qa = (1 << a_bits) - 1, qw = (1 << wb) - 1;
    if (qa * qw * w->K > INT32_MAX) return QLLM_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(a->codes) & 15u) || (reinterpret_cast<uintptr_t>(w->codes) & 15u))
        return QLLM_ERR_ALIGN;
    if (workspace_bytes < qllm_gemm_workspace_floor_bytes(N, w->K, w->O, a_bits)) return QLLM_ERR_WORKSPACE;
    if (N == 0) return QLLM_OK;

    GemmArgs g{};
    g.a_codes = a->codes;
    g.w_codes = w->codes;
    g.a_row_bytes = qllm_packed_row_bytes(w->K, a_bits);
    g.w_row_bytes = qllm_packed_row_bytes(w->K, wb);
    g.ax = a->scale; g.bx = a->zero; g.rs = a->rowsum;
    g.aw = w->scale; g.bw = w->zero; g.cs = w->colsum;
    g.N = (int32_t)N; g.O = (int32_t)w->O; g.K = (int32_t)w->K;
    g.Kpad = (int32_t)((w->K + QLLM_K_PAD - 1) / QLLM_K_PAD * QLLM_K_PAD);
    g.y = y; g.ldy = ldy; g.acc_dump = acc_dump;
    g.splits = (a_bits == 4 && wb == 4) ? k_splits(N, w->K, w->O, a_bits) : 1;
    g.partial = static_cast<int32_t *>(workspace);
    if (g.splits > 1 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u))) return workspace ? QLLM_ERR_ALIGN : QLLM_ERR_WORKSPACE;
    // the FP6 matrix-core path: 4-bit codes, more than 32 tokens, K not split, the weight's tiles at hand and room
    // for the activations' in the workspace
    // (where K is split, the parts' accumulators come first in the workspace and the tiles behind them)
    const int64_t tiles_at = g.splits > 1 ? ((int64_t)g.splits * N * w->O * (int64_t)sizeof(int32_t) + 255) / 256 * 256 : 0;
    if (a_bits == 4 && wb == 4 && w->tiles6 && N > 64 && workspace && 225 * w->K < (1 << 24) &&
        workspace_bytes >= tiles_at + qllm_tiles6_bytes(N, w->K) && qllm_tiles6_bytes(N, w->K) < (1ll << 32) &&
        qllm_tiles6_bytes(w->O, w->K) < (1ll << 32)) { // the kernel addresses either operand with 32-bit offsets
        if ((reinterpret_cast<uintptr_t>(workspace) & 15u) || (reinterpret_cast<uintptr_t>(w->tiles6) & 15u)) return QLLM_ERR_ALIGN;
        g.a_tiles = static_cast<const uint8_t *>(workspace) + tiles_at;
        g.w_tiles = w->tiles6;
    }
    // the byte-operand path of the other bit pairs: more than 32 tokens, the weight's tiles at hand and room for the
    // activations' in the workspace
    if (!(a_bits == 4 && wb == 4) && w->tiles8 && N > 32 && workspace && workspace_bytes >= qllm_tiles8_bytes(N, w->K) &&
        qllm_tiles8_bytes(N, w->K) < (1ll << 32) && qllm_tiles8_bytes(w->O, w->K) < (1ll << 32)) {
        if ((reinterpret_cast<uintptr_t>(workspace) & 15u) || (reinterpret_cast<uintptr_t>(w->tiles8) & 15u)) return QLLM_ERR_ALIGN;
        g.a_tiles8 = static_cast<const uint8_t *>(workspace);
        g.w_tiles8 = w->tiles8;
        // K split over workgroups where few tiles would leave most CUs idle, if the workspace also holds the parts
        const int32_t s8 = t8_splits(N, w->K, w->O);
        const int64_t at = (qllm_tiles8_bytes(N, w->K) + 255) / 256 * 256;
        if (s8 > 1 && workspace_bytes >= at + (int64_t)s8 * N * w->O * (int64_t)sizeof(int32_t)) {
            g.splits = s8;
            g.partial = reinterpret_cast<int32_t *>(static_cast<uint8_t *>(workspace) + at);
        }
    }
    g.small_zero = small_zero_bound(w->K, a_bits, wb);
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (a_bits == 4) return launch<4, 4>(g, y_dtype, stream);
    if (a_bits == 6) return launch<6, 6>(g, y_dtype, stream);
    if (wb == 8) return launch<8, 8>(g, y_dtype, stream);
    return launch<8, 4>(g, y_dtype, stream);
}

extern "C" int64_t qllm_tiles6_bytes(int64_t rows, int64_t K)
{
    if (rows < 0 || K <= 0) return QLLM_ERR_SHAPE;
    const int64_t Kpad = (K + QLLM_K_PAD - 1) / QLLM_K_PAD * QLLM_K_PAD;
    return (rows + 15) / 16 * (Kpad / T6_KT) * T6_BLOCK;
}

extern "C" int32_t qllm_pack_tiles6(const uint8_t *codes, int64_t rows, int64_t K, uint8_t *tiles, void *hip_stream)
{
    if (!codes || !tiles) return QLLM_ERR_NULL;
    if (rows < 0 || rows > INT32_MAX || K <= 0 || K > (1 << 24)) return QLLM_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(codes) & 15u) || (reinterpret_cast<uintptr_t>(tiles) & 15u)) return QLLM_ERR_ALIGN;
    if (rows == 0) return QLLM_OK;
    const int64_t Kpad = (K + QLLM_K_PAD - 1) / QLLM_K_PAD * QLLM_K_PAD;
    return launch_tiles6(codes, qllm_packed_row_bytes(K, 4), rows, Kpad, tiles, reinterpret_cast<hipStream_t>(hip_stream));
}

extern "C" int64_t qllm_tiles8_bytes(int64_t rows, int64_t K)
{
    if (rows < 0 || K <= 0) return QLLM_ERR_SHAPE;
    return (rows + 15) / 16 * ((K + T8_KT - 1) / T8_KT) * T8_BLOCK;
}

extern "C" int32_t qllm_pack_tiles8(const uint8_t *codes, int32_t bits, int64_t rows, int64_t K, uint8_t *tiles, void *hip_stream)
{
    if (!codes || !tiles) return QLLM_ERR_NULL;
    if (bits != 4 && bits != 6 && bits != 8) return QLLM_ERR_BITS;
    if (rows < 0 || rows > INT32_MAX || K <= 0 || K > (1 << 24)) return QLLM_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(codes) & 15u) || (reinterpret_cast<uintptr_t>(tiles) & 15u)) return QLLM_ERR_ALIGN;
    if (rows == 0) return QLLM_OK;
    return launch_tiles8(codes, bits, rows, K, tiles, reinterpret_cast<hipStream_t>(hip_stream));
}

namespace {

// What the layer needs at least (quantized activations + what the GEMM needs whatever path it takes), and the
// room that lets the GEMM take its FP6 path when the weight comes with tiles.
int64_t layer_workspace_floor(int64_t N, int64_t K, int64_t O, int32_t a_bits)
{
    const int64_t gw = qllm_gemm_workspace_floor_bytes(N, K, O, a_bits);
    if (gw < 0) return gw;
    const int64_t rb = qllm_packed_row_bytes(K, a_bits);
    auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
    return up(N * rb) + 3 * up(N * 4) + up(gw);
}

} // namespace

extern "C" int64_t qllm_workspace_floor_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits)
{
    return layer_workspace_floor(N, K, O, a_bits);
}

extern "C" int64_t qllm_workspace_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits)
{
    const int64_t floor_bytes = layer_workspace_floor(N, K, O, a_bits);
    if (floor_bytes < 0) return floor_bytes;
    auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
    return floor_bytes - up(qllm_gemm_workspace_floor_bytes(N, K, O, a_bits)) + up(qllm_gemm_workspace_bytes(N, K, O, a_bits));
}

extern "C" int32_t qllm_reassembled_linear(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                           int32_t norm, const float *gamma, const float *beta, float eps,
                                           const qllm_map *map, int32_t a_bits, const qllm_weight *w, void *y,
                                           int32_t y_dtype, int64_t ldy, void *workspace, int64_t workspace_bytes,
                                           void *hip_stream)
{
    if (!map || !w) return QLLM_ERR_NULL;
    if (w->K != map->C_out) return QLLM_ERR_SHAPE;
    if (N < 0) return QLLM_ERR_SHAPE;
    const int64_t need = layer_workspace_floor(N, map->C_out, w->O, a_bits); // more lets the GEMM take its FP6 path
    if (need < 0) return (int32_t)need;
    if (N == 0) return QLLM_OK; // nothing to do, whatever the workspace
    if (!workspace || workspace_bytes < need) return QLLM_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QLLM_ERR_ALIGN;
    auto up = [](int64_t v) { return (v + 255) / 256 * 256; };
    uint8_t *p = static_cast<uint8_t *>(workspace);
    qllm_qact q;
    q.codes = p;
    p += up(N * qllm_packed_row_bytes(map->C_out, a_bits));
    q.scale = reinterpret_cast<float *>(p);
    p += up(N * 4);
    q.zero = reinterpret_cast<int32_t *>(p);
    p += up(N * 4);
    q.rowsum = reinterpret_cast<int32_t *>(p);
    p += up(N * 4);
    int32_t rc = qllm_norm_reassemble_quant(x, x_dtype, N, C, ldx, norm, gamma, beta, eps, map, a_bits, &q, hip_stream);
    if (rc != QLLM_OK) return rc;
    return qllm_int_gemm(&q, a_bits, N, w, y, y_dtype, ldy, nullptr, p, workspace_bytes - (p - static_cast<uint8_t *>(workspace)),
                         hip_stream);
}

// ---- the layer for callers that cannot allocate: its workspace is a device array of this library

namespace {

// Device memory beyond the inputs and outputs of the layer: the quantized activations between the two kernels
// and, where the sum over K is split over workgroups, their partial accumulators.  One copy per GPU, held from
// the moment the code object is loaded on it until the process ends.  In host code this name is only a handle:
// the address on the current device comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[QLLM_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_lock;
void *scratch_at[MAX_DEVICES]; // the array's address on each device, asked for once

int32_t scratch_pointer(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        qllm_note_hip_error("static workspace: current device", e != hipSuccess ? hipGetErrorName(e) : "device number out of range");
        return QLLM_ERR_HIP;
    }
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_at[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            qllm_note_hip_error("static workspace: address of the device array", e != hipSuccess ? hipGetErrorName(e) : "null address");
            return QLLM_ERR_HIP;
        }
        scratch_at[dev] = p;
    }
    *out = scratch_at[dev];
    return QLLM_OK;
}

} // namespace

extern "C" int32_t qllm_reassembled_linear_static(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                                  int32_t norm, const float *gamma, const float *beta, float eps,
                                                  const qllm_map *map, int32_t a_bits, const qllm_weight *w, void *y,
                                                  int32_t y_dtype, int64_t ldy, void *hip_stream)
{
    if (!map || !w) return QLLM_ERR_NULL;
    if (w->K != map->C_out) return QLLM_ERR_SHAPE;
    if (N < 0) return QLLM_ERR_SHAPE;
    const int64_t need = layer_workspace_floor(N, map->C_out, w->O, a_bits);
    if (need < 0) return (int32_t)need;
    if (need > (int64_t)QLLM_STATIC_WORKSPACE_BYTES) return QLLM_ERR_WORKSPACE; // too large a batch for the built-in workspace
    if (N == 0) return QLLM_OK;
    void *ws = nullptr;
    const int32_t rc = scratch_pointer(&ws);
    if (rc != QLLM_OK) return rc;
    return qllm_reassembled_linear(x, x_dtype, N, C, ldx, norm, gamma, beta, eps, map, a_bits, w, y, y_dtype, ldy, ws,
                                   (int64_t)QLLM_STATIC_WORKSPACE_BYTES, hip_stream);
}
