/*
 * CPU oracle for the reassembled low-bit linear layer of QLLM (arXiv 2310.08041).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, loop-by-loop statement of what the
 * hot path computes, written from the paper's equations.  Only the test-suite, the smoke check
 * and the cpu_baseline leg of the benchmark may load it.  It shares no code, header, table or
 * helper with the HIP library; the HIP library never calls it.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC (see oracle/build.py).
 * -ffp-contract=off matters: every fp32 product and sum below is rounded on its own.
 *
 * All pointers are host pointers.  Every function returns 0 on success, a positive code on a
 * malformed argument.  Rows are independent; loops over rows may run under OpenMP, which does
 * not change any result (no reduction crosses a row).
 *
 * Steps and where the paper defines them:
 *   norm                    Sec. 4.3 "Inference efficiency" (a normalisation layer precedes the
 *                           runtime disassembly/assembly layers; its formula is the textbook one)
 *   channel disassembly     Sec. 4.1.1, Eq. (3); T = ceil(max|x| / theta)
 *   channel assembly        Sec. 4.1.2, Eq. (4); the A/B (even/odd) indexing of the runtime
 *                           pseudo-code figure in the appendix
 *   uniform quantizer       Preliminaries, Eq. (2); per token for activations and per output
 *                           channel for weights (Sec. 5 "Quantization settings")
 *   quantized linear layer  Eq. (1) applied to the codes; Y~ = quant(X^) quant(W^) (Sec. 4.1.3)
 *   weight reassembly       Eq. (3) (rows duplicated), Eq. (4) (rows summed), Appendix B
 *   gated activation        the producer of a down projection's input in the models of Sec. 5
 *                           (silu(gate) * up; its arithmetic is this build's, stated where it is defined)
 *
 * Fixed arithmetic (the paper states none; these are this build's readings, listed in the design
 * notes): row statistics in fp64, rounded once to fp32; every element-wise step in fp32 with
 * separate roundings; round-half-to-even; the quantizer multiplies by inv = fl32(1/alpha) and
 * rounds the EXACT product x*inv to the nearest integer.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_NORM_NONE = 0, ORACLE_NORM_LAYER = 1, ORACLE_NORM_RMS = 2 };

/* ---------------------------------------------------------------- bf16 <-> fp32 */

static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* round-to-nearest-even truncation of an fp32 value to bfloat16 bits (finite inputs) */
static uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static float load_elem(const void *x, int dtype, int64_t idx)
{
    if (dtype == ORACLE_BF16) return bf16_bits_to_f32(((const uint16_t *)x)[idx]);
    return ((const float *)x)[idx];
}

int oracle_round_to_bf16(const float *src, int64_t n, uint16_t *dst)
{
    if (!src || !dst || n < 0) return 1;
    for (int64_t i = 0; i < n; ++i) dst[i] = f32_to_bf16_bits(src[i]);
    return 0;
}

int oracle_widen_bf16(const uint16_t *src, int64_t n, float *dst)
{
    if (!src || !dst || n < 0) return 1;
    for (int64_t i = 0; i < n; ++i) dst[i] = bf16_bits_to_f32(src[i]);
    return 0;
}

/* ---------------------------------------------------------------- step a1: norm
 * LayerNorm : mu = mean(x), var = mean((x-mu)^2) (biased), y = ((x-mu)*rstd)*gamma + beta
 * RMSNorm   : rstd = 1/sqrt(mean(x^2)+eps),               y = (x*rstd)*gamma
 * NONE      : y = x
 * Sums, mu, var and rstd are formed in fp64; mu and rstd are rounded once to fp32 and the
 * element-wise part runs in fp32, one rounding per operation, in the order written.
 * beta == NULL means "no shift" (the add is skipped).  y is [N, C] dense fp32.
 */
int oracle_norm(const void *x, int x_dtype, int64_t N, int64_t C, int64_t ldx, int norm,
                const float *gamma, const float *beta, float eps, float *y)
{
    if (!x || !y || N < 0 || C <= 0 || ldx < C) return 1;
    if (x_dtype != ORACLE_F32 && x_dtype != ORACLE_BF16) return 2;
    if (norm != ORACLE_NORM_NONE && norm != ORACLE_NORM_LAYER && norm != ORACLE_NORM_RMS) return 3;
    if (norm != ORACLE_NORM_NONE && !gamma) return 4;

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const int64_t base = n * ldx;
        float *yr = y + n * C;
        if (norm == ORACLE_NORM_NONE) {
            for (int64_t c = 0; c < C; ++c) yr[c] = load_elem(x, x_dtype, base + c);
        } else if (norm == ORACLE_NORM_LAYER) {
            double s = 0.0;
            for (int64_t c = 0; c < C; ++c) s += (double)load_elem(x, x_dtype, base + c);
            const double mu64 = s / (double)C;
            double q = 0.0;
            for (int64_t c = 0; c < C; ++c) {
                const double d = (double)load_elem(x, x_dtype, base + c) - mu64;
                q += d * d;
            }
            const double var = q / (double)C;
            const float mu = (float)mu64;
            const float rstd = (float)(1.0 / sqrt(var + (double)eps));
            for (int64_t c = 0; c < C; ++c) {
                float t = load_elem(x, x_dtype, base + c) - mu;
                t = t * rstd;
                t = t * gamma[c];
                if (beta) t = t + beta[c];
                yr[c] = t;
            }
        } else {
            double q = 0.0;
            for (int64_t c = 0; c < C; ++c) {
                const double v = (double)load_elem(x, x_dtype, base + c);
                q += v * v;
            }
            const float rstd = (float)(1.0 / sqrt(q / (double)C + (double)eps));
            for (int64_t c = 0; c < C; ++c) {
                float t = load_elem(x, x_dtype, base + c) * rstd;
                t = t * gamma[c];
                yr[c] = t;
            }
        }
    }
    return 0;
}

/* per-channel max |y| over the N rows of a dense fp32 [N, C] matrix: the calibration statistic
 * "max(|x_M|)" of Sec. 4.1.1 and the vector m of Algorithm 1. */
int oracle_channel_absmax(const float *y, int64_t N, int64_t C, float *absmax)
{
    if (!y || !absmax || N < 0 || C <= 0) return 1;
    for (int64_t c = 0; c < C; ++c) absmax[c] = 0.0f;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c) {
            const float a = fabsf(y[n * C + c]);
            if (a > absmax[c]) absmax[c] = a;
        }
    return 0;
}

/* ---------------------------------------------------------------- step a2: channel disassembly
 * T_c = ceil(max|x_c| / theta) (Sec. 4.1.1), at least 1; the quotient is taken in fp64. */
int oracle_num_split(const float *absmax, int64_t C, float theta, int32_t *T)
{
    if (!absmax || !T || C <= 0 || !(theta > 0.0f)) return 1;
    for (int64_t c = 0; c < C; ++c) {
        double t = ceil((double)absmax[c] / (double)theta);
        if (!(t >= 1.0)) t = 1.0;
        if (t > 1e9) return 2;
        T[c] = (int32_t)t;
    }
    return 0;
}

/* Eq. (3): channel c becomes T_c adjacent sub-channels, each y_c * (1/T_c).
 * d is [N, Cp] with Cp = sum_c T_c (the caller sizes it). */
int oracle_disassemble(const float *y, int64_t N, int64_t C, const int32_t *T, float *d, int64_t Cp)
{
    if (!y || !T || !d || N < 0 || C <= 0) return 1;
    int64_t total = 0;
    for (int64_t c = 0; c < C; ++c) {
        if (T[c] < 1) return 2;
        total += T[c];
    }
    if (total != Cp) return 3;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        int64_t pos = 0;
        for (int64_t c = 0; c < C; ++c) {
            const float s = (float)(1.0 / (double)T[c]);
            const float v = y[n * C + c] * s;
            for (int32_t t = 0; t < T[c]; ++t) d[n * Cp + pos++] = v;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- step a3: channel assembly
 * The disassembled axis (Cp positions) is split into set A = even positions and set B = odd
 * positions.  Pair k merges A-member src_idx[k] (position 2*src_idx[k]) into B-member dst_idx[k]
 * (position 2*dst_idx[k]+1).  Several A-members may name the same B-member.  The B-member's value
 * becomes the mean of itself and everything merged into it (Eq. (4) for a pair); the merged
 * A-positions disappear; every other position keeps its place and order.
 *
 * The mean of a group of g values is evaluated as (1/g)*v_dst + (1/g)*v_src1 + ... with
 * (1/g) = fl32(1.0/g), sources in ascending A-index, each product and each sum rounded to fp32.
 *
 * keep_out (nullable, [Chat]) receives the disassembled position each output channel came from.
 */
typedef struct {
    int32_t *merged_into; /* [Cp] position of the B-member an A-position was merged into, or -1 */
    int32_t *group;       /* [Cp] 1 + number of A-members merged into this position */
    int32_t *first_src;   /* [Cp] lowest merged A-position of this destination, or -1 */
    int32_t *next_src;    /* [Cp] next higher A-position merged into the same destination, or -1 */
} merge_plan;

static void free_plan(merge_plan *pl)
{
    free(pl->merged_into); free(pl->group); free(pl->first_src); free(pl->next_src);
    memset(pl, 0, sizeof *pl);
}

static int assemble_plan(int64_t Cp, const int32_t *src_idx, const int32_t *dst_idx, int64_t r,
                         merge_plan *pl)
{
    const int64_t nA = (Cp + 1) / 2, nB = Cp / 2;
    const size_t bytes = sizeof(int32_t) * (size_t)(Cp > 0 ? Cp : 1);
    pl->merged_into = (int32_t *)malloc(bytes);
    pl->group = (int32_t *)malloc(bytes);
    pl->first_src = (int32_t *)malloc(bytes);
    pl->next_src = (int32_t *)malloc(bytes);
    if (!pl->merged_into || !pl->group || !pl->first_src || !pl->next_src) { free_plan(pl); return 9; }
    for (int64_t p = 0; p < Cp; ++p) {
        pl->merged_into[p] = -1; pl->group[p] = 1; pl->first_src[p] = -1; pl->next_src[p] = -1;
    }
    for (int64_t k = 0; k < r; ++k) {
        if (src_idx[k] < 0 || src_idx[k] >= nA || dst_idx[k] < 0 || dst_idx[k] >= nB) {
            free_plan(pl); return 4;
        }
        const int64_t sp = 2 * (int64_t)src_idx[k], dp = 2 * (int64_t)dst_idx[k] + 1;
        if (pl->merged_into[sp] != -1) { free_plan(pl); return 5; } /* A-member merged twice */
        pl->merged_into[sp] = (int32_t)dp;
        pl->group[dp] += 1;
    }
    /* chain the sources of every destination in ascending position: walk down, push in front */
    for (int64_t q = Cp - 1; q >= 0; --q) {
        const int32_t dp = pl->merged_into[q];
        if (dp == -1) continue;
        pl->next_src[q] = pl->first_src[dp];
        pl->first_src[dp] = (int32_t)q;
    }
    return 0;
}

int64_t oracle_assembled_count(int64_t Cp, int64_t r) { return Cp - r; }

int oracle_assemble(const float *d, int64_t N, int64_t Cp, const int32_t *src_idx,
                    const int32_t *dst_idx, int64_t r, float *xhat, int64_t Chat, int32_t *keep_out)
{
    if (!d || !xhat || N < 0 || Cp <= 0 || r < 0 || (r > 0 && (!src_idx || !dst_idx))) return 1;
    if (Chat != Cp - r) return 3;
    merge_plan pl;
    int rc = assemble_plan(Cp, src_idx, dst_idx, r, &pl);
    if (rc) return rc;

    if (keep_out) {
        int64_t o = 0;
        for (int64_t p = 0; p < Cp; ++p)
            if (pl.merged_into[p] == -1) keep_out[o++] = (int32_t)p;
    }
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float *dr = d + n * Cp;
        float *out = xhat + n * Chat;
        int64_t o = 0;
        for (int64_t p = 0; p < Cp; ++p) {
            if (pl.merged_into[p] != -1) continue; /* merged A-member: removed */
            if (pl.group[p] == 1) { out[o++] = dr[p]; continue; }
            const float s = (float)(1.0 / (double)pl.group[p]);
            float acc = s * dr[p];
            for (int32_t q = pl.first_src[p]; q != -1; q = pl.next_src[q]) /* ascending A-index */
                acc = acc + s * dr[q];
            out[o++] = acc;
        }
    }
    free_plan(&pl);
    return 0;
}

/* ---------------------------------------------------------------- a2+a3 as one map
 * The composition of Eq. (3) and Eq. (4) written as, for every reassembled channel, a list of
 * (source channel, scale): x^[ch] = sum_k scale_k * y[src_k].  Built here from (T, src_idx,
 * dst_idx) so that the literal two-stage form above can be checked against it, and the HIP
 * library's own builder against both.
 * Sub-channels of a disassembled channel take no part in merging (Sec. 4.1.2, last sentences):
 * naming one as source or destination is an error.
 * row_ptr has Chat+1 entries; src/scale have nnz = Chat + r entries (the caller sizes them from
 * Cp and r).  Entry order inside a row: destination first, then sources by ascending A-index.
 */
int oracle_build_map(const int32_t *T, int64_t C, const int32_t *src_idx, const int32_t *dst_idx,
                     int64_t r, int32_t *row_ptr, int32_t *src, float *scale, int64_t *Chat_out,
                     int64_t *nnz_out)
{
    if (!T || !row_ptr || !src || !scale || C <= 0 || r < 0 || (r > 0 && (!src_idx || !dst_idx))) return 1;
    int64_t Cp = 0;
    for (int64_t c = 0; c < C; ++c) {
        if (T[c] < 1) return 2;
        Cp += T[c];
    }
    int32_t *chan_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)Cp);
    if (!chan_of) return 9;
    {
        int64_t p = 0;
        for (int64_t c = 0; c < C; ++c)
            for (int32_t t = 0; t < T[c]; ++t) chan_of[p++] = (int32_t)c;
    }
    merge_plan pl;
    int rc = assemble_plan(Cp, src_idx, dst_idx, r, &pl);
    if (rc) { free(chan_of); return rc; }
    for (int64_t p = 0; p < Cp; ++p) {
        const int involved = (pl.merged_into[p] != -1) || (pl.group[p] > 1);
        if (involved && T[chan_of[p]] != 1) { free(chan_of); free_plan(&pl); return 6; }
    }
    int64_t o = 0, e = 0;
    for (int64_t p = 0; p < Cp; ++p) {
        if (pl.merged_into[p] != -1) continue;
        row_ptr[o++] = (int32_t)e;
        if (pl.group[p] == 1) {
            src[e] = chan_of[p];
            scale[e] = (float)(1.0 / (double)T[chan_of[p]]);
            ++e;
        } else {
            const float s = (float)(1.0 / (double)pl.group[p]);
            src[e] = chan_of[p]; scale[e] = s; ++e;
            for (int32_t q = pl.first_src[p]; q != -1; q = pl.next_src[q]) {
                src[e] = chan_of[q]; scale[e] = s; ++e;
            }
        }
    }
    row_ptr[o] = (int32_t)e;
    if (Chat_out) *Chat_out = o;
    if (nnz_out) *nnz_out = e;
    free(chan_of); free_plan(&pl);
    return 0;
}

/* x^[n, ch] = scale_0*y[src_0] + scale_1*y[src_1] + ... , left to right, fp32, one rounding each */
int oracle_apply_map(const float *y, int64_t N, int64_t C, const int32_t *row_ptr, const int32_t *src,
                     const float *scale, int64_t Chat, float *xhat)
{
    if (!y || !row_ptr || !src || !scale || !xhat || N < 0 || C <= 0 || Chat <= 0) return 1;
    for (int64_t o = 0; o < Chat; ++o) {
        if (row_ptr[o + 1] <= row_ptr[o]) return 2;
        for (int32_t e = row_ptr[o]; e < row_ptr[o + 1]; ++e)
            if (src[e] < 0 || src[e] >= C) return 3;
    }
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float *yr = y + n * C;
        float *out = xhat + n * Chat;
        for (int64_t o = 0; o < Chat; ++o) {
            int32_t e = row_ptr[o];
            float acc = scale[e] * yr[src[e]];
            for (++e; e < row_ptr[o + 1]; ++e) acc = acc + scale[e] * yr[src[e]];
            out[o] = acc;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- step a4: Eq. (2) on one vector
 * alpha = (max - min) / (2^b - 1)           fp32 subtraction, fp32 division
 * beta  = -round(min / alpha)               as round(min * inv), inv = fl32(1/alpha)
 * code  = clamp(round(x / alpha) + beta, 0, 2^b - 1)   as round(x * inv) + beta
 * round() is to nearest, ties to even, applied to the exact product (two fp32 factors multiply
 * exactly in fp64).  A constant vector (max == min) takes alpha = 1.
 * stride lets the same routine walk a column of a row-major matrix (weights).
 */
static int64_t rne_exact_product(float a, float b)
{
    return (int64_t)rint((double)a * (double)b);
}

static void quantize_vector(const float *x, int64_t K, int64_t stride, int qmax, uint8_t *codes,
                            float *alpha_out, int32_t *beta_out, int32_t *sum_out)
{
    float mn = x[0], mx = x[0];
    for (int64_t k = 1; k < K; ++k) {
        const float v = x[k * stride];
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    const float range = mx - mn;
    float alpha = range / (float)qmax;
    if (!(range > 0.0f)) alpha = 1.0f;
    const float inv = 1.0f / alpha;
    int64_t beta = -rne_exact_product(mn, inv);
    if (beta > INT32_MAX) beta = INT32_MAX;
    if (beta < -INT32_MAX) beta = -INT32_MAX;
    int64_t sum = 0;
    for (int64_t k = 0; k < K; ++k) {
        int64_t q = rne_exact_product(x[k * stride], inv) + beta;
        if (q < 0) q = 0;
        if (q > qmax) q = qmax;
        codes[k] = (uint8_t)q;
        sum += q;
    }
    *alpha_out = alpha;
    *beta_out = (int32_t)beta;
    *sum_out = (int32_t)sum;
}

static int bits_ok(int bits) { return bits >= 2 && bits <= 8; }

/* per-token quantization of x^ [N, K] (row stride ldx): codes [N, K] one byte each */
int oracle_quantize_rows(const float *x, int64_t N, int64_t K, int64_t ldx, int bits, uint8_t *codes,
                         float *alpha, int32_t *beta, int32_t *rowsum)
{
    if (!x || !codes || !alpha || !beta || !rowsum || N < 0 || K <= 0 || ldx < K) return 1;
    if (!bits_ok(bits)) return 2;
    const int qmax = (1 << bits) - 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        quantize_vector(x + n * ldx, K, 1, qmax, codes + n * K, alpha + n, beta + n, rowsum + n);
    return 0;
}

/* per-output-channel quantization of W^ [K, O] (the paper's [in, out] layout):
 * wcodes [O, K], alpha_w/beta_w/colsum [O]; min and max run over the input channels of column o */
int oracle_quantize_weight(const float *What, int64_t K, int64_t O, int bits, uint8_t *wcodes,
                           float *alpha_w, int32_t *beta_w, int32_t *colsum)
{
    if (!What || !wcodes || !alpha_w || !beta_w || !colsum || K <= 0 || O <= 0) return 1;
    if (!bits_ok(bits)) return 2;
    const int qmax = (1 << bits) - 1;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < O; ++o)
        quantize_vector(What + o, K, O, qmax, wcodes + o * K, alpha_w + o, beta_w + o, colsum + o);
    return 0;
}

/* ---------------------------------------------------------------- storage format of the codes
 * 8 bit: one byte per code.  4 bit: code 2j in bits 0..3 and code 2j+1 in bits 4..7 of byte j.
 * 6 bit: codes 4j..4j+3 fill the 24 bits of bytes 3j..3j+2, little endian, code 4j lowest.
 * A row occupies row_bytes >= ceil(K*bits/8) bytes; the tail is zero.
 */
int oracle_pack_codes(const uint8_t *codes, int64_t R, int64_t K, int bits, uint8_t *packed,
                      int64_t row_bytes)
{
    if (!codes || !packed || R < 0 || K <= 0) return 1;
    if (bits != 4 && bits != 6 && bits != 8) return 2;
    if (row_bytes < (K * bits + 7) / 8) return 3;
    for (int64_t rI = 0; rI < R; ++rI) {
        uint8_t *p = packed + rI * row_bytes;
        memset(p, 0, (size_t)row_bytes);
        for (int64_t k = 0; k < K; ++k) {
            const uint32_t v = codes[rI * K + k];
            if (v >> bits) return 4;
            const int64_t bit = k * bits;
            p[bit / 8] |= (uint8_t)(v << (bit % 8));
            if ((bit % 8) + bits > 8) p[bit / 8 + 1] |= (uint8_t)(v >> (8 - bit % 8));
        }
    }
    return 0;
}

int oracle_unpack_codes(const uint8_t *packed, int64_t R, int64_t K, int bits, int64_t row_bytes,
                        uint8_t *codes)
{
    if (!codes || !packed || R < 0 || K <= 0) return 1;
    if (bits != 4 && bits != 6 && bits != 8) return 2;
    if (row_bytes < (K * bits + 7) / 8) return 3;
    for (int64_t rI = 0; rI < R; ++rI) {
        const uint8_t *p = packed + rI * row_bytes;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t bit = k * bits;
            uint32_t w = p[bit / 8];
            if ((bit % 8) + bits > 8) w |= (uint32_t)p[bit / 8 + 1] << 8;
            codes[rI * K + k] = (uint8_t)((w >> (bit % 8)) & ((1u << bits) - 1u));
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- weight reassembly (offline)
 * W is [C, O] as in Eq. (1).  Disassembly duplicates row c T_c times (Eq. (3), Appendix B);
 * assembly replaces the destination row by the sum of the group's rows and removes the merged
 * source rows (Eq. (4): "W_ik + W_jk represents the merged weight").  Sums run destination first,
 * then sources in ascending A-index, in fp32.
 */
int oracle_reassemble_weight(const float *W, int64_t C, int64_t O, const int32_t *T,
                             const int32_t *src_idx, const int32_t *dst_idx, int64_t r, float *What,
                             int64_t Chat)
{
    if (!W || !T || !What || C <= 0 || O <= 0 || r < 0 || (r > 0 && (!src_idx || !dst_idx))) return 1;
    int64_t Cp = 0;
    for (int64_t c = 0; c < C; ++c) {
        if (T[c] < 1) return 2;
        Cp += T[c];
    }
    if (Chat != Cp - r) return 3;
    int32_t *chan_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)Cp);
    if (!chan_of) return 9;
    {
        int64_t p = 0;
        for (int64_t c = 0; c < C; ++c)
            for (int32_t t = 0; t < T[c]; ++t) chan_of[p++] = (int32_t)c;
    }
    merge_plan pl;
    int rc = assemble_plan(Cp, src_idx, dst_idx, r, &pl);
    if (rc) { free(chan_of); return rc; }
    int64_t o = 0;
    for (int64_t p = 0; p < Cp; ++p) {
        if (pl.merged_into[p] != -1) continue;
        float *out = What + o * O;
        const float *w0 = W + (int64_t)chan_of[p] * O;
        for (int64_t j = 0; j < O; ++j) out[j] = w0[j];
        for (int32_t q = pl.first_src[p]; q != -1; q = pl.next_src[q]) {
            const float *w1 = W + (int64_t)chan_of[q] * O;
            for (int64_t j = 0; j < O; ++j) out[j] = out[j] + w1[j];
        }
        ++o;
    }
    free(chan_of); free_plan(&pl);
    return 0;
}

/* ---------------------------------------------------------------- step a5: Eq. (1) on the codes
 * acc[n, o] = sum_k a[n, k] * w[o, k]; unsigned codes; exact integers. Returns 7 if a sum leaves
 * the int32 range. */
int oracle_int_gemm(const uint8_t *a, const uint8_t *w, int64_t N, int64_t K, int64_t O, int32_t *acc)
{
    if (!a || !w || !acc || N < 0 || K <= 0 || O < 0) return 1;
    int overflow = 0;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t o = 0; o < O; ++o) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int64_t)a[n * K + k] * (int64_t)w[o * K + k];
            if (s > INT32_MAX) overflow = 1;
            acc[n * O + o] = (int32_t)s;
        }
    return overflow ? 7 : 0;
}

/* ---------------------------------------------------------------- step a6: dequantising epilogue
 * Eq. (2) read backwards gives x ~ alpha*(code - beta) for both operands, so by Eq. (1)
 *   Y[n,o] = alpha_x[n]*alpha_w[o] * sum_k (a[n,k]-beta_x[n]) * (w[o,k]-beta_w[o])
 *          = alpha_x[n]*alpha_w[o] * (acc - beta_x*colsum_w[o] - beta_w[o]*rowsum_x[n] + K*beta_x*beta_w)
 * The bracket is an exact int64; it is converted to fp32 (nearest-even), multiplied by alpha_x
 * and then by alpha_w, in fp32.
 */
int oracle_epilogue(const int32_t *acc, int64_t N, int64_t O, int64_t K, const float *alpha_x,
                    const int32_t *beta_x, const int32_t *rowsum_x, const float *alpha_w,
                    const int32_t *beta_w, const int32_t *colsum_w, float *y)
{
    if (!acc || !alpha_x || !beta_x || !rowsum_x || !alpha_w || !beta_w || !colsum_w || !y) return 1;
    if (N < 0 || O < 0 || K <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t o = 0; o < O; ++o) {
            const int64_t bx = beta_x[n], bw = beta_w[o];
            const int64_t bracket = (int64_t)acc[n * O + o] - bx * (int64_t)colsum_w[o] -
                                    bw * (int64_t)rowsum_x[n] + K * bx * bw;
            float v = (float)bracket;
            v = v * alpha_x[n];
            v = v * alpha_w[o];
            y[n * O + o] = v;
        }
    return 0;
}

/* The same output without the algebra: the zero-point-corrected products summed one by one. */
int oracle_dequant_linear_direct(const uint8_t *a, const uint8_t *w, int64_t N, int64_t K, int64_t O,
                                 const float *alpha_x, const int32_t *beta_x, const float *alpha_w,
                                 const int32_t *beta_w, float *y)
{
    if (!a || !w || !alpha_x || !beta_x || !alpha_w || !beta_w || !y) return 1;
    if (N < 0 || O < 0 || K <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t o = 0; o < O; ++o) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += ((int64_t)a[n * K + k] - beta_x[n]) * ((int64_t)w[o * K + k] - beta_w[o]);
            float v = (float)s;
            v = v * alpha_x[n];
            v = v * alpha_w[o];
            y[n * O + o] = v;
        }
    return 0;
}

/* ---------------------------------------------------------------- the whole path, a1..a6
 * Runs the steps above one after the other through full-size temporaries.  Any output pointer
 * may be NULL except where a later step needs it (they are allocated internally then).
 * The map is given in the paper's form (T, src_idx, dst_idx); a2 and a3 run literally.
 * wcodes is [O, Chat] one byte per code.
 */
int oracle_reassembled_linear(const void *x, int x_dtype, int64_t N, int64_t C, int64_t ldx, int norm,
                              const float *gamma, const float *beta, float eps, const int32_t *T,
                              const int32_t *src_idx, const int32_t *dst_idx, int64_t r, int a_bits,
                              const uint8_t *wcodes, const float *alpha_w, const int32_t *beta_w,
                              const int32_t *colsum_w, int64_t O, uint8_t *codes_out /*[N,Chat]*/,
                              float *alpha_x_out, int32_t *beta_x_out, int32_t *rowsum_out,
                              int32_t *acc_out /*[N,O]*/, float *y_out /*[N,O]*/)
{
    if (!x || !T || C <= 0 || N < 0) return 1;
    int64_t Cp = 0;
    for (int64_t c = 0; c < C; ++c) Cp += T[c];
    const int64_t Chat = Cp - r;
    if (Chat <= 0) return 3;
    int rc = 0;
    float *y = (float *)malloc(sizeof(float) * (size_t)(N * C + 1));
    float *d = (float *)malloc(sizeof(float) * (size_t)(N * Cp + 1));
    float *xh = (float *)malloc(sizeof(float) * (size_t)(N * Chat + 1));
    uint8_t *codes = codes_out ? codes_out : (uint8_t *)malloc((size_t)(N * Chat + 1));
    float *ax = alpha_x_out ? alpha_x_out : (float *)malloc(sizeof(float) * (size_t)(N + 1));
    int32_t *bx = beta_x_out ? beta_x_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(N + 1));
    int32_t *rs = rowsum_out ? rowsum_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(N + 1));
    int32_t *acc = NULL;
    if (!y || !d || !xh || !codes || !ax || !bx || !rs) { rc = 9; goto done; }
    if ((rc = oracle_norm(x, x_dtype, N, C, ldx, norm, gamma, beta, eps, y))) goto done;
    if ((rc = oracle_disassemble(y, N, C, T, d, Cp))) goto done;
    if ((rc = oracle_assemble(d, N, Cp, src_idx, dst_idx, r, xh, Chat, NULL))) goto done;
    if ((rc = oracle_quantize_rows(xh, N, Chat, Chat, a_bits, codes, ax, bx, rs))) goto done;
    if (wcodes && O > 0 && (acc_out || y_out)) {
        acc = acc_out ? acc_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(N * O + 1));
        if (!acc) { rc = 9; goto done; }
        if ((rc = oracle_int_gemm(codes, wcodes, N, Chat, O, acc))) goto done;
        if (y_out) {
            if (!alpha_w || !beta_w || !colsum_w) { rc = 1; goto done; }
            rc = oracle_epilogue(acc, N, O, Chat, ax, bx, rs, alpha_w, beta_w, colsum_w, y_out);
        }
    }
done:
    free(y); free(d); free(xh);
    if (!codes_out) free(codes);
    if (!alpha_x_out) free(ax);
    if (!beta_x_out) free(bx);
    if (!rowsum_out) free(rs);
    if (acc && !acc_out) free(acc);
    return rc;
}

/*
 * Appendix A step 2 with the plain squared L2 distance between activation columns (the matching the
 * benchmark configurations name: "nearest-L2 channel pairs"): for every member i of set A, the member j
 * of set B with the smallest D(i, j) = sum over the n calibration tokens of (y[t, a_i] - y[t, b_j])^2,
 * the lowest j on ties.  Differences, squares and sums in double, tokens in ascending order.
 * With W != NULL the distance is that of Eq. (5) instead, |x_i - x_j|^2 |W_i - W_j|^2 / 4 (W is
 * [C, ldw], O features): the error Eq. (4) leaves in the layer's output when i is merged into j.
 */
int oracle_nearest_member(const float *y, int64_t n, int64_t ldy, const float *W, int64_t O, int64_t ldw,
                          const int32_t *chan_a, int64_t nA, const int32_t *chan_b, int64_t nB,
                          int64_t *best_j, double *best_d)
{
    if (!y || !chan_a || !chan_b || !best_j || !best_d) return 1;
    if (n <= 0 || nA < 0 || nB <= 0 || (W && O <= 0)) return 2;
    /* the columns of set B, gathered once: [nB][n] */
    double *xb = (double *)malloc((size_t)nB * (size_t)n * sizeof(double));
    if (!xb) return 3;
    for (int64_t j = 0; j < nB; ++j)
        for (int64_t t = 0; t < n; ++t) xb[j * n + t] = (double)y[t * ldy + chan_b[j]];
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t i = 0; i < nA; ++i) {
        double *xa = (double *)malloc((size_t)n * sizeof(double));
        for (int64_t t = 0; t < n; ++t) xa[t] = (double)y[t * ldy + chan_a[i]];
        const float *wa = W ? W + (int64_t)chan_a[i] * ldw : NULL;
        double bd = 0.0;
        int64_t bj = -1;
        for (int64_t j = 0; j < nB; ++j) {
            double dx = 0.0;
            for (int64_t t = 0; t < n; ++t) {
                const double e = xa[t] - xb[j * n + t];
                dx += e * e;
            }
            double d = dx;
            if (W) {
                const float *wb = W + (int64_t)chan_b[j] * ldw;
                double dw = 0.0;
                for (int64_t k = 0; k < O; ++k) {
                    const double e = (double)wa[k] - (double)wb[k];
                    dw += e * e;
                }
                d = 0.25 * dx * dw;
            }
            if (bj < 0 || d < bd) { /* strict: the first of equal minima stays */
                bd = d;
                bj = j;
            }
        }
        free(xa);
        best_j[i] = bj;
        best_d[i] = bd;
    }
    free(xb);
    return 0;
}

/* ---------------------------------------------------------------- the gated activation before a down projection
 *
 * The models of Sec. 5 (LLaMA-1/2) feed their down projection with x = silu(gate) * up, silu(g) = g / (1 + e^-g):
 * the producer of the activations that the headline shape reassembles.  The paper says nothing of its
 * arithmetic; this build fixes it as the following sequence of fp32 operations, each rounded once (fma = one
 * rounding), so that a GPU can reproduce it bit for bit:
 *     z  = min(max(-g, -86), 88)                       (e^z stays a normal number)
 *     n  = rint(z * log2(e));  r = fma(n, -ln2_hi, z);  r = fma(n, -ln2_lo, r)        (|r| <= ln2 / 2)
 *     p  = the degree-5 polynomial of the Cephes expf in r, by Horner's rule with fma;  e = fma(p, r*r, r) + 1
 *     e  = e * 2^n;   d = 1 + e;   s = g / d (correctly rounded);   s = -0 where g < -88
 *     x  = s * up, rounded to bfloat16 (nearest even)
 * gate and up are bfloat16.  The fp32 value before the last rounding is within 2 ulp of the real-number
 * silu(g) * up for the inputs the tests sweep (tests/test_oracle_swiglu.py).
 */
static float silu_times_up(float g, float up)
{
    const float LOG2E = 1.44269504088896341f, LN2_HI = 0.693359375f, LN2_LO = -2.12194440e-4f;
    float z = -g;
    z = fminf(fmaxf(z, -86.0f), 88.0f);
    const float n = rintf(z * LOG2E);
    float r = fmaf(n, -LN2_HI, z);
    r = fmaf(n, -LN2_LO, r);
    float p = 1.9875691500e-4f;
    p = fmaf(p, r, 1.3981999507e-3f);
    p = fmaf(p, r, 8.3334519073e-3f);
    p = fmaf(p, r, 4.1665795894e-2f);
    p = fmaf(p, r, 1.6666665459e-1f);
    p = fmaf(p, r, 5.0000001201e-1f);
    float e = fmaf(p, r * r, r);
    e = e + 1.0f;
    const uint32_t scale_bits = (uint32_t)((int32_t)n + 127) << 23; /* 2^n, n in [-124, 127] */
    float scale;
    memcpy(&scale, &scale_bits, sizeof scale);
    e = e * scale;
    const float d = 1.0f + e;
    float s = g / d;
    if (g < -88.0f) s = -0.0f;
    return s * up;
}

/* gate, up: [N, ld*] bfloat16 bits; x: [N, ldx] bfloat16 bits; f32 (may be NULL): [N, C] the values before the last rounding */
int oracle_swiglu(const uint16_t *gate, int64_t ld_gate, const uint16_t *up, int64_t ld_up, int64_t N, int64_t C,
                  uint16_t *x, int64_t ldx, float *f32)
{
    if (!gate || !up || !x || N < 0 || C <= 0 || ld_gate < C || ld_up < C || ldx < C) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c) {
            const float v = silu_times_up(bf16_bits_to_f32(gate[n * ld_gate + c]), bf16_bits_to_f32(up[n * ld_up + c]));
            if (f32) f32[n * C + c] = v;
            x[n * ldx + c] = f32_to_bf16_bits(v);
        }
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
