/*
 * libqllm: the reassembled low-bit linear layer of QLLM (arXiv 2310.08041) for AMD MI355X (gfx950).
 *
 *   norm -> channel disassembly -> channel assembly -> per-token b-bit quantization
 *        -> integer GEMM against per-output-channel quantized weights -> dequantising epilogue
 *
 * C ABI.  All sizes are int64_t, all status returns int32_t (qllm_status, 0 = ok).  Unless a
 * parameter says "host", every pointer is a DEVICE pointer owned by the caller; the library
 * allocates no device memory and keeps no state.  Device work is enqueued on the HIP stream the
 * caller passes (a hipStream_t cast to void*, NULL = the default stream) and the call returns
 * without synchronising.  Outputs are overwritten, never accumulated into.  Arguments that can be
 * checked on the host (sizes, enums, null pointers, alignment) are checked before anything is
 * launched; nothing is launched when a check fails.  The contents of device arrays (the map, the
 * codes) are trusted: pass maps made by qllm_build_map_host or checked by qllm_check_map_host.
 *
 * Notation: N tokens, C_in channels entering the layer, C_out = K reassembled channels, O output
 * features, b bits, qmax = 2^b - 1.
 *
 * Fixed arithmetic.  The paper leaves precision open; this library computes
 *   - row statistics (sums for mean / variance / mean square) in fp64, rounded once to fp32;
 *   - every element-wise step in fp32, one rounding per operation, no fused multiply-add;
 *   - Eq. (2) as alpha = (max-min)/qmax (fp32), inv = 1/alpha (fp32),
 *     code = clamp(rne(x*inv) + beta, 0, qmax), beta = -rne(min*inv), where rne() rounds the
 *     EXACT product to the nearest integer, ties to even; a constant row takes alpha = 1;
 *   - integer accumulators exactly (int32), the epilogue bracket exactly (int64).
 */
#ifndef QLLM_H
#define QLLM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QLLM_OK = 0,
    QLLM_ERR_NULL = -1,      /* a required pointer is NULL */
    QLLM_ERR_SHAPE = -2,     /* a size is negative, zero where it may not be, inconsistent or above a limit */
    QLLM_ERR_BITS = -3,      /* bit width outside {4, 6, 8}, or an unsupported pair of widths */
    QLLM_ERR_DTYPE = -4,     /* unknown qllm_dtype / qllm_norm value */
    QLLM_ERR_MAP = -5,       /* malformed reassembly map or merge list */
    QLLM_ERR_ALIGN = -6,     /* a buffer or stride misses the required alignment */
    QLLM_ERR_WORKSPACE = -7, /* workspace missing or smaller than qllm_workspace_bytes says */
    QLLM_ERR_HIP = -8        /* the HIP runtime reported an error (launch, attribute, device) */
} qllm_status;

typedef enum { QLLM_F32 = 0, QLLM_BF16 = 1 } qllm_dtype;
typedef enum { QLLM_NORM_NONE = 0, QLLM_NORM_LAYER = 1, QLLM_NORM_RMS = 2 } qllm_norm;

/* Largest channel counts the fused kernel accepts (one token row is staged on chip in fp32). */
#define QLLM_MAX_CHANNELS 32768
/* Rows of packed codes are padded with zero codes to a multiple of this many codes. */
#define QLLM_K_PAD 256
/* The fused kernel handles channels in groups of this many. */
#define QLLM_MAP_GROUP 8
#define QLLM_PLAN_HEAD 16      /* int32 words of header at the start of a plan (qllm_plan_map_host) */

/*
 * Reassembly map: channel disassembly (Sec. 4.1.1, Eq. 3) followed by channel assembly
 * (Sec. 4.1.2, Eq. 4), composed into one sparse matrix in CSR form over the OUTPUT channels:
 *     x^[n, ch] = sum_{e = row_ptr[ch]}^{row_ptr[ch+1]-1} scale[e] * y[n, src[e]]
 * evaluated left to right in fp32.  A sub-channel of a channel split T ways has one entry with
 * scale 1/T; a channel merged from a group of g has g entries with scale 1/g; every other channel
 * has one entry with scale 1.  theta does not appear: it is consumed when the map is built.
 */
typedef struct {
    int64_t C_in;           /* channels of y */
    int64_t C_out;          /* reassembled channels, 1 .. QLLM_MAX_CHANNELS */
    int64_t nnz;            /* entries, >= C_out */
    const int32_t *row_ptr; /* [C_out+1] increasing, row_ptr[0] = 0, row_ptr[C_out] = nnz, no empty row */
    const int32_t *src;     /* [nnz] 0 <= src < C_in */
    const float *scale;     /* [nnz] */
    const int32_t *plan;    /* optional: device copy of the array qllm_plan_map_host makes from this very
                               map (an index of it for the fused kernel: which output channels copy an input
                               channel, which are computed, how groups of 8 are put together).  NULL: the
                               kernel walks the CSR for every channel (much slower). */
    int32_t plan_head[QLLM_PLAN_HEAD]; /* host copy of the plan's first QLLM_PLAN_HEAD words (ignored with NULL) */
} qllm_map;

/*
 * Packed codes (activations and weights use the same format).  A row holds K codes followed by
 * zero codes up to a multiple of QLLM_K_PAD; qllm_packed_row_bytes(K, bits) is the row stride.
 *   8 bit: one byte per code.
 *   4 bit: code 2j in bits 0..3, code 2j+1 in bits 4..7 of byte j.
 *   6 bit: codes 4j..4j+3 in the 24 bits of bytes 3j..3j+2, little endian, code 4j lowest.
 * Code buffers must be 16-byte aligned.
 */

/* Per-output-channel quantized weights, built offline (qllm_quantize_weight_host): Eq. (2) applied
 * to each output channel of the reassembled weight (Sec. 5, "Quantization settings"). */
typedef struct {
    int64_t O;              /* output features */
    int64_t K;              /* reassembled input channels; must equal map.C_out */
    int32_t bits;           /* 4, 6 or 8 */
    const uint8_t *codes;   /* [O, qllm_packed_row_bytes(K, bits)] */
    const float *scale;     /* [O] alpha_w */
    const int32_t *zero;    /* [O] beta_w */
    const int32_t *colsum;  /* [O] sum_k codes[o, k] */
    const uint8_t *tiles6;  /* optional, bits == 4 only: device copy of the codes in the layout qllm_pack_tiles6
                               makes, qllm_tiles6_bytes(O, K) bytes, 16-byte aligned.  With it (and room in the
                               workspace, see qllm_int_gemm) the GEMM runs on the FP6 matrix cores.  NULL: int8. */
    const uint8_t *tiles8;  /* optional, any bits (unused when the activations are 4-bit too): device copy of the
                               codes, one byte each, in the layout qllm_pack_tiles8 makes, qllm_tiles8_bytes(O, K)
                               bytes, 16-byte aligned.  With it (and room in the workspace) the GEMM of 6- and 8-bit
                               activations feeds the int8 matrix cores without unpacking anything on the way.
                               NULL: the packed codes are expanded inside the GEMM. */
} qllm_weight;

/* Per-token quantized activations: output of the fused kernel, input of the GEMM. */
typedef struct {
    uint8_t *codes;         /* [N, qllm_packed_row_bytes(K, bits)] */
    float *scale;           /* [N] alpha_x */
    int32_t *zero;          /* [N] beta_x (not clamped to [0, qmax]) */
    int32_t *rowsum;        /* [N] sum_k codes[n, k] */
} qllm_qact;

/* ------------------------------------------------------------------------------------------
 * Steps a1..a4 in one kernel: norm (the layer that precedes the runtime reassembly, Sec. 4.3),
 * channel disassembly (Eq. 3), channel assembly (Eq. 4), per-token asymmetric quantization (Eq. 2).
 *
 *   x        [N, ldx] row-major, x_dtype (QLLM_BF16 = raw bfloat16 bits); ldx >= C in elements.
 *   norm     LAYER: y = ((x-mu)*rstd)*gamma + beta, biased variance, beta may be NULL (no shift)
 *            RMS  : y = (x*rstd)*gamma        NONE: y = x (gamma, beta ignored)
 *   gamma, beta  [C] fp32.      eps is added to the variance / mean square under the root.
 *   map      map->C_in must equal C.
 *   bits     4, 6 or 8.
 *   out      caller-allocated; fully overwritten, padding codes included.
 * Errors: NULL / SHAPE / BITS / DTYPE / ALIGN / HIP as described above.  N == 0 is a no-op.
 * Rows whose values are not finite give unspecified codes.
 */
int32_t qllm_norm_reassemble_quant(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                   int32_t norm, const float *gamma, const float *beta, float eps,
                                   const qllm_map *map, int32_t bits, const qllm_qact *out,
                                   void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Steps a5..a6: Eq. (1) on the codes, acc[n,o] = sum_k a[n,k]*w[o,k] on the int8 matrix cores,
 * and the epilogue that undoes Eq. (2) on both operands,
 *   Y[n,o] = ((float)(acc - beta_x[n]*colsum_w[o] - beta_w[o]*rowsum_x[n] + K*beta_x[n]*beta_w[o])
 *             * alpha_x[n]) * alpha_w[o]                               (= quant(X^) quant(W^), Sec. 4.1.3)
 *
 *   a, a_bits   quantized activations [N, K]; a_bits must equal w->bits, or be 8 with w->bits 4.
 *   y           [N, ldy] y_dtype (fp32, or bf16 rounded to nearest even); ldy >= O in elements.
 *   acc_dump    NULL, or [N, O] int32 that receives the raw accumulators.
 *   workspace   scratch, 16-byte aligned, contents undefined afterwards.  qllm_gemm_workspace_bytes(N,
 *               w->K, w->O, a_bits) bytes serve every path; at least qllm_gemm_workspace_floor_bytes(...)
 *               are required (may be NULL when that is 0: it is non-zero only where the sum over K is
 *               split over workgroups), else QLLM_ERR_WORKSPACE.
 *
 * The FP6 path.  For 4-bit codes on both sides and N > 64 the same acc[n,o] is also available from the FP6
 * matrix cores at close to twice the int8 rate: a code c, zero-extended to 6 bits, is the E2M3 number c/8, the
 * products a*w/64 and all their partial sums (multiples of 1/64 below 2^18, K <= 74564) are exact in fp32, and
 * 64 times the fp32 accumulator is the integer accumulator of Eq. (1), bit for bit.  It is taken when
 * w->tiles6 is set and the workspace holds, behind the qllm_gemm_workspace_floor_bytes(...) bytes rounded up to a
 * multiple of 256, at least qllm_tiles6_bytes(N, w->K) bytes (the activations are re-laid into them first, a few
 * per cent of the GEMM's time); otherwise the int8 path runs.  Same results either way.
 *
 * Byte operands.  For the other bit pairs (6/6, 8/8, 8-bit activations on 4-bit weights; Sec. 5, "Quantization
 * settings") and N > 32 the int8 matrix cores can be fed straight from one-byte-per-code copies of both operands:
 * taken when w->tiles8 is set and the workspace holds at least qllm_tiles8_bytes(N, w->K) bytes (the activations
 * are re-laid into it first); otherwise the packed codes are expanded inside the GEMM.  Same results either way.
 * With qllm_gemm_workspace_bytes(...) bytes this path also splits the sum over K over workgroups where a small
 * batch would leave most of the chip idle (the parts' accumulators follow the activations' bytes in the workspace).
 */
int32_t qllm_int_gemm(const qllm_qact *a, int32_t a_bits, int64_t N, const qllm_weight *w, void *y,
                      int32_t y_dtype, int64_t ldy, int32_t *acc_dump, void *workspace,
                      int64_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * The whole layer a1..a6: qllm_norm_reassemble_quant into workspace, then qllm_int_gemm, on one
 * stream.  workspace: 256-byte aligned; qllm_workspace_bytes(N, map->C_out, w->O, a_bits) bytes serve every
 * path (the quantized activations, the GEMM's own need, and for 4-bit codes the room its FP6 path wants);
 * with less, down to qllm_workspace_floor_bytes(...), the layer still runs, the GEMM on its int8 path.
 * Arguments as in the two calls above.
 */
int32_t qllm_reassembled_linear(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                int32_t norm, const float *gamma, const float *beta, float eps,
                                const qllm_map *map, int32_t a_bits, const qllm_weight *w, void *y,
                                int32_t y_dtype, int64_t ldy, void *workspace, int64_t workspace_bytes,
                                void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * qllm_reassembled_linear for callers that cannot allocate device memory or have none to spare for a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without the workspace, same kernels, same results bit for bit; the workspace is a device array
 * inside the library, QLLM_STATIC_WORKSPACE_BYTES per GPU, held until the process ends.  The call allocates and
 * frees nothing.  QLLM_ERR_WORKSPACE if qllm_workspace_floor_bytes(N, map->C_out, w->O, a_bits) exceeds that size
 * (decode and small-batch shapes fit: 16 tokens x 8192 channels need 0.1 MB, 512 tokens x 28672 channels at 4
 * bits 7.4 MB).  All calls on one GPU share the array: two of them in flight at once on different streams race;
 * calls on one stream are ordered like any other work.  The first call on a device asks the runtime for the
 * array's address there (no allocation, but not under stream capture): make that call before capturing.
 */
#define QLLM_STATIC_WORKSPACE_BYTES (32 << 20)
int32_t qllm_reassembled_linear_static(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                       int32_t norm, const float *gamma, const float *beta, float eps,
                                       const qllm_map *map, int32_t a_bits, const qllm_weight *w, void *y,
                                       int32_t y_dtype, int64_t ldy, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Offline, on the device: which channels to merge (Sec. 4.1.2, Appendix A steps 1-2).  The caller
 * has split the candidates into set A and set B (Appendix A step 1; on the disassembled axis, even and
 * odd positions, sub-channels of split channels left out) and names each member's channel.  For every
 * member i of A this finds its nearest member of B under the distance of Eq. (5),
 *     D(i, j) = | x_i (W_i - W_j) / 2 + x_j (W_j - W_i) / 2 |^2 = |x_i - x_j|^2 |W_i - W_j|^2 / 4,
 * x_c = column c of y over the n calibration tokens, W_c = row c of W over the O output features.
 * Arithmetic in double precision on the fp64 matrix cores; ties go to the lower j.
 * With W == NULL (O, ldw ignored) the distance is the plain D(i, j) = |x_i - x_j|^2: matching on the
 * activations alone, for layers whose weights are not at hand.
 *   y        [n, ldy] fp32 activations after the norm (ldy >= C); W [C, ldw] fp32 (ldw >= O)
 *   chan_a   [nA], chan_b [nB] int32 channel numbers in [0, C) (device arrays, trusted)
 *   best_j   [nA] int32: index into chan_b;   best_d [nA] double: the distance
 *   workspace  qllm_match_workspace_bytes(nA, nB) bytes, 8-byte aligned
 * Errors: NULL / SHAPE (also nB == 0 with nA > 0) / WORKSPACE / ALIGN / HIP.  nA == 0 is a no-op.
 * qllm_select_edges_host (host pointers) is Appendix A step 3: the r shortest edges, ties to the lower
 * member of A; pick_out receives min(r, nA) indices into set A in ascending order and the count is
 * returned (negative = qllm_status).
 */
int64_t qllm_match_workspace_bytes(int64_t nA, int64_t nB);
int32_t qllm_match_nearest(const float *y, int64_t n, int64_t ldy, const float *W, int64_t C, int64_t O,
                           int64_t ldw, const int32_t *chan_a, int64_t nA, const int32_t *chan_b, int64_t nB,
                           int32_t *best_j, double *best_d, void *workspace, int64_t workspace_bytes,
                           void *hip_stream);
int64_t qllm_select_edges_host(const double *best_d, int64_t nA, int64_t r, int32_t *pick_out);

/* The host-side steps around that search.  HOST pointers.
 * qllm_matching_sets_host: Appendix A step 1 on the disassembled axis (channel c occupies num_split[c]
 *   adjacent positions): set A = even positions, set B = odd positions, and only channels that were not split
 *   take part (Sec. 4.1.2).  Outputs, each sized C by the caller: the members' channels and positions, in
 *   ascending order, and their counts.  QLLM_ERR_MAP for a split count below 1.
 * qllm_pairs_host: Appendix A step 3 in the indexing of the paper's run-time pseudo-code: the min(r, nA)
 *   shortest edges (ties to the lower member of A, as qllm_select_edges_host), written as src_idx[k] = number of
 *   the A-member among the even positions, dst_idx[k] = number of its B-member among the odd positions, ascending
 *   in src_idx: the arguments qllm_build_map_host takes.  best_j / best_d as qllm_match_nearest returns them
 *   (copied to the host).  Returns the count (negative = qllm_status).
 * qllm_theta_for_expansion_host: the largest float32 theta whose disassembly adds at least extra_target
 *   channels, sum_c (T_c - 1) >= extra_target (Sec. 5.2 fixes theta through the expansion ratio; the count never
 *   grows with theta).  QLLM_ERR_SHAPE if no theta above max(m) / 2^20 does.
 * qllm_theta_grid_host: Algorithm 1's candidates theta_p = min(m) + p / P (max(m) - min(m)), p = 1 .. P, formed in
 *   double and rounded once. */
int32_t qllm_matching_sets_host(const int32_t *num_split, int64_t C, int32_t *chan_a, int32_t *pos_a, int64_t *nA,
                                int32_t *chan_b, int32_t *pos_b, int64_t *nB);
int64_t qllm_pairs_host(const double *best_d, const int32_t *best_j, const int32_t *pos_a, const int32_t *pos_b, int64_t nA,
                        int64_t nB, int64_t r, int32_t *src_idx, int32_t *dst_idx);
int32_t qllm_theta_for_expansion_host(const float *chan_absmax, int64_t C, int64_t extra_target, float *theta);
int32_t qllm_theta_grid_host(const float *chan_absmax, int64_t C, int32_t P, float *thetas);

/* What Algorithm 1 scores a candidate theta with, for one linear layer: the squared error of the quantized
 * layer's output against the full-precision layer (the paper scores a whole attention block through Eq. (6);
 * a single linear layer has no softmax to go through, so the error is taken at the layer's own output).
 * DEVICE pointers.
 *   qllm_linear_f64   out[n, o] = sum_c y[n, c] W[c, o], products and sums in double, c ascending.
 *                     y [N, ldy] fp32, W [C, ldw] fp32, out [N, ldo] double.
 *   qllm_sq_error     *result (one device double) = sum over n, o of (got[n, o] - ref[n, o])^2 in double, in a
 *                     fixed order.  got [N, ldg] fp32 or bf16, ref [N, ldr] double; workspace of
 *                     qllm_sq_error_workspace_bytes(N) bytes, 8-byte aligned. */
int32_t qllm_linear_f64(const float *y, int64_t N, int64_t C, int64_t ldy, const float *W, int64_t O, int64_t ldw,
                        double *out, int64_t ldo, void *hip_stream);
int64_t qllm_sq_error_workspace_bytes(int64_t N);
int32_t qllm_sq_error(const void *got, int32_t got_dtype, int64_t N, int64_t O, int64_t ldg, const double *ref,
                      int64_t ldr, double *result, void *workspace, int64_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * The gated activation that feeds a down projection in the models of Sec. 5 (LLaMA): x = silu(gate) * up with
 * silu(g) = g / (1 + e^-g); the producer of the input that the layer above then reassembles and quantizes.
 *   gate, up  device, [N, ld_gate] / [N, ld_up] raw bfloat16 bits; x device, [N, ldx] bfloat16; ld* >= C in elements.
 * The arithmetic is fixed (fp32, one rounding per operation, an expf by range reduction and a degree-5
 * polynomial, a correctly rounded division; within 2 ulp of silu before the product): the same bits on every run
 * and as the CPU statement of the same sequence.  16-byte aligned buffers with strides that are multiples of 8
 * take the fast path (16-byte accesses); anything 2-byte aligned works.  Gates below -88 give a zero.
 * Errors: NULL / SHAPE / ALIGN / HIP.  N == 0: no-op.
 */
int32_t qllm_swiglu(const void *gate, int64_t ld_gate, const void *up, int64_t ld_up, int64_t N, int64_t C, void *x,
                    int64_t ldx, void *hip_stream);

/* Sizes.  Negative return = qllm_status. */
int64_t qllm_packed_row_bytes(int64_t K, int32_t bits);
int64_t qllm_gemm_workspace_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits);
int64_t qllm_gemm_workspace_floor_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits);
int64_t qllm_workspace_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits);
int64_t qllm_workspace_floor_bytes(int64_t N, int64_t K, int64_t O, int32_t a_bits);

/* ------------------------------------------------------------------------------------------
 * 4-bit codes re-laid for the FP6 matrix-core path of qllm_int_gemm (Eq. 1 on the codes; see there).
 *   codes   device, [rows, qllm_packed_row_bytes(K, 4)] in the packed format above, 16-byte aligned.
 *   tiles   device, qllm_tiles6_bytes(rows, K) bytes, 16-byte aligned, fully overwritten:
 *           rows in blocks of 16 (the last one filled with zero codes), K in tiles of 128 codes up to the
 *           padded row length; block b, K-tile t is the 1536 bytes at (b * tiles_per_row + t) * 1536; for
 *           l = 0..63, r = l % 16, q = l / 16 the 32 codes 128 t + 32 q + e (e = 0..31) of row 16 b + r form a
 *           192-bit little-endian number with code e in bits 6 e .. 6 e + 3 (bits 6 e + 4, 6 e + 5 zero); its
 *           first 16 bytes lie at 16 l of the block, its last 8 at 1024 + 8 l.
 * For a weight: once, offline, into qllm_weight.tiles6.  Errors: NULL / SHAPE / ALIGN / HIP.  rows == 0: no-op.
 */
int64_t qllm_tiles6_bytes(int64_t rows, int64_t K);
int32_t qllm_pack_tiles6(const uint8_t *codes, int64_t rows, int64_t K, uint8_t *tiles, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * Codes re-laid one byte each for the byte-operand path of qllm_int_gemm (Eq. 1 on the codes; see there).
 *   codes   device, [rows, qllm_packed_row_bytes(K, bits)] in the packed format above, 16-byte aligned; bits 4, 6, 8.
 *   tiles   device, qllm_tiles8_bytes(rows, K) bytes, 16-byte aligned, fully overwritten:
 *           rows in blocks of 16, K in tiles of 64 codes (ceil(K / 64) of them); block b, K-tile t is the 1024 bytes
 *           at (b * tiles_per_row + t) * 1024; for l = 0..63, r = l % 16, q = l / 16 the code 64 t + 16 q + e
 *           (e = 0..15) of row 16 b + r is the byte at 16 l + e: the code itself for 4- and 6-bit codes, the code
 *           XOR 0x80 (code - 128 as a signed byte) for 8-bit codes.  Rows past the matrix and places past K are
 *           zero bytes.
 * For a weight: once, offline, into qllm_weight.tiles8.  Errors: NULL / BITS / SHAPE / ALIGN / HIP.  rows == 0: no-op.
 */
int64_t qllm_tiles8_bytes(int64_t rows, int64_t K);
int32_t qllm_pack_tiles8(const uint8_t *codes, int32_t bits, int64_t rows, int64_t K, uint8_t *tiles, void *hip_stream);

const char *qllm_status_string(int32_t status);

/* After a call on this thread returned QLLM_ERR_HIP: the HIP runtime's own name for what went wrong
 * and the library step that met it (a static or thread-local string; "" if there was none). */
const char *qllm_last_hip_error(void);

/* ------------------------------------------------------------------------------------------
 * Offline helpers.  HOST pointers throughout; plain CPU code; no GPU needed.
 */

/* Builds the map from the calibration statistics, in the paper's own terms:
 *   T_c = max(1, ceil(chan_absmax[c] / theta))                      (Sec. 4.1.1)
 *   the disassembled axis (sum_c T_c positions) is split into set A (even positions) and set B
 *   (odd positions); pair k merges A-member src_idx[k] into B-member dst_idx[k] (Sec. 4.1.2,
 *   Appendix A, and the indexing of the runtime pseudo-code figure); several A-members may share
 *   a B-member; sub-channels of a split channel may not take part (QLLM_ERR_MAP).
 * Outputs (caller-sized: row_ptr C + extra + 1, src/scale C + extra entries, where
 * extra = sum(T_c - 1) can be obtained by a first call with row_ptr == NULL): the CSR arrays,
 * C_out = C + extra - r, nnz = C + extra, the T vector (num_split_out may be NULL).
 * Entry order inside a merged row: destination first, then sources by ascending position.
 */
int32_t qllm_build_map_host(const float *chan_absmax, int64_t C, float theta, const int32_t *src_idx,
                            const int32_t *dst_idx, int64_t r, int32_t *row_ptr, int32_t *src,
                            float *scale, int64_t *C_out, int64_t *nnz, int32_t *num_split_out);

/* The comparison of Sec. 4.1.2: the same disassembly (Eq. 3), but the r listed members of set A (src_idx, as for
 * qllm_build_map_host) are DROPPED instead of merged into a member of set B, so every row of the map has one
 * entry and nnz = sum(T) - r = C_out.  Arguments, the sizing call (row_ptr == NULL) and errors as for
 * qllm_build_map_host.  The result is an ordinary map: the kernels, qllm_plan_map_host and
 * qllm_quantize_weight_host take it like any other. */
int32_t qllm_build_pruned_map_host(const float *chan_absmax, int64_t C, float theta, const int32_t *src_idx, int64_t r,
                                   int32_t *row_ptr, int32_t *src, float *scale, int64_t *C_out, int64_t *nnz,
                                   int32_t *num_split);

/* Indexes a CSR map for the fused kernel (see qllm_map.plan).  Call once with plan == NULL to get
 * *plan_len (int32 words) and *n_general, then with plan pointing at that many words.  The plan
 * depends only on the map; upload it next to the CSR arrays and keep its first QLLM_PLAN_HEAD words
 * in qllm_map.plan_head.
 *
 * The kernel quantizes every input channel where it sits and then moves CODES, so the plan sorts the
 * output channels into three kinds:
 *   copied    one entry with scale exactly 1: the channel's code is the code of its source channel;
 *   computed  one entry with another scale (a sub-channel, Eq. 3) or two entries of equal scale (a merged
 *             pair, Eq. 4): the value is formed from the sources and quantized on its own;
 *   long      any other row: summed entry by entry, then as a computed channel (rows of up to 64 entries by
 *             the lanes of one wavefront in one go, longer ones block by block).
 * and the groups of 8 output channels into "plain" (8 copied channels with consecutive sources d .. d+7:
 * one 8-code window of the input-order codes) and "composite" (anything else: a few windows, each masked
 * to the channels it supplies, plus the codes of its computed and long channels).
 *
 * Layout (int32 words; every part starts at a multiple of 4 words, in this order):
 *   [0..15]  header: magic, version, C_in, C_out, n_work = groups of 8 output channels including the zero
 *            padding to 256 codes, n_comp = composite groups (*n_general), n_chunks = ceil(C_in/8), n_long,
 *            n_pub, n_spec, n_dest, n_segw, offset of chunks, plan_len, n_xl = rows of more than 64 entries,
 *            n_xle = their entries
 *   work     [n_work] at word 16: kind << 30 | group << 17 | field.  kind 0 (plain): field = d; kind 1
 *            (composite): field = offset of the group's segment list inside `segs`; kind 2: padding (all
 *            codes zero).  Sorted by kind, then by group
 *   chunks   [n_chunks]: bits 0..7: bit j set = input channel 8*chunk + j is the source of some copied
 *            channel; bits 8..31: p if some computed or long channel reads a channel of this chunk (the
 *            kernel then stages the chunk's x at floats 8p .. 8p+7 of its on-chip table; p = 0 ..
 *            n_pub-1 in chunk order), 0xffffff otherwise.  Float 8*n_pub of that table is a zero.  A map whose
 *            lists could not be held on chip at every setting of the kernel has all chunks staged instead
 *            (n_pub == n_chunks, p == chunk): a staged position is then the channel number
 *   spec     [n_spec][2]: a computed channel: {s0 | s1 << 16, scale}, s = staged position of the source
 *            channel (s1 = 8*n_pub, the zero, for one entry)
 *   dest     [n_dest]: where the code of computed channel i (i < n_spec), of long row i - n_spec, or (last) of a
 *            row of more than 64 entries goes: number of its composite group << 3 | position in the group
 *   longs    [n_long][4]: {s, value slot or -1, scale, pos | most << 8}: entry pos (0, 1, ...) of a long row;
 *            the row's last entry names its slot in `dest`, the others -1.  The kernel gives entry e to lane
 *            e % 64 of a wavefront and adds a row up lane by lane, so the table holds padding entries
 *            {0, -1, 0.0f, 0 | most << 8} wherever a row would otherwise straddle a multiple of 64; n_long
 *            counts them; most = the largest pos among the (up to) 64 entries that share a wavefront
 *   segs     [n_segw]: per composite group {count | number << 8, then count x {d, mask, 0}}: the group's
 *            copied channels at positions k with bit k of mask set have sources d + k (d may be negative or
 *            reach past C_in - 8: only the masked positions are real channels)
 *   recs     [n_comp][8]: the same once more as records of fixed size, by composite group number:
 *            {count | offset of the group's list in segs << 8, d0, mask0, d1, mask1, group, 0, 0} (what the kernel
 *            reads for the first two segments; a group with more takes the rest from segs)
 *   xlrows   [n_xl][4]: a row of more than 64 entries: {its first entry in xlent, entries, its slot in dest, 0}
 *   xlent    [n_xle][2]: {s, scale}, the rows' entries in order
 * QLLM_ERR_MAP: malformed map, or one whose counts do not fit the fields above.
 */
int32_t qllm_plan_map_host(const int32_t *row_ptr, const int32_t *src, const float *scale, int64_t C_in,
                           int64_t C_out, int32_t *plan, int64_t *plan_len, int64_t *n_general);

/* Verifies a host copy of a map: monotone row_ptr without empty rows, sources in range, finite scales. */
int32_t qllm_check_map_host(const int32_t *row_ptr, const int32_t *src, const float *scale,
                            int64_t C_in, int64_t C_out, int64_t nnz);

/* Folds the reassembly into a preceding linear layer (Appendix B): when the activations that enter
 * the quantized layer are the output of a linear layer y = x Wp^T + bp, disassembly and assembly can
 * be applied to that layer's output channels once, offline, instead of to every token at run time:
 *   Wp^[ch, :] = sum over the entries e of map row ch of scale[e] * Wp[src[e], :]      (same for bp)
 * (columns of the paper's W^{l-1} divided by T and repeated for a split channel, averaged for merged
 * ones).  The run-time path is then plain quantization + GEMM: call the library with norm NONE and
 * the identity map on x Wp^^T + bp^.
 * All pointers host.  Wp is [C_in, K_prev] row-major fp32 (one row per OUTPUT channel of the preceding
 * layer = input channel of the quantized one), bp is [C_in] or NULL; W_out is [C_out, K_prev], b_out
 * [C_out] (ignored when bp is NULL).  Sums are formed in double precision in entry order and rounded
 * once.  QLLM_ERR_MAP for a malformed map (checked as by qllm_check_map_host). */
int32_t qllm_fold_linear_host(const float *Wp, const float *bp, int64_t C_in, int64_t K_prev,
                              const int32_t *row_ptr, const int32_t *src, const float *scale, int64_t C_out,
                              float *W_out, float *b_out);

/* Reassembles and quantizes the weights of one layer (offline half of Sec. 4.1.1 / 4.1.2):
 *   W^[ch, :] = sum of W[src[e], :] over the entries e of map row ch (rows duplicated for
 *   sub-channels as in Eq. (3), summed for merged channels as in Eq. (4)), then Eq. (2) per output
 *   channel over ch.  W is [C_in, O] row-major fp32 (input channels x output features, the layout
 *   of Eq. (1)).  Outputs: codes [O, qllm_packed_row_bytes(C_out, bits)] packed, scale/zero/colsum [O].
 */
int32_t qllm_quantize_weight_host(const float *W, int64_t C_in, int64_t O, const int32_t *row_ptr,
                                  const int32_t *src, int64_t C_out, int32_t bits, uint8_t *codes,
                                  float *scale, int32_t *zero, int32_t *colsum);

/* Packs / unpacks rows of one-byte codes into the storage format above (R rows of K codes). */
int32_t qllm_pack_codes_host(const uint8_t *codes, int64_t R, int64_t K, int32_t bits, uint8_t *packed);
int32_t qllm_unpack_codes_host(const uint8_t *packed, int64_t R, int64_t K, int32_t bits, uint8_t *codes);

/* Which form of the fused kernel qllm_norm_reassemble_quant runs for this map and these arguments (a host-side
 * answer: nothing is launched, no device memory is read; map->plan may be a device pointer, map->plan_head is
 * read on the host).  The per-channel work of Sec. 4.1 (Eq. 3, Eq. 4) is the same in all three; they differ in
 * where the map's lists live while a row is worked on.
 *   QLLM_FUSED_WALKS_MAP       no plan, or it fits neither way: every output channel walks its CSR row
 *   QLLM_FUSED_LISTS_IN_LDS    the planned kernel with the plan's lists copied to LDS once per workgroup
 *   QLLM_FUSED_LISTS_STREAMED  the planned kernel reading the lists from global memory (L2) row by row: maps
 *                              with thousands of computed channels on the longest rows
 * x is assumed 16-byte aligned; ldx in elements as in qllm_norm_reassemble_quant; has_beta != 0: a LayerNorm shift
 * is given.  Returns one of the three (>= 0) or a QLLM_ERR_* (< 0) for arguments qllm_norm_reassemble_quant
 * would reject too. */
#define QLLM_FUSED_WALKS_MAP 0
#define QLLM_FUSED_LISTS_IN_LDS 1
#define QLLM_FUSED_LISTS_STREAMED 2
int32_t qllm_fused_kernel_choice(const qllm_map *map, int32_t x_dtype, int64_t N, int64_t ldx, int32_t norm,
                                 int32_t has_beta, int32_t bits);

/* ------------------------------------------------------------------------------------------
 * Calibration statistic on the device: the norm of each row as in qllm_norm_reassemble_quant,
 * then absmax[c] = max(absmax[c], max_n |y[n,c]|) (Sec. 4.1.1 "max(|x_M|)"; vector m of Algorithm 1).
 * absmax [C] fp32 must be initialised by the caller (zeros for a fresh statistic).  y_dump, if not
 * NULL, receives the first n_dump rows of y as [n_dump, C] fp32.
 */
int32_t qllm_norm_channel_absmax(const void *x, int32_t x_dtype, int64_t N, int64_t C, int64_t ldx,
                                 int32_t norm, const float *gamma, const float *beta, float eps,
                                 float *absmax, float *y_dump, int64_t n_dump, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* QLLM_H */
