// Offline channel matching on the device: Appendix A steps 1-2 (every member of set A gets an edge to
// its most similar member of set B) with the distance of Sec. 4.1.2, Eq. (5).
//
// Eq. (5) is the squared norm of the error that merging channels i and j leaves in the layer's
// output, x_i (W_i - W_j) / 2 + x_j (W_j - W_i) / 2 = (x_i - x_j) (W_i - W_j)^T / 2, an outer product of
// a vector over the calibration tokens and a vector over the output features, so
//     D(i, j) = |x_i - x_j|^2 |W_i - W_j|^2 / 4,    |a - b|^2 = |a|^2 + |b|^2 - 2 a.b.
// The two sets of inner products are Gram matrices: dense contractions, done here on the fp64 matrix
// cores (v_mfma_f64_16x16x4_f64) so that the argmin is taken in the precision the definition is
// written in.  Nothing of size |A| x |B| is ever stored: a workgroup owns 64 members of A, walks over
// B in tiles of 128, forms both Gram tiles, the distances, and keeps a running minimum per row.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "qllm.h"

extern "C" void qllm_note_hip_error(const char *step, const char *name);

namespace {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int TA = 64, TB = 128, KT = 32, THREADS = 256;
// The fp64 tiles of the register path: K-steps of KTX values, row stride KTX + 1 doubles (odd, against bank
// conflicts), two buffers of both tiles.  KTX = 32: 101376 bytes, one workgroup per CU.  The kernel whose weight
// pass goes straight into LDS runs its token pass with KTX = 16 (52224 bytes), so that its LDS need is the weight
// ring's and two workgroups share a CU.
constexpr size_t tile_lds(int ktx) { return (size_t)2 * (TA + TB) * (ktx + 1) * sizeof(double); }

struct MatchArgs {
    const float *y;  // [n, ldy]: activations, token-major
    const float *w;  // [C, ldw]: weights, one row per input channel
    int64_t ldy, ldw;
    int32_t n, O, nA, nB;
    const int32_t *chan_a, *chan_b;
    const double *norms; // workspace: |x|^2 of A members [nA], |W|^2 of A [nA], |x|^2 of B [nB], |W|^2 of B [nB]
    int32_t *best_j;
    double *best_d;
    // the members of set B are dealt out to `splits` workgroups per tile of A; each writes its own
    // minimum here ([splits][nA]) and match_combine_kernel takes the minimum of those
    int32_t splits;
    double *part_d;
    int32_t *part_j;
};

// ---- squared norms of every set member's activation column and weight row, in double
__global__ __launch_bounds__(THREADS) void match_norms_kernel(const MatchArgs g, double *out)
{
    __shared__ double red[2][THREADS / 64];
    const int m = blockIdx.x, tid = threadIdx.x;
    const bool in_a = m < g.nA;
    const int c = in_a ? g.chan_a[m] : g.chan_b[m - g.nA];
    double sx = 0.0, sw = 0.0;
    for (int t = tid; t < g.n; t += THREADS) {
        const double v = (double)g.y[(int64_t)t * g.ldy + c];
        sx += v * v;
    }
    if (g.w) {
        const float *wr = g.w + (int64_t)c * g.ldw;
        for (int k = tid; k < g.O; k += THREADS) {
            const double v = (double)wr[k];
            sw += v * v;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        sx += __shfl_xor(sx, off);
        sw += __shfl_xor(sw, off);
    }
    if ((tid & 63) == 0) {
        red[0][tid >> 6] = sx;
        red[1][tid >> 6] = sw;
    }
    __syncthreads();
    if (tid == 0) {
        double a = 0.0, b = 0.0;
        for (int q = 0; q < THREADS / 64; ++q) {
            a += red[0][q];
            b += red[1][q];
        }
        if (in_a) {
            out[m] = a;
            out[g.nA + m] = b;
        } else {
            out[2 * (int64_t)g.nA + (m - g.nA)] = a;
            out[2 * (int64_t)g.nA + g.nB + (m - g.nA)] = b;
        }
    }
}

// One K-step of operands: 64 x 32 values of the A tile (8 per lane), 128 x 32 of the B tile (16 per lane).
// XPASS: element (member i, token t) = y[t][chan[i]], consecutive lanes take consecutive members;
// otherwise element (member i, feature k) = w[chan[i]][k], a lane takes four consecutive features
// (one 16-byte load when VEC: rows 16-byte aligned; four 4-byte loads otherwise).
template <bool XPASS, bool VEC, int ROWS, int PER>
__device__ __forceinline__ void fetch_tile(const MatchArgs &g, const int32_t *chan, int k0, int tid, float (&p)[PER])
{
    const int K = XPASS ? g.n : g.O;
    if constexpr (XPASS) {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = tid + q * THREADS, i = e & (ROWS - 1), k = e / ROWS;
            const bool ok = k0 + k < K;
            const float v = g.y[(int64_t)(ok ? k0 + k : 0) * g.ldy + chan[i]];
            p[q] = ok ? v : 0.0f;
        }
    } else {
#pragma unroll
        for (int q = 0; q < PER / 4; ++q) {
            const int e = tid + q * THREADS, i = e / (KT / 4), k = 4 * (e % (KT / 4));
            const float *row = g.w + (int64_t)chan[i] * g.ldw;
            if (VEC && k0 + k + 3 < K) {
                const float4 v = *reinterpret_cast<const float4 *>(row + k0 + k);
                p[4 * q] = v.x; p[4 * q + 1] = v.y; p[4 * q + 2] = v.z; p[4 * q + 3] = v.w;
            } else {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const bool ok = k0 + k + d < K;
                    const float v = row[ok ? k0 + k + d : 0];
                    p[4 * q + d] = ok ? v : 0.0f;
                }
            }
        }
    }
}

template <bool XPASS, int ROWS, int PAD, int PER>
__device__ __forceinline__ void stage_tile(double *tile, int tid, const float (&p)[PER])
{
    if constexpr (XPASS) {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = tid + q * THREADS, i = e & (ROWS - 1), k = e / ROWS;
            tile[i * PAD + k] = (double)p[q];
        }
    } else {
#pragma unroll
        for (int q = 0; q < PER / 4; ++q) {
            const int e = tid + q * THREADS, i = e / (KT / 4), k = 4 * (e % (KT / 4));
#pragma unroll
            for (int d = 0; d < 4; ++d) tile[i * PAD + k + d] = (double)p[4 * q + d];
        }
    }
}

// acc[ti][tj] += A tile rows 16 ti.. times B tile rows 32 wave + 16 tj.., over K (n tokens or O features),
// in K-steps of KTX values (the weight rows' 16-byte loads are laid out for KTX == KT)
template <bool XPASS, bool VEC, int KTX>
__device__ __forceinline__ void gram_pass(const MatchArgs &g, const int32_t *ca, const int32_t *cb, double *tiles, int tid,
                                          v4d (&acc)[4][2])
{
    static_assert(XPASS || KTX == KT, "weight rows are fetched in K-steps of KT");
    constexpr int PAD = KTX + 1, NA_STEP = TA * KTX / THREADS, NB_STEP = TB * KTX / THREADS;
    double *as = tiles, *bs = tiles + 2 * TA * PAD;
    const int lane = tid & 63, wave = tid >> 6;
    const int K = XPASS ? g.n : g.O;
    const int steps = (K + KTX - 1) / KTX;
    float pa[NA_STEP], pb[NB_STEP];
    fetch_tile<XPASS, VEC, TA, NA_STEP>(g, ca, 0, tid, pa);
    fetch_tile<XPASS, VEC, TB, NB_STEP>(g, cb, 0, tid, pb);
    for (int s = 0; s < steps; ++s) {
        double *a_buf = as + (s & 1) * TA * PAD, *b_buf = bs + (s & 1) * TB * PAD;
        stage_tile<XPASS, TA, PAD, NA_STEP>(a_buf, tid, pa);
        stage_tile<XPASS, TB, PAD, NB_STEP>(b_buf, tid, pb);
        // one barrier per step: the buffer written now was last read two steps ago, before the previous barrier
        __syncthreads();
        if (s + 1 < steps) {
            fetch_tile<XPASS, VEC, TA, NA_STEP>(g, ca, (s + 1) * KTX, tid, pa);
            fetch_tile<XPASS, VEC, TB, NB_STEP>(g, cb, (s + 1) * KTX, tid, pb);
        }
#pragma unroll
        for (int kk = 0; kk < KTX / 4; ++kk) {
            double a[4], b[2];
#pragma unroll
            for (int ti = 0; ti < 4; ++ti) a[ti] = a_buf[(16 * ti + (lane & 15)) * PAD + 4 * kk + (lane >> 4)];
#pragma unroll
            for (int tj = 0; tj < 2; ++tj) b[tj] = b_buf[(32 * wave + 16 * tj + (lane & 15)) * PAD + 4 * kk + (lane >> 4)];
#pragma unroll
            for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                for (int tj = 0; tj < 2; ++tj)
                    acc[ti][tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
        }
    }
    __syncthreads(); // the next pass starts writing buffer 0 again
}

// The weight pass when every row allows 16-byte loads and O is a multiple of the K-step: the operands
// go from global memory straight into LDS (global_load_lds_dwordx4: lane l of a wave lands at the
// wave's LDS base + 16 l), as fp32, two K-steps ahead in a ring of three stages, and are widened to
// double when the matrix-core operands are read.  No staging registers, no conversion and store pass.
// Three stages (72 KB) and the token pass in K-steps of 16 leave room for a second workgroup on the CU:
// two waves per SIMD, so that one's wait for its operand reads is the other's matrix-core time.
// A stage holds 192 rows (64 of the A tile, 128 of the B tile) of 32 floats; a wave load covers 8 rows;
// the 16-byte chunk c of row R sits at position c ^ ((R >> 1) & 7), chosen on the global side (which
// chunk a lane fetches), so that the 64 lanes of an operand read fall on 64 different banks.
constexpr int MAX_SPLITS = 16;
constexpr int STAGE_F = (TA + TB) * KT, NSTAGE = 3;                 // floats per stage (24 KB), stages
constexpr int KTX_DMA = 16;                                         // K-step of the token pass in the same kernel
constexpr size_t RING_LDS = (size_t)NSTAGE * STAGE_F * sizeof(float);
constexpr int WAIT_VM6_LGKM0 = 6 | (7 << 4) | (0 << 8);            // s_waitcnt vmcnt(6) lgkmcnt(0)
constexpr int WAIT_VM0_ONLY = 0 | (7 << 4) | (15 << 8);            // s_waitcnt vmcnt(0)
static_assert(tile_lds(KTX_DMA) <= RING_LDS, "the token pass's fp64 tiles fit where the fp32 ring is");

__device__ __forceinline__ void gram_pass_w_dma(const MatchArgs &g, const int32_t *ca, const int32_t *cb, float *ring, int tid,
                                                v4d (&acc)[4][2])
{
    const int lane = tid & 63, wave = tid >> 6;
    const int steps = g.O / KT;
    // this wave's six loads per K-step: blocks wave, wave + 4, .. of 8 rows each (blocks 0..7: A tile)
    const float *src[6];
#pragma unroll
    for (int t = 0; t < 6; ++t) {
        const int row = 8 * (wave + 4 * t) + (lane >> 3);
        const int chan = row < TA ? ca[row] : cb[row - TA];
        src[t] = g.w + (int64_t)chan * g.ldw + 4 * ((lane & 7) ^ ((row >> 1) & 7));
    }
    auto fetch = [&](int s, int stage) { // K-step s (clamped to the last one) -> stage s % 3
        const int sc = min(s, steps - 1);
        float *dst = ring + stage * STAGE_F;
#pragma unroll
        for (int t = 0; t < 6; ++t)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[t] + (int64_t)sc * KT),
                                             (__attribute__((address_space(3))) void *)(dst + 8 * (wave + 4 * t) * KT), 16, 0, 0);
    };
    const int r = lane & 15, kq = lane >> 4, f = (r >> 1) & 7;
    fetch(0, 0);
    fetch(1, 1);
    int stage = 0; // s % 3
    for (int s = 0; s < steps; ++s) {
        // loads complete in order: at most the newest step outstanding = step s has landed (this wave's
        // share; the barrier adds the others').  The stage written next was read in step s - 1.
        __builtin_amdgcn_s_waitcnt(WAIT_VM6_LGKM0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        fetch(s + 2, stage == 0 ? 2 : stage - 1);
        const float *sb = ring + stage * STAGE_F;
        stage = stage == 2 ? 0 : stage + 1;
#pragma unroll
        for (int kk = 0; kk < KT / 4; ++kk) {
            const int off = 4 * (kk ^ f) + kq;
            double a[4], b[2];
#pragma unroll
            for (int ti = 0; ti < 4; ++ti) a[ti] = (double)sb[(16 * ti + r) * KT + off];
#pragma unroll
            for (int tj = 0; tj < 2; ++tj) b[tj] = (double)sb[(TA + 32 * wave + 16 * tj + r) * KT + off];
#pragma unroll
            for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                for (int tj = 0; tj < 2; ++tj)
                    acc[ti][tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
        }
    }
    // the loads past the last step went to stages nobody reads; they must have landed before the
    // memory is used for anything else (the next tile's first pass, or another workgroup)
    __builtin_amdgcn_s_waitcnt(WAIT_VM0_ONLY);
    __syncthreads();
}

// MODE 0: 4-byte loads; 1: 16-byte loads of weight rows; 2: weight rows straight into LDS.
// L2: no weights, the distance is |x_i - x_j|^2 alone.
template <int MODE, bool L2 = false>
__global__ __launch_bounds__(THREADS, MODE == 2 ? 2 : 1) void match_nearest_kernel(const MatchArgs g)
{
    extern __shared__ __align__(16) double tiles[];
    constexpr int KTX = MODE == 2 ? KTX_DMA : KT; // K-step of the token pass
    __shared__ double na_x[TA], na_w[TA], nb_x[TB], nb_w[TB];
    __shared__ int32_t ca[TA], cb[TB];
    __shared__ double fin_d[THREADS / 64][TA];
    __shared__ int32_t fin_j[THREADS / 64][TA];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroup number -> (tile of A, split of B).  Workgroups are handed to the eight XCDs round robin
    // and each XCD has its own L2: the `splits` workgroups that share a tile of A (and sweep the same
    // 64 weight rows, each against its own part of B) get numbers that are equal modulo 8, so that
    // they run side by side on one XCD and the rows come from HBM once for all of them.
    const int group = blockIdx.x / (8 * g.splits), in_group = blockIdx.x % (8 * g.splits);
    const int a_tile = group * 8 + (in_group & 7), split = in_group >> 3;
    const int n_a_tiles = (g.nA + TA - 1) / TA, n_b_tiles = (g.nB + TB - 1) / TB;
    if (a_tile >= n_a_tiles) return; // the last group of eight may be short; whole workgroups leave, before any barrier
    const int a0 = a_tile * TA;
    const int b_begin = (int)((int64_t)n_b_tiles * split / g.splits) * TB;
    const int b_end = min(g.nB, (int)((int64_t)n_b_tiles * (split + 1) / g.splits) * TB);
    if (tid < TA) {
        const int m = min(a0 + tid, g.nA - 1); // past the end: the last member again, its result is dropped
        ca[tid] = g.chan_a[m];
        na_x[tid] = g.norms[m];
        na_w[tid] = g.norms[g.nA + m];
    }

    // running minimum for the 16 rows this lane sees: rows 16 ti + (lane >> 4) + 4 r
    double best_d[4][4];
    int32_t best_j[4][4];
#pragma unroll
    for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            best_d[ti][r] = __builtin_huge_val();
            best_j[ti][r] = 0x7fffffff;
        }

    for (int b0 = b_begin; b0 < b_end; b0 += TB) {
        __syncthreads(); // everybody is done with the previous tile's cb / norms
        if (tid < TB) {
            const int m = min(b0 + tid, g.nB - 1);
            cb[tid] = g.chan_b[m];
            nb_x[tid] = g.norms[2 * (int64_t)g.nA + m];
            nb_w[tid] = g.norms[2 * (int64_t)g.nA + g.nB + m];
        }
        __syncthreads();
        v4d gx[4][2], gw[4][2];
#pragma unroll
        for (int ti = 0; ti < 4; ++ti)
#pragma unroll
            for (int tj = 0; tj < 2; ++tj) gx[ti][tj] = gw[ti][tj] = v4d{0.0, 0.0, 0.0, 0.0};
        gram_pass<true, MODE != 0, KTX>(g, ca, cb, tiles, tid, gx);
        if constexpr (L2) {
        } else if constexpr (MODE == 2) {
            gram_pass_w_dma(g, ca, cb, reinterpret_cast<float *>(tiles), tid, gw);
        } else {
            gram_pass<false, MODE != 0, KT>(g, ca, cb, tiles, tid, gw);
        }
        // distances of this tile; element r of an accumulator: row (lane >> 4) + 4 r, column lane & 15
        // (checked against the oracle: the fp64 operation interleaves the rows of its four result registers)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj) {
            const int jl = 32 * wave + 16 * tj + (lane & 15), j = b0 + jl;
            const double bx = nb_x[jl], bw = nb_w[jl];
#pragma unroll
            for (int ti = 0; ti < 4; ++ti)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int il = 16 * ti + (lane >> 4) + 4 * r;
                    double sx = na_x[il] + bx - 2.0 * gx[ti][tj][r];
                    double sw = na_w[il] + bw - 2.0 * gw[ti][tj][r];
                    sx = sx < 0.0 ? 0.0 : sx; // round-off of a difference that is zero
                    sw = sw < 0.0 ? 0.0 : sw;
                    const double d = L2 ? sx : 0.25 * sx * sw;
                    if (j < g.nB && (d < best_d[ti][r] || (d == best_d[ti][r] && j < best_j[ti][r]))) {
                        best_d[ti][r] = d;
                        best_j[ti][r] = j;
                    }
                }
        }
    }

    // the 16 lanes that share lane >> 4 hold different columns of the same rows; then the four waves
#pragma unroll
    for (int ti = 0; ti < 4; ++ti)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            double d = best_d[ti][r];
            int32_t j = best_j[ti][r];
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                const double od = __shfl_xor(d, off);
                const int32_t oj = __shfl_xor(j, off);
                if (od < d || (od == d && oj < j)) {
                    d = od;
                    j = oj;
                }
            }
            if ((lane & 15) == 0) {
                fin_d[wave][16 * ti + (lane >> 4) + 4 * r] = d;
                fin_j[wave][16 * ti + (lane >> 4) + 4 * r] = j;
            }
        }
    __syncthreads();
    if (tid < TA && a0 + tid < g.nA) {
        double d = fin_d[0][tid];
        int32_t j = fin_j[0][tid];
#pragma unroll
        for (int w = 1; w < THREADS / 64; ++w)
            if (fin_d[w][tid] < d || (fin_d[w][tid] == d && fin_j[w][tid] < j)) {
                d = fin_d[w][tid];
                j = fin_j[w][tid];
            }
        g.part_d[(int64_t)split * g.nA + a0 + tid] = d; // a split without members of B leaves (inf, INT_MAX)
        g.part_j[(int64_t)split * g.nA + a0 + tid] = j;
    }
}

// minimum over the splits; their parts of B ascend with the split number, so ties go to the lower split
__global__ __launch_bounds__(THREADS) void match_combine_kernel(const MatchArgs g)
{
    const int64_t i = (int64_t)blockIdx.x * THREADS + threadIdx.x;
    if (i >= g.nA) return;
    double d = g.part_d[i];
    int32_t j = g.part_j[i];
    for (int s = 1; s < g.splits; ++s) {
        const double ds = g.part_d[(int64_t)s * g.nA + i];
        if (ds < d) {
            d = ds;
            j = g.part_j[(int64_t)s * g.nA + i];
        }
    }
    g.best_d[i] = d;
    g.best_j[i] = j;
}

} // namespace

extern "C" int64_t qllm_match_workspace_bytes(int64_t nA, int64_t nB)
{
    if (nA < 0 || nB < 0) return QLLM_ERR_SHAPE;
    // squared norms (two per member), and a (distance, index) pair per member of A and split of B
    return 2 * (nA + nB) * (int64_t)sizeof(double) + MAX_SPLITS * nA * (int64_t)(sizeof(double) + sizeof(int32_t));
}

extern "C" int32_t qllm_match_nearest(const float *y, int64_t n, int64_t ldy, const float *W, int64_t C, int64_t O,
                                      int64_t ldw, const int32_t *chan_a, int64_t nA, const int32_t *chan_b,
                                      int64_t nB, int32_t *best_j, double *best_d, void *workspace,
                                      int64_t workspace_bytes, void *hip_stream)
{
    if (!y || !chan_a || !chan_b || !best_j || !best_d) return QLLM_ERR_NULL;
    if (n <= 0 || C <= 0 || ldy < C || nA < 0 || nB < 0) return QLLM_ERR_SHAPE;
    if (W && (O <= 0 || ldw < O)) return QLLM_ERR_SHAPE;
    if (n > INT32_MAX || O > INT32_MAX || C > INT32_MAX || nA > INT32_MAX - TA || nB > INT32_MAX - TB) return QLLM_ERR_SHAPE;
    if (nA == 0) return QLLM_OK;
    if (nB == 0) return QLLM_ERR_SHAPE; // nothing to match against
    if (workspace_bytes < qllm_match_workspace_bytes(nA, nB) || !workspace) return QLLM_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 7u) return QLLM_ERR_ALIGN;
    MatchArgs g{};
    g.y = y; g.w = W; g.ldy = ldy; g.ldw = ldw;
    g.n = (int32_t)n; g.O = (int32_t)O; g.nA = (int32_t)nA; g.nB = (int32_t)nB;
    g.chan_a = chan_a; g.chan_b = chan_b;
    g.norms = static_cast<const double *>(workspace);
    g.best_j = best_j; g.best_d = best_d;
    const int64_t n_b_tiles = (nB + TB - 1) / TB;
    g.splits = (int32_t)(n_b_tiles < MAX_SPLITS ? n_b_tiles : MAX_SPLITS);
    g.part_d = static_cast<double *>(workspace) + 2 * (nA + nB);
    g.part_j = reinterpret_cast<int32_t *>(g.part_d + (int64_t)MAX_SPLITS * nA);
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    hipLaunchKernelGGL(match_norms_kernel, dim3((unsigned)(nA + nB)), dim3(THREADS), 0, stream, g,
                       static_cast<double *>(workspace));
    // 16-byte loads of weight rows where every row allows them, straight into LDS where the K-steps come out even
    const bool vec = W && (reinterpret_cast<uintptr_t>(W) & 15u) == 0 && (ldw & 3) == 0;
    const int mode = !W ? 3 : vec ? (O % KT == 0 ? 2 : 1) : 0; // 3: plain L2, no weights
    const void *fn = mode == 3   ? reinterpret_cast<const void *>(&match_nearest_kernel<0, true>)
                     : mode == 2 ? reinterpret_cast<const void *>(&match_nearest_kernel<2>)
                     : mode == 1 ? reinterpret_cast<const void *>(&match_nearest_kernel<1>)
                                 : reinterpret_cast<const void *>(&match_nearest_kernel<0>);
    const size_t lds = mode == 2 ? RING_LDS : tile_lds(KT);
    { // the LDS limit is raised once per kernel; later calls (also under stream capture) only launch
        static std::mutex lock;
        static bool raised[4] = {false, false, false, false};
        std::lock_guard<std::mutex> hold(lock);
        if (!raised[mode]) {
            const hipError_t ea = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (ea != hipSuccess) {
                (void)hipGetLastError();
                qllm_note_hip_error("channel matching: raising the LDS limit", hipGetErrorName(ea));
                return QLLM_ERR_HIP;
            }
            raised[mode] = true;
        }
    }
    const int64_t n_a_tiles = (nA + TA - 1) / TA;
    const dim3 grid((unsigned)((n_a_tiles + 7) / 8 * 8 * g.splits));
    if (mode == 3) hipLaunchKernelGGL((match_nearest_kernel<0, true>), grid, dim3(THREADS), lds, stream, g);
    else if (mode == 2) hipLaunchKernelGGL(match_nearest_kernel<2>, grid, dim3(THREADS), lds, stream, g);
    else if (mode == 1) hipLaunchKernelGGL(match_nearest_kernel<1>, grid, dim3(THREADS), lds, stream, g);
    else hipLaunchKernelGGL(match_nearest_kernel<0>, grid, dim3(THREADS), lds, stream, g);
    hipLaunchKernelGGL(match_combine_kernel, dim3((unsigned)((nA + THREADS - 1) / THREADS)), dim3(THREADS), 0, stream, g);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        qllm_note_hip_error("channel matching: launch", hipGetErrorName(e));
        return QLLM_ERR_HIP;
    }
    return QLLM_OK;
}
