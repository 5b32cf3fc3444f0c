// Offline, host-side half of libqllm: building the reassembly map from calibration statistics and
// reassembling + quantizing the weights.  Plain C++, no GPU calls.
//
// Paper: channel disassembly Sec. 4.1.1 (Eq. 3), channel assembly Sec. 4.1.2 (Eq. 4) with the
// bipartite A/B split of Appendix A, uniform quantizer Eq. (2), per-output-channel weights
// (Sec. 5 "Quantization settings"), weight-side rewrites of Appendix B.
#include "qllm.h"
#include "plan_budget.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

inline bool bits_supported(int32_t bits) { return bits == 4 || bits == 6 || bits == 8; }

// What every disassembled position is, and what happens to it in assembly.
struct Position {
    int32_t channel;   // source channel of y
    int32_t splits;    // T of that channel
    int32_t target;    // B-position this A-position is merged into, or -1
    int32_t members;   // 1 + number of A-positions merged into this position
};

template <class F>
void parallel_blocks(int64_t n_blocks, F &&body)
{
    unsigned hw = std::thread::hardware_concurrency();
    int64_t n_thr = std::max<int64_t>(1, std::min<int64_t>({(int64_t)(hw ? hw : 1), 16, n_blocks}));
    if (n_thr == 1) {
        for (int64_t b = 0; b < n_blocks; ++b) body(b);
        return;
    }
    std::vector<std::thread> pool;
    for (int64_t t = 0; t < n_thr; ++t)
        pool.emplace_back([&, t] {
            for (int64_t b = t; b < n_blocks; b += n_thr) body(b);
        });
    for (auto &th : pool) th.join();
}

// Eq. (2) for one vector held with a stride; rne() acts on the exact product (fp32 x fp32 fits fp64).
struct QuantParams {
    float alpha, inv;
    int64_t beta;
};

inline int64_t rne_product(float a, float b) { return (int64_t)std::nearbyint((double)a * (double)b); }

inline QuantParams quant_params(float mn, float mx, int qmax)
{
    QuantParams p;
    const float range = mx - mn;
    p.alpha = range > 0.0f ? range / (float)qmax : 1.0f;
    p.inv = 1.0f / p.alpha;
    p.beta = -rne_product(mn, p.inv);
    const int64_t lim = std::numeric_limits<int32_t>::max();
    p.beta = std::min(lim, std::max(-lim, p.beta));
    return p;
}

inline uint32_t quant_code(float v, const QuantParams &p, int qmax)
{
    int64_t q = rne_product(v, p.inv) + p.beta;
    return (uint32_t)std::min<int64_t>(qmax, std::max<int64_t>(0, q));
}

inline void put_code(uint8_t *row, int64_t k, int32_t bits, uint32_t code)
{
    if (bits == 8) {
        row[k] = (uint8_t)code;
    } else if (bits == 4) {
        row[k >> 1] |= (uint8_t)(code << ((k & 1) * 4));
    } else { // 6 bit: four codes per three bytes
        const int64_t bit = k * 6;
        const int sh = (int)(bit & 7);
        row[bit >> 3] |= (uint8_t)(code << sh);
        if (sh > 2) row[(bit >> 3) + 1] |= (uint8_t)(code >> (8 - sh));
    }
}

inline uint32_t get_code(const uint8_t *row, int64_t k, int32_t bits)
{
    if (bits == 8) return row[k];
    if (bits == 4) return (row[k >> 1] >> ((k & 1) * 4)) & 15u;
    const int64_t bit = k * 6;
    const int sh = (int)(bit & 7);
    uint32_t w = row[bit >> 3];
    if (sh > 2) w |= (uint32_t)row[(bit >> 3) + 1] << 8;
    return (w >> sh) & 63u;
}

} // namespace

// Text of the last HIP failure seen by this thread (written by the launch sites).
thread_local char g_hip_error[160] = "";

extern "C" void qllm_note_hip_error(const char *step, const char *name)
{
    std::snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", step, name);
}

extern "C" {

const char *qllm_last_hip_error(void) { return g_hip_error; }

int64_t qllm_packed_row_bytes(int64_t K, int32_t bits)
{
    if (!bits_supported(bits)) return QLLM_ERR_BITS;
    if (K <= 0) return QLLM_ERR_SHAPE;
    return round_up(K, QLLM_K_PAD) * bits / 8;
}

const char *qllm_status_string(int32_t status)
{
    switch (status) {
    case QLLM_OK: return "ok";
    case QLLM_ERR_NULL: return "a required pointer is NULL";
    case QLLM_ERR_SHAPE: return "bad size or leading dimension";
    case QLLM_ERR_BITS: return "unsupported bit width";
    case QLLM_ERR_DTYPE: return "unknown dtype or norm kind";
    case QLLM_ERR_MAP: return "malformed reassembly map";
    case QLLM_ERR_ALIGN: return "buffer or stride not aligned";
    case QLLM_ERR_WORKSPACE: return "workspace missing or too small";
    case QLLM_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int32_t qllm_plan_map_host(const int32_t *row_ptr, const int32_t *src, const float *scale, int64_t C_in,
                           int64_t C_out, int32_t *plan, int64_t *plan_len, int64_t *n_general)
{
    if (!row_ptr || !src || !scale || !plan_len || !n_general) return QLLM_ERR_NULL;
    if (C_in <= 0 || C_out <= 0 || C_in > QLLM_MAX_CHANNELS || C_out > QLLM_MAX_CHANNELS) return QLLM_ERR_SHAPE;
    const int64_t G = QLLM_MAP_GROUP, HEAD = QLLM_PLAN_HEAD;
    const int64_t n_groups = (C_out + G - 1) / G, n_chunks = (C_in + G - 1) / G;
    constexpr int64_t WAVE = 64;
    enum { PASS = 0, COMPACT = 1, LONG = 2 };
    // What an output channel is to the fused kernel: a copy of one input channel (its code is the code of
    // that input channel), a value of one entry or of two entries of equal scale, or a longer sum.
    auto classify = [&](int64_t ch) {
        const int32_t e0 = row_ptr[ch], n = row_ptr[ch + 1] - e0;
        if (n == 1) return scale[e0] == 1.0f ? PASS : COMPACT;
        return n == 2 && std::memcmp(&scale[e0], &scale[e0 + 1], 4) == 0 ? COMPACT : LONG;
    };
    auto plain_source = [&](int64_t g) -> int32_t { // first source of a plain group, or -1
        const int64_t c0 = g * G;
        if (c0 + G > C_out) return -1;
        const int32_t e0 = row_ptr[c0];
        if (row_ptr[c0 + G] - e0 != G) return -1;
        for (int j = 0; j < G; ++j)
            if (row_ptr[c0 + j] != e0 + j || src[e0 + j] != src[e0] + j || scale[e0 + j] != 1.0f) return -1;
        return src[e0] + G <= C_in && src[e0] >= 0 ? src[e0] : -1;
    };
    // A long row occupies consecutive lanes of ONE wavefront of the kernel, so the table of long-row entries is
    // padded wherever a row would otherwise straddle a multiple of 64.
    auto place_long = [&](int64_t at, int64_t n) { return at % WAVE + n > WAVE ? (at + WAVE - 1) / WAVE * WAVE : at; };

    // ---- first pass: sizes
    std::vector<int32_t> pub_slot((size_t)n_chunks, -1), desc((size_t)n_groups);
    std::vector<uint8_t> pass((size_t)n_chunks, 0);
    int64_t n_comp = 0, n_long = 0, n_spec = 0, n_rows_long = 0, n_segw = 0, n_xl = 0, n_xle = 0;
    std::vector<std::pair<int32_t, int32_t>> long_rows; // {entries, channel}
    for (int64_t ch = 0; ch < C_out; ++ch) {
        const int32_t e0 = row_ptr[ch], n = row_ptr[ch + 1] - e0;
        if (n < 1) return QLLM_ERR_MAP;
        for (int32_t e = e0; e < e0 + n; ++e)
            if (src[e] < 0 || src[e] >= C_in) return QLLM_ERR_MAP;
        const int kind = classify(ch);
        if (kind == PASS) {
            pass[(size_t)(src[e0] / G)] |= (uint8_t)(1 << (src[e0] % G));
            continue;
        }
        for (int32_t e = e0; e < e0 + n; ++e) pub_slot[(size_t)(src[e] / G)] = 0; // the kernel stages this chunk's x
        if (kind == COMPACT) {
            ++n_spec;
        } else if (n > WAVE) { // too long for one pass of a wavefront: listed apart and summed block by block
            ++n_xl;
            n_xle += n;
        } else {
            long_rows.push_back({n, (int32_t)ch});
            ++n_rows_long;
        }
    }
    // The wavefront that owns 64 entries of the table repeats its addition as often as the longest row among them
    // has entries, so rows of like length go together: longest first (channel order among equals).
    std::stable_sort(long_rows.begin(), long_rows.end(), [](const auto &x, const auto &y) { return x.first > y.first; });
    std::vector<int32_t> long_start((size_t)C_out, -1);
    for (const auto &row : long_rows) {
        n_long = place_long(n_long, row.first);
        long_start[(size_t)row.second] = (int32_t)n_long;
        n_long += row.first;
    }
    for (int64_t g = 0; g < n_groups; ++g) {
        const int32_t d = desc[(size_t)g] = plain_source(g);
        if (d >= 0) continue;
        // segments of a composite group: the copied channels, grouped by d = source - position
        int32_t ds[8];
        int n_seg = 0;
        for (int64_t ch = g * G; ch < std::min(C_out, (g + 1) * G); ++ch) {
            if (classify(ch) != PASS) continue;
            const int32_t dk = src[row_ptr[ch]] - (int32_t)(ch - g * G);
            int s = 0;
            while (s < n_seg && ds[s] != dk) ++s;
            if (s == n_seg) ds[n_seg++] = dk;
        }
        n_segw += 1 + 3 * n_seg;
        ++n_comp;
    }
    // Chunks that hold a source of a computed channel are staged.  If the lists would then not fit in LDS next
    // to the row at the kernel's most demanding setting (8-bit codes, LayerNorm with a shift), all chunks are: a
    // staged position then is the channel number, which lets the kernel fetch gamma and beta of a source by it
    // while the lists stay in global memory.
    int64_t n_pub = 0;
    for (int64_t c = 0; c < n_chunks; ++c) n_pub += pub_slot[(size_t)c] == 0;
    {
        const int64_t units = std::max(n_chunks, (C_out + QLLM_K_PAD - 1) / QLLM_K_PAD * QLLM_K_PAD / G);
        const qllm_detail::PlanCounts p{n_comp, n_long, n_pub, n_chunks, n_spec, n_spec + n_rows_long + n_xl, n_segw};
        if (qllm_detail::fused_lists_lds_bytes(p, 2, 3, units + 256) > qllm_detail::FUSED_MAX_LDS)
            std::fill(pub_slot.begin(), pub_slot.end(), 0);
    }
    n_pub = 0;
    for (int64_t c = 0; c < n_chunks; ++c)
        if (pub_slot[(size_t)c] == 0) pub_slot[(size_t)c] = (int32_t)n_pub++;
    const int64_t n_dest = n_spec + n_rows_long + n_xl;
    if (n_long > 0xffffff || G * n_pub + 4 > 0xffff || n_segw > 0x1ffff || n_comp > 0xffffff || n_xle > 0xffffff) return QLLM_ERR_MAP;
    *n_general = n_comp;
    const int64_t n_work = (C_out + QLLM_K_PAD - 1) / QLLM_K_PAD * QLLM_K_PAD / G; // groups incl. zero padding
    auto round4 = [](int64_t v) { return (v + 3) / 4 * 4; };
    const int64_t off_work = HEAD, off_chunks = round4(off_work + n_work), off_spec = round4(off_chunks + n_chunks);
    const int64_t off_dest = round4(off_spec + 2 * n_spec), off_longs = round4(off_dest + n_dest);
    const int64_t off_segs = off_longs + 4 * n_long, off_recs = round4(off_segs + n_segw);
    const int64_t off_xlrows = off_recs + 8 * n_comp, off_xlent = off_xlrows + 4 * n_xl;
    *plan_len = off_xlent + 2 * n_xle;
    if (!plan) return QLLM_OK;

    // ---- second pass: the tables
    std::fill(plan, plan + *plan_len, 0);
    const int64_t head[QLLM_PLAN_HEAD] = {0x514c4d50, 8, C_in, C_out, n_work, n_comp, n_chunks, n_long,
                                          n_pub, n_spec, n_dest, n_segw, off_chunks, *plan_len, n_xl, n_xle};
    for (int64_t k = 0; k < HEAD; ++k) plan[k] = (int32_t)head[k];
    int32_t *work = plan + off_work, *chunks = plan + off_chunks, *spec = plan + off_spec, *dest = plan + off_dest;
    int32_t *longs = plan + off_longs, *segs = plan + off_segs, *recs = plan + off_recs;
    int32_t *xlrows = plan + off_xlrows, *xlent = plan + off_xlent;
    for (int64_t e = 0; e < n_long; ++e) longs[4 * e + 1] = -1; // padding entries are {0, -1, 0.0f, 0}
    const uint32_t zero_at = (uint32_t)(G * n_pub); // the staged zero sits right after the published chunks
    auto staged = [&](int32_t channel) { return (uint32_t)(pub_slot[(size_t)(channel / G)] * G + channel % G); };
    for (int64_t c = 0; c < n_chunks; ++c)
        chunks[c] = (int32_t)(((uint32_t)pub_slot[(size_t)c] << 8) | pass[(size_t)c]); // no slot: 0xffffff
    int64_t comp = 0, spec_at = 0, long_row = 0, long_at = 0, seg_at = 0, xl_row = 0, xl_at = 0;
    for (int64_t g = 0; g < n_groups; ++g) {
        if (desc[(size_t)g] >= 0) continue;
        int32_t *hdr = segs + seg_at;
        int n_seg = 0;
        for (int64_t ch = g * G; ch < std::min(C_out, (g + 1) * G); ++ch) {
            const int k = (int)(ch - g * G);
            const int32_t e0 = row_ptr[ch], n = row_ptr[ch + 1] - e0;
            const int kind = classify(ch);
            if (kind == PASS) {
                const int32_t dk = src[e0] - k;
                int s = 0;
                while (s < n_seg && hdr[1 + 3 * s] != dk) ++s;
                if (s == n_seg) hdr[1 + 3 * n_seg++] = dk;
                hdr[2 + 3 * s] |= 1 << k;
            } else if (kind == COMPACT) { // {staged source | second staged source << 16, scale}; destination apart
                const uint32_t second = n == 2 ? staged(src[e0 + 1]) : zero_at;
                spec[2 * spec_at] = (int32_t)(staged(src[e0]) | (second << 16));
                std::memcpy(&spec[2 * spec_at + 1], &scale[e0], 4);
                dest[spec_at++] = (int32_t)((comp << 3) | k);
            } else if (n > WAVE) { // {first entry, entries, value slot, 0} and the entries {staged source, scale}
                const int64_t id = n_spec + n_rows_long + xl_row;
                dest[id] = (int32_t)((comp << 3) | k);
                xlrows[4 * xl_row] = (int32_t)xl_at;
                xlrows[4 * xl_row + 1] = n;
                xlrows[4 * xl_row + 2] = (int32_t)id;
                ++xl_row;
                for (int32_t e = e0; e < e0 + n; ++e, ++xl_at) {
                    xlent[2 * xl_at] = (int32_t)staged(src[e]);
                    std::memcpy(&xlent[2 * xl_at + 1], &scale[e], 4);
                }
            } else { // entries go to the table of long rows: {staged source, value slot or -1, scale, position}
                long_at = long_start[(size_t)ch];
                const int64_t id = n_spec + long_row++;
                dest[id] = (int32_t)((comp << 3) | k);
                for (int32_t e = e0; e < e0 + n; ++e, ++long_at) {
                    longs[4 * long_at] = (int32_t)staged(src[e]);
                    longs[4 * long_at + 1] = e == e0 + n - 1 ? (int32_t)id : -1;
                    std::memcpy(&longs[4 * long_at + 2], &scale[e], 4);
                    longs[4 * long_at + 3] = e - e0;
                }
            }
        }
        hdr[0] = (int32_t)((uint32_t)n_seg | ((uint32_t)comp << 8));
        // the same group as one record of fixed size: {count | list offset << 8, d0, mask0, d1, mask1, group, 0, 0}
        int32_t *rc = recs + 8 * comp;
        rc[0] = (int32_t)((uint32_t)n_seg | ((uint32_t)seg_at << 8));
        for (int sg = 0; sg < std::min(n_seg, 2); ++sg) {
            rc[1 + 2 * sg] = hdr[1 + 3 * sg];
            rc[2 + 2 * sg] = hdr[2 + 3 * sg];
        }
        rc[5] = (int32_t)g;
        desc[(size_t)g] = (int32_t)(-(seg_at + 1));
        seg_at += 1 + 3 * n_seg;
        ++comp;
    }
    // every entry of a block of 64 also carries the block's largest position: the number of additions
    // the wavefront that owns the block has to make
    for (int64_t b0 = 0; b0 < n_long; b0 += WAVE) {
        int32_t most = 0;
        for (int64_t e = b0; e < std::min(n_long, b0 + WAVE); ++e) most = std::max(most, longs[4 * e + 3]);
        for (int64_t e = b0; e < std::min(n_long, b0 + WAVE); ++e) longs[4 * e + 3] |= most << 8;
    }
    // work list of the code-producing step, one entry per group of 8 output channels (zero padding
    // included): kind << 30 | group << 17 | field.  Plain groups first, then composite groups, then
    // padding groups, so that all but two wavefronts of the kernel are of one kind.
    int64_t at = 0;
    for (int64_t g = 0; g < n_groups; ++g)
        if (desc[g] >= 0) work[at++] = (int32_t)(((uint32_t)g << 17) | (uint32_t)desc[g]);
    for (int64_t g = 0; g < n_groups; ++g)
        if (desc[g] < 0) work[at++] = (int32_t)((1u << 30) | ((uint32_t)g << 17) | (uint32_t)(-(desc[g] + 1)));
    for (int64_t g = n_groups; g < n_work; ++g) work[at++] = (int32_t)((2u << 30) | ((uint32_t)g << 17));
    return QLLM_OK;
}

// ---------------------------------------------------------------- offline: thresholds, matching sets, edges

namespace {

inline int64_t split_count(float m, float theta)
{
    const double q = std::ceil((double)m / (double)theta); // Sec. 4.1.1: T = ceil(max|x| / theta), at least 1
    return q < 1.0 ? 1 : (int64_t)q;
}

int64_t extra_channels(const float *m, int64_t C, float theta)
{
    int64_t extra = 0;
    for (int64_t c = 0; c < C; ++c) extra += split_count(m[c], theta) - 1;
    return extra;
}

inline float from_bits(uint32_t u)
{
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

inline uint32_t to_bits(float f)
{
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return u;
}

} // namespace

int32_t qllm_theta_for_expansion_host(const float *chan_absmax, int64_t C, int64_t extra_target, float *theta)
{
    if (!chan_absmax || !theta) return QLLM_ERR_NULL;
    if (C <= 0 || extra_target <= 0) return QLLM_ERR_SHAPE;
    float top = 0.0f;
    for (int64_t c = 0; c < C; ++c) {
        if (!(chan_absmax[c] >= 0.0f) || !std::isfinite(chan_absmax[c])) return QLLM_ERR_SHAPE;
        top = std::max(top, chan_absmax[c]);
    }
    // Channels added never increase with theta, and positive floats order like their bit patterns: step
    // through the patterns between max(m) / 2^20 (every T at most 2^20) and max(m) (nothing is split).
    uint32_t lo = to_bits(top * 9.5367431640625e-07f), hi = to_bits(top);
    if (top <= 0.0f || extra_channels(chan_absmax, C, from_bits(lo)) < extra_target) return QLLM_ERR_SHAPE;
    while (hi - lo > 1) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if (extra_channels(chan_absmax, C, from_bits(mid)) >= extra_target) lo = mid;
        else hi = mid;
    }
    *theta = from_bits(lo);
    return QLLM_OK;
}

int32_t qllm_theta_grid_host(const float *chan_absmax, int64_t C, int32_t P, float *thetas)
{
    if (!chan_absmax || !thetas) return QLLM_ERR_NULL;
    if (C <= 0 || P <= 0) return QLLM_ERR_SHAPE;
    double lo = chan_absmax[0], hi = chan_absmax[0];
    for (int64_t c = 1; c < C; ++c) {
        lo = std::min(lo, (double)chan_absmax[c]);
        hi = std::max(hi, (double)chan_absmax[c]);
    }
    for (int32_t p = 1; p <= P; ++p) thetas[p - 1] = (float)(lo + ((double)p / (double)P) * (hi - lo));
    return QLLM_OK;
}

int32_t qllm_matching_sets_host(const int32_t *num_split, int64_t C, int32_t *chan_a, int32_t *pos_a, int64_t *nA,
                                int32_t *chan_b, int32_t *pos_b, int64_t *nB)
{
    if (!num_split || !chan_a || !pos_a || !nA || !chan_b || !pos_b || !nB) return QLLM_ERR_NULL;
    if (C <= 0) return QLLM_ERR_SHAPE;
    int64_t at = 0, na = 0, nb = 0; // position on the disassembled axis
    for (int64_t c = 0; c < C; ++c) {
        const int32_t T = num_split[c];
        if (T < 1) return QLLM_ERR_MAP;
        if (T == 1) { // only channels that were not split take part
            if (at > INT32_MAX) return QLLM_ERR_SHAPE;
            if (at % 2 == 0) {
                chan_a[na] = (int32_t)c;
                pos_a[na++] = (int32_t)at;
            } else {
                chan_b[nb] = (int32_t)c;
                pos_b[nb++] = (int32_t)at;
            }
        }
        at += T;
    }
    *nA = na;
    *nB = nb;
    return QLLM_OK;
}

int64_t qllm_pairs_host(const double *best_d, const int32_t *best_j, const int32_t *pos_a, const int32_t *pos_b, int64_t nA,
                        int64_t nB, int64_t r, int32_t *src_idx, int32_t *dst_idx)
{
    if (nA < 0 || nB < 0 || r < 0) return QLLM_ERR_SHAPE;
    if (r == 0 || nA == 0 || nB == 0) return 0;
    if (!best_d || !best_j || !pos_a || !pos_b || !src_idx || !dst_idx) return QLLM_ERR_NULL;
    std::vector<int32_t> pick((size_t)std::min(r, nA));
    const int64_t n = qllm_select_edges_host(best_d, nA, r, pick.data());
    if (n < 0) return n;
    for (int64_t k = 0; k < n; ++k) {
        const int32_t i = pick[(size_t)k], j = best_j[i];
        if (j < 0 || j >= nB || pos_a[i] % 2 != 0 || pos_b[j] % 2 != 1) return QLLM_ERR_MAP;
        src_idx[k] = pos_a[i] / 2;       // member number in set A: the even positions
        dst_idx[k] = (pos_b[j] - 1) / 2; // member number in set B: the odd positions
    }
    return n;
}

int32_t qllm_check_map_host(const int32_t *row_ptr, const int32_t *src, const float *scale,
                            int64_t C_in, int64_t C_out, int64_t nnz)
{
    if (!row_ptr || !src || !scale) return QLLM_ERR_NULL;
    if (C_in <= 0 || C_out <= 0 || nnz < C_out) return QLLM_ERR_SHAPE;
    if (row_ptr[0] != 0 || row_ptr[C_out] != nnz) return QLLM_ERR_MAP;
    for (int64_t c = 0; c < C_out; ++c)
        if (row_ptr[c + 1] <= row_ptr[c]) return QLLM_ERR_MAP;
    for (int64_t e = 0; e < nnz; ++e)
        if (src[e] < 0 || src[e] >= C_in || !std::isfinite(scale[e])) return QLLM_ERR_MAP;
    return QLLM_OK;
}

} // extern "C"

namespace {

// Disassembly (Eq. 3) followed by assembly (Eq. 4) as a CSR map; with `prune` the listed A-members are dropped
// instead of merged into their B-members (the comparison of Sec. 4.1.2) and dst_idx is not read.
int32_t build_map(const float *chan_absmax, int64_t C, float theta, const int32_t *src_idx, const int32_t *dst_idx,
                  int64_t r, bool prune, int32_t *row_ptr, int32_t *src, float *scale, int64_t *C_out, int64_t *nnz,
                  int32_t *num_split_out)
{
    if (!chan_absmax || !C_out || !nnz) return QLLM_ERR_NULL;
    if (r > 0 && (!src_idx || (!prune && !dst_idx))) return QLLM_ERR_NULL;
    if (C <= 0 || r < 0 || !(theta > 0.0f)) return QLLM_ERR_SHAPE;

    // T = ceil(max|x| / theta), never below 1 (Sec. 4.1.1)
    std::vector<int32_t> T((size_t)C);
    int64_t total = 0;
    for (int64_t c = 0; c < C; ++c) {
        const double q = std::ceil((double)chan_absmax[c] / (double)theta);
        if (!(q <= 1e9)) return QLLM_ERR_SHAPE; // also catches NaN
        T[c] = q >= 1.0 ? (int32_t)q : 1;
        total += T[c];
    }
    if (total > std::numeric_limits<int32_t>::max() || r > total) return QLLM_ERR_SHAPE;
    *C_out = total - r;
    *nnz = prune ? total - r : total;
    if (num_split_out) std::copy(T.begin(), T.end(), num_split_out);
    if (!row_ptr) return QLLM_OK; // sizing call
    if (!src || !scale) return QLLM_ERR_NULL;
    if (*C_out <= 0) return QLLM_ERR_SHAPE;

    std::vector<Position> pos((size_t)total);
    {
        int64_t p = 0;
        for (int64_t c = 0; c < C; ++c)
            for (int32_t t = 0; t < T[c]; ++t) pos[p++] = Position{(int32_t)c, T[c], -1, 1};
    }
    const int64_t n_a = (total + 1) / 2, n_b = total / 2;
    for (int64_t k = 0; k < r; ++k) {
        if (src_idx[k] < 0 || src_idx[k] >= n_a) return QLLM_ERR_MAP;
        Position &a = pos[2 * (size_t)src_idx[k]];
        if (a.target != -1) return QLLM_ERR_MAP; // an A-member can be merged (dropped) once
        if (a.splits != 1) return QLLM_ERR_MAP;  // sub-channels stay out of assembly
        if (prune) {
            a.target = -2; // dropped
            continue;
        }
        if (dst_idx[k] < 0 || dst_idx[k] >= n_b) return QLLM_ERR_MAP;
        Position &b = pos[2 * (size_t)dst_idx[k] + 1];
        if (b.splits != 1) return QLLM_ERR_MAP;
        a.target = 2 * dst_idx[k] + 1;
        b.members += 1;
    }
    // sources of every destination, ascending: bucket the A-positions by target
    std::vector<int32_t> first((size_t)total + 1, 0);
    for (int64_t p = 0; p < total; p += 2)
        if (pos[p].target >= 0) first[(size_t)pos[p].target + 1] += 1;
    for (int64_t p = 0; p < total; ++p) first[p + 1] += first[p];
    std::vector<int32_t> merged_src((size_t)std::max<int64_t>(r, 1));
    {
        std::vector<int32_t> fill(first.begin(), first.end() - 1);
        for (int64_t p = 0; p < total; p += 2)
            if (pos[p].target >= 0) merged_src[fill[pos[p].target]++] = (int32_t)p;
    }
    int64_t ch = 0, e = 0;
    for (int64_t p = 0; p < total; ++p) {
        const Position &q = pos[p];
        if (q.target != -1) continue; // merged away, or dropped
        row_ptr[ch++] = (int32_t)e;
        if (q.members == 1) {
            src[e] = q.channel;
            scale[e++] = (float)(1.0 / (double)q.splits);
        } else {
            const float s = (float)(1.0 / (double)q.members);
            src[e] = q.channel;
            scale[e++] = s;
            for (int32_t i = first[p]; i < first[p + 1]; ++i) {
                src[e] = pos[merged_src[i]].channel;
                scale[e++] = s;
            }
        }
    }
    row_ptr[ch] = (int32_t)e;
    if (ch != *C_out || e != *nnz) return QLLM_ERR_MAP;
    return QLLM_OK;
}

} // namespace

extern "C" {

int32_t qllm_build_map_host(const float *chan_absmax, int64_t C, float theta, const int32_t *src_idx,
                            const int32_t *dst_idx, int64_t r, int32_t *row_ptr, int32_t *src,
                            float *scale, int64_t *C_out, int64_t *nnz, int32_t *num_split_out)
{
    return build_map(chan_absmax, C, theta, src_idx, dst_idx, r, false, row_ptr, src, scale, C_out, nnz, num_split_out);
}

int32_t qllm_build_pruned_map_host(const float *chan_absmax, int64_t C, float theta, const int32_t *src_idx, int64_t r,
                                   int32_t *row_ptr, int32_t *src, float *scale, int64_t *C_out, int64_t *nnz,
                                   int32_t *num_split_out)
{
    return build_map(chan_absmax, C, theta, src_idx, nullptr, r, true, row_ptr, src, scale, C_out, nnz, num_split_out);
}

int32_t qllm_pack_codes_host(const uint8_t *codes, int64_t R, int64_t K, int32_t bits, uint8_t *packed)
{
    if (!codes || !packed) return QLLM_ERR_NULL;
    if (!bits_supported(bits)) return QLLM_ERR_BITS;
    if (R < 0 || K <= 0) return QLLM_ERR_SHAPE;
    const int64_t rb = qllm_packed_row_bytes(K, bits);
    for (int64_t i = 0; i < R; ++i) {
        uint8_t *row = packed + i * rb;
        std::memset(row, 0, (size_t)rb);
        for (int64_t k = 0; k < K; ++k) {
            if (codes[i * K + k] >> bits) return QLLM_ERR_BITS;
            put_code(row, k, bits, codes[i * K + k]);
        }
    }
    return QLLM_OK;
}

int32_t qllm_unpack_codes_host(const uint8_t *packed, int64_t R, int64_t K, int32_t bits, uint8_t *codes)
{
    if (!codes || !packed) return QLLM_ERR_NULL;
    if (!bits_supported(bits)) return QLLM_ERR_BITS;
    if (R < 0 || K <= 0) return QLLM_ERR_SHAPE;
    const int64_t rb = qllm_packed_row_bytes(K, bits);
    for (int64_t i = 0; i < R; ++i)
        for (int64_t k = 0; k < K; ++k) codes[i * K + k] = (uint8_t)get_code(packed + i * rb, k, bits);
    return QLLM_OK;
}

int64_t qllm_select_edges_host(const double *best_d, int64_t nA, int64_t r, int32_t *pick_out)
{
    if (nA < 0 || r < 0) return QLLM_ERR_SHAPE;
    const int64_t take = std::min(r, nA);
    if (take == 0) return 0;
    if (!best_d || !pick_out) return QLLM_ERR_NULL;
    std::vector<int32_t> order((size_t)nA);
    for (int64_t i = 0; i < nA; ++i) order[(size_t)i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return best_d[a] < best_d[b]; });
    std::sort(order.begin(), order.begin() + take);
    for (int64_t k = 0; k < take; ++k) pick_out[k] = order[(size_t)k];
    return take;
}

int32_t qllm_fold_linear_host(const float *Wp, const float *bp, int64_t C_in, int64_t K_prev,
                              const int32_t *row_ptr, const int32_t *src, const float *scale, int64_t C_out,
                              float *W_out, float *b_out)
{
    if (!Wp || !row_ptr || !src || !scale || !W_out || (bp && !b_out)) return QLLM_ERR_NULL;
    if (C_in <= 0 || K_prev <= 0 || C_out <= 0) return QLLM_ERR_SHAPE;
    if (row_ptr[0] != 0) return QLLM_ERR_MAP;
    for (int64_t c = 0; c < C_out; ++c)
        if (row_ptr[c + 1] <= row_ptr[c]) return QLLM_ERR_MAP;
    const int32_t st = qllm_check_map_host(row_ptr, src, scale, C_in, C_out, row_ptr[C_out]);
    if (st != QLLM_OK) return st;
    constexpr int64_t BLK = 16; // output rows per task
    parallel_blocks((C_out + BLK - 1) / BLK, [&](int64_t b) {
        std::vector<double> acc((size_t)K_prev);
        for (int64_t c = b * BLK; c < std::min(C_out, (b + 1) * BLK); ++c) {
            std::fill(acc.begin(), acc.end(), 0.0);
            double bacc = 0.0;
            for (int32_t e = row_ptr[c]; e < row_ptr[c + 1]; ++e) {
                const double sc = (double)scale[e];
                const float *w = Wp + (int64_t)src[e] * K_prev;
                for (int64_t k = 0; k < K_prev; ++k) acc[(size_t)k] += sc * (double)w[k];
                if (bp) bacc += sc * (double)bp[src[e]];
            }
            float *out = W_out + c * K_prev;
            for (int64_t k = 0; k < K_prev; ++k) out[k] = (float)acc[(size_t)k];
            if (bp) b_out[c] = (float)bacc;
        }
    });
    return QLLM_OK;
}

int32_t qllm_quantize_weight_host(const float *W, int64_t C_in, int64_t O, const int32_t *row_ptr,
                                  const int32_t *src, int64_t C_out, int32_t bits, uint8_t *codes,
                                  float *scale, int32_t *zero, int32_t *colsum)
{
    if (!W || !row_ptr || !src || !codes || !scale || !zero || !colsum) return QLLM_ERR_NULL;
    if (!bits_supported(bits)) return QLLM_ERR_BITS;
    if (C_in <= 0 || O <= 0 || C_out <= 0) return QLLM_ERR_SHAPE;
    if (row_ptr[0] != 0) return QLLM_ERR_MAP;
    for (int64_t c = 0; c < C_out; ++c) {
        if (row_ptr[c + 1] <= row_ptr[c]) return QLLM_ERR_MAP;
        for (int32_t e = row_ptr[c]; e < row_ptr[c + 1]; ++e)
            if (src[e] < 0 || src[e] >= C_in) return QLLM_ERR_MAP;
    }
    const int qmax = (1 << bits) - 1;
    const int64_t rb = qllm_packed_row_bytes(C_out, bits);
    constexpr int64_t BLK = 64; // output channels handled together: one cache line of every weight row
    const int64_t n_blocks = (O + BLK - 1) / BLK;

    parallel_blocks(n_blocks, [&](int64_t b) {
        const int64_t o0 = b * BLK, nb = std::min(BLK, O - o0);
        std::vector<float> what((size_t)(C_out * nb)); // reassembled weight, this block of columns
        std::vector<float> mn((size_t)nb, std::numeric_limits<float>::infinity());
        std::vector<float> mx((size_t)nb, -std::numeric_limits<float>::infinity());
        for (int64_t c = 0; c < C_out; ++c) {
            float *dst = &what[(size_t)(c * nb)];
            int32_t e = row_ptr[c];
            const float *w0 = W + (int64_t)src[e] * O + o0;
            for (int64_t j = 0; j < nb; ++j) dst[j] = w0[j];
            for (++e; e < row_ptr[c + 1]; ++e) { // merged channel: rows add up (Eq. 4)
                const float *w1 = W + (int64_t)src[e] * O + o0;
                for (int64_t j = 0; j < nb; ++j) dst[j] = dst[j] + w1[j];
            }
            for (int64_t j = 0; j < nb; ++j) {
                mn[j] = std::min(mn[j], dst[j]);
                mx[j] = std::max(mx[j], dst[j]);
            }
        }
        for (int64_t j = 0; j < nb; ++j) {
            const QuantParams p = quant_params(mn[j], mx[j], qmax);
            uint8_t *row = codes + (o0 + j) * rb;
            std::memset(row, 0, (size_t)rb);
            int64_t sum = 0;
            for (int64_t c = 0; c < C_out; ++c) {
                const uint32_t q = quant_code(what[(size_t)(c * nb + j)], p, qmax);
                put_code(row, c, bits, q);
                sum += q;
            }
            scale[o0 + j] = p.alpha;
            zero[o0 + j] = (int32_t)p.beta;
            colsum[o0 + j] = (int32_t)sum;
        }
    });
    return QLLM_OK;
}

} // extern "C"
