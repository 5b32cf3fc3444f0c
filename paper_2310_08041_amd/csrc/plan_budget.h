// LDS need of the planned fused kernel with a plan's lists held on chip: shared by the launcher (which form of
// the kernel fits) and the plan builder (whether to stage only the chunks that hold sources, or all of them,
// so that the form that streams the lists can run).  Plain C++, no HIP.
#ifndef QLLM_PLAN_BUDGET_H
#define QLLM_PLAN_BUDGET_H

#include <cstdint>

namespace qllm_detail {

// dynamic LDS a launch may ask for: 160 KB per CU, less the kernel's static reduction slots
constexpr int64_t FUSED_MAX_LDS = 159 * 1024;

struct PlanCounts {
    int64_t n_comp, n_long, n_pub, n_chunks, n_spec, n_dest, n_segw;
};

// words_per_chunk: LDS dwords per packed chunk of 8 codes (1 for 4-bit, 2 for 6- and 8-bit codes);
// staging_sets: x alone, with gamma, with gamma and beta (1..3); slots: chunks per lane x lanes of the launch
// (one word per slot for its chunk, two for its output group).
inline int64_t fused_lists_lds_bytes(const PlanCounts &p, int64_t words_per_chunk, int64_t staging_sets, int64_t slots)
{
    const int64_t w = words_per_chunk, n_stage = 8 * p.n_pub + 4, n_dest4 = (p.n_dest + 3) / 4 * 4;
    return (staging_sets * n_stage + n_dest4) * 4 + p.n_long * 16 + p.n_comp * 32 + p.n_spec * 8 +
           (p.n_comp * w + w + (p.n_chunks + 1) * w) * 4 + (p.n_dest + p.n_segw + 3 * slots + 1) * 4; // + 1: the two-word slots start at an even word
}

// The same with the lists left in global memory and the whole row staged in the input's own type.
inline int64_t fused_streamed_lds_bytes(const PlanCounts &p, int64_t words_per_chunk, int64_t C, int64_t elem_bytes, int64_t slots)
{
    const int64_t w = words_per_chunk, n_dest4 = (p.n_dest + 3) / 4 * 4;
    return ((C + 8) * elem_bytes + 15) / 16 * 16 + n_dest4 * 4 + (p.n_comp * w + w + (p.n_chunks + 1) * w) * 4 + (3 * slots + 1) * 4;
}

} // namespace qllm_detail

#endif
