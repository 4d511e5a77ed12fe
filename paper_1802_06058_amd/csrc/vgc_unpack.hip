// Decode-and-sum half of CommunicateAndUpdate() (Section 4.3): one launch adds one worker's
// message into the dense gradient buffer.  Indices inside a message are distinct, so plain
// read-modify-write is race free and the float32 result does not depend on scheduling; messages
// are ordered by the stream.
#include "vgc_internal.h"

namespace vgc {

__global__ __launch_bounds__(256) void k_unpack_add(const uint32_t* __restrict__ words, uint64_t n_words,
                                                    const vgc_group_hdr* __restrict__ hdrs,
                                                    const PlanGroup* __restrict__ groups, uint32_t n_groups,
                                                    float scale, float* __restrict__ dense) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const vgc_group_hdr last = hdrs[n_groups - 1];
    uint64_t total = last.word_offset + last.count;
    if (total > n_words) total = n_words;
    if (i >= total) return;
    // the group whose word range holds i: the last one whose first word is at or before i
    uint32_t lo = 0, hi = n_groups - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (hdrs[mid].word_offset <= i) lo = mid; else hi = mid - 1;
    }
    const vgc_group_hdr h = hdrs[lo];
    const PlanGroup pg = groups[lo];
    const uint32_t w = __builtin_nontemporal_load(words + i);
    const uint32_t idx = w & 0x0FFFFFFFu;
    const uint32_t d = (w >> 28) & 7u;
    // a well-formed message never trips these; a damaged one is skipped rather than written out of range
    if (idx >= pg.size || h.exp_field <= d || h.exp_field > 254u || i >= h.word_offset + h.count) return;
    const float val = __uint_as_float(((h.exp_field - d) << 23) | (w & 0x80000000u));
    const float contrib = scale * val;
    float* p = dense + pg.offset + idx;
    *p = *p + contrib;
}

int launch_unpack_add(const uint32_t* words, uint64_t n_words, const vgc_group_hdr* hdrs,
                      const PlanGroup* groups, uint32_t n_groups, float scale, float* dense,
                      hipStream_t stream) {
    if (n_words == 0) return VGC_OK;
    const uint64_t blocks = (n_words + 255) / 256;
    if (blocks > 0x7FFFFFFFull) {
        set_error("vgc_unpack_add: %llu words exceed the launch limit", (unsigned long long)n_words);
        return VGC_ERR_SIZE;
    }
    hipLaunchKernelGGL(k_unpack_add, dim3((uint32_t)blocks), dim3(256), 0, stream, words, n_words, hdrs, groups,
                       n_groups, scale, dense);
    return hip_check(hipGetLastError(), "launch k_unpack_add");
}

}  // namespace vgc
