// Decode-and-sum half of CommunicateAndUpdate() (Section 4.3): one launch adds one worker's
// message into the dense gradient buffer.  Indices inside a message are distinct, so plain
// read-modify-write is race free and the float32 result does not depend on scheduling; messages
// are ordered by the stream.
#include "vgc_internal.h"

namespace vgc {

__global__ __launch_bounds__(256) void k_unpack_add(PlanCheck pc, const uint32_t* __restrict__ words, uint64_t n_words,
                                                    const vgc_group_hdr* __restrict__ hdrs,
                                                    const PlanGroup* __restrict__ groups, uint32_t n_groups,
                                                    float scale, float* __restrict__ dense) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (!plan_ok(pc)) return;
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

int launch_unpack_add(PlanCheck pc, const uint32_t* words, uint64_t n_words, const vgc_group_hdr* hdrs,
                      const PlanGroup* groups, uint32_t n_groups, float scale, float* dense,
                      hipStream_t stream) {
    if (n_words == 0) return VGC_OK;
    const uint64_t blocks = (n_words + 255) / 256;
    if (blocks > 0x7FFFFFFFull) {
        set_error("vgc_unpack_add: %llu words exceed the launch limit", (unsigned long long)n_words);
        return VGC_ERR_SIZE;
    }
    hipLaunchKernelGGL(k_unpack_add, dim3((uint32_t)blocks), dim3(256), 0, stream, pc, words, n_words, hdrs, groups,
                       n_groups, scale, dense);
    return hip_check(hipGetLastError(), "launch k_unpack_add");
}

}  // namespace vgc

// ------------------------------------------------------------------------------------------------
// Several messages in one pass over the dense buffer.  When the messages together touch most cache
// lines of the dense buffer (the synthetic workloads send 20-35 % of all elements per worker), one
// launch per message re-reads and re-writes the whole buffer p times.  Here one wave owns a run of
// consecutive tiles of one group: it keeps the current tile (2048 floats) in LDS, and for every
// message, in message order, streams that message's words of the tile from a cursor and adds them.
// The float32 additions an element receives are the same, in the same order, as p single-message
// launches would perform, so the result is bit-identical.
// ------------------------------------------------------------------------------------------------
namespace vgc {


template <int kMax>
struct BatchArgs {
    const uint32_t* words[kMax];
    const vgc_group_hdr* hdrs[kMax];
    uint64_t n_words[kMax];
    uint32_t p;
};

// What happens to a tile once every message has been added into it.
//   kToDense       it is the tile of the dense gradient buffer: written back.
//   kMomentumSgd   it is the decoded gradient ghat (elements nobody sent are zero, Section 4.1):
//                  m <- mu m - lr ghat;  w <- w + m.
//   kAdam          m <- b1 m + (1 - b1) ghat;  v <- b2 v + (1 - b2) ghat^2;
//                  w <- w - lr (m / bias1) / (sqrt(v / bias2) + eps),  bias_i = 1 - b_i^t.
// One float32 rounding per operation, in the order written (no contraction).
enum { kToDense = 0, kMomentumSgd = 1, kAdam = 2 };

struct UpdateArgs {
    float* w;
    float* s1;
    float* s2;
    float lr, mu, b1, b2, omb1, omb2, bias1, bias2, eps;
};

template <int kMode>
__device__ __forceinline__ void update_element(const UpdateArgs& O, float ghat, float& w, float& s1, float& s2) {
    if (kMode == kMomentumSgd) {
        const float t1 = O.mu * s1;
        const float t2 = O.lr * ghat;
        s1 = t1 - t2;
        w = w + s1;
    } else {
        const float a = O.b1 * s1, b = O.omb1 * ghat;
        s1 = a + b;
        const float g2 = ghat * ghat;
        const float c = O.b2 * s2, d = O.omb2 * g2;
        s2 = c + d;
        const float mhat = s1 / O.bias1;
        const float vhat = s2 / O.bias2;
        const float denom = sqrtf(vhat) + O.eps;
        const float step = (O.lr * mhat) / denom;
        w = w - step;
    }
}

typedef float f4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint64_t shfl64(uint64_t x, int src) {
    const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)x, src);
    const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)(x >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}

template <int kMax, int kMode>
__global__ __launch_bounds__(256) void k_unpack_add_batch(PlanCheck pc, BatchArgs<kMax> A, const PlanGroup* __restrict__ groups,
                                                          const PlanRun* __restrict__ runs, uint32_t n_runs,
                                                          float scale, float* __restrict__ dense, int overwrite,
                                                          UpdateArgs O, uint32_t tiles_per_wave) {
    // wave-wide word loads in flight per message: eight where the words are most of what the wave waits for, four
    // where the optimizer's arrays are in flight as well (there the words loaded past the tile's end cost more)
    constexpr int kRounds = kMode == kToDense ? 8 : 4;
    // A message's words of a tile are requested before their number is known.  The first request of a tile is sized
    // from the message's density in the group (mean + 3 standard deviations of a tile's count if the sent elements
    // were spread evenly, at most kFirst x 64 words); if the tile holds more, requests of kRounds x 64 follow.  Words
    // requested past the tile's end are requested again with the next tile: they are what this sizing keeps small.
    constexpr int kFirst = 16;
    __shared__ __attribute__((aligned(16))) float sh_tile[4][kTile];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    // a run of kRunTiles tiles is shared by kRunTiles / tiles_per_wave waves (small parameter sets have few runs)
    const uint32_t per_run = (uint32_t)kRunTiles / tiles_per_wave;
    const uint32_t gw = blockIdx.x * 4 + wave;
    const uint32_t run = gw / per_run;
    if (run >= n_runs || !plan_ok(pc)) return;
    float* T = sh_tile[wave];
    const uint32_t k = runs[run].group;
    const PlanGroup pg = groups[k];
    const uint32_t nt_group = (pg.size + kTile - 1) / kTile;
    const uint32_t run_end = min(runs[run].first_tile + (uint32_t)kRunTiles, nt_group);
    const uint32_t t0 = runs[run].first_tile + (gw % per_run) * tiles_per_wave;   // first tile of this wave, counted inside the group
    if (t0 >= run_end) return;
    const uint32_t t1 = min(t0 + tiles_per_wave, run_end);

    // per message (lane w < p): segment of group k and the cursor = first word with index >= run start
    uint64_t cur = 0, seg_end = 0;
    uint32_t expf = 0, first_rounds = 1;
    if (lane < A.p) {
        const vgc_group_hdr h = A.hdrs[lane][k];
        const float mu = (float)h.count * ((float)kTile / (float)pg.size);
        first_rounds = min((uint32_t)kFirst, (uint32_t)((mu + 3.0f * sqrtf(mu)) * (1.0f / 64.0f)) + 1u);
        uint64_t lo = h.word_offset, hi = h.word_offset + h.count;
        if (hi > A.n_words[lane]) hi = A.n_words[lane];
        if (lo > hi) lo = hi;
        seg_end = hi;
        expf = h.exp_field;
        const uint32_t first = t0 * kTile;
        const uint32_t* W = A.words[lane];
        while (lo < hi) {                                    // lower bound on the 28-bit index
            const uint64_t mid = (lo + hi) >> 1;
            if ((W[mid] & 0x0FFFFFFFu) < first) lo = mid + 1; else hi = mid;
        }
        cur = lo;
    }

    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t start = t * kTile;
        const uint32_t m = min(kTile, pg.size - start);
        const uint64_t e0 = pg.offset + start;
        float* base = (kMode == kToDense) ? dense + e0 : O.w + e0;
        bool vec = (m == kTile) && ((reinterpret_cast<uintptr_t>(base) & 15u) == 0);
        // the optimizer's arrays are requested now and arrive while the messages are decoded
        f4u W4[kMode == kToDense ? 1 : 8], S1[kMode == kToDense ? 1 : 8], S2[kMode == kAdam ? 8 : 1];
        if (kMode != kToDense) {
            vec = vec && ((reinterpret_cast<uintptr_t>(O.s1 + e0) & 15u) == 0) &&
                  (kMode != kAdam || (reinterpret_cast<uintptr_t>(O.s2 + e0) & 15u) == 0);
            if (vec) {
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    W4[q] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(O.w + e0) + q * 64 + lane);
                    S1[q] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(O.s1 + e0) + q * 64 + lane);
                    if (kMode == kAdam) S2[q] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(O.s2 + e0) + q * 64 + lane);
                }
            }
        }
        // ---- tile -> LDS ----
        if (overwrite || kMode != kToDense) {
#pragma unroll
            for (int q = 0; q < 8; ++q) reinterpret_cast<f4u*>(T)[q * 64 + lane] = (f4u){0.f, 0.f, 0.f, 0.f};
        } else if (vec) {
            f4u x[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) x[q] = __builtin_nontemporal_load(reinterpret_cast<const f4u*>(base) + q * 64 + lane);
#pragma unroll
            for (int q = 0; q < 8; ++q) reinterpret_cast<f4u*>(T)[q * 64 + lane] = x[q];
        } else {
            for (uint32_t i = lane; i < kTile; i += 64) T[i] = (i < m) ? base[i] : 0.f;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- messages in order ----
        const uint32_t tile_end = start + m;
        for (uint32_t w = 0; w < A.p; ++w) {
            uint64_t c = shfl64(cur, (int)w);                // wave-uniform cursor of message w
            const uint64_t se = shfl64(seg_end, (int)w);
            const uint32_t ef = (uint32_t)__shfl((int)expf, (int)w);
            const uint32_t* W = A.words[w];
            {                                                // first request: first_rounds x 64 words
                const uint32_t fr = (uint32_t)__shfl((int)first_rounds, (int)w);
                uint32_t wd[kFirst];
#pragma unroll
                for (int j = 0; j < kFirst; ++j) {
                    const uint64_t i = c + (uint32_t)j * 64u + lane;
                    wd[j] = ((uint32_t)j < fr && i < se) ? __builtin_nontemporal_load(W + i) : 0xFFFFFFFFu;
                }
                uint32_t used = 0;
#pragma unroll
                for (int j = 0; j < kFirst; ++j) {
                    if ((uint32_t)j < fr) {
                        const uint64_t i = c + (uint32_t)j * 64u + lane;
                        const uint32_t idx = wd[j] & 0x0FFFFFFFu;
                        const uint32_t d = (wd[j] >> 28) & 7u;
                        const bool in_tile = (i < se) && (idx < tile_end);
                        if (in_tile && idx >= start && ef > d && ef <= 254u) {
                            const float val = __uint_as_float(((ef - d) << 23) | (wd[j] & 0x80000000u));
                            const float contrib = scale * val;
                            T[idx - start] = T[idx - start] + contrib;
                        }
                        used += (uint32_t)__popcll(__ballot(in_tile));
                    }
                }
                c += used;
                if (used != fr * 64u) {                      // the tile's words ended inside the request
                    if (lane == w) cur = c;
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    continue;
                }
            }
            bool more = true;
            while (more) {
                uint32_t wd[kRounds];
#pragma unroll
                for (int j = 0; j < kRounds; ++j) {
                    const uint64_t i = c + (uint32_t)j * 64u + lane;
                    wd[j] = (i < se) ? __builtin_nontemporal_load(W + i) : 0xFFFFFFFFu;
                }
                uint32_t used = 0;
#pragma unroll
                for (int j = 0; j < kRounds; ++j) {
                    const uint64_t i = c + (uint32_t)j * 64u + lane;
                    const uint32_t idx = wd[j] & 0x0FFFFFFFu;
                    const uint32_t d = (wd[j] >> 28) & 7u;
                    const bool in_tile = (i < se) && (idx < tile_end);
                    // a well-formed message has idx >= start here and exp_field > d; anything else is skipped
                    if (in_tile && idx >= start && ef > d && ef <= 254u) {
                        const float val = __uint_as_float(((ef - d) << 23) | (wd[j] & 0x80000000u));
                        const float contrib = scale * val;
                        T[idx - start] = T[idx - start] + contrib;
                    }
                    used += (uint32_t)__popcll(__ballot(in_tile));
                }
                c += used;
                more = (used == (uint32_t)kRounds * 64u);
            }
            if (lane == w) cur = c;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }

        // ---- LDS -> tile ----
        if (kMode == kToDense) {
            if (vec) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    __builtin_nontemporal_store(reinterpret_cast<f4u*>(T)[q * 64 + lane], reinterpret_cast<f4u*>(base) + q * 64 + lane);
            } else {
                for (uint32_t i = lane; i < m; i += 64) base[i] = T[i];
            }
        } else if (vec) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const f4u G = reinterpret_cast<f4u*>(T)[q * 64 + lane];
                f4u w4 = W4[q], a4 = S1[q], b4 = S2[kMode == kAdam ? q : 0];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float w = w4[c], a = a4[c], b = b4[c];
                    update_element<kMode>(O, G[c], w, a, b);
                    w4[c] = w; a4[c] = a; b4[c] = b;
                }
                __builtin_nontemporal_store(w4, reinterpret_cast<f4u*>(O.w + e0) + q * 64 + lane);
                __builtin_nontemporal_store(a4, reinterpret_cast<f4u*>(O.s1 + e0) + q * 64 + lane);
                if (kMode == kAdam) __builtin_nontemporal_store(b4, reinterpret_cast<f4u*>(O.s2 + e0) + q * 64 + lane);
            }
        } else {
            for (uint32_t i = lane; i < m; i += 64) {
                float w = O.w[e0 + i], a = O.s1[e0 + i], b = (kMode == kAdam) ? O.s2[e0 + i] : 0.f;
                update_element<kMode>(O, T[i], w, a, b);
                O.w[e0 + i] = w;
                O.s1[e0 + i] = a;
                if (kMode == kAdam) O.s2[e0 + i] = b;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Tiles one wave takes: a whole run when there are plenty of runs, fewer (a power of two) when the parameter
// set is small, so that there are about 16 K waves to spread over the chip.
static uint32_t tiles_per_wave(uint64_t n_runs) {
    uint32_t tpw = kRunTiles;
    while (tpw > 1 && n_runs * (kRunTiles / tpw) < 16384) tpw /= 2;
    return tpw;
}

template <int kMax>
static BatchArgs<kMax> batch_args(const uint32_t* const* words, const uint64_t* n_words, const vgc_group_hdr* const* hdrs,
                                  uint32_t first, uint32_t p) {
    BatchArgs<kMax> A;
    A.p = p - first < (uint32_t)kMax ? p - first : (uint32_t)kMax;
    for (uint32_t w = 0; w < (uint32_t)kMax; ++w) {
        const bool on = w < A.p;
        A.words[w] = on ? words[first + w] : nullptr;
        A.hdrs[w] = on ? hdrs[first + w] : nullptr;
        A.n_words[w] = on ? n_words[first + w] : 0;
    }
    return A;
}

int launch_unpack_add_batch(PlanCheck pc, const uint32_t* const* words, const uint64_t* n_words, const vgc_group_hdr* const* hdrs,
                            uint32_t p, const PlanGroup* groups, const PlanRun* runs, uint64_t n_runs,
                            float scale, int overwrite, float* dense, hipStream_t stream) {
    const uint32_t tpw = tiles_per_wave(n_runs);
    const uint32_t blocks = (uint32_t)((n_runs * (kRunTiles / tpw) + 3) / 4);
    const uint32_t chunks = p ? (p + kBatchMax - 1) / kBatchMax : 1;     // p == 0: only the optional clear
    for (uint32_t ch = 0; ch < chunks; ++ch) {
        const BatchArgs<kBatchMax> A = batch_args<kBatchMax>(words, n_words, hdrs, ch * kBatchMax, p);
        hipLaunchKernelGGL((k_unpack_add_batch<kBatchMax, kToDense>), dim3(blocks), dim3(256), 0, stream, pc, A, groups, runs,
                           (uint32_t)n_runs, scale, dense, (overwrite && ch == 0) ? 1 : 0, UpdateArgs{}, tpw);
    }
    return hip_check(hipGetLastError(), "launch k_unpack_add_batch");
}

int launch_unpack_apply(PlanCheck pc, const uint32_t* const* words, const uint64_t* n_words, const vgc_group_hdr* const* hdrs,
                        uint32_t p, const PlanGroup* groups, const PlanRun* runs, uint64_t n_runs, float scale,
                        int kind, float lr, float mu, float b1, float b2, float omb1, float omb2, float bias1, float bias2,
                        float eps, float* param, float* state1, float* state2, hipStream_t stream) {
    const uint32_t tpw = tiles_per_wave(n_runs);
    const uint32_t blocks = (uint32_t)((n_runs * (kRunTiles / tpw) + 3) / 4);
    const BatchArgs<kApplyMax> A = batch_args<kApplyMax>(words, n_words, hdrs, 0, p);
    UpdateArgs O;
    O.w = param; O.s1 = state1; O.s2 = state2;
    O.lr = lr; O.mu = mu; O.b1 = b1; O.b2 = b2; O.omb1 = omb1; O.omb2 = omb2; O.bias1 = bias1; O.bias2 = bias2; O.eps = eps;
    if (kind == VGC_OPT_ADAM)
        hipLaunchKernelGGL((k_unpack_add_batch<kApplyMax, kAdam>), dim3(blocks), dim3(256), 0, stream, pc, A, groups, runs,
                           (uint32_t)n_runs, scale, static_cast<float*>(nullptr), 1, O, tpw);
    else
        hipLaunchKernelGGL((k_unpack_add_batch<kApplyMax, kMomentumSgd>), dim3(blocks), dim3(256), 0, stream, pc, A, groups, runs,
                           (uint32_t)n_runs, scale, static_cast<float*>(nullptr), 1, O, tpw);
    return hip_check(hipGetLastError(), "launch k_unpack_add_batch (update)");
}

}  // namespace vgc
