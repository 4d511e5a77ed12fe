// Accumulate / test / reset-or-decay pass of Alg. 1 (criterion of Eq. 2, decay of Section 4.4),
// fused with the first half of Encode(): rounding to a power of two by the integer recipe of
// Section 4.4 and a tile-local, index-ordered compaction of the sent elements.
//
// One workgroup owns one tile of 2048 consecutive elements of one group.  It reads g, s, r, v once
// (non-temporal, 16 B per lane where alignment allows), writes r and v once, and leaves in the
// scratch: the tile's send bitmap, the tile's largest exponent among sent elements, a 9-bin
// histogram of exponent codes relative to it, and one 16-bit staged entry per sent element in
// ascending position order.  The group-wide exponent floor(log2 M_k) is only known after every
// tile has run, so the final 3-bit code is fixed by the pack kernels from the tile-relative one.
#include "vgc_tile_core.h"

namespace vgc {

// Loads the thread's eight elements of the four arrays (non-temporal, 16 bytes per lane where the tile is whole
// and aligned) and hands them to the tile core.
template <bool kVec, bool kHybrid>
__device__ __forceinline__ void tile_body(const float* __restrict__ g, const float* __restrict__ s,
                                          float* __restrict__ r, float* __restrict__ v,
                                          uint32_t m, TileHdr* __restrict__ hdr,
                                          uint32_t* __restrict__ bitmap, uint16_t* __restrict__ staging,
                                          float alpha, float zeta, float tau) {
    __shared__ TileLds sh;
    const uint32_t tid = threadIdx.x;
    constexpr int E = kElemsPerThread;
    float G[E], S[E], R[E], V[E];
    if (kVec) {
        f4 G4[2], S4[2], R4[2], V4[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t i = u * 256 + tid;
            G4[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g) + i);
            S4[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(s) + i);
            R4[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(r) + i);
            V4[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(v) + i);
        }
#pragma unroll
        for (int e = 0; e < E; ++e) { G[e] = G4[e >> 2][e & 3]; S[e] = S4[e >> 2][e & 3]; R[e] = R4[e >> 2][e & 3]; V[e] = V4[e >> 2][e & 3]; }
    } else {
#pragma unroll
        for (int u = 0; u < E; ++u) {
            const uint32_t i = u * 256 + tid;
            G[u] = S[u] = R[u] = V[u] = 0.0f;
            if (i < m) {
                G[u] = __builtin_nontemporal_load(g + i);
                S[u] = __builtin_nontemporal_load(s + i);
                R[u] = __builtin_nontemporal_load(r + i);
                V[u] = __builtin_nontemporal_load(v + i);
            }
        }
    }
    tile_core<kVec, kHybrid, false>(G, S, R, V, r, v, m, true, hdr, bitmap, staging, alpha, zeta, tau, sh, tid);
}

template <bool kHybrid>
__global__ __launch_bounds__(256) void k_accumulate_select(
    PlanCheck pc, uint32_t* __restrict__ flags, const float* __restrict__ g, const float* __restrict__ s, float* __restrict__ r, float* __restrict__ v,
    const PlanGroup* __restrict__ groups, const PlanTile* __restrict__ tiles,
    TileHdr* __restrict__ hdrs, uint32_t* __restrict__ bitmap, uint16_t* __restrict__ staging,
    float alpha, float zeta, float tau, int ptrs_vec_aligned, uint32_t tile0) {
    const uint64_t t = (uint64_t)tile0 + blockIdx.x;            // tile0: first tile of the launch (a range of groups)
    const bool ok = plan_ok(pc);                                // uniform: a few scalar loads
    if (blockIdx.x == 0 && threadIdx.x == 0) flags[0] = ok ? 0u : 1u;
    if (!ok) return;
    const PlanTile pt = tiles[t];
    const PlanGroup pg = groups[pt.group];
    const uint64_t base = pg.offset + pt.start;
    const uint32_t m = min(kTile, pg.size - pt.start);
    TileHdr* hdr = hdrs + t;
    uint32_t* bm = bitmap + t * (kTile / 32);
    uint16_t* st = staging + t * kTile;
    if (m == kTile && (base & 3u) == 0 && ptrs_vec_aligned)
        tile_body<true, kHybrid>(g + base, s + base, r + base, v + base, m, hdr, bm, st, alpha, zeta, tau);
    else
        tile_body<false, kHybrid>(g + base, s + base, r + base, v + base, m, hdr, bm, st, alpha, zeta, tau);
}

int launch_accumulate_select(PlanCheck pc, uint32_t* flags, const float* g, const float* s, float* r, float* v,
                             const PlanGroup* groups, const PlanTile* tiles, uint64_t tile0, uint64_t n_tiles,
                             TileHdr* hdrs, uint32_t* bitmap, uint16_t* staging,
                             float alpha, float zeta, float tau, bool hybrid, bool ptrs_vec_aligned,
                             hipStream_t stream) {
    if (n_tiles == 0) return VGC_OK;
    if (tile0 + n_tiles > 0x7FFFFFFFull) {
        set_error("vgc_accumulate_select: %llu tiles exceed the launch limit", (unsigned long long)n_tiles);
        return VGC_ERR_SIZE;
    }
    if (hybrid)
        hipLaunchKernelGGL(k_accumulate_select<true>, dim3((uint32_t)n_tiles), dim3(kThreads), 0, stream,
                           pc, flags, g, s, r, v, groups, tiles, hdrs, bitmap, staging, alpha, zeta, tau, ptrs_vec_aligned ? 1 : 0, (uint32_t)tile0);
    else
        hipLaunchKernelGGL(k_accumulate_select<false>, dim3((uint32_t)n_tiles), dim3(kThreads), 0, stream,
                           pc, flags, g, s, r, v, groups, tiles, hdrs, bitmap, staging, alpha, zeta, 0.0f, ptrs_vec_aligned ? 1 : 0, (uint32_t)tile0);
    return hip_check(hipGetLastError(), "launch k_accumulate_select");
}

}  // namespace vgc
