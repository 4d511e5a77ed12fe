// The per-tile core of the accumulate / test / reset-or-decay pass of Alg. 1 (and of Alg. 2), shared by the
// kernel that streams g and s from memory (vgc_select.hip) and by the one that takes them straight from the
// matrix cores (vgc_fused_fc.hip): given the tile's g, s, r, v in registers it evaluates the loop body, stores
// r and v, and leaves the tile's send bitmap, exponent statistics and index-ordered staged entries in the scratch.
#ifndef VGC_TILE_CORE_H
#define VGC_TILE_CORE_H

#include "vgc_internal.h"

namespace vgc {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t rank_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Alg. 1 loop body for one element; every operation is a single float32 rounding
// (the files that include this are compiled without floating-point contraction).
__device__ __forceinline__ bool alg1_step(float g, float s, float r, float v, float alpha, float zeta,
                                          float& r_out, float& v_out, uint32_t& acc_bits) {
    const float rp = r + g;
    const float vp = v + s;
    const float lhs = rp * rp;
    const float rhs = alpha * vp;
    const bool send = lhs > rhs;
    r_out = send ? 0.0f : rp;
    v_out = send ? 0.0f : zeta * vp;
    acc_bits = __float_as_uint(rp);
    return send;
}

// Alg. 2 loop body (hybrid with the threshold method, Section 4.5) for one element:
//   send = |r'| > tau and r'^2 > alpha v';  sent: r = r' - sign(r') tau,  v = max((v' - (2|r'|) tau) + tau^2, 0);
//   v *= zeta always.  What is staged for a sent element is +-1.0f: the message carries signs in units of
//   tau, so the exponent machinery of the basic algorithm sees one constant magnitude (header 2^0, code 0).
__device__ __forceinline__ bool alg2_step(float g, float s, float r, float v, float alpha, float zeta, float tau,
                                          float& r_out, float& v_out, uint32_t& acc_bits) {
    const float rp = r + g;
    const float vp = v + s;
    const float lhs = rp * rp;
    const float rhs = alpha * vp;
    const bool send = (fabsf(rp) > tau) && (lhs > rhs);
    const float r_sent = rp - copysignf(tau, rp);
    const float two_r_tau = (2.0f * fabsf(rp)) * tau;
    const float v_sent = fmaxf((vp - two_r_tau) + (tau * tau), 0.0f);
    r_out = send ? r_sent : rp;
    v_out = zeta * (send ? v_sent : vp);
    acc_bits = (__float_as_uint(rp) & 0x80000000u) | 0x3F800000u;
    return send;
}

template <bool kHybrid>
__device__ __forceinline__ bool step_any(float g, float s, float r, float v, float alpha, float zeta, float tau,
                                         float& r_out, float& v_out, uint32_t& acc_bits) {
    if (kHybrid) return alg2_step(g, s, r, v, alpha, zeta, tau, r_out, v_out, acc_bits);
    return alg1_step(g, s, r, v, alpha, zeta, r_out, v_out, acc_bits);
}

// LDS working set of one 256-thread group running tile_core.
struct TileLds {
    uint32_t wmax[4];
    uint32_t seg[32];
    uint32_t hist[4][kRelBins];
    __attribute__((aligned(16))) uint16_t stage[kTile];
};

// Which elements of a tile thread `tid` (0..255) of the group owns, as element e = 0..7 of its arrays:
//   kVec:  tile element (e / 4) * 1024 + 4 * tid + e % 4   (two 16-byte pieces per array)
//   !kVec: tile element e * 256 + tid                       (4-byte accesses, any alignment, bounds-checked by m)
// In both layouts the elements of segment (u, wave) are a contiguous index range and segments are ordered by u*4 + wave.
template <bool kVec> __device__ __forceinline__ uint32_t tile_element(uint32_t tid, int e) {
    return kVec ? ((uint32_t)(e >> 2) * 1024u + 4u * tid + (uint32_t)(e & 3)) : ((uint32_t)e * 256u + tid);
}

// G, S, R, V: the thread's eight elements of g, s, r, v (zeros where the element is past m).  r, v: the tile's
// first element in memory; m: elements the tile has.  kGuarded: `live` may be false for a group of threads that
// only keeps the barriers company (nothing is stored then).  Contains three workgroup barriers.
template <bool kVec, bool kHybrid, bool kGuarded>
__device__ __forceinline__ void tile_core(const float (&G)[8], const float (&S)[8], const float (&R)[8], const float (&V)[8],
                                          float* __restrict__ r, float* __restrict__ v, uint32_t m, bool live,
                                          TileHdr* __restrict__ hdr, uint32_t* __restrict__ bitmap,
                                          uint16_t* __restrict__ staging, float alpha, float zeta, float tau,
                                          TileLds& sh, uint32_t tid) {
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    constexpr int E = kElemsPerThread;
    const bool on = !kGuarded || live;

    uint32_t bits[E];
    uint32_t sendmask = 0;
    if (kVec) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            f4 ro, vo;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float a, b;
                const bool send = step_any<kHybrid>(G[u * 4 + c], S[u * 4 + c], R[u * 4 + c], V[u * 4 + c], alpha, zeta, tau, a, b, bits[u * 4 + c]);
                ro[c] = a;
                vo[c] = b;
                sendmask |= (send ? 1u : 0u) << (u * 4 + c);
            }
            if (on) {
                __builtin_nontemporal_store(ro, reinterpret_cast<f4*>(r) + u * 256 + tid);
                __builtin_nontemporal_store(vo, reinterpret_cast<f4*>(v) + u * 256 + tid);
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < E; ++u) {
            const uint32_t i = u * 256 + tid;
            float a, b;
            const bool send = step_any<kHybrid>(G[u], S[u], R[u], V[u], alpha, zeta, tau, a, b, bits[u]) && (i < m);
            sendmask |= (send ? 1u : 0u) << u;
            if (i < m && on) {
                __builtin_nontemporal_store(a, r + i);
                __builtin_nontemporal_store(b, v + i);
            }
        }
    }
    if (kGuarded && !live) sendmask = 0;

    // ---- send bitmap of the tile (bit i = element i) and the tile's largest truncated exponent ----
    uint32_t etr = 0;
    if (kHybrid) {
        // every sent element is staged as +-1.0f: the largest exponent field is that of 1.0f wherever anything is sent
        etr = __ballot(sendmask != 0u) ? 127u : 0u;
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e)
            if (sendmask & (1u << e)) etr = max(etr, (bits[e] & 0x7FFFFFFFu) >> 23);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) etr = max(etr, (uint32_t)__shfl_xor((int)etr, off));
    }
    if (lane == 0) sh.wmax[wave] = etr;

    if (kVec) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            uint32_t x = ((sendmask >> (u * 4)) & 0xFu) << (4 * (lane & 7u));
            x |= (uint32_t)__shfl_xor((int)x, 1);
            x |= (uint32_t)__shfl_xor((int)x, 2);
            x |= (uint32_t)__shfl_xor((int)x, 4);
            if ((lane & 7u) == 0 && on) bitmap[(u * 1024 + wave * 256) / 32 + (lane >> 3)] = x;
        }
    } else {
#pragma unroll
        for (int u = 0; u < E; ++u) {
            const uint64_t b = __ballot((sendmask >> u) & 1u);
            if (lane == 0 && on) {
                uint2 w = make_uint2((uint32_t)b, (uint32_t)(b >> 32));
                *reinterpret_cast<uint2*>(bitmap + (u * 256 + wave * 64) / 32) = w;
            }
        }
    }
    __syncthreads();
    etr = max(max(sh.wmax[0], sh.wmax[1]), max(sh.wmax[2], sh.wmax[3]));

    // ---- tile-relative exponent code of every sent element (Section 4.4 rounding recipe) ----
    uint32_t entry[E];
    uint32_t stagedmask = 0;
    if (kHybrid) {
        // 1.0f rounds to 2^0 and the tile's maximum is 2^0: the relative code is 1 for every sent element
#pragma unroll
        for (int e = 0; e < E; ++e) entry[e] = (1u << 12) | ((bits[e] >> 31) << 11) | tile_element<kVec>(tid, e);
        stagedmask = sendmask;
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const uint32_t ab = bits[e] & 0x7FFFFFFFu;
            const uint32_t ernd = (ab + 0x00400000u) >> 23;   // add one at the mantissa's top bit, drop the mantissa
            const uint32_t rel = etr + 1u - ernd;             // >= 0 for sent elements: ernd <= own exponent + 1 <= etr + 1
            const bool staged = ((sendmask >> e) & 1u) && ernd >= 1u && rel <= 8u;
            const uint32_t pos = tile_element<kVec>(tid, e);
            entry[e] = ((rel & 15u) << 12) | ((bits[e] >> 31) << 11) | pos;
            stagedmask |= (staged ? 1u : 0u) << e;
        }
    }

    // histogram of rel over the wave (uniform values; scalar popcounts)
    if (kHybrid) {
        // every staged element is +-1.0f and so is the tile's maximum: rel = 1 for all of them
        uint32_t cnt = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) cnt += __popcll(__ballot((stagedmask >> e) & 1u));
        if (lane < kRelBins) sh.hist[wave][lane] = (lane == 1u) ? cnt : 0u;
    } else {
#pragma unroll
        for (int j = 0; j < (int)kRelBins; ++j) {
            uint32_t cnt = 0;
#pragma unroll
            for (int e = 0; e < E; ++e)
                cnt += __popcll(__ballot(((stagedmask >> e) & 1u) && ((entry[e] >> 12) == (uint32_t)j)));
            if (lane == 0) sh.hist[wave][j] = cnt;
        }
    }

    // rank of each staged element inside its segment, and segment totals
    uint32_t rank[E];
    constexpr int kSeg = kVec ? 2 : 8;
    if (kVec) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            uint32_t below = 0, total = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint64_t b = __ballot((stagedmask >> (u * 4 + c)) & 1u);
                below += rank_below(b);
                total += __popcll(b);
            }
            uint32_t acc = below;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                rank[u * 4 + c] = acc;
                acc += (stagedmask >> (u * 4 + c)) & 1u;
            }
            if (lane == 0) sh.seg[u * 4 + wave] = total;
        }
    } else {
#pragma unroll
        for (int u = 0; u < E; ++u) {
            const uint64_t b = __ballot((stagedmask >> u) & 1u);
            rank[u] = rank_below(b);
            if (lane == 0) sh.seg[u * 4 + wave] = (uint32_t)__popcll(b);
        }
    }
    __syncthreads();

    // exclusive scan over the kSeg*4 segment totals, redundantly in every wave
    uint32_t x = (lane < (uint32_t)(kSeg * 4)) ? sh.seg[lane] : 0u;
    uint32_t incl = x;
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
        const uint32_t y = (uint32_t)__shfl_up((int)incl, off);
        if (lane >= (uint32_t)off) incl += y;
    }
    const uint32_t excl = incl - x;
    const uint32_t n_staged = (uint32_t)__shfl((int)incl, 31);
    // compact in LDS, then write the tile's entries as whole 16-byte pieces (the tile's staging area is
    // 4 KiB-aligned; slots between the count and the next multiple of 8 receive stale values that the
    // reader ignores)
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int u = kVec ? (e >> 2) : e;
        const uint32_t segbase = (uint32_t)__shfl((int)excl, u * 4 + (int)wave);
        if ((stagedmask >> e) & 1u) sh.stage[segbase + rank[e]] = (uint16_t)entry[e];
    }
    __syncthreads();
    if (tid * 8 < n_staged && on)
        __builtin_nontemporal_store(reinterpret_cast<const uint4v*>(sh.stage)[tid], reinterpret_cast<uint4v*>(staging) + tid);

    if (tid == 0 && on) {
        uint32_t h[kRelBins];
#pragma unroll
        for (int j = 0; j < (int)kRelBins; ++j) h[j] = sh.hist[0][j] + sh.hist[1][j] + sh.hist[2][j] + sh.hist[3][j];
        uint4 lo = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        uint4 hi = make_uint4(h[8] | (etr << 16), 0u, 0u, 0u);
        reinterpret_cast<uint4*>(hdr)[0] = lo;
        reinterpret_cast<uint4*>(hdr)[1] = hi;
    }
}

}  // namespace vgc
#endif
