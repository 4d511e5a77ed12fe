// Second half of Encode() (Sections 4.2 and 4.4): fix floor(log2 M_k) per group, turn the staged
// tile-relative exponent codes into the final 3-bit codes, drop what falls below 2^(E_k-7), and
// write the words of every group contiguously, in ascending index order.
//
// A group is cut into segments of up to kSegTiles tiles so that a very large weight matrix is
// scanned by several workgroups.
//
//   k_seg_max      (only when some group has several segments) largest tile exponent per segment.
//   k_seg_scan     one workgroup per segment: E_k = max of the tile exponents, then per tile the
//                  number of words it keeps and its exclusive prefix inside the segment.
//   k_header_scan  one workgroup: exclusive scan of the group counts -> headers, status and the
//                  position of every segment's first word.
//   k_emit         one wave per tile: read the staged entries, filter, re-rank, write words.
#include "vgc_internal.h"

namespace vgc {

__device__ __forceinline__ uint32_t rank_below64(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Inclusive scan over a 1024-thread workgroup; returns the inclusive value, total through `total`.
__device__ __forceinline__ uint32_t block_scan_1024(uint32_t x, uint32_t* sh /*[16]*/, uint32_t& total) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    uint32_t incl = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t y = (uint32_t)__shfl_up((int)incl, off);
        if (lane >= (uint32_t)off) incl += y;
    }
    __syncthreads();                       // protects sh against the previous use
    if (lane == 63) sh[wave] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const uint32_t c = sh[w];
        if ((uint32_t)w < wave) base += c;
        tot += c;
    }
    total = tot;
    return incl + base;
}

// Workgroup maximum of the tile exponents of `cnt` (<= kSegTiles) tile records.
__device__ __forceinline__ uint32_t seg_max_exponent(const TileHdr* __restrict__ H, uint32_t cnt, uint32_t* sh /*[17]*/) {
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {                           // eight independent loads in flight
        const uint32_t i = (uint32_t)j * 1024 + tid;
        w[j] = (i < cnt) ? H[i].w[4] : 0u;
    }
    uint32_t e = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) e = max(e, w[j] >> 16);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) e = max(e, (uint32_t)__shfl_xor((int)e, off));
    __syncthreads();
    if (lane == 0) sh[wave] = e;
    __syncthreads();
    if (tid == 0) {
        uint32_t m = 0;
        for (int q = 0; q < 16; ++q) m = max(m, sh[q]);
        sh[16] = m;
    }
    __syncthreads();
    return sh[16];
}

// Only for groups of more than one segment: the largest tile exponent of every segment, so that the
// scan kernel's workgroups can each derive E_k of the whole group.
__global__ __launch_bounds__(1024) void k_seg_max(PlanCheck pc, const PlanGroup* __restrict__ groups, const PlanSeg* __restrict__ segs,
                                                  const TileHdr* __restrict__ hdrs, SegTmp* __restrict__ stmp) {
    __shared__ uint32_t sh[17];
    if (!plan_ok(pc)) return;
    const PlanSeg ps = segs[blockIdx.x];
    const PlanGroup pg = groups[ps.group];
    const uint32_t nt = (pg.size + kTile - 1) / kTile;
    if (nt <= kSegTiles) return;                            // single segment: the scan kernel finds E_k itself
    const uint32_t cnt = min(kSegTiles, nt - ps.first_tile);
    const uint32_t m = seg_max_exponent(hdrs + pg.first_tile + ps.first_tile, cnt, sh);
    if (threadIdx.x == 0) stmp[blockIdx.x].max_e = m;
}

// One workgroup per segment: E_k, then per tile the number of words it keeps and its exclusive
// prefix inside the segment.  Each thread owns 8 consecutive tile records: they are loaded together,
// scanned in registers, and only the per-thread totals go through the workgroup scan.
__global__ __launch_bounds__(1024) void k_seg_scan(PlanCheck pc, const PlanGroup* __restrict__ groups, const PlanSeg* __restrict__ segs,
                                                   TileHdr* __restrict__ hdrs, SegTmp* __restrict__ stmp) {
    __shared__ uint32_t sh[17];
    if (!plan_ok(pc)) return;
    const PlanSeg ps = segs[blockIdx.x];
    const PlanGroup pg = groups[ps.group];
    const uint32_t nt = (pg.size + kTile - 1) / kTile;
    const uint32_t cnt = min(kSegTiles, nt - ps.first_tile);
    TileHdr* H = hdrs + pg.first_tile + ps.first_tile;
    const uint32_t tid = threadIdx.x;

    // the loads of the records do not depend on E_k: issue them first
    uint4 lo[8];
    uint32_t w4[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t i = tid * 8 + j;
        lo[j] = make_uint4(0u, 0u, 0u, 0u);
        w4[j] = 0u;
        if (i < cnt) {
            lo[j] = reinterpret_cast<const uint4*>(H + i)[0];
            w4[j] = H[i].w[4];
        }
    }

    uint32_t E = 0;
    if (nt <= kSegTiles) {
        E = seg_max_exponent(H, cnt, sh);
    } else {
        const uint32_t n_seg = (nt + kSegTiles - 1) / kSegTiles;       // at most 16
        for (uint32_t q = 0; q < n_seg; ++q) E = max(E, stmp[ps.group_first_seg + q].max_e);
    }

    uint32_t kept[8], shift[8], mine = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        shift[j] = E - (w4[j] >> 16);
        kept[j] = 0;
        if (E != 0 && shift[j] <= 8) {
            const uint32_t h[9] = {lo[j].x & 0xFFFFu, lo[j].x >> 16, lo[j].y & 0xFFFFu, lo[j].y >> 16, lo[j].z & 0xFFFFu,
                                   lo[j].z >> 16, lo[j].w & 0xFFFFu, lo[j].w >> 16, w4[j] & 0xFFFFu};
            const uint32_t lim = 8 - shift[j];              // entries with rel <= lim are encoded
#pragma unroll
            for (int q = 0; q < 9; ++q) kept[j] += ((uint32_t)q <= lim) ? h[q] : 0u;
        }
        mine += kept[j];
    }
    uint32_t total;
    const uint32_t incl = block_scan_1024(mine, sh, total);
    uint32_t prefix = incl - mine;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t i = tid * 8 + j;
        if (i < cnt) {
            H[i].w[5] = prefix;
            H[i].w[6] = shift[j];
            H[i].w[7] = kept[j];
        }
        prefix += kept[j];
    }
    if (tid == 0) {
        stmp[blockIdx.x].exp_field = E;
        stmp[blockIdx.x].count = total;
    }
}

// One workgroup: group counts from the segment counts, exclusive scan over the groups -> headers,
// status, and the position of every segment's first word.
__global__ __launch_bounds__(1024) void k_header_scan(PlanCheck pc, const uint32_t* __restrict__ flags,
                                                      const PlanGroup* __restrict__ groups, SegTmp* __restrict__ stmp,
                                                      uint32_t n_groups,
                                                      vgc_group_hdr* __restrict__ hdrs_out,
                                                      vgc_pack_status* __restrict__ status, uint64_t words_cap) {
    __shared__ uint32_t sh[16];
    if (!plan_ok(pc) || flags[0] != 0u) {                   // the plan belongs to another group list: an empty message
        for (uint32_t k = threadIdx.x; k < n_groups; k += 1024) {
            vgc_group_hdr h;
            h.exp_field = 0; h.count = 0; h.word_offset = 0;
            hdrs_out[k] = h;
        }
        if (threadIdx.x == 0) {
            vgc_pack_status st;
            st.total_words = 0; st.overflow = 0; st.plan_mismatch = 1;
            *status = st;
        }
        return;
    }
    uint64_t running = 0;
    uint32_t seg_cursor = 0;                                // first segment of the chunk's first group
    for (uint32_t base = 0; base < n_groups; base += 1024) {
        const uint32_t k = base + threadIdx.x;
        // first segment of every group of the chunk: scan of the segment counts per group
        uint32_t n_seg = 0;
        if (k < n_groups) {
            const uint32_t nt = (groups[k].size + kTile - 1) / kTile;
            n_seg = (nt + kSegTiles - 1) / kSegTiles;
        }
        uint32_t seg_total;
        const uint32_t seg_incl = block_scan_1024(n_seg, sh, seg_total);
        const uint32_t first_seg = seg_cursor + seg_incl - n_seg;
        uint32_t count = 0, exp_field = 0;
        for (uint32_t q = 0; q < n_seg; ++q) count += stmp[first_seg + q].count;
        if (n_seg && count) exp_field = stmp[first_seg].exp_field;
        // a chunk of 1024 groups holds at most 1024 * 2^28 words: scan the low and high parts separately
        const uint32_t lo = count & 0xFFFFu, hi = count >> 16;
        uint32_t tot_lo, tot_hi;
        const uint32_t incl_lo = block_scan_1024(lo, sh, tot_lo);
        const uint32_t incl_hi = block_scan_1024(hi, sh, tot_hi);
        const uint64_t incl = (uint64_t)incl_lo + ((uint64_t)incl_hi << 16);
        if (k < n_groups) {
            vgc_group_hdr h;
            h.exp_field = exp_field;
            h.count = count;
            h.word_offset = running + incl - count;
            hdrs_out[k] = h;
            uint64_t b = h.word_offset;
            for (uint32_t q = 0; q < n_seg; ++q) {
                stmp[first_seg + q].base = b;
                b += stmp[first_seg + q].count;
            }
        }
        running += (uint64_t)tot_lo + ((uint64_t)tot_hi << 16);
        seg_cursor += seg_total;
    }
    if (threadIdx.x == 0) {
        vgc_pack_status st;
        st.total_words = running;
        st.overflow = running > words_cap ? 1u : 0u;
        st.plan_mismatch = 0;
        *status = st;
    }
}

__global__ __launch_bounds__(256) void k_emit(PlanCheck pc, const PlanTile* __restrict__ tiles, uint64_t n_tiles,
                                              const TileHdr* __restrict__ hdrs, const uint16_t* __restrict__ staging,
                                              const SegTmp* __restrict__ stmp,
                                              uint32_t* __restrict__ words, uint64_t words_cap) {
    constexpr int kAhead = 8;                               // rounds of 64 entries loaded before anything is known
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t t = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= n_tiles || !plan_ok(pc)) return;
    const uint16_t* st = staging + t * kTile;
    // Every tile owns kTile staging slots, so the first rounds can be fetched before the tile's count
    // is known (slots past the count hold stale data and are ignored): the loads overlap the header's.
    uint32_t e[kAhead];
#pragma unroll
    for (int j = 0; j < kAhead; ++j) e[j] = __builtin_nontemporal_load(st + j * 64 + lane);
    const uint32_t hw = (lane < 8) ? hdrs[t].w[lane] : 0u;  // one 32-byte read per wave
    const PlanTile pt = tiles[t];
    uint32_t w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = (uint32_t)__shfl((int)hw, i);
    const uint32_t kept = w[7];
    if (kept == 0) return;
    const uint32_t cnt = (w[0] & 0xFFFFu) + (w[0] >> 16) + (w[1] & 0xFFFFu) + (w[1] >> 16) + (w[2] & 0xFFFFu) +
                         (w[2] >> 16) + (w[3] & 0xFFFFu) + (w[3] >> 16) + (w[4] & 0xFFFFu);
    const uint32_t shift = w[6];
    const uint32_t lim = 8 - shift;                         // kept != 0 implies shift <= 8
    uint64_t out = stmp[pt.seg].base + w[5];
    for (uint32_t j0 = 0; j0 < cnt; j0 += 64 * kAhead) {
        if (j0) {
#pragma unroll
            for (int j = 0; j < kAhead; ++j) {
                const uint32_t jj = j0 + j * 64 + lane;
                e[j] = (jj < kTile) ? (uint32_t)__builtin_nontemporal_load(st + jj) : 0xFFFFu;
            }
        }
#pragma unroll
        for (int j = 0; j < kAhead; ++j) {
            const uint32_t jj = j0 + j * 64 + lane;
            const uint32_t rel = e[j] >> 12;
            const bool keep = (jj < cnt) && (rel <= lim);
            const uint32_t sr = shift + rel;
            const uint32_t d = sr ? sr - 1u : 0u;           // E_k minus min(rounded exponent, E_k)
            const uint32_t word = (((e[j] >> 11) & 1u) << 31) | (d << 28) | (pt.start + (e[j] & 0x7FFu));
            const uint64_t b = __ballot(keep);
            const uint64_t pos = out + rank_below64(b);
            if (keep && pos < words_cap) __builtin_nontemporal_store(word, words + pos);
            out += (uint32_t)__popcll(b);
        }
    }
}

int launch_pack_scans(PlanCheck pc, const uint32_t* flags, const PlanGroup* groups, const PlanSeg* segs, uint32_t n_groups,
                      uint32_t n_segs, bool multi_seg, TileHdr* hdrs, SegTmp* stmp, vgc_group_hdr* hdrs_out,
                      vgc_pack_status* status_out, uint64_t words_cap, hipStream_t stream) {
    if (multi_seg) hipLaunchKernelGGL(k_seg_max, dim3(n_segs), dim3(1024), 0, stream, pc, groups, segs, hdrs, stmp);
    hipLaunchKernelGGL(k_seg_scan, dim3(n_segs), dim3(1024), 0, stream, pc, groups, segs, hdrs, stmp);
    hipLaunchKernelGGL(k_header_scan, dim3(1), dim3(1024), 0, stream, pc, flags, groups, stmp, n_groups, hdrs_out,
                       status_out, words_cap);
    return hip_check(hipGetLastError(), "launch pack scans");
}

int launch_pack(PlanCheck pc, const uint32_t* flags, const PlanGroup* groups, const PlanTile* tiles, const PlanSeg* segs, uint64_t n_tiles,
                uint32_t n_groups, uint32_t n_segs, bool multi_seg,
                TileHdr* hdrs, SegTmp* stmp, const uint16_t* staging,
                uint32_t* words_out, uint64_t words_cap, vgc_group_hdr* hdrs_out,
                vgc_pack_status* status_out, hipStream_t stream) {
    const int rc = launch_pack_scans(pc, flags, groups, segs, n_groups, n_segs, multi_seg, hdrs, stmp, hdrs_out, status_out, words_cap, stream);
    if (rc != VGC_OK) return rc;
    const uint64_t blocks = (n_tiles + 3) / 4;
    hipLaunchKernelGGL(k_emit, dim3((uint32_t)blocks), dim3(256), 0, stream, pc, tiles, n_tiles, hdrs, staging,
                       stmp, words_out, words_cap);
    return hip_check(hipGetLastError(), "launch pack kernels");
}

}  // namespace vgc
