// Compressed index encoding of a message (Section 4.2 ends by noting that the index bits can be reduced further by
// compressing the indexes; the paper gives no algorithm, the format is this library's own).  Elements are in
// ascending index order, so each is stored as its distance from the previous element of its tile:
//     gap  = position in tile - position of the tile's previous element - 1   (the first element counts from -1)
//     code = sign << 3 | d                                                   (the 4-bit value of Section 4.2)
//     gap < 8: one byte gap << 4 | code;  else two bytes 0x80 | (gap & 7) << 4 | code, gap >> 3   (gap <= 2047)
// plus a directory: bytes per tile (uint16) and the byte offset of every run of 64 tiles (uint64).  The chain of
// distances restarts in every tile, so one wave encodes or decodes a tile without looking at any other.
//
//   k_compact_count   one wave per tile: bytes the tile's kept entries take -> tile_bytes
//   k_compact_runsum  one wave per run: bytes of the run's tiles
//   k_compact_scan    one workgroup: exclusive scan over the runs -> run offsets, group byte offsets, total
//   k_compact_emit    one wave per tile: the bytes
//   k_unpack_compact  one wave per run, tile in LDS, messages in order (the batched decoder for this format)
#include "vgc_internal.h"

namespace vgc {

__device__ __forceinline__ uint64_t lanes_below(uint32_t lane) { return (1ull << lane) - 1ull; }

// The staged entries of tile t that the group keeps, 64 at a time, as (first byte, second byte, two bytes?, byte
// offset inside the tile).  Calls `sink(keep, b0, b1, is_long, offset)` once per round in every lane; returns the
// tile's bytes.
template <class Sink>
__device__ __forceinline__ uint32_t encode_tile(const TileHdr* __restrict__ hdrs, const uint16_t* __restrict__ staging,
                                                uint64_t t, uint32_t lane, Sink sink) {
    const uint32_t hw = (lane < 8) ? hdrs[t].w[lane] : 0u;
    uint32_t w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = (uint32_t)__shfl((int)hw, i);
    if (w[7] == 0) return 0;                                   // nothing kept
    const uint32_t cnt = (w[0] & 0xFFFFu) + (w[0] >> 16) + (w[1] & 0xFFFFu) + (w[1] >> 16) + (w[2] & 0xFFFFu) +
                         (w[2] >> 16) + (w[3] & 0xFFFFu) + (w[3] >> 16) + (w[4] & 0xFFFFu);
    const uint32_t shift = w[6], lim = 8 - shift;              // kept != 0 implies shift <= 8
    const uint16_t* st = staging + t * kTile;
    int32_t prev = -1;                                         // position of the last kept entry so far (uniform)
    uint32_t bytes = 0;
    for (uint32_t j0 = 0; j0 < cnt; j0 += 64) {
        const uint32_t j = j0 + lane;
        const uint32_t e = (j < cnt) ? (uint32_t)st[j] : 0xFFFFu;
        const uint32_t rel = e >> 12;
        const bool keep = (j < cnt) && (rel <= lim);
        const uint32_t sr = shift + rel;
        const uint32_t d = sr ? sr - 1u : 0u;                  // E_k minus min(rounded exponent, E_k)
        const uint32_t code = (((e >> 11) & 1u) << 3) | d;
        const int32_t pos = (int32_t)(e & 0x7FFu);
        const uint64_t b = __ballot(keep), lower = b & lanes_below(lane);
        const int src = lower ? 63 - __builtin_clzll(lower) : 0;
        const int32_t before = __shfl(pos, src);
        const uint32_t gap = (uint32_t)(pos - (lower ? before : prev) - 1);
        const bool is_long = keep && gap >= 8u;
        const uint64_t bl = __ballot(is_long);
        const uint32_t offset = bytes + (uint32_t)__popcll(lower) + (uint32_t)__popcll(bl & lanes_below(lane));
        const uint32_t b0 = (is_long ? 0x80u : 0u) | ((gap & 7u) << 4) | code, b1 = gap >> 3;
        sink(keep, b0, b1, is_long, offset);
        if (b) prev = __shfl(pos, 63 - __builtin_clzll(b));
        bytes += (uint32_t)__popcll(b) + (uint32_t)__popcll(bl);
    }
    return bytes;
}

__global__ __launch_bounds__(256) void k_compact_count(PlanCheck pc, uint64_t n_tiles, const TileHdr* __restrict__ hdrs,
                                                       const uint16_t* __restrict__ staging, uint16_t* __restrict__ tile_bytes) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t t = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= n_tiles || !plan_ok(pc)) return;
    const uint32_t bytes = encode_tile(hdrs, staging, t, lane, [](bool, uint32_t, uint32_t, bool, uint32_t) {});
    if (lane == 0) tile_bytes[t] = (uint16_t)bytes;
}

// run_offsets[r] <- bytes of run r (turned into offsets by the scan)
__global__ __launch_bounds__(256) void k_compact_runsum(PlanCheck pc, const PlanGroup* __restrict__ groups, const PlanRun* __restrict__ runs,
                                                        uint64_t n_runs, const uint16_t* __restrict__ tile_bytes,
                                                        uint64_t* __restrict__ run_offsets) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t r = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= n_runs || !plan_ok(pc)) return;
    const PlanGroup pg = groups[runs[r].group];
    const uint32_t nt = (pg.size + kTile - 1) / kTile;
    const uint32_t i = runs[r].first_tile + lane;
    uint32_t x = (i < nt) ? (uint32_t)tile_bytes[(uint64_t)pg.first_tile + i] : 0u;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += (uint32_t)__shfl_xor((int)x, off);
    if (lane == 0) run_offsets[r] = x;
}

// One workgroup: exclusive scan over the runs' bytes in place, the groups' byte offsets, the total.
__global__ __launch_bounds__(1024) void k_compact_scan(PlanCheck pc, const PlanGroup* __restrict__ groups, const PlanTile* __restrict__ tiles,
                                                       uint64_t n_runs, uint32_t n_groups, uint64_t* __restrict__ run_offsets,
                                                       vgc_group_hdr* __restrict__ hdrs_out, vgc_pack_status* __restrict__ status,
                                                       uint64_t stream_cap) {
    __shared__ uint64_t sh[1024];
    __shared__ uint64_t carry;
    if (!plan_ok(pc) || status->plan_mismatch) return;          // the header scan has already reported it
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (uint64_t base = 0; base < n_runs; base += 1024) {
        const uint64_t r = base + threadIdx.x;
        const uint64_t x = r < n_runs ? run_offsets[r] : 0;
        sh[threadIdx.x] = x;
        __syncthreads();
        for (uint32_t off = 1; off < 1024; off <<= 1) {        // inclusive scan in LDS
            const uint64_t y = threadIdx.x >= off ? sh[threadIdx.x - off] : 0;
            __syncthreads();
            sh[threadIdx.x] += y;
            __syncthreads();
        }
        if (r < n_runs) run_offsets[r] = carry + sh[threadIdx.x] - x;
        __syncthreads();
        if (threadIdx.x == 1023) carry += sh[1023];
        __syncthreads();
    }
    __threadfence_block();
    for (uint32_t k = threadIdx.x; k < n_groups; k += 1024) hdrs_out[k].word_offset = run_offsets[tiles[groups[k].first_tile].run];
    if (threadIdx.x == 0) {
        status->total_words = carry;                            // bytes of the stream
        status->overflow = carry > stream_cap ? 1u : 0u;
    }
}

__global__ __launch_bounds__(256) void k_compact_emit(PlanCheck pc, const PlanGroup* __restrict__ groups, const PlanTile* __restrict__ tiles,
                                                      const PlanRun* __restrict__ runs, uint64_t n_tiles, const TileHdr* __restrict__ hdrs,
                                                      const uint16_t* __restrict__ staging, const uint16_t* __restrict__ tile_bytes,
                                                      const uint64_t* __restrict__ run_offsets, uint8_t* __restrict__ stream, uint64_t stream_cap) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t t = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= n_tiles || !plan_ok(pc)) return;
    if (hdrs[t].w[7] == 0) return;
    // where the tile's bytes go: the run's offset plus the bytes of the run's earlier tiles
    const PlanTile pt = tiles[t];
    const uint64_t run_first = (uint64_t)groups[pt.group].first_tile + runs[pt.run].first_tile;
    uint32_t x = (run_first + lane < t) ? (uint32_t)tile_bytes[run_first + lane] : 0u;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += (uint32_t)__shfl_xor((int)x, off);
    const uint64_t out = run_offsets[pt.run] + x;
    encode_tile(hdrs, staging, t, lane, [&](bool keep, uint32_t b0, uint32_t b1, bool is_long, uint32_t offset) {
        const uint64_t o = out + offset;
        if (keep && o < stream_cap) stream[o] = (uint8_t)b0;
        if (is_long && o + 1 < stream_cap) stream[o + 1] = (uint8_t)b1;
    });
}

int launch_pack_compact(PlanCheck pc, const PlanGroup* groups, const PlanTile* tiles, const PlanRun* runs, uint64_t n_tiles,
                        uint64_t n_runs, uint32_t n_groups, const TileHdr* hdrs, const uint16_t* staging, uint8_t* stream_out,
                        uint64_t stream_cap, uint16_t* tile_bytes_out, uint64_t* run_offsets_out, vgc_group_hdr* hdrs_out,
                        vgc_pack_status* status_out, hipStream_t stream) {
    const uint32_t tb = (uint32_t)((n_tiles + 3) / 4), rb = (uint32_t)((n_runs + 3) / 4);
    hipLaunchKernelGGL(k_compact_count, dim3(tb), dim3(256), 0, stream, pc, n_tiles, hdrs, staging, tile_bytes_out);
    hipLaunchKernelGGL(k_compact_runsum, dim3(rb), dim3(256), 0, stream, pc, groups, runs, n_runs, tile_bytes_out, run_offsets_out);
    hipLaunchKernelGGL(k_compact_scan, dim3(1), dim3(1024), 0, stream, pc, groups, tiles, n_runs, n_groups, run_offsets_out, hdrs_out,
                       status_out, stream_cap);
    hipLaunchKernelGGL(k_compact_emit, dim3(tb), dim3(256), 0, stream, pc, groups, tiles, runs, n_tiles, hdrs, staging, tile_bytes_out,
                       run_offsets_out, stream_out, stream_cap);
    return hip_check(hipGetLastError(), "launch compact pack kernels");
}

// ------------------------------------------------------------------------------------------------
// decoder: several messages in one pass over the dense buffer, message order kept per element
// ------------------------------------------------------------------------------------------------
struct CompactArgs {
    const uint8_t* streams[kBatchMax];
    const uint16_t* tile_bytes[kBatchMax];
    const uint64_t* run_offsets[kBatchMax];
    const vgc_group_hdr* hdrs[kBatchMax];
    uint64_t n_bytes[kBatchMax];
    uint32_t p;
};

typedef float f4c __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_unpack_compact(PlanCheck pc, CompactArgs A, const PlanGroup* __restrict__ groups,
                                                        const PlanRun* __restrict__ runs, uint32_t n_runs, float scale,
                                                        float* __restrict__ dense, int overwrite) {
    __shared__ __attribute__((aligned(16))) float sh_tile[4][kTile];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t run = blockIdx.x * 4 + wave;
    if (run >= n_runs || !plan_ok(pc)) return;
    float* T = sh_tile[wave];
    const uint32_t k = runs[run].group;
    const PlanGroup pg = groups[k];
    const uint32_t nt_group = (pg.size + kTile - 1) / kTile;
    const uint32_t t0 = runs[run].first_tile, t1 = min(t0 + (uint32_t)kRunTiles, nt_group);
    // lane w < p: byte cursor of message w, and the exponent field of the group in that message
    uint64_t cur = 0;
    uint32_t expf = 0;
    if (lane < A.p) {
        cur = A.run_offsets[lane][run];
        expf = A.hdrs[lane][k].exp_field;
    }
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t start = t * kTile;
        const uint32_t m = min(kTile, pg.size - start);
        float* base = dense + pg.offset + start;
        const bool vec = (m == kTile) && ((reinterpret_cast<uintptr_t>(base) & 15u) == 0);
        if (overwrite) {
#pragma unroll
            for (int q = 0; q < 8; ++q) reinterpret_cast<f4c*>(T)[q * 64 + lane] = (f4c){0.f, 0.f, 0.f, 0.f};
        } else if (vec) {
#pragma unroll
            for (int q = 0; q < 8; ++q) reinterpret_cast<f4c*>(T)[q * 64 + lane] = __builtin_nontemporal_load(reinterpret_cast<const f4c*>(base) + q * 64 + lane);
        } else {
            for (uint32_t i = lane; i < kTile; i += 64) T[i] = (i < m) ? base[i] : 0.f;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const uint32_t nb_mine = (lane < A.p) ? (uint32_t)A.tile_bytes[lane][(uint64_t)pg.first_tile + t] : 0u;
        for (uint32_t w = 0; w < A.p; ++w) {
            const uint64_t c0 = ((uint64_t)(uint32_t)__shfl((int)(uint32_t)(cur >> 32), (int)w) << 32) | (uint32_t)__shfl((int)(uint32_t)cur, (int)w);
            const uint32_t nb = (uint32_t)__shfl((int)nb_mine, (int)w);
            const uint32_t ef = (uint32_t)__shfl((int)expf, (int)w);
            const uint8_t* S = A.streams[w] + c0;
            const uint64_t left = A.n_bytes[w] > c0 ? A.n_bytes[w] - c0 : 0;      // a damaged directory never reads past the stream
            int32_t pos_base = -1;                              // position of the last element decoded so far
            uint32_t done = 0;
            while (done < nb) {                                 // 64 bytes at a time, always starting at an element
                const uint32_t i = done + lane;
                const bool valid = i < nb && i < left;
                const uint32_t byte = valid ? (uint32_t)S[i] : 0u;
                // a byte starts an element iff the bytes with bit 7 set directly before it are an even number: such a
                // byte opens a two-byte element when it is itself a start, and is its second byte otherwise
                const uint64_t L = __ballot(valid && (byte & 0x80u));
                const uint64_t zeros_below = ~L & lanes_below(lane);
                const int last_zero = zeros_below ? 63 - __builtin_clzll(zeros_below) : -1;
                const bool is_start = valid && ((((int)lane - 1 - last_zero) & 1) == 0);
                const bool is_long = is_start && (byte & 0x80u);
                const uint32_t next = (uint32_t)__shfl_down((int)byte, 1);
                const bool cut = is_long && lane == 63u;        // its second byte is in the next 64: leave it for the next round
                const uint32_t gap = ((byte >> 4) & 7u) | (is_long ? next << 3 : 0u);
                uint32_t incl = (is_start && !cut) ? gap + 1u : 0u;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const uint32_t y = (uint32_t)__shfl_up((int)incl, off);
                    if (lane >= (uint32_t)off) incl += y;
                }
                const int32_t pos = pos_base + (int32_t)incl;
                const uint32_t d = byte & 7u;
                if (is_start && !cut && (uint32_t)pos < m && ef > d && ef <= 254u) {
                    const float val = __uint_as_float(((ef - d) << 23) | ((byte & 8u) << 28));
                    const float contrib = scale * val;
                    T[pos] = T[pos] + contrib;
                }
                pos_base += (int32_t)__shfl((int)incl, 63);
                done += __ballot(cut) ? 63u : 64u;
            }
            if (lane == w) cur += nb;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (vec) {
#pragma unroll
            for (int q = 0; q < 8; ++q)
                __builtin_nontemporal_store(reinterpret_cast<f4c*>(T)[q * 64 + lane], reinterpret_cast<f4c*>(base) + q * 64 + lane);
        } else {
            for (uint32_t i = lane; i < m; i += 64) base[i] = T[i];
        }
        __builtin_amdgcn_wave_barrier();
    }
}

int launch_unpack_compact_batch(PlanCheck pc, const uint8_t* const* streams, const uint64_t* stream_bytes, const uint16_t* const* tile_bytes,
                                const uint64_t* const* run_offsets, const vgc_group_hdr* const* hdrs, uint32_t p,
                                const PlanGroup* groups, const PlanRun* runs, uint64_t n_runs, float scale, int overwrite,
                                float* dense, hipStream_t stream) {
    const uint32_t blocks = (uint32_t)((n_runs + 3) / 4);
    const uint32_t chunks = p ? (p + kBatchMax - 1) / kBatchMax : 1;
    for (uint32_t ch = 0; ch < chunks; ++ch) {
        CompactArgs A;
        const uint32_t first = ch * kBatchMax;
        A.p = p - first < (uint32_t)kBatchMax ? p - first : (uint32_t)kBatchMax;
        for (uint32_t w = 0; w < (uint32_t)kBatchMax; ++w) {
            const bool on = w < A.p;
            A.streams[w] = on ? streams[first + w] : nullptr;
            A.n_bytes[w] = on ? stream_bytes[first + w] : 0;
            A.tile_bytes[w] = on ? tile_bytes[first + w] : nullptr;
            A.run_offsets[w] = on ? run_offsets[first + w] : nullptr;
            A.hdrs[w] = on ? hdrs[first + w] : nullptr;
        }
        hipLaunchKernelGGL(k_unpack_compact, dim3(blocks), dim3(256), 0, stream, pc, A, groups, runs, (uint32_t)n_runs, scale, dense,
                           (overwrite && ch == 0) ? 1 : 0);
    }
    return hip_check(hipGetLastError(), "launch k_unpack_compact");
}

}  // namespace vgc
