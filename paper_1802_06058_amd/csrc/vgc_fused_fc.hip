// The statistic of a fully-connected layer fused into the accumulate / test / reset-or-decay pass of Alg. 1:
// g = c X^T D and s = c^2 (X.X)^T (D.D) (the first two lines of the loop body, Section 5's 2 N |B|
// multiply-adds each) are formed on the matrix cores and consumed in place by the rest of the loop body
// (r += g, v += s, the test of Eq. 2, reset or decay, and the first half of Encode()), so that neither g nor
// s of the layer ever reaches HBM: 16 bytes per parameter (r and v read and written) instead of 32.
//
// A workgroup (8 waves) owns 16 tiles of the select pass, i.e. 16 x 2048 consecutive-per-tile elements of the
// weight [J, C]: 16 rows x 2048 columns when C is a multiple of 2048 (a tile is a piece of a row), 16 R whole
// rows when C = 2048 / R (a tile is R rows).  The K = |B| contraction is short, so the operands are read
// from a pre-transposed copy (K contiguous per row / column: one 16-byte load per MFMA fragment, no LDS) that a
// small kernel prepares, and all 16 tiles' g and s stay in the accumulators (2 x 64 registers per lane).  They
// then pass through LDS four tiles at a time, which turns the MFMA layout into the tile order the select
// pass works in, and each half of the workgroup runs the tile core on one tile at a time while the r and v
// of the next tile are already in flight.
#include "vgc_tile_core.h"

namespace vgc {

typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef uint32_t u4v __attribute__((ext_vector_type(4)));

// [B, W] row-major -> [W, Kp] with the B values of a column contiguous and zeros up to Kp.  One thread per
// (column, 16-byte piece of K); neighbouring threads take neighbouring columns, so the reads coalesce.
template <typename T>
__global__ __launch_bounds__(256) void k_fc_transpose(const T* __restrict__ src, uint32_t B, uint32_t W, uint32_t Kp,
                                                      T* __restrict__ dst) {
    constexpr uint32_t kPer = 16 / sizeof(T);
    const uint64_t idx = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const uint32_t pieces = Kp / kPer;
    if (idx >= (uint64_t)W * pieces) return;
    const uint32_t w = (uint32_t)(idx % W), kc = (uint32_t)(idx / W);
    T out[kPer];
#pragma unroll
    for (uint32_t i = 0; i < kPer; ++i) {
        const uint32_t k = kc * kPer + i;
        out[i] = k < B ? src[(size_t)k * W + w] : (T)0;
    }
    *reinterpret_cast<u4v*>(dst + (size_t)w * Kp + (size_t)kc * kPer) = *reinterpret_cast<const u4v*>(out);
}

// Squares of packed bf16 values: float32 products, rounded to nearest-even bf16 (2^-9 relative per factor) by the
// hardware's packed conversion.
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
typedef float f2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t sq_bf16x2(uint32_t w) {
    const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xFFFF0000u);
    const f2v p = {lo * lo, hi * hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf2v));
}
__device__ __forceinline__ u4v sq_bf16x8(u4v x) {
    u4v y;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = sq_bf16x2(x[e]);
    return y;
}

constexpr int kFusedTiles = 16;                     // tiles per workgroup
constexpr int kLdsPitch = kTile + 8;                // floats per staged tile: slots 2 q and 2 q + 2 start 16 banks apart

struct FusedArgs {
    const void* XT;          // [J, Kp]
    const void* DT;          // [C, Kp]
    uint32_t J, C, Kp;
    float cg, cs;
    float* r;                // whole parameter space
    float* v;
    float* g_out;            // optional [J, C] of this layer
    float* s_out;
    uint32_t group;
    float alpha, zeta;
};

// One tile of the block as a wave sees it.
struct TileRef {
    uint64_t base;           // first element in the flat parameter space
    uint32_t t;              // tile number in the plan (scratch records)
    uint32_t in_group;       // tile number inside the group
    uint32_t m;              // elements
    bool live;               // false: past the end of the layer (the wave only keeps the barriers company)
    bool vec;                // whole, 16-byte aligned tile: 16-byte accesses
};

// Alg. 1's loop body on one tile by ONE wave, from g and s staged in LDS (lg, ls: this wave's slot) and r, v in memory.
// No workgroup barrier inside: the eight waves of a workgroup each run their own tile.  Element e = 4 u + c of a lane
// is tile element 256 u + 4 lane + c (whole aligned tiles: 16-byte accesses; R4, V4 hold chunks u = 0, 1 on entry, the
// rest is loaded two chunks ahead), so chunk u is a contiguous range of 256 elements in (lane, c) order.  The slot's g
// area is reused for the index-ordered staged entries once g has been consumed.
__device__ __forceinline__ void wave_tile_vec(const FusedArgs& A, const TileRef& q, float* lg, const float* ls, f4 (&R4)[4], f4 (&V4)[4],
                                              TileHdr* __restrict__ hdrs, uint32_t* __restrict__ bitmap, uint16_t* __restrict__ staging,
                                              uint32_t lane) {
    float* r = A.r + q.base;
    float* v = A.v + q.base;
    uint32_t* bm = bitmap + (size_t)q.t * (kTile / 32);
    uint32_t bits[32];
    uint32_t sendmask = 0, etr = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const f4 g4 = reinterpret_cast<const f4*>(lg)[u * 64 + lane];
        const f4 s4 = reinterpret_cast<const f4*>(ls)[u * 64 + lane];
        const f4 r4 = R4[u & 3], v4 = V4[u & 3];
        if (u + 4 < 8) {                                     // chunk u + 4 into the registers chunk u leaves
            R4[u & 3] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(r) + (u + 4) * 64 + lane);
            V4[u & 3] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(v) + (u + 4) * 64 + lane);
        }
        if (A.g_out) {
            const size_t o = (size_t)q.in_group * kTile;
            reinterpret_cast<f4*>(A.g_out + o)[u * 64 + lane] = g4;
            reinterpret_cast<f4*>(A.s_out + o)[u * 64 + lane] = s4;
        }
        f4 ro, vo;
        uint32_t nib = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float a, b;
            const bool send = alg1_step(g4[c], s4[c], r4[c], v4[c], A.alpha, A.zeta, a, b, bits[u * 4 + c]);
            ro[c] = a;
            vo[c] = b;
            nib |= (send ? 1u : 0u) << c;
            if (send) etr = max(etr, (bits[u * 4 + c] & 0x7FFFFFFFu) >> 23);
        }
        __builtin_nontemporal_store(ro, reinterpret_cast<f4*>(r) + u * 64 + lane);
        __builtin_nontemporal_store(vo, reinterpret_cast<f4*>(v) + u * 64 + lane);
        sendmask |= nib << (4 * u);
        // send bitmap: bit 256 u + 4 lane + c; eight lanes make one word
        uint32_t x = nib << (4 * (lane & 7u));
        x |= (uint32_t)__shfl_xor((int)x, 1);
        x |= (uint32_t)__shfl_xor((int)x, 2);
        x |= (uint32_t)__shfl_xor((int)x, 4);
        if ((lane & 7u) == 0) bm[u * 8 + (lane >> 3)] = x;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) etr = max(etr, (uint32_t)__shfl_xor((int)etr, off));

    // ---- tile-relative exponent codes (Section 4.4's rounding recipe), histogram, index-ordered compaction ----
    uint16_t* stage = reinterpret_cast<uint16_t*>(lg);
    uint64_t hist = 0;                                       // nine 6-bit counters (a lane has at most 32 entries)
    uint32_t base = 0;                                       // entries of the chunks before u (uniform)
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        uint32_t entry[4], below = 0, total = 0, st = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int e = u * 4 + c;
            const uint32_t ab = bits[e] & 0x7FFFFFFFu;
            const uint32_t ernd = (ab + 0x00400000u) >> 23;  // add one at the mantissa's top bit, drop the mantissa
            const uint32_t rel = etr + 1u - ernd;            // >= 0 for sent elements
            const bool staged = ((sendmask >> e) & 1u) && ernd >= 1u && rel <= 8u;
            entry[c] = ((rel & 15u) << 12) | ((bits[e] >> 31) << 11) | (uint32_t)(u * 256 + c) + 4u * lane;
            hist += staged ? (1ull << (staged ? 6u * rel : 0u)) : 0ull;
            const uint64_t b = __ballot(staged);
            below += rank_below(b);
            total += (uint32_t)__popcll(b);
            st |= (staged ? 1u : 0u) << c;
        }
        uint32_t pos = base + below;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if ((st >> c) & 1u) stage[pos] = (uint16_t)entry[c];
            pos += (st >> c) & 1u;
        }
        base += total;
    }
    // wave totals of the nine bins: 12-bit fields in two 64-bit words (bins 0..4, 5..8)
    uint64_t h_lo = 0, h_hi = 0;
#pragma unroll
    for (int j = 0; j < 5; ++j) h_lo |= ((hist >> (6 * j)) & 63ull) << (12 * j);
#pragma unroll
    for (int j = 5; j < 9; ++j) h_hi |= ((hist >> (6 * j)) & 63ull) << (12 * (j - 5));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        h_lo += ((uint64_t)(uint32_t)__shfl_xor((int)(uint32_t)(h_lo >> 32), off) << 32) | (uint32_t)__shfl_xor((int)(uint32_t)h_lo, off);
        h_hi += ((uint64_t)(uint32_t)__shfl_xor((int)(uint32_t)(h_hi >> 32), off) << 32) | (uint32_t)__shfl_xor((int)(uint32_t)h_hi, off);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    uint16_t* out = staging + (size_t)q.t * kTile;
    for (uint32_t piece = lane; piece * 8u < base; piece += 64u)
        __builtin_nontemporal_store(reinterpret_cast<const uint4v*>(stage)[piece], reinterpret_cast<uint4v*>(out) + piece);
    if (lane == 0) {
        uint32_t h[kRelBins];
#pragma unroll
        for (int j = 0; j < 5; ++j) h[j] = (uint32_t)(h_lo >> (12 * j)) & 0xFFFu;
#pragma unroll
        for (int j = 5; j < 9; ++j) h[j] = (uint32_t)(h_hi >> (12 * (j - 5))) & 0xFFFu;
        uint4 lo = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        uint4 hi = make_uint4(h[8] | (etr << 16), 0u, 0u, 0u);
        reinterpret_cast<uint4*>(hdrs + q.t)[0] = lo;
        reinterpret_cast<uint4*>(hdrs + q.t)[1] = hi;
    }
}

// The same for a tile that is partial or not 16-byte aligned: element e of a lane is tile element 64 e + lane
// (4-byte accesses, bounds-checked by m), chunk e is a contiguous range of 64 elements in lane order.
__device__ __forceinline__ void wave_tile_any(const FusedArgs& A, const TileRef& q, float* lg, const float* ls,
                                              TileHdr* __restrict__ hdrs, uint32_t* __restrict__ bitmap, uint16_t* __restrict__ staging,
                                              uint32_t lane) {
    float* r = A.r + q.base;
    float* v = A.v + q.base;
    uint32_t* bm = bitmap + (size_t)q.t * (kTile / 32);
    uint32_t bits[32];
    uint32_t sendmask = 0, etr = 0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const uint32_t i = (uint32_t)e * 64u + lane;
        const bool in = i < q.m;
        const float g1 = lg[i], s1 = ls[i];
        const float r1 = in ? __builtin_nontemporal_load(r + i) : 0.f, v1 = in ? __builtin_nontemporal_load(v + i) : 0.f;
        if (A.g_out && in) {
            A.g_out[(size_t)q.in_group * kTile + i] = g1;
            A.s_out[(size_t)q.in_group * kTile + i] = s1;
        }
        float a, b;
        const bool send = alg1_step(g1, s1, r1, v1, A.alpha, A.zeta, a, b, bits[e]) && in;
        if (in) {
            __builtin_nontemporal_store(a, r + i);
            __builtin_nontemporal_store(b, v + i);
        }
        sendmask |= (send ? 1u : 0u) << e;
        if (send) etr = max(etr, (bits[e] & 0x7FFFFFFFu) >> 23);
        const uint64_t bal = __ballot(send);
        if (lane == 0) *reinterpret_cast<uint2*>(bm + 2 * e) = make_uint2((uint32_t)bal, (uint32_t)(bal >> 32));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) etr = max(etr, (uint32_t)__shfl_xor((int)etr, off));
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // every lane's reads of lg precede the entries written over it
    __builtin_amdgcn_wave_barrier();
    uint16_t* stage = reinterpret_cast<uint16_t*>(lg);
    uint32_t h[kRelBins];
#pragma unroll
    for (int j = 0; j < (int)kRelBins; ++j) h[j] = 0;
    uint32_t base = 0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const uint32_t ab = bits[e] & 0x7FFFFFFFu;
        const uint32_t ernd = (ab + 0x00400000u) >> 23;
        const uint32_t rel = etr + 1u - ernd;
        const bool staged = ((sendmask >> e) & 1u) && ernd >= 1u && rel <= 8u;
        const uint32_t entry = ((rel & 15u) << 12) | ((bits[e] >> 31) << 11) | ((uint32_t)e * 64u + lane);
#pragma unroll
        for (int j = 0; j < (int)kRelBins; ++j) h[j] += (uint32_t)__popcll(__ballot(staged && rel == (uint32_t)j));
        const uint64_t b = __ballot(staged);
        if (staged) stage[base + rank_below(b)] = (uint16_t)entry;
        base += (uint32_t)__popcll(b);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    uint16_t* out = staging + (size_t)q.t * kTile;
    for (uint32_t piece = lane; piece * 8u < base; piece += 64u)
        __builtin_nontemporal_store(reinterpret_cast<const uint4v*>(stage)[piece], reinterpret_cast<uint4v*>(out) + piece);
    if (lane == 0) {
        uint4 lo = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        uint4 hi = make_uint4(h[8] | (etr << 16), 0u, 0u, 0u);
        reinterpret_cast<uint4*>(hdrs + q.t)[0] = lo;
        reinterpret_cast<uint4*>(hdrs + q.t)[1] = hi;
    }
}

// kR: rows of [J, C] per tile (1: C is a multiple of 2048 and a tile is a piece of a row; 2, 4, 8: C = 2048 / kR).
template <int kR, bool kBf16>
__global__ __launch_bounds__(512) void k_fused_fc_select(PlanCheck pc, uint32_t* __restrict__ flags, FusedArgs A,
                                                         const PlanGroup* __restrict__ groups,
                                                         TileHdr* __restrict__ hdrs, uint32_t* __restrict__ bitmap,
                                                         uint16_t* __restrict__ staging) {
    __shared__ __attribute__((aligned(16))) float lds_g[8][kLdsPitch];
    __shared__ __attribute__((aligned(16))) float lds_s[8][kLdsPitch];

    const bool ok = plan_ok(pc);
    if (blockIdx.x == 0 && threadIdx.x == 0) flags[0] = ok ? 0u : 1u;
    if (!ok) return;

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform per wave: scalar registers, scalar branches
    const uint32_t lrow = lane & 15u, lgrp = lane >> 4;
    const PlanGroup pg = groups[A.group];
    constexpr uint32_t Cb = kTile / kR;                       // columns one block spans
    constexpr uint32_t CT = Cb / 16;                          // 16-column MFMA tiles per row tile
    const uint32_t ncb = kR == 1 ? A.C / kTile : 1u;          // column blocks
    const uint32_t cb = kR == 1 ? blockIdx.x % ncb : 0u, rb = kR == 1 ? blockIdx.x / ncb : blockIdx.x;
    const uint32_t j0 = rb * 16u * kR;                        // first row of the block
    const uint32_t colbase = cb * kTile;
    const uint32_t nt_group = (pg.size + kTile - 1) / kTile;

    // The block's 16 tiles pass through LDS eight at a time; wave w runs the tile in slot w.  Accumulator element i of MFMA
    // tile t of a lane is row 16 rt + 4 lgrp + i, column 16 (ct0 + t) + lrow of the block; it belongs to tile tl = row / kR at
    // position (row % kR) Cb + column.  For kR = 1 pass p takes elements i = 2 p, 2 p + 1 of every lane (tiles 4 lgrp + i, slot
    // 2 lgrp + i % 2: all lanes write), otherwise the tiles 8 p .. 8 p + 7.
    auto ref_of = [&](int p) -> TileRef {
        const uint32_t tl = kR == 1 ? 4u * (wave >> 1) + 2u * (uint32_t)p + (wave & 1u) : 8u * (uint32_t)p + wave;
        TileRef q;
        q.in_group = kR == 1 ? (j0 + tl) * ncb + cb : (uint32_t)blockIdx.x * kFusedTiles + tl;
        q.live = kR == 1 ? (j0 + tl) < A.J : q.in_group < nt_group;
        if (!q.live) q.in_group = 0;
        q.t = pg.first_tile + q.in_group;
        q.base = pg.offset + (uint64_t)q.in_group * kTile;
        q.m = min(kTile, pg.size - q.in_group * kTile);
        q.vec = q.live && q.m == kTile && ((reinterpret_cast<uintptr_t>(A.r + q.base) | reinterpret_cast<uintptr_t>(A.v + q.base)) & 15u) == 0 &&
                (!A.g_out || ((reinterpret_cast<uintptr_t>(A.g_out) | reinterpret_cast<uintptr_t>(A.s_out)) & 15u) == 0);
        return q;
    };
    // r and v of the first four chunks of a tile, requested early: they arrive while the matrix cores (pass 0) or the
    // previous tile's compaction (pass 1) are busy
    f4 R4[4], V4[4];
    auto prefetch = [&](const TileRef& q) {
        if (q.vec) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                R4[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.r + q.base) + u * 64 + lane);
                V4[u] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.v + q.base) + u * 64 + lane);
            }
        }
    };
    TileRef q0 = ref_of(0);
    prefetch(q0);

    // ---- contraction: this wave's 16 MFMA tiles (one row tile, 16 column tiles) ----
    const uint32_t rt = (16u * wave) / CT, ct0 = (16u * wave) % CT;
    f4v acc_g[16], acc_s[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) { acc_g[t] = (f4v){0.f, 0.f, 0.f, 0.f}; acc_s[t] = (f4v){0.f, 0.f, 0.f, 0.f}; }
    const uint32_t arow = j0 + 16u * rt + lrow;
    const bool arow_ok = arow < A.J;
    if (kBf16) {
        const uint16_t* XT = static_cast<const uint16_t*>(A.XT);
        const uint16_t* DT = static_cast<const uint16_t*>(A.DT);
        const uint16_t* ap = XT + (size_t)(arow_ok ? arow : 0u) * A.Kp + 8u * lgrp;
        const uint16_t* bp = DT + (size_t)(colbase + 16u * ct0 + lrow) * A.Kp + 8u * lgrp;
        for (uint32_t k0 = 0; k0 < A.Kp; k0 += 32) {
            u4v a = *reinterpret_cast<const u4v*>(ap + k0);
            if (!arow_ok) a = (u4v){0u, 0u, 0u, 0u};
            const u4v a2 = sq_bf16x8(a);
#pragma unroll
            for (int tb = 0; tb < 16; tb += 8) {
                u4v b[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) b[t] = *reinterpret_cast<const u4v*>(bp + (size_t)(tb + t) * 16u * A.Kp + k0);
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const u4v b2 = sq_bf16x8(b[t]);
                    acc_g[tb + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8v, a), __builtin_bit_cast(bf8v, b[t]), acc_g[tb + t], 0, 0, 0);
                    acc_s[tb + t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8v, a2), __builtin_bit_cast(bf8v, b2), acc_s[tb + t], 0, 0, 0);
                }
            }
        }
    } else {
        // float32: v_mfma_f32_16x16x4_f32 takes one k per lane group; a lane loads four consecutive k at once and
        // k-step i of a group of 16 uses element i, so lane group q supplies k = 16 step + 4 q + i (the same
        // assignment for both operands, every k exactly once)
        const float* XT = static_cast<const float*>(A.XT);
        const float* DT = static_cast<const float*>(A.DT);
        const float* ap = XT + (size_t)(arow_ok ? arow : 0u) * A.Kp + 4u * lgrp;
        const float* bp = DT + (size_t)(colbase + 16u * ct0 + lrow) * A.Kp + 4u * lgrp;
        for (uint32_t k0 = 0; k0 < A.Kp; k0 += 16) {
            f4v a = *reinterpret_cast<const f4v*>(ap + k0);
            if (!arow_ok) a = (f4v){0.f, 0.f, 0.f, 0.f};
            const f4v a2 = a * a;
#pragma unroll
            for (int tb = 0; tb < 16; tb += 8) {
                f4v b[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) b[t] = *reinterpret_cast<const f4v*>(bp + (size_t)(tb + t) * 16u * A.Kp + k0);
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const f4v b2 = b[t] * b[t];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        acc_g[tb + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[t][i], acc_g[tb + t], 0, 0, 0);
                        acc_s[tb + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[i], b2[i], acc_s[tb + t], 0, 0, 0);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 16; ++t) { acc_g[t] = acc_g[t] * A.cg; acc_s[t] = acc_s[t] * A.cs; }

#pragma unroll
    for (int p = 0; p < 2; ++p) {
        if (p) __syncthreads();                               // every wave is done with the slots of pass 0
        if (kR == 1) {
#pragma unroll
            for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                for (int t = 0; t < 16; ++t) {
                    const uint32_t col = 16u * (ct0 + t) + lrow;
                    lds_g[2u * lgrp + ii][col] = acc_g[t][2 * p + ii];
                    lds_s[2u * lgrp + ii][col] = acc_s[t][2 * p + ii];
                }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t row = 16u * rt + 4u * lgrp + i, tl = row / kR;
                if ((tl >> 3) == (uint32_t)p) {
#pragma unroll
                    for (int t = 0; t < 16; ++t) {
                        const uint32_t pos = (row % kR) * Cb + 16u * (ct0 + t) + lrow;
                        lds_g[tl & 7u][pos] = acc_g[t][i];
                        lds_s[tl & 7u][pos] = acc_s[t][i];
                    }
                }
            }
        }
        __syncthreads();
        const TileRef q = p == 0 ? q0 : ref_of(1);
        if (p == 1) prefetch(q);
        if (q.vec) wave_tile_vec(A, q, lds_g[wave], lds_s[wave], R4, V4, hdrs, bitmap, staging, lane);
        else if (q.live) wave_tile_any(A, q, lds_g[wave], lds_s[wave], hdrs, bitmap, staging, lane);
    }
}

// Shapes the fused kernel takes: C a multiple of 2048 (a tile is a piece of a row) or C = 1024, 512, 256 (a tile is
// 2, 4, 8 whole rows).  0 = not supported.
static int fused_rows_per_tile(uint32_t C) {
    if (C % kTile == 0) return 1;
    if (C == 1024) return 2;
    if (C == 512) return 4;
    if (C == 256) return 8;
    return 0;
}

static uint32_t fused_kp(int dtype, uint32_t B) { return dtype == VGC_BF16 ? (B + 31u) / 32u * 32u : (B + 15u) / 16u * 16u; }

size_t fused_fc_workspace_bytes(int dtype, uint32_t B, uint32_t J, uint32_t C) {
    if (fused_rows_per_tile(C) == 0 || B == 0 || J == 0) return 0;
    const size_t es = dtype == VGC_BF16 ? 2 : 4;
    return ((size_t)J + C) * fused_kp(dtype, B) * es;
}

int launch_fused_fc_select(PlanCheck pc, uint32_t* flags, int dtype, const void* X, const void* D, uint32_t B, uint32_t J, uint32_t C,
                           float c, float* r, float* v, const PlanGroup* groups, uint32_t group, TileHdr* hdrs, uint32_t* bitmap,
                           uint16_t* staging, float alpha, float zeta, void* workspace, float* g_out, float* s_out, hipStream_t stream) {
    const int kr = fused_rows_per_tile(C);
    if (kr == 0) { set_error("vgc_sqgrad_accumulate_select: C = %u is neither a multiple of 2048 nor 256, 512 or 1024", C); return VGC_ERR_SIZE; }
    const uint32_t Kp = fused_kp(dtype, B);
    const size_t es = dtype == VGC_BF16 ? 2 : 4;
    char* ws = static_cast<char*>(workspace);
    void* XT = ws;
    void* DT = ws + (size_t)J * Kp * es;
    const uint32_t per = 16 / (uint32_t)es;
    const uint64_t nx = (uint64_t)J * (Kp / per), nd = (uint64_t)C * (Kp / per);
    if (dtype == VGC_BF16) {
        hipLaunchKernelGGL(k_fc_transpose<uint16_t>, dim3((uint32_t)((nx + 255) / 256)), dim3(256), 0, stream, (const uint16_t*)X, B, J, Kp, (uint16_t*)XT);
        hipLaunchKernelGGL(k_fc_transpose<uint16_t>, dim3((uint32_t)((nd + 255) / 256)), dim3(256), 0, stream, (const uint16_t*)D, B, C, Kp, (uint16_t*)DT);
    } else {
        hipLaunchKernelGGL(k_fc_transpose<float>, dim3((uint32_t)((nx + 255) / 256)), dim3(256), 0, stream, (const float*)X, B, J, Kp, (float*)XT);
        hipLaunchKernelGGL(k_fc_transpose<float>, dim3((uint32_t)((nd + 255) / 256)), dim3(256), 0, stream, (const float*)D, B, C, Kp, (float*)DT);
    }
    FusedArgs A;
    A.XT = XT; A.DT = DT; A.J = J; A.C = C; A.Kp = Kp; A.cg = c; A.cs = c * c; A.r = r; A.v = v; A.g_out = g_out; A.s_out = s_out;
    A.group = group; A.alpha = alpha; A.zeta = zeta;
    const uint64_t rows_per_block = 16ull * kr;
    const uint64_t nblk = (J + rows_per_block - 1) / rows_per_block * (kr == 1 ? C / kTile : 1u);
    if (nblk > 0x7FFFFFFFull) { set_error("vgc_sqgrad_accumulate_select: shape exceeds the launch limit"); return VGC_ERR_SIZE; }
#define VGC_FUSED(KR, BF)                                                                                                     \
    hipLaunchKernelGGL((k_fused_fc_select<KR, BF>), dim3((uint32_t)nblk), dim3(512), 0, stream, pc, flags, A, groups, hdrs, \
                       bitmap, staging)
    const bool bf = dtype == VGC_BF16;
    if (kr == 1) { if (bf) VGC_FUSED(1, true); else VGC_FUSED(1, false); }
    else if (kr == 2) { if (bf) VGC_FUSED(2, true); else VGC_FUSED(2, false); }
    else if (kr == 4) { if (bf) VGC_FUSED(4, true); else VGC_FUSED(4, false); }
    else { if (bf) VGC_FUSED(8, true); else VGC_FUSED(8, false); }
#undef VGC_FUSED
    return hip_check(hipGetLastError(), "launch k_fused_fc_select");
}

}  // namespace vgc
