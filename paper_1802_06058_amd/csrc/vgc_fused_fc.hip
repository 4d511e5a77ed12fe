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

// Square of two packed bf16 values: float32 product, rounded to nearest-even bf16 (2^-9 relative per factor).
__device__ __forceinline__ uint32_t sq_bf16x2(uint32_t w) {
    const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xFFFF0000u);
    const uint32_t a = __float_as_uint(lo * lo), b = __float_as_uint(hi * hi);
    return ((a + 0x7FFFu + ((a >> 16) & 1u)) >> 16) | ((b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u);
}
__device__ __forceinline__ u4v sq_bf16x8(u4v x) {
    u4v y;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = sq_bf16x2(x[e]);
    return y;
}

constexpr int kFusedTiles = 16;                     // tiles per workgroup
constexpr int kLdsPitch = kTile + 16;               // floats per staged tile: the four tiles of a pass start 16 banks apart

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

// kR: rows of [J, C] per tile (1: C is a multiple of 2048 and a tile is a piece of a row; 2, 4, 8: C = 2048 / kR).
template <int kR, bool kBf16>
__global__ __launch_bounds__(512) void k_fused_fc_select(PlanCheck pc, uint32_t* __restrict__ flags, FusedArgs A,
                                                         const PlanGroup* __restrict__ groups,
                                                         TileHdr* __restrict__ hdrs, uint32_t* __restrict__ bitmap,
                                                         uint16_t* __restrict__ staging) {
    __shared__ __attribute__((aligned(16))) float lds_g[4][kLdsPitch];
    __shared__ __attribute__((aligned(16))) float lds_s[4][kLdsPitch];
    __shared__ TileLds sh[2];

    const bool ok = plan_ok(pc);
    if (blockIdx.x == 0 && threadIdx.x == 0) flags[0] = ok ? 0u : 1u;
    if (!ok) return;

    const uint32_t tid = threadIdx.x, lane = tid & 63u, tid_h = tid & 255u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6), half = wave >> 2;      // uniform per wave: scalar registers, scalar branches
    const uint32_t lrow = lane & 15u, lgrp = lane >> 4;
    const PlanGroup pg = groups[A.group];
    constexpr uint32_t Cb = kTile / kR;                       // columns one block spans
    constexpr uint32_t CT = Cb / 16;                          // 16-column MFMA tiles per row tile
    const uint32_t ncb = kR == 1 ? A.C / kTile : 1u;          // column blocks
    const uint32_t cb = kR == 1 ? blockIdx.x % ncb : 0u, rb = kR == 1 ? blockIdx.x / ncb : blockIdx.x;
    const uint32_t j0 = rb * 16u * kR;                        // first row of the block
    const uint32_t colbase = cb * kTile;
    const uint32_t nt_group = (pg.size + kTile - 1) / kTile;

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

    // ---- the block's tiles.  Accumulator element i of MFMA tile t is row 16 rt + 4 lgrp + i, column 16 (ct0 + t) + lrow
    // of the block; it belongs to tile tl = row / kR at position (row % kR) Cb + column.  Four tiles pass through LDS at a
    // time: for kR = 1 pass p takes the tiles with tl % 4 = p (accumulator element p of every lane: all lanes write),
    // otherwise the tiles 4 p .. 4 p + 3.  Step s = (pass, round): half h of the workgroup runs tile slot 2 round + h.
    auto tile_of = [&](int p, uint32_t slot) -> uint32_t { return kR == 1 ? 4u * slot + (uint32_t)p : 4u * (uint32_t)p + slot; };
    struct Ref { uint64_t base; uint32_t t, m, in_group; bool live, vec; };
    auto ref_of = [&](int step) -> Ref {
        const uint32_t tl = tile_of(step >> 1, 2u * (uint32_t)(step & 1) + half);
        Ref q;
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
    auto load_rv = [&](const Ref& q, float (&R)[8], float (&V)[8]) {
        if (q.vec) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const f4 r4 = q.live ? __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.r + q.base) + u * 256 + tid_h) : (f4){0.f, 0.f, 0.f, 0.f};
                const f4 v4 = q.live ? __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.v + q.base) + u * 256 + tid_h) : (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < 4; ++c) { R[u * 4 + c] = r4[c]; V[u * 4 + c] = v4[c]; }
            }
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t i = u * 256 + tid_h;
                const bool in = q.live && i < q.m;
                R[u] = in ? __builtin_nontemporal_load(A.r + q.base + i) : 0.f;
                V[u] = in ? __builtin_nontemporal_load(A.v + q.base + i) : 0.f;
            }
        }
    };

    float Rn[8], Vn[8];
    Ref cur = ref_of(0);
    load_rv(cur, Rn, Vn);
#pragma unroll
    for (int step = 0; step < 8; ++step) {
        const int p = step >> 1;
        if ((step & 1) == 0) {
            if (kR == 1) {
#pragma unroll
                for (int t = 0; t < 16; ++t) {
                    const uint32_t col = 16u * (ct0 + t) + lrow;
                    lds_g[lgrp][col] = acc_g[t][p];
                    lds_s[lgrp][col] = acc_s[t][p];
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t row = 16u * rt + 4u * lgrp + i, tl = row / kR;
                    if ((tl >> 2) == (uint32_t)p) {
#pragma unroll
                        for (int t = 0; t < 16; ++t) {
                            const uint32_t pos = (row % kR) * Cb + 16u * (ct0 + t) + lrow;
                            lds_g[tl & 3u][pos] = acc_g[t][i];
                            lds_s[tl & 3u][pos] = acc_s[t][i];
                        }
                    }
                }
            }
            __syncthreads();
        }
        float R[8], V[8], G[8], S[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { R[e] = Rn[e]; V[e] = Vn[e]; }
        const Ref q = cur;
        if (step + 1 < 8) {
            cur = ref_of(step + 1);
            load_rv(cur, Rn, Vn);
        }
        const uint32_t slot = 2u * (uint32_t)(step & 1) + half;
        if (q.vec) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const f4 g4 = reinterpret_cast<const f4*>(lds_g[slot])[u * 256 + tid_h];
                const f4 s4 = reinterpret_cast<const f4*>(lds_s[slot])[u * 256 + tid_h];
#pragma unroll
                for (int c = 0; c < 4; ++c) { G[u * 4 + c] = g4[c]; S[u * 4 + c] = s4[c]; }
                if (A.g_out && q.live) {
                    const size_t o = (size_t)q.in_group * kTile;
                    reinterpret_cast<f4*>(A.g_out + o)[u * 256 + tid_h] = g4;
                    reinterpret_cast<f4*>(A.s_out + o)[u * 256 + tid_h] = s4;
                }
            }
            tile_core<true, false, true>(G, S, R, V, A.r + q.base, A.v + q.base, q.m, q.live, hdrs + q.t, bitmap + (size_t)q.t * (kTile / 32),
                                         staging + (size_t)q.t * kTile, A.alpha, A.zeta, 0.0f, sh[half], tid_h);
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t i = u * 256 + tid_h;
                G[u] = lds_g[slot][i];
                S[u] = lds_s[slot][i];
                if (A.g_out && q.live && i < q.m) {
                    const size_t o = (size_t)q.in_group * kTile + i;
                    A.g_out[o] = G[u];
                    A.s_out[o] = S[u];
                }
            }
            tile_core<false, false, true>(G, S, R, V, A.r + q.base, A.v + q.base, q.m, q.live, hdrs + q.t, bitmap + (size_t)q.t * (kTile / 32),
                                          staging + (size_t)q.t * kTile, A.alpha, A.zeta, 0.0f, sh[half], tid_h);
        }
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
