// The conv statistic (Section 4.1's per-sample sums for a weight tensor, Section 4.2) of a network's first
// layer, read from the NHWC input: few input channels (an RGB image: Cin = 3), so a pixel's channels are
// not a multiple of 16 bytes and the kernels that move 16-byte pieces of a filter tap do not apply.  Such
// a layer has a small J = kh kw Cin (27 for a 3 x 3 filter, 147 for 7 x 7) and few multiply-adds; what it
// costs is reading the output gradient once, so the kernel is a plain one: a workgroup owns one sample,
// one part of its positions and 64 output channels; per chunk of 32 to 128 positions it gathers the patch
// rows U[p, j] (pixel by pixel for three channels, element by element otherwise) and the rows of D into
// LDS, rows = positions, and multiplies them on the matrix cores; the unsquared partial product of the part
// goes to the workspace and k_sqgrad_reduce_parts adds the parts of each sample, squares, and sums over the
// samples in a fixed order.  What a thread gathers for the chunk after the current one waits in registers
// while the current one is multiplied.
#include "vgc_internal.h"

namespace vgc {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef short s4v __attribute__((ext_vector_type(4)));
typedef short s8v __attribute__((ext_vector_type(8)));
typedef uint32_t u4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s4v* lds_s4v_ptr;

constexpr int kStemJMax = 160;         // J is padded to a multiple of 32
constexpr int kStemBN = 64;            // output channels per workgroup

struct StemGeom {
    uint32_t H, W, Cin, kw, sh, sw, ph, pw, Ho, Wo, J, Jpad;
};

// Positions per chunk: as many as keep the elements a thread holds in registers for the next chunk few
// (16 bytes of D per 256 / (64 / piece) positions, one element of U per position group).
__host__ __device__ constexpr int stem_kc(int esize, int jt) {
    return esize == 2 ? (jt == 1 ? 128 : (jt == 2 ? 64 : 32)) : (jt == 1 ? 64 : 32);
}

// LDS row pitches in bytes (rows are positions; 16 bytes of padding keep four consecutive rows off each other's banks)
__host__ __device__ inline uint32_t stem_pitch_u(uint32_t Jpad, uint32_t esize) { return Jpad * esize + 16u; }
__host__ __device__ inline uint32_t stem_pitch_d(uint32_t esize) { return kStemBN * esize + 16u; }

// kJT = Jpad / 32 (1..5) fixes the workgroup's size (four waves, eight from three row tiles on: ten 32 x 32 tiles on
// four waves would be three on the slowest), the position groups kG = threads / Jpad rounded down to a power of two
// (how many threads share a column of U) and the tiles a wave holds at most, kT = ceil(2 kJT / waves).
__host__ __device__ constexpr int stem_threads(int jt) { return jt >= 3 ? 512 : 256; }

// The three channels of a pixel, aligned like one element: fetched with one 12-byte load (float32) or whatever the
// compiler makes of 6 bytes at a 2-byte boundary (bfloat16).
template <typename T> struct StemPixel3;
template <> struct __attribute__((packed, aligned(4))) StemPixel3<float> { float c[3]; };
template <> struct __attribute__((packed, aligned(2))) StemPixel3<uint16_t> { uint16_t c[3]; };
// pixels a thread holds for the next chunk at most (kPix3)
__host__ __device__ constexpr int stem_pix_max(int esize) { return esize == 2 ? 8 : 4; }

// Position groups of the pixel-wise gather: the largest power of two that threads / taps and the chunk allow.
__host__ __device__ inline uint32_t stem_pix_groups(uint32_t threads, uint32_t taps, uint32_t kc) {
    uint32_t g = 1;
    while (2u * g * taps <= threads && 2u * g <= kc) g *= 2u;
    return g;
}

// kPix3 (Cin = 3): the patch rows are gathered pixel by pixel (one load per tap and position) instead of element by
// element.
template <typename T, int kJT, bool kPix3 = false>
__global__ __launch_bounds__(stem_threads(kJT)) void k_conv_stem(const T* __restrict__ act, const T* __restrict__ D, uint32_t B, uint32_t C,
                                                   StemGeom G, uint32_t parts, float* __restrict__ ws) {
    (void)B;                                                            // (the grid carries the sample count)
    constexpr int kPiece = 16 / (int)sizeof(T), kKC = stem_kc((int)sizeof(T), kJT);
    constexpr int kNT = stem_threads(kJT), kWaves = kNT / 64;
    constexpr int kDTotal = kKC * kStemBN / kPiece;                     // 16-byte pieces of D per chunk
    constexpr int kDPieces = (kDTotal + kNT - 1) / kNT;                 // ... per thread
    extern __shared__ __attribute__((aligned(16))) uint8_t sh[];       // [kKC rows of U][kKC rows of D], rows = positions
    const uint32_t pitch_u = stem_pitch_u(G.Jpad, sizeof(T)), pitch_d = stem_pitch_d(sizeof(T));
    uint8_t* const Ush = sh;
    uint8_t* const Dsh = sh + (size_t)kKC * pitch_u;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t tiles_c = (C + kStemBN - 1) / kStemBN;
    const uint32_t tile_c = blockIdx.x % tiles_c, part = (blockIdx.x / tiles_c) % parts, z = blockIdx.x / (tiles_c * parts);
    const uint32_t P = G.Ho * G.Wo, n_chunks = (P + kKC - 1) / kKC;
    const uint32_t per_part = (n_chunks + parts - 1) / parts;
    const uint32_t q_begin = min(n_chunks, part * per_part), q_end = min(n_chunks, q_begin + per_part);
    const T* act_z = act + (size_t)z * G.H * G.W * G.Cin;
    const T* D_z = D + (size_t)z * P * C;
    const uint32_t c0 = tile_c * kStemBN;

    // ---- what this thread fetches per chunk; the chunk after the current one waits in registers ----
    // D: piece i of the thread is row pl = e / (64 / kPiece), columns c0 + kPiece (e % (64 / kPiece)) .. + kPiece - 1,
    // e = tid + threads x i.
    // U: thread tid < groups * Jpad (groups = kG <= threads / Jpad) owns column j = tid % Jpad of the chunk's [kKC, Jpad] block and
    // the positions pg, pg + groups, ... (pg = tid / Jpad); the column's tap and channel are fixed, so what is left per
    // element is the position's (y, x), carried along from the chunk's first position, and the bounds tests.
    constexpr int kG = kJT == 1 ? 8 : (kJT == 2 ? 4 : (kJT <= 4 ? 4 : 2));   // 256 / 32, 256 / 64, 512 / 96, 512 / 128, 512 / 160
    constexpr int kT = (2 * kJT + kWaves - 1) / kWaves;
    constexpr int kUMax = kKC / kG;                                     // elements of a thread per chunk
    constexpr uint32_t groups = kG;
    u4v d_next[kDPieces];
    T u_next[kUMax];
    const uint32_t uj = tid % G.Jpad, upg = tid / G.Jpad;
    const uint32_t n_u = upg < groups ? (uint32_t)kUMax : 0u;
    const bool u_col = uj < G.J;
    const uint32_t utap = uj / G.Cin, uci = uj - utap * G.Cin, uky = utap / G.kw, ukx = utap - uky * G.kw;
    const int32_t dy = (int32_t)uky - (int32_t)G.ph, dx = (int32_t)ukx - (int32_t)G.pw;
    // kPix3: thread tid < pgroups * taps owns tap tid % taps (columns 3 tap .. + 2) and the positions ppg, ppg + pgroups, ...
    const uint32_t n_taps = kPix3 ? G.J / 3u : 1u, pgroups = stem_pix_groups(kNT, n_taps, kKC);
    const uint32_t ptap = tid % n_taps, ppg = tid / n_taps, pky = ptap / G.kw, pkx = ptap - pky * G.kw;
    constexpr int kStemPixMax = stem_pix_max((int)sizeof(T));
    const uint32_t n_pix = kPix3 && ppg < pgroups ? (uint32_t)kKC / pgroups : 0u;     // <= kStemPixMax (the launcher checks)
    const int32_t pdy = (int32_t)pky - (int32_t)G.ph, pdx = (int32_t)pkx - (int32_t)G.pw;
    StemPixel3<T> pix_next[kPix3 ? kStemPixMax : 1];
    if (kPix3) {                                                        // the columns J .. Jpad - 1 are never staged
        for (uint32_t e = tid * 16u; e < (uint32_t)kKC * pitch_u; e += (uint32_t)kNT * 16u) *reinterpret_cast<u4v*>(Ush + e) = (u4v){0u, 0u, 0u, 0u};
    }
    auto fetch = [&](uint32_t q) {
        const uint32_t p0 = q * kKC;
#pragma unroll
        for (int i = 0; i < kDPieces; ++i) {
            constexpr uint32_t ppr = kStemBN / kPiece;                  // pieces per row
            const uint32_t e = tid + (uint32_t)kNT * i, pl = e / ppr, col = c0 + (e % ppr) * kPiece, p = p0 + pl;
            d_next[i] = (u4v){0u, 0u, 0u, 0u};
            if (e < (uint32_t)kDTotal && p < P && col < C) d_next[i] = *reinterpret_cast<const u4v*>(D_z + (size_t)p * C + col);   // C is a multiple of kPiece
        }
        const uint32_t y0 = p0 / G.Wo, x0 = p0 - y0 * G.Wo;             // (uniform)
        if constexpr (kPix3) {
            uint32_t y = y0, x = x0 + ppg;
#pragma unroll
            for (int i = 0; i < kStemPixMax; ++i) {
                pix_next[i] = StemPixel3<T>{{(T)0, (T)0, (T)0}};
                if ((uint32_t)i < n_pix) {
                    while (x >= G.Wo) { x -= G.Wo; ++y; }
                    const uint32_t iy = (uint32_t)((int32_t)(y * G.sh) + pdy), ix = (uint32_t)((int32_t)(x * G.sw) + pdx);
                    if (y < G.Ho && iy < G.H && ix < G.W) pix_next[i] = *reinterpret_cast<const StemPixel3<T>*>(act_z + ((size_t)iy * G.W + ix) * 3u);
                    x += pgroups;
                }
            }
            return;
        }
        uint32_t y = y0, x = x0 + upg;
#pragma unroll
        for (int i = 0; i < kUMax; ++i) {
            u_next[i] = (T)0;
            if ((uint32_t)i < n_u) {
                while (x >= G.Wo) { x -= G.Wo; ++y; }
                const uint32_t iy = (uint32_t)((int32_t)(y * G.sh) + dy), ix = (uint32_t)((int32_t)(x * G.sw) + dx);   // huge when negative
                if (u_col && y < G.Ho && iy < G.H && ix < G.W) u_next[i] = act_z[((size_t)iy * G.W + ix) * G.Cin + uci];
                x += groups;
            }
        }
    };
    auto stage = [&]() {                                                // registers -> LDS, rows = positions
#pragma unroll
        for (int i = 0; i < kDPieces; ++i) {
            constexpr uint32_t ppr = kStemBN / kPiece;
            const uint32_t e = tid + (uint32_t)kNT * i, pl = e / ppr, cl = (e % ppr) * kPiece;
            if (e < (uint32_t)kDTotal) *reinterpret_cast<u4v*>(Dsh + pl * pitch_d + cl * sizeof(T)) = d_next[i];
        }
        if constexpr (kPix3) {
#pragma unroll
            for (int i = 0; i < kStemPixMax; ++i)
                if ((uint32_t)i < n_pix) {
                    T* dst = reinterpret_cast<T*>(Ush + (ppg + (uint32_t)i * pgroups) * pitch_u + ptap * 3u * sizeof(T));
                    dst[0] = pix_next[i].c[0]; dst[1] = pix_next[i].c[1]; dst[2] = pix_next[i].c[2];
                }
            return;
        }
#pragma unroll
        for (int i = 0; i < kUMax; ++i)
            if ((uint32_t)i < n_u) *reinterpret_cast<T*>(Ush + (upg + (uint32_t)i * groups) * pitch_u + uj * sizeof(T)) = u_next[i];
    };

    // ---- tiles of the workgroup's [Jpad, 64] block, dealt to the waves ----
    // bfloat16: 32 x 32 tiles, tile = wave + waves x t.  float32: 16 x 16 tiles (v_mfma_f32_16x16x4_f32 runs at the
    // rate of the 32 x 32 x 2 one), which deal evenly: a wave owns 16 columns (wave % 4) and kT16 row tiles, all
    // 2 kJT of them with four waves, one half of them each with eight (ten 32 x 32 tiles on eight waves left two
    // waves with twice the work of the others).
    const uint32_t n_jt = G.Jpad / 32u, n_tiles = n_jt * 2u;
    constexpr int kT16 = kWaves == 4 ? 2 * kJT : kJT;
    f16v acc[kT];
    f4v acc16[kT16];
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int t = 0; t < kT; ++t) acc[t] = (f16v){0};
    } else {
#pragma unroll
        for (int t = 0; t < kT16; ++t) acc16[t] = (f4v){0};
    }
    const uint32_t ct16 = wave & 3u, jt16 = kWaves == 4 ? 0u : (wave >> 2) * (uint32_t)kJT;   // first row tile of the wave
    // bfloat16: the transposing LDS read hands lane l the 8 consecutive positions 8 (l / 32) .. + 7 of column l % 32 from
    // rows that are positions: within 16 lanes, lane r points at row r / 4, columns 4 (r % 4) .. + 3
    const uint32_t r16 = lane & 15u, g16 = lane >> 4, mhalf = g16 & 1u, khalf = g16 >> 1;
    const uint32_t frow = khalf * 8u + (r16 >> 2), fcol = mhalf * 16u + (r16 & 3u) * 4u;

    if (q_begin < q_end) fetch(q_begin);
    for (uint32_t q = q_begin; q < q_end; ++q) {
        __syncthreads();                                                // the previous chunk's fragments have been read
        stage();
        __syncthreads();
        if (q + 1 < q_end) fetch(q + 1);                                // in flight during the multiplications
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int t = 0; t < kT; ++t) {
                const uint32_t tile = wave + (uint32_t)kWaves * t;
                if (tile < n_tiles) {                                   // wave-uniform
                    const uint32_t jt = tile >> 1, ct = tile & 1u;
                    const uint8_t* ua = Ush + frow * pitch_u + (jt * 32u + fcol) * 2u;
                    const uint8_t* db = Dsh + frow * pitch_d + (ct * 32u + fcol) * 2u;
#pragma unroll
                    for (int ks = 0; ks < kKC / 16; ++ks) {
                        const s4v alo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(ua + ks * 16 * pitch_u));
                        const s4v ahi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(ua + (ks * 16 + 4) * pitch_u));
                        const s4v blo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(db + ks * 16 * pitch_d));
                        const s4v bhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(db + (ks * 16 + 4) * pitch_d));
                        const s8v av = {alo[0], alo[1], alo[2], alo[3], ahi[0], ahi[1], ahi[2], ahi[3]};
                        const s8v bv = {blo[0], blo[1], blo[2], blo[3], bhi[0], bhi[1], bhi[2], bhi[3]};
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8v, av), __builtin_bit_cast(bf8v, bv), acc[t], 0, 0, 0);
                    }
                }
            }
        } else {
            // float32: of each four positions lane l supplies U[k = l / 16][m = l % 16] and D[k][n = l % 16]
            const uint8_t* ua = Ush + (lane >> 4) * pitch_u + (jt16 * 16u + (lane & 15u)) * 4u;
            const uint8_t* db = Dsh + (lane >> 4) * pitch_d + (ct16 * 16u + (lane & 15u)) * 4u;
#pragma unroll
            for (int ks = 0; ks < kKC / 4; ++ks) {
                const float b = *reinterpret_cast<const float*>(db + ks * 4 * pitch_d);
#pragma unroll
                for (int t = 0; t < kT16; ++t) {
                    const float a = *reinterpret_cast<const float*>(ua + ks * 4 * pitch_u + t * 64);
                    acc16[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc16[t], 0, 0, 0);
                }
            }
        }
    }

    // ---- the part's unsquared product to the workspace: plane (z, part) of [J, C] ----
    float* out = ws + ((size_t)z * parts + part) * (size_t)G.J * C;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int t = 0; t < kT; ++t) {
            const uint32_t tile = wave + (uint32_t)kWaves * t;
            if (tile < n_tiles) {
                const uint32_t jt = tile >> 1, ct = tile & 1u;
                const uint32_t col = c0 + ct * 32u + (lane & 31u);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t row = jt * 32u + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                    if (row < G.J && col < C) out[(size_t)row * C + col] = acc[t][i];
                }
            }
        }
    } else {
        const uint32_t col = c0 + ct16 * 16u + (lane & 15u);
#pragma unroll
        for (int t = 0; t < kT16; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t row = (jt16 + (uint32_t)t) * 16u + 4u * (lane >> 4) + (uint32_t)i;
                if (row < G.J && col < C) out[(size_t)row * C + col] = acc16[t][i];
            }
    }
}

bool conv_stem_supported(int dtype, uint32_t Cin, uint32_t C, uint32_t kh, uint32_t kw) {
    const uint32_t piece = dtype == VGC_BF16 ? 8u : 4u;
    const uint64_t J = (uint64_t)kh * kw * Cin;
    // 5 row tiles x 2 column tiles are at most three tiles per wave
    return (dtype == VGC_BF16 || dtype == VGC_F32) && Cin % piece != 0 && C % piece == 0 && J <= (uint64_t)kStemJMax;
}

// Parts the positions of a sample are split into: about 2048 workgroups, at least four chunks per part.
static uint32_t stem_parts(int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    const uint64_t tiles_c = (C + kStemBN - 1) / kStemBN;
    const uint32_t kc = (uint32_t)stem_kc(dtype == VGC_BF16 ? 2 : 4, (int)((J + 31u) / 32u));
    const uint32_t n_chunks = (P + kc - 1) / kc;
    uint64_t parts = 2048 / ((uint64_t)B * tiles_c);
    if (parts > n_chunks / 4) parts = n_chunks / 4;
    return parts < 1 ? 1u : (uint32_t)parts;
}

size_t conv_stem_workspace_bytes(int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    return (size_t)B * stem_parts(dtype, B, P, J, C) * J * C * sizeof(float);
}

int launch_conv_stem(int dtype, const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C,
                     uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw, uint32_t Ho, uint32_t Wo,
                     float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    const uint32_t P = Ho * Wo, J = kh * kw * Cin;
    if (!workspace || workspace_bytes < conv_stem_workspace_bytes(dtype, B, P, J, C)) {
        set_error("vgc_sqgrad_conv2d: a layer whose input channels are not a multiple of 16 bytes needs the workspace "
                  "vgc_sqgrad_conv2d_workspace_bytes() asks for");
        return VGC_ERR_SIZE;
    }
    const uint32_t parts = stem_parts(dtype, B, P, J, C);
    const uint64_t nblk = (uint64_t)B * parts * ((C + kStemBN - 1) / kStemBN);
    if (nblk > 0x7FFFFFFFull) { set_error("vgc_sqgrad_conv2d: shape exceeds the launch limit"); return VGC_ERR_SIZE; }
    StemGeom G;
    G.H = H; G.W = W; G.Cin = Cin; G.kw = kw; G.sh = sh; G.sw = sw; G.ph = ph; G.pw = pw; G.Ho = Ho; G.Wo = Wo;
    G.J = J; G.Jpad = (J + 31u) / 32u * 32u;
    float* ws = static_cast<float*>(workspace);
    const uint32_t jt = G.Jpad / 32u;
#define VGC_LAUNCH_STEM_P(T_, JT_, PIX_)                                                                                      \
    hipLaunchKernelGGL((k_conv_stem<T_, JT_, PIX_>), dim3((uint32_t)nblk), dim3(stem_threads(JT_)),                           \
                       (size_t)stem_kc((int)sizeof(T_), JT_) * (stem_pitch_u(G.Jpad, sizeof(T_)) + stem_pitch_d(sizeof(T_))), stream, \
                       (const T_*)act, (const T_*)D, B, C, G, parts, ws)
    // RGB input: pixel by pixel, where a thread's share of a chunk's pixels fits what the kernel holds
#define VGC_LAUNCH_STEM(T_, JT_)                                                                                              \
    do {                                                                                                                      \
        const uint32_t kc_ = (uint32_t)stem_kc((int)sizeof(T_), JT_);                                                         \
        if (Cin == 3 && kc_ / stem_pix_groups((uint32_t)stem_threads(JT_), J / 3u, kc_) <= (uint32_t)stem_pix_max((int)sizeof(T_))) \
            VGC_LAUNCH_STEM_P(T_, JT_, true);                                                                                 \
        else VGC_LAUNCH_STEM_P(T_, JT_, false);                                                                               \
    } while (0)
    if (dtype == VGC_BF16) {
        if (jt == 1) VGC_LAUNCH_STEM(uint16_t, 1); else if (jt == 2) VGC_LAUNCH_STEM(uint16_t, 2);
        else if (jt == 3) VGC_LAUNCH_STEM(uint16_t, 3); else if (jt == 4) VGC_LAUNCH_STEM(uint16_t, 4);
        else VGC_LAUNCH_STEM(uint16_t, 5);
    } else {
        if (jt == 1) VGC_LAUNCH_STEM(float, 1); else if (jt == 2) VGC_LAUNCH_STEM(float, 2);
        else if (jt == 3) VGC_LAUNCH_STEM(float, 3); else if (jt == 4) VGC_LAUNCH_STEM(float, 4);
        else VGC_LAUNCH_STEM(float, 5);
    }
#undef VGC_LAUNCH_STEM
#undef VGC_LAUNCH_STEM_P
    launch_sqgrad_reduce_parts(ws, B, parts, (size_t)J * C, c, c * c, g_out, s_out, stream);
    return hip_check(hipGetLastError(), "launch k_conv_stem");
}

}  // namespace vgc
