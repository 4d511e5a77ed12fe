// LDS-tiled MFMA kernels for the per-parameter sums of Alg. 1 (g = c sum_z G_z, s = c^2 sum_z G_z.G_z):
//
//   k_fc_bf16     FC form, bf16 inputs.  G_z is the outer product x_z d_z^T, so s = c^2 (X.X)^T (D.D) and
//                 g = c X^T D are two contractions over K = B (Section 5's 2 N |B| multiply-adds each).
//                 The squares are taken in float32 and rounded to bf16 (2^-9 relative per factor, well
//                 inside the 1e-2 budget for bf16 inputs); v_mfma_f32_32x32x16_bf16, float32 accumulate.
//                 With K this small the kernel is bound by writing [J, C] floats, not by the matrix cores.
//   k_tiled_f32   float32 inputs, both forms, v_mfma_f32_32x32x2_f32 (float32 products and sums, which is
//                 what the 1e-5 tolerance on s needs).  FC: two MFMA chains on (x, d) and (x^2, d^2).
//                 Conv: per-sample product in the accumulators, squared into s when the sample ends.
//
// Block tile 128 x 128 of [J, C], 4 waves (2 x 2), operands staged through LDS k-major (rows of the
// source matrices as they are in memory).  Rows past the end of a sample's matrix are outside the
// bounded range of the buffer loads and read as zero.
#include "vgc_internal.h"

namespace vgc {

typedef short s4v __attribute__((ext_vector_type(4)));
typedef short s8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef uint32_t u4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s4v* lds_s4v_ptr;
typedef __amdgpu_buffer_rsrc_t rsrc_t;

constexpr int kT = 128;                  // block tile edge
constexpr int kPitch16 = kT + 32;        // bf16 row pitch (elements): rows start 16 banks apart

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// ds_read_b64_tr_b16 operand fetch: see vgc_sqgrad_tiled.hip for the lane mapping.
__device__ __forceinline__ bf8v frag16(const uint16_t* tile, int ks, int mbase, uint32_t lane) {
    const uint32_t r = lane & 15u, grp = lane >> 4;
    const uint16_t* p = tile + (ks * 16 + (grp >> 1) * 8 + (r >> 2)) * kPitch16 + mbase + (grp & 1u) * 16 + 4 * (r & 3u);
    const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p));
    const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p + 4 * kPitch16));
    s8v v;
    v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
    v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
    return __builtin_bit_cast(bf8v, v);
}

// Square of two packed bf16 values: float32 product, rounded to nearest-even bf16.
__device__ __forceinline__ uint32_t square_bf16x2(uint32_t w) {
    const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xFFFF0000u);
    const uint32_t a = __float_as_uint(lo * lo), b = __float_as_uint(hi * hi);
    const uint32_t ra = (a + 0x7FFFu + ((a >> 16) & 1u)) >> 16;
    const uint32_t rb = (b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u;
    return ra | rb;
}

__device__ __forceinline__ void store_tile(float fs, float fg, const f16v (&s_acc)[2][2], const f16v (&g_acc)[2][2],
                                           bool want_g, float* __restrict__ so, float* __restrict__ go,
                                           uint32_t j0, uint32_t c0, uint32_t J, uint32_t C, uint32_t wm, uint32_t wn,
                                           uint32_t lane) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const uint32_t col = c0 + wn * 64 + nt * 32 + (lane & 31u);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t row = j0 + wm * 64 + mt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                if (row < J && col < C) {
                    const size_t o = (size_t)row * C + col;
                    __builtin_nontemporal_store(fs * s_acc[mt][nt][i], so + o);
                    if (want_g) __builtin_nontemporal_store(fg * g_acc[mt][nt][i], go + o);
                }
            }
        }
}

// ------------------------------------------------------------------------------------------------
// FC, bf16
// ------------------------------------------------------------------------------------------------
template <bool kWantG>
__global__ __launch_bounds__(256, 2) void k_fc_bf16(const uint16_t* __restrict__ X, const uint16_t* __restrict__ D,
                                                    uint32_t B, uint32_t J, uint32_t C, float cg, float cs,
                                                    float* __restrict__ g_out, float* __restrict__ s_out) {
    constexpr int kRows = 32;
    __shared__ __attribute__((aligned(16))) uint16_t shX[kRows * kPitch16], shD[kRows * kPitch16];
    __shared__ __attribute__((aligned(16))) uint16_t shX2[kRows * kPitch16], shD2[kRows * kPitch16];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, wm = wave >> 1, wn = wave & 1u;
    const uint32_t tiles_c = (C + kT - 1) / kT;
    const uint32_t j0 = (blockIdx.x / tiles_c) * kT, c0 = (blockIdx.x % tiles_c) * kT;
    const rsrc_t rx = make_rsrc(X, B * J * 2u), rd = make_rsrc(D, B * C * 2u);

    f16v s_acc[2][2], g_acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) { s_acc[a][b] = (f16v){0}; g_acc[a][b] = (f16v){0}; }

    for (uint32_t z0 = 0; z0 < B; z0 += kRows) {
        u4v vx[2], vd[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t idx = tid + 256u * i, row = idx >> 4, col = (idx & 15u) * 8u;
            vx[i] = __builtin_bit_cast(u4v, __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(((z0 + row) * J + j0 + col) * 2u), 0, 0));
            vd[i] = __builtin_bit_cast(u4v, __builtin_amdgcn_raw_buffer_load_b128(rd, (int)(((z0 + row) * C + c0 + col) * 2u), 0, 0));
        }
        if (z0) __syncthreads();                        // the previous chunk has been consumed
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t idx = tid + 256u * i, off = (idx >> 4) * kPitch16 + (idx & 15u) * 8u;
            // columns past the matrix edge wrapped into the next row: they feed outputs that are not stored
            if (kWantG) {
                *reinterpret_cast<u4v*>(shX + off) = vx[i];
                *reinterpret_cast<u4v*>(shD + off) = vd[i];
            }
            u4v x2, d2;
#pragma unroll
            for (int e = 0; e < 4; ++e) { x2[e] = square_bf16x2(vx[i][e]); d2[e] = square_bf16x2(vd[i][e]); }
            *reinterpret_cast<u4v*>(shX2 + off) = x2;
            *reinterpret_cast<u4v*>(shD2 + off) = d2;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < kRows / 16; ++ks) {
            bf8v a2[2], b2[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) { a2[t] = frag16(shX2, ks, wm * 64 + t * 32, lane); b2[t] = frag16(shD2, ks, wn * 64 + t * 32, lane); }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    s_acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2[mt], b2[nt], s_acc[mt][nt], 0, 0, 0);
            if (kWantG) {
                bf8v a[2], b[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) { a[t] = frag16(shX, ks, wm * 64 + t * 32, lane); b[t] = frag16(shD, ks, wn * 64 + t * 32, lane); }
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        g_acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt], b[nt], g_acc[mt][nt], 0, 0, 0);
            }
        }
    }
    store_tile(cs, cg, s_acc, g_acc, kWantG, s_out, g_out, j0, c0, J, C, wm, wn, lane);
}

// ------------------------------------------------------------------------------------------------
// float32, FC and conv
// ------------------------------------------------------------------------------------------------
constexpr int kR32 = 16;                 // rows per LDS stage

// One staged chunk in registers: kR32 rows of a BM-wide and of a BN-wide float matrix, PA resp. PB 16-byte
// pieces per thread of a workgroup of NT threads.  Piece idx of an operand W columns wide sits in row
// idx / (W / 4), columns 4 (idx % (W / 4)) .. + 3.
template <int PA, int PB> struct Chunk32 { f4v a[PA], b[PB]; };

template <int BM, int BN, int NT, int PA, int PB>
__device__ __forceinline__ void load32(Chunk32<PA, PB>& R, rsrc_t ra, rsrc_t rb, uint32_t J, uint32_t C, uint32_t p0,
                                       uint32_t j0, uint32_t c0, uint32_t tid) {
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const uint32_t idx = tid + (uint32_t)NT * i, row = idx / (BM / 4), col = (idx % (BM / 4)) * 4u;
        R.a[i] = __builtin_bit_cast(f4v, __builtin_amdgcn_raw_buffer_load_b128(ra, (int)(((p0 + row) * J + j0 + col) * 4u), 0, 0));
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
        const uint32_t idx = tid + (uint32_t)NT * i, row = idx / (BN / 4), col = (idx % (BN / 4)) * 4u;
        R.b[i] = __builtin_bit_cast(f4v, __builtin_amdgcn_raw_buffer_load_b128(rb, (int)(((p0 + row) * C + c0 + col) * 4u), 0, 0));
    }
}

template <int BM, int BN, int NT, int PA, int PB>
__device__ __forceinline__ void stage32(float* A, float* Bm, const Chunk32<PA, PB>& R, uint32_t tid) {
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const uint32_t idx = tid + (uint32_t)NT * i;
        *reinterpret_cast<f4v*>(A + (idx / (BM / 4)) * (BM + 32) + (idx % (BM / 4)) * 4u) = R.a[i];
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
        const uint32_t idx = tid + (uint32_t)NT * i;
        *reinterpret_cast<f4v*>(Bm + (idx / (BN / 4)) * (BN + 32) + (idx % (BN / 4)) * 4u) = R.b[i];
    }
}

// kConv: X is [B, P, J], D is [B, P, C], samples z_begin .. z_end-1 of this workgroup's split.
// !kConv: X is [B, J], D is [B, C]; treated as one "sample" with P = B rows and no per-sample square
//         (the two chains run on the values and on their squares instead).
// kImplicit (with kConv): X is the layer's NHWC input [B, H, W, Cin] seen through the geometry G, J = kh kw Cin; the
//         lane's piece of 4 columns lies inside one filter tap (Cin is a multiple of 4) and its offset in the input
//         is formed per chunk from the output position of its row, which is kept incrementally.
// BM x BN: the block tile (64 or 128 each), one wave per 64 x 64 of it; rows of LDS are padded by 32 floats.
// kTail: the k-steps of a sample's last chunk that lie wholly past its rows are skipped (see conv_f32_tail).
// kDepth: sets of staging registers, i.e. chunks requested ahead of the one being staged (2, or 3 where the registers allow).
template <bool kConv, bool kWantG, bool kImplicit, int BM = 128, int BN = 128, bool kTail = false, int kDepth = 2>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64, 2)
void k_tiled_f32(const float* __restrict__ X, const float* __restrict__ D,
                 uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                 uint32_t splits, uint32_t split_p, float cg, float cs,
                 float* __restrict__ g_out, float* __restrict__ s_out,
                 float* __restrict__ ws, ConvGeom G) {
    constexpr int NT = (BM / 64) * (BN / 64) * 64;                   // threads of the workgroup
    constexpr int PA = kR32 * BM / 4 / NT, PB = kR32 * BN / 4 / NT;  // 16-byte pieces per thread and chunk
    constexpr int kPitchA = BM + 32, kPitchB = BN + 32;
    __shared__ __attribute__((aligned(16))) float shA[2][kR32 * kPitchA];
    __shared__ __attribute__((aligned(16))) float shB[2][kR32 * kPitchB];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6, wm = wave / (BN / 64), wn = wave % (BN / 64);
    const uint32_t tiles_c = (C + BN - 1) / BN, tiles_j = (J + BM - 1) / BM;
    const uint32_t nblk = gridDim.x, per = nblk / 8u, rem = nblk % 8u;
    const uint32_t xcd = blockIdx.x % 8u, slot = blockIdx.x / 8u;
    const uint32_t logical = xcd * per + min(xcd, rem) + slot;       // contiguous range of tiles per XCD
    const uint32_t tile_c = logical % tiles_c, tile_j = (logical / tiles_c) % tiles_j, split = logical / (tiles_c * tiles_j);
    const uint32_t j0 = tile_j * BM, c0 = tile_c * BN;
    const uint32_t rowsP = kConv ? P : B;                            // K extent of one "sample"
    // split_p > 1 (conv only): the workgroup owns part `part` of the positions of the single sample split / split_p
    // and leaves the unsquared partial product in the workspace
    const uint32_t n_chunks = (rowsP + kR32 - 1) / kR32;
    const uint32_t part = split_p > 1 ? split % split_p : 0u;
    const uint32_t chunks_per_part = (n_chunks + split_p - 1) / split_p;
    const uint32_t c_begin = min(n_chunks, part * chunks_per_part);
    // sample ranges of the splits differ by at most one sample
    const uint32_t z_begin = !kConv ? 0u : (split_p > 1 ? split / split_p : (uint32_t)((uint64_t)split * B / splits));
    const uint32_t z_end = !kConv ? 1u : (split_p > 1 ? z_begin + 1u : (uint32_t)((uint64_t)(split + 1u) * B / splits));
    const uint32_t total = split_p > 1 ? min(n_chunks, c_begin + chunks_per_part) - c_begin : (z_end - z_begin) * n_chunks;

    f16v acc[2][2], s_acc[2][2], g_acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) { acc[a][b] = (f16v){0}; s_acc[a][b] = (f16v){0}; g_acc[a][b] = (f16v){0}; }

    // implicit form: per load, the tap of the lane's columns and the output position of its row
    uint32_t y0A[PA], x0A[PA], yA[PA], xA[PA];
    int32_t tapX[PA], tapOff[PA];
    if (kImplicit) {
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const uint32_t idx = tid + (uint32_t)NT * i, row = idx / (BM / 4), colj = j0 + (idx % (BM / 4)) * 4u;
            const uint32_t tap = colj / G.Cin, ky = tap / G.kw;
            const uint32_t pos0 = c_begin * kR32 + row;           // the lane's row in the workgroup's first chunk
            y0A[i] = yA[i] = pos0 / G.Wo;
            x0A[i] = xA[i] = pos0 - y0A[i] * G.Wo;
            const int32_t ty = (int32_t)ky - (int32_t)G.ph;
            tapX[i] = (int32_t)(tap - ky * G.kw) - (int32_t)G.pw;
            tapOff[i] = (ty * (int32_t)G.W + tapX[i]) * (int32_t)G.Cin + (int32_t)(colj - tap * G.Cin);
            if (colj >= J) tapX[i] = -0x400000;              // a column past J: never inside the input
        }
    }
    Chunk32<PA, PB> R[kDepth];
    uint32_t zl = z_begin, pcl = c_begin, issued = 0;
    auto issue = [&](int slot_) {
        const bool live = issued < total;
        const uint32_t zz = live ? zl : z_begin;
        const rsrc_t rb = make_rsrc(D + (size_t)zz * rowsP * C, live ? rowsP * C * 4u : 0u);
        if (kImplicit) {
            const uint32_t sample = G.H * G.W * G.Cin;
            const rsrc_t ra = make_rsrc(X + (size_t)zz * sample, live ? sample * 4u : 0u);
#pragma unroll
            for (int i = 0; i < PA; ++i) {
                // rows of the input outside the image give an offset that is negative or past the sample: the load
                // answers with zeros; columns outside and positions past P are masked
                const int32_t ys = __mul24((int32_t)yA[i], (int32_t)G.sh), xs = __mul24((int32_t)xA[i], (int32_t)G.sw);
                const bool inside = ((uint32_t)(xs + tapX[i]) < G.W) & (yA[i] < G.Ho);
                const int32_t off = __mul24(__mul24(ys, (int32_t)G.W) + xs, (int32_t)G.Cin) + tapOff[i];
                const uint32_t voff = ((uint32_t)off << 2) | (inside ? 0u : 0xFFFFFFFFu);
                R[slot_].a[i] = __builtin_bit_cast(f4v, __builtin_amdgcn_raw_buffer_load_b128(ra, (int)voff, 0, 0));
            }
#pragma unroll
            for (int i = 0; i < PB; ++i) {
                const uint32_t idx = tid + (uint32_t)NT * i, row = idx / (BN / 4), col = (idx % (BN / 4)) * 4u;
                R[slot_].b[i] = __builtin_bit_cast(f4v, __builtin_amdgcn_raw_buffer_load_b128(rb, (int)(((pcl * kR32 + row) * C + c0 + col) * 4u), 0, 0));
            }
        } else {
            const rsrc_t ra = make_rsrc(X + (size_t)zz * rowsP * J, live ? rowsP * J * 4u : 0u);
            load32<BM, BN, NT>(R[slot_], ra, rb, J, C, pcl * kR32, j0, c0, tid);
        }
        const bool wrap = (++pcl == n_chunks);
        if (wrap) { pcl = 0; ++zl; }
        if (kImplicit) {
#pragma unroll
            for (int i = 0; i < PA; ++i) {                    // the lane's row of the next chunk: kR32 positions further
                const uint32_t x = xA[i] + G.step_x, xw = x - G.Wo;
                const uint32_t carry = x >= G.Wo ? 1u : 0u;
                const uint32_t keep = wrap ? 0u : 0xFFFFFFFFu;
                xA[i] = (min(x, xw) & keep) | (x0A[i] & ~keep);
                yA[i] = ((yA[i] + G.step_y + carry) & keep) | (y0A[i] & ~keep);
            }
        }
        ++issued;
    };
#pragma unroll
    for (int d = 0; d < kDepth; ++d) issue(d);
    stage32<BM, BN, NT>(shA[0], shB[0], R[0], tid);
    issue(0);
    __syncthreads();

    const uint32_t col = lane & 31u, kh = lane >> 5;
    uint32_t left = split_p > 1 ? 0u : n_chunks;                     // chunks until the sample's product is complete (0: never)
    // kTail: a sample's last chunk holds rowsP - (n_chunks - 1) kR32 rows and zeros after them; of its k-steps (two
    // rows each) the first two, four or all eight are multiplied, whichever covers the rows.  Adding the zero
    // products would change nothing; the tests split the chunk into three runs for the scheduler, which is why
    // shapes with little to skip take the kernel without them.
    const uint32_t tail_steps = (rowsP - (n_chunks - 1u) * kR32 + 1u) / 2u;
    uint32_t cpos = split_p > 1 ? c_begin : 0u;                      // the chunk's place in its sample
    // chunk q sits in LDS buffer q % 2 and came through register set q % kDepth; the loop is unrolled over both
    constexpr int kUnroll = kDepth % 2 == 0 ? kDepth : 2 * kDepth;
    for (uint32_t q0 = 0; q0 < total; q0 += kUnroll) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (u > 0 && q0 + (uint32_t)u >= total) break;
            const uint32_t buf = (uint32_t)(u & 1);                 // q = q0 + u, and q0 is even
            const float* A = shA[buf];
            const float* Bm = shB[buf];
            auto k_step = [&](uint32_t ks) __attribute__((always_inline)) {
                float a[2], b[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    a[t] = A[(ks * 2 + kh) * kPitchA + wm * 64 + t * 32 + col];
                    b[t] = Bm[(ks * 2 + kh) * kPitchB + wn * 64 + t * 32 + col];
                }
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) {
                        if (kConv) {
                            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
                        } else {
                            s_acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt] * a[mt], b[nt] * b[nt], s_acc[mt][nt], 0, 0, 0);
                            if (kWantG) g_acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt], b[nt], g_acc[mt][nt], 0, 0, 0);
                        }
                    }
            };
            if (kTail) {
                const uint32_t steps = cpos == n_chunks - 1u ? tail_steps : (uint32_t)(kR32 / 2);
                cpos = cpos + 1u == n_chunks ? 0u : cpos + 1u;
                k_step(0u);
                k_step(1u);
                if (steps > 2u) {
                    k_step(2u);
                    k_step(3u);
                }
                if (steps > 4u) {
#pragma unroll
                    for (int ks = 4; ks < kR32 / 2; ++ks) k_step((uint32_t)ks);
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < kR32 / 2; ++ks) k_step((uint32_t)ks);
            }
            const int ns = (u + 1) % kDepth;
            stage32<BM, BN, NT>(shA[buf ^ 1u], shB[buf ^ 1u], R[ns], tid);
            issue(ns);
            if (kConv && --left == 0) {                           // sample finished: G_z is complete in acc
                left = n_chunks;                                  // (a surplus chunk of zeros may "finish" a sample: adds nothing)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const float x = acc[mt][nt][i];
                            s_acc[mt][nt][i] += x * x;
                            if (kWantG) g_acc[mt][nt][i] += x;
                        }
                        acc[mt][nt] = (f16v){0};
                    }
            }
            __syncthreads();
        }
    }

    const bool direct = (splits == 1);
    const size_t JC = (size_t)J * C;
    if (split_p > 1) {                                               // the partial product itself, for k_sqgrad_reduce_parts
        store_tile(1.0f, 1.0f, acc, acc, false, ws + (size_t)split * JC, nullptr, j0, c0, J, C, wm, wn, lane);
        return;
    }
    float* so = direct ? s_out : ws + (size_t)split * 2 * JC;
    float* go = direct ? g_out : ws + (size_t)split * 2 * JC + JC;
    store_tile(direct ? cs : 1.0f, direct ? cg : 1.0f, s_acc, g_acc, kWantG, so, go, j0, c0, J, C, wm, wn, lane);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
bool fc_tiled_supported(int dtype, uint32_t B, uint32_t J, uint32_t C) {
    const uint64_t limit = 0x7FFFFFFFull;                            // buffer ranges and offsets are 32-bit
    if (dtype == VGC_BF16) return J % 8 == 0 && C % 8 == 0 && (uint64_t)(B + 32) * J * 2 < limit && (uint64_t)(B + 32) * C * 2 < limit;
    return J % 4 == 0 && C % 4 == 0 && (uint64_t)(B + 16) * J * 4 < limit && (uint64_t)(B + 16) * C * 4 < limit;
}

bool conv_f32_tiled_supported(uint32_t P, uint32_t J, uint32_t C) {
    const uint64_t limit = 0x7FFFFFFFull;
    return J % 4 == 0 && C % 4 == 0 && (uint64_t)(P + 16) * J * 4 < limit && (uint64_t)(P + 16) * C * 4 < limit;
}

// Block tile of the float32 conv kernel for a shape: 64 instead of 128 rows (columns) where that wastes at
// least a fifth fewer of them (J or C at most 64, or just past a multiple of 128).
struct F32Tile { uint32_t bm, bn; };
static uint32_t f32_tile_edge(uint32_t n) {
    const uint32_t pad128 = (n + 127) / 128 * 128, pad64 = (n + 63) / 64 * 64;
    return pad64 * 5 <= pad128 * 4 ? 64u : 128u;
}
static F32Tile conv_f32_tile(uint32_t J, uint32_t C) { return F32Tile{f32_tile_edge(J), f32_tile_edge(C)}; }
static uint64_t conv_f32_tiles(const F32Tile& t, uint32_t J, uint32_t C) {
    return (uint64_t)((J + t.bm - 1) / t.bm) * ((C + t.bn - 1) / t.bn);
}
// Workgroups resident at once: 256 compute units x (8 waves, and 160 KB of LDS at two staged chunks per workgroup).
static uint64_t conv_f32_slots(const F32Tile& t) {
    const uint64_t waves = (uint64_t)(t.bm / 64) * (t.bn / 64);
    const uint64_t lds = 2ull * kR32 * (t.bm + 32 + t.bn + 32) * sizeof(float);
    const uint64_t by_waves = 8 / waves, by_lds = (160ull * 1024) / lds;
    return 256 * (by_waves < by_lds ? by_waves : by_lds);
}

uint32_t conv_f32_splits(uint32_t B, uint32_t J, uint32_t C) {
    const F32Tile t = conv_f32_tile(J, C);
    const uint64_t tiles = conv_f32_tiles(t, J, C);
    const uint64_t slots = conv_f32_slots(t);
    double best = 1e300;
    uint32_t best_s = 1;
    for (uint32_t s = 1; s <= B; ++s) {
        const uint32_t zper = (B + s - 1) / s, s2 = (B + zper - 1) / zper;
        if (s2 != s) continue;
        const uint64_t rounds = (tiles * s2 + slots - 1) / slots;
        const double cost = (double)rounds * zper + (s2 > 1 ? 0.5 * s2 * (double)tiles / slots + 0.5 : 0.0);
        if (cost < best - 1e-9) { best = cost; best_s = s2; }
    }
    return best_s;
}

int launch_fc_tiled(int dtype, const void* X, const void* D, uint32_t B, uint32_t J, uint32_t C, float c,
                    float* g_out, float* s_out, hipStream_t stream) {
    const uint64_t nblk = (uint64_t)((J + kT - 1) / kT) * ((C + kT - 1) / kT);
    if (nblk > 0x7FFFFFFFull) { set_error("vgc_sqgrad: shape exceeds the launch limit"); return VGC_ERR_SIZE; }
    const float cg = c, cs = c * c;
    if (dtype == VGC_BF16) {
        if (g_out) hipLaunchKernelGGL(k_fc_bf16<true>, dim3((uint32_t)nblk), dim3(256), 0, stream, (const uint16_t*)X, (const uint16_t*)D, B, J, C, cg, cs, g_out, s_out);
        else hipLaunchKernelGGL(k_fc_bf16<false>, dim3((uint32_t)nblk), dim3(256), 0, stream, (const uint16_t*)X, (const uint16_t*)D, B, J, C, cg, cs, g_out, s_out);
    } else {
        if (g_out) hipLaunchKernelGGL((k_tiled_f32<false, true, false>), dim3((uint32_t)nblk), dim3(256), 0, stream, (const float*)X, (const float*)D, B, 1u, J, C, 1u, 1u, cg, cs, g_out, s_out, (float*)nullptr, ConvGeom{});
        else hipLaunchKernelGGL((k_tiled_f32<false, false, false>), dim3((uint32_t)nblk), dim3(256), 0, stream, (const float*)X, (const float*)D, B, 1u, J, C, 1u, 1u, cg, cs, g_out, s_out, (float*)nullptr, ConvGeom{});
    }
    return hip_check(hipGetLastError(), "launch fc tiled");
}

// Positions split: the rule of conv_split_p of the bf16 kernel with this kernel's tiles and slots.
uint32_t conv_f32_split_p(uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    const F32Tile t = conv_f32_tile(J, C);
    const uint64_t tiles = conv_f32_tiles(t, J, C);
    const uint64_t slots = conv_f32_slots(t);
    const uint32_t n_chunks = (P + kR32 - 1) / kR32;
    if (tiles * B * 3 > slots * 2 || n_chunks < 16) return 1;
    // up to half a round: as many parts as fill one round; up to two thirds: just under two rounds
    const uint64_t sp = tiles * B * 2 <= slots ? slots / (tiles * B) : 2 * slots / (tiles * B);
    return (uint32_t)(sp < n_chunks / 8 ? sp : n_chunks / 8);
}

// Whether a shape takes the kernel that skips the empty k-steps of each sample's last chunk: where they are at
// least an eighth of all (7 x 7 positions: 6 of 32; 14 x 14: 6 of 104, less than the tests cost).
static bool conv_f32_tail(uint32_t P) {
    const uint32_t n_chunks = (P + kR32 - 1) / kR32, steps = (P - (n_chunks - 1) * kR32 + 1) / 2;
    const uint32_t run = steps <= 2 ? 2u : steps <= 4 ? 4u : (uint32_t)(kR32 / 2);
    return (kR32 / 2 - run) * 8u >= n_chunks * (kR32 / 2);
}

size_t conv_f32_workspace_bytes(uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    const uint32_t sp = conv_f32_split_p(B, P, J, C);
    if (sp > 1) return (size_t)B * sp * J * C * sizeof(float);
    const uint32_t splits = conv_f32_splits(B, J, C);
    return splits > 1 ? (size_t)splits * 2 * J * C * sizeof(float) : 0;
}

template <bool kImplicit>
static int launch_conv_f32_any(const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
                               float* g_out, float* s_out, void* workspace, size_t workspace_bytes, const ConvGeom& G,
                               hipStream_t stream) {
    const size_t JC = (size_t)J * C;
    uint32_t split_p = conv_f32_split_p(B, P, J, C);
    if (split_p > 1 && (!workspace || workspace_bytes < (size_t)B * split_p * JC * sizeof(float))) split_p = 1;
    uint32_t splits = split_p > 1 ? B * split_p : conv_f32_splits(B, J, C);
    if (split_p == 1 && splits > 1 && (!workspace || workspace_bytes < (size_t)splits * 2 * JC * sizeof(float))) splits = 1;
    const F32Tile t = conv_f32_tile(J, C);
    const uint64_t nblk = conv_f32_tiles(t, J, C) * splits;
    if (nblk > 0x7FFFFFFFull) { set_error("vgc_sqgrad: shape exceeds the launch limit"); return VGC_ERR_SIZE; }
    const float cg = c, cs = c * c;
    float* ws = static_cast<float*>(workspace);
    // with the positions split the partial products are unsquared: the variant without g serves both
    const bool with_g = g_out && split_p == 1;
    const float* Xf = static_cast<const float*>(X);
    const float* Df = static_cast<const float*>(D);
#define VGC_LAUNCH_F32_T(BM_, BN_, TAIL_)                                                                                  \
    do {                                                                                                                   \
        const dim3 grid((uint32_t)nblk), block((BM_ / 64) * (BN_ / 64) * 64);                                              \
        if (with_g) hipLaunchKernelGGL((k_tiled_f32<true, true, kImplicit, BM_, BN_, TAIL_>), grid, block, 0, stream, Xf,  \
                                       Df, B, P, J, C, splits, split_p, cg, cs, g_out, s_out, ws, G);                      \
        else hipLaunchKernelGGL((k_tiled_f32<true, false, kImplicit, BM_, BN_, TAIL_, (BM_ == 128 && BN_ == 128) ? 3 : 2>), \
                                grid, block, 0, stream, Xf, Df, B, P, J, C, splits, split_p, cg, cs, g_out, s_out, ws, G); \
    } while (0)
#define VGC_LAUNCH_F32(BM_, BN_)                                                                                           \
    do {                                                                                                                   \
        if (tail) VGC_LAUNCH_F32_T(BM_, BN_, true);                                                                        \
        else VGC_LAUNCH_F32_T(BM_, BN_, false);                                                                            \
    } while (0)
    const bool tail = conv_f32_tail(P);
    if (t.bm == 128 && t.bn == 128) VGC_LAUNCH_F32(128, 128);
    else if (t.bm == 128) VGC_LAUNCH_F32(128, 64);
    else if (t.bn == 128) VGC_LAUNCH_F32(64, 128);
    else VGC_LAUNCH_F32(64, 64);
#undef VGC_LAUNCH_F32_T
#undef VGC_LAUNCH_F32
    if (split_p > 1) launch_sqgrad_reduce_parts(ws, B, split_p, JC, cg, cs, g_out, s_out, stream);
    else if (splits > 1) launch_sqgrad_reduce(ws, splits, JC, cg, cs, g_out, s_out, stream);
    return hip_check(hipGetLastError(), "launch k_tiled_f32");
}

int launch_conv_f32_tiled(const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
                          float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    return launch_conv_f32_any<false>(X, D, B, P, J, C, c, g_out, s_out, workspace, workspace_bytes, ConvGeom{}, stream);
}

int launch_conv2d_f32(const void* act, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
                      float* g_out, float* s_out, void* workspace, size_t workspace_bytes, ConvGeom G, hipStream_t stream) {
    G.step_y = kR32 / G.Wo;
    G.step_x = kR32 % G.Wo;
    return launch_conv_f32_any<true>(act, D, B, P, J, C, c, g_out, s_out, workspace, workspace_bytes, G, stream);
}

}  // namespace vgc
