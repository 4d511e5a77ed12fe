// LDS-tiled MFMA kernels for the per-parameter sums of Alg. 1 (g = c sum_z G_z, s = c^2 sum_z G_z.G_z,
// G_z the gradient of sample z's loss, Section 4.1), shared-weight form: G_z = U_z^T D_z with K = P.
//
// A workgroup (4 waves, 2 x 2) owns a 128 x 128 tile of [J, C] and a range of samples.  For every
// sample it runs the K loop over the P positions in chunks of 32 rows staged through LDS (double
// buffered, one barrier per chunk), keeping the per-sample product in MFMA accumulators; when the
// sample is finished the accumulators are squared into s (and added into g) and cleared, so a
// per-sample gradient never leaves registers.  The sample range can be split over blockIdx.z to fill
// the chip when [J, C] has few tiles; the partial sums then go to a workspace and are added in fixed
// order by k_sqgrad_reduce.
//
// bf16 path: v_mfma_f32_32x32x16_bf16.  Lane l of that instruction holds, for row m = l % 32, the 8
// consecutive k = 8 * (l / 32) .. + 7.  Memory has the other order (k-major rows, m contiguous), so
// the operands are fetched with the LDS transposing read ds_read_b64_tr_b16: within 16 lanes, lane r
// supplies the address of 4 consecutive b16 and lane i receives element i % 4 from the addresses of
// lanes i / 4 + 4 j, j = 0..3.  With lane r pointing at row k0 + r / 4, columns m0 + 4 (r % 4) .. + 3,
// lane i receives k0 .. k0 + 3 for column m0 + i.
#include "vgc_internal.h"

namespace vgc {

typedef short s4v __attribute__((ext_vector_type(4)));
typedef short s8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef uint32_t u4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s4v* lds_s4v_ptr;

#ifndef VGC_CONV_KC
#define VGC_CONV_KC 32
#endif
constexpr int kKC = VGC_CONV_KC;         // positions per LDS stage

// Row pitch (bf16 elements) of a staged tile of width W: W + 32, i.e. consecutive rows start 16 banks
// apart, so the 4 rows x 2 column halves one half-wave reads with a transposing load fall on distinct banks.
template <int W> struct Pitch { static constexpr int value = W + 32; };

template <int W>
__device__ __forceinline__ bf8v lds_frag_bf16(const uint16_t* tile, int ks, int mbase, uint32_t lane) {
    constexpr int kPitch = Pitch<W>::value;
    const uint32_t r = lane & 15u, grp = lane >> 4;
    const uint32_t mhalf = grp & 1u, khalf = grp >> 1;
    const uint16_t* p = tile + (ks * 16 + khalf * 8 + (r >> 2)) * kPitch + mbase + mhalf * 16 + 4 * (r & 3u);
    const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p));
    const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p + 4 * kPitch));
    s8v v;
    v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
    v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
    return __builtin_bit_cast(bf8v, v);
}

// One staged chunk of an operand: rows p0 .. p0+31 of a [P, W] bf16 matrix, columns w0 .. w0+TW-1,
// moved by NT threads in 16-byte pieces.
template <int TW, int NT> struct ChunkRegs { u4v v[kKC * TW / 8 / NT]; };

// Buffer loads with the sample's [P, W] matrix as the bounded range: rows past P fall outside the range
// and read as zero in hardware, so there is no branch around a load and the compiler can count the
// outstanding loads exactly (it waits only for the register set about to be staged).  Columns past W
// wrap into the next row; they only feed outputs that are never stored.
typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t sample_rsrc(const uint16_t* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, (int)bytes, 0x00020000);
}

template <int TW, int NT>
__device__ __forceinline__ void load_chunk(ChunkRegs<TW, NT>& R, rsrc_t rs, uint32_t W, uint32_t p0, uint32_t w0, uint32_t tid) {
    constexpr int kPer = kKC * TW / 8 / NT, kCols = TW / 8;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const uint32_t idx = tid + (uint32_t)NT * i, row = idx / kCols, col = w0 + (idx % kCols) * 8u;
        const uint32_t off = ((p0 + row) * W + col) * 2u;
        R.v[i] = __builtin_bit_cast(u4v, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0));
    }
}

template <int TW, int NT>
__device__ __forceinline__ void store_chunk(uint16_t* tile, const ChunkRegs<TW, NT>& R, uint32_t tid) {
    constexpr int kPer = kKC * TW / 8 / NT, kCols = TW / 8, kPitch = Pitch<TW>::value;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const uint32_t idx = tid + (uint32_t)NT * i, row = idx / kCols, col = (idx % kCols) * 8u;
        *reinterpret_cast<u4v*>(tile + row * kPitch + col) = R.v[i];
    }
}


// BM x BN block tile of [J, C]; one wave per 64 x 64 sub-tile.
template <int BM, int BN, bool kWantG>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64, 2)
void k_conv_bf16(const uint16_t* __restrict__ U, const uint16_t* __restrict__ D,
                 uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                 uint32_t z_per_split, uint32_t splits, float cg, float cs,
                 float* __restrict__ g_out, float* __restrict__ s_out, float* __restrict__ ws) {
    constexpr int NT = (BM / 64) * (BN / 64) * 64;
    constexpr int kPA = Pitch<BM>::value, kPB = Pitch<BN>::value;
    __shared__ __attribute__((aligned(16))) uint16_t shA[2][kKC * kPA];
    __shared__ __attribute__((aligned(16))) uint16_t shB[2][kKC * kPB];

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t wm = wave / (BN / 64), wn = wave % (BN / 64);
    // Workgroups are dealt to the 8 XCDs round-robin by linear id.  Give every XCD a contiguous range
    // of (split, row tile, column tile) so that the workgroups sharing a sample range and a row tile
    // also share an L2.
    const uint32_t tiles_c = (C + BN - 1) / BN, tiles_j = (J + BM - 1) / BM;
    const uint32_t nblk = gridDim.x, per = nblk / 8u, rem = nblk % 8u;
    const uint32_t xcd = blockIdx.x % 8u, slot = blockIdx.x / 8u;
    const uint32_t logical = xcd * per + min(xcd, rem) + slot;
    const uint32_t tile_c = logical % tiles_c, tile_j = (logical / tiles_c) % tiles_j, split = logical / (tiles_c * tiles_j);
    const uint32_t j0 = tile_j * BM, c0 = tile_c * BN;
    const uint32_t z_begin = split * z_per_split;
    const uint32_t z_end = min(B, z_begin + z_per_split);
    const uint32_t n_chunks = (P + kKC - 1) / kKC;
    const uint32_t total = (z_end - z_begin) * n_chunks;

    f16v acc[2][2], s_acc[2][2], g_acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            acc[a][b] = (f16v){0};
            s_acc[a][b] = (f16v){0};
            if (kWantG) g_acc[a][b] = (f16v){0};
        }

    constexpr int kDepth = 2;                            // chunks in flight from global memory per thread
    constexpr int kKS = kKC / 16;                        // MFMA k-steps per chunk
    ChunkRegs<BM, NT> ra[kDepth];
    ChunkRegs<BN, NT> rb[kDepth];
    uint32_t zl = z_begin, pcl = 0, issued = 0;          // cursor of the next chunk to request from global memory
    auto issue = [&](int slot_) {                       // past the last chunk the range is empty: zeros come back
        const bool live = issued < total;
        const uint32_t zz = live ? zl : z_begin, pq = pcl;
        load_chunk<BM, NT>(ra[slot_], sample_rsrc(U + (size_t)zz * P * J, live ? P * J * 2u : 0u), J, pq * kKC, j0, tid);
        load_chunk<BN, NT>(rb[slot_], sample_rsrc(D + (size_t)zz * P * C, live ? P * C * 2u : 0u), C, pq * kKC, c0, tid);
        if (++pcl == n_chunks) { pcl = 0; ++zl; }
        ++issued;
    };
    auto sample_end = [&]() {                            // G_z is complete in acc: square into s, add into g, clear
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
    };
    // The loop bodies are free of branches around memory operations (the trip count is rounded up to a
    // multiple of the unroll factor; the surplus chunks are all zeros and add nothing), which keeps the
    // compiler's count of outstanding loads exact.
    uint32_t pc = 0, zdone = z_begin;

    if constexpr (!kWantG) {
        // Pipelined across the barrier: the operand fragments of chunk q+1 are read from LDS while the
        // MFMAs of chunk q run from registers, and chunk q+2 is staged into the buffer chunk q came from.
        bf8v F[2][kKS][2][2];                            // [ping-pong][k-step][A / B][32-wide tile]
        auto read_frags = [&](int pp, uint32_t buf) {
#pragma unroll
            for (int ks = 0; ks < kKS; ++ks)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    F[pp][ks][0][t] = lds_frag_bf16<BM>(shA[buf], ks, wm * 64 + t * 32, lane);
                    F[pp][ks][1][t] = lds_frag_bf16<BN>(shB[buf], ks, wn * 64 + t * 32, lane);
                }
        };
        issue(0);
        issue(1);
        store_chunk<BM, NT>(shA[0], ra[0], tid);
        store_chunk<BN, NT>(shB[0], rb[0], tid);
        issue(0);
        __syncthreads();
        read_frags(0, 0);
        store_chunk<BM, NT>(shA[1], ra[1], tid);
        store_chunk<BN, NT>(shB[1], rb[1], tid);
        issue(1);
        __syncthreads();
        // A wave issues in order, and the two waves of a SIMD run in lockstep between barriers: if the
        // MFMAs sat in one block and the LDS traffic in another, the matrix pipe would idle during the
        // LDS phase and vice versa.  So the instruction stream is interleaved by hand: after every MFMA
        // one operand fragment (two transposing reads) of the next chunk is requested, and the staging
        // writes and the next global loads go in the middle of the MFMA sequence.
        static_assert(kKS == 2, "the interleaving below is written for two k-steps per chunk");
        for (uint32_t q0 = 0; q0 < total; q0 += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {                // chunk q = q0 + u lives in fragment set u, LDS buffer u
                const uint32_t nb = (uint32_t)(u ^ 1);
#pragma unroll
                for (int i = 0; i < 8; ++i) {            // MFMA i = (ks, mt, nt); fragment i = (ks, A/B, t) of chunk q+1
                    const int ks = i >> 2, mt = (i >> 1) & 1, nt = i & 1;
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F[u][ks][0][mt], F[u][ks][1][nt], acc[mt][nt], 0, 0, 0);
                    const int fk = i >> 2, fo = (i >> 1) & 1, ft = i & 1;
                    if (fo == 0) F[u ^ 1][fk][0][ft] = lds_frag_bf16<BM>(shA[nb], fk, wm * 64 + ft * 32, lane);
                    else F[u ^ 1][fk][1][ft] = lds_frag_bf16<BN>(shB[nb], fk, wn * 64 + ft * 32, lane);
                    if (i == 3) {
                        store_chunk<BM, NT>(shA[u], ra[u], tid);  // chunk q+2, then its registers take chunk q+4
                        store_chunk<BN, NT>(shB[u], rb[u], tid);
                        issue(u);
                    }
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {            // pin the order above for the instruction scheduler
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);      // two LDS reads
                    if (i == 3) {
                        __builtin_amdgcn_sched_group_barrier(0x200, kKC * (BM + BN) / 8 / NT, 0);   // the LDS writes
                        __builtin_amdgcn_sched_group_barrier(0x020, kKC * (BM + BN) / 8 / NT, 0);   // the global loads
                    }
                }
                if (++pc == n_chunks && zdone < z_end) { pc = 0; ++zdone; sample_end(); }
                __syncthreads();
            }
        }
    } else {
        issue(0);
        issue(1);
        store_chunk<BM, NT>(shA[0], ra[0], tid);
        store_chunk<BN, NT>(shB[0], rb[0], tid);
        issue(0);
        __syncthreads();
        for (uint32_t q0 = 0; q0 < total; q0 += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {                // chunk q = q0 + u is in LDS buffer u
#pragma unroll
                for (int ks = 0; ks < kKS; ++ks) {
                    bf8v fa[2], fb[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        fa[t] = lds_frag_bf16<BM>(shA[u], ks, wm * 64 + t * 32, lane);
                        fb[t] = lds_frag_bf16<BN>(shB[u], ks, wn * 64 + t * 32, lane);
                    }
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int nt = 0; nt < 2; ++nt)
                            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mt], fb[nt], acc[mt][nt], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);       // MFMAs issue before the wait for the global loads
                store_chunk<BM, NT>(shA[u ^ 1], ra[u ^ 1], tid);   // chunk q+1, then its registers take chunk q+3
                store_chunk<BN, NT>(shB[u ^ 1], rb[u ^ 1], tid);
                issue(u ^ 1);
                if (++pc == n_chunks && zdone < z_end) { pc = 0; ++zdone; sample_end(); }
                __syncthreads();
            }
        }
    }

    // ---- epilogue: scaled result, or unscaled partial sums for the fixed-order reduction ----
    const bool direct = (splits == 1);
    const size_t JC = (size_t)J * C;
    float* so = direct ? s_out : ws + (size_t)split * 2 * JC;
    float* go = direct ? g_out : ws + (size_t)split * 2 * JC + JC;
    const float fs = direct ? cs : 1.0f, fg = direct ? cg : 1.0f;
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
                    if (kWantG) __builtin_nontemporal_store(fg * g_acc[mt][nt][i], go + o);
                }
            }
        }
}

// Adds the per-split partial sums in split order and applies the scale factors.
__global__ __launch_bounds__(256) void k_sqgrad_reduce(const float* __restrict__ ws, uint32_t splits, size_t JC,
                                                       float cg, float cs, float* __restrict__ g_out,
                                                       float* __restrict__ s_out) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= JC) return;
    float s = 0.f, g = 0.f;
    for (uint32_t k = 0; k < splits; ++k) {
        s += ws[(size_t)k * 2 * JC + i];
        if (g_out) g += ws[(size_t)k * 2 * JC + JC + i];
    }
    s_out[i] = cs * s;
    if (g_out) g_out[i] = cg * g;
}

// Block tile for a shape: wide in J (256) when J has room, 64 / 128 in C following C.
struct ConvTile { int bm, bn; };
static ConvTile conv_tile(uint32_t J, uint32_t C) {
    ConvTile t;
    t.bn = (C <= 64) ? 64 : 128;
    // 256 rows unless 128 wastes clearly less of the last tile
    const uint32_t pad256 = (J + 255) / 256 * 256, pad128 = (J + 127) / 128 * 128;
    t.bm = (J >= 256 && pad256 * 10 <= pad128 * 11) ? 256 : 128;
    return t;
}

// How many ways to split the samples.  Workgroups run in rounds of `slots` (compute units x resident
// workgroups); the cost of a choice is rounds x samples per workgroup, plus one pass over the partial
// sums per split for the reduction (weighted as a fraction of one sample's work on a tile).
uint32_t conv_splits(uint32_t B, uint32_t J, uint32_t C) {
    const ConvTile t = conv_tile(J, C);
    const uint64_t tiles = (uint64_t)((J + t.bm - 1) / t.bm) * ((C + t.bn - 1) / t.bn);
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n_cu = v;
        else n_cu = 256;
    }
    const uint64_t waves_per_wg = (uint64_t)(t.bm / 64) * (t.bn / 64);
    const uint64_t slots = (uint64_t)n_cu * (8 / waves_per_wg);
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

size_t sqgrad_workspace_bytes(int kind, int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    if (kind != VGC_CONV) return 0;
    uint32_t splits = 1;
    if (conv_tiled_supported(dtype, P, J, C)) splits = conv_splits(B, J, C);
    else if (dtype == VGC_F32 && conv_f32_tiled_supported(P, J, C)) splits = conv_f32_splits(B, J, C);
    return splits > 1 ? (size_t)splits * 2 * J * C * sizeof(float) : 0;
}

bool conv_tiled_supported(int dtype, uint32_t P, uint32_t J, uint32_t C) {
    const uint64_t limit = 0x7FFFFFFFull;               // buffer ranges and offsets are 32-bit
    return dtype == VGC_BF16 && (J % 8 == 0) && (C % 8 == 0) && (uint64_t)(P + 64) * J * 2 < limit &&
           (uint64_t)(P + 64) * C * 2 < limit;
}

void launch_sqgrad_reduce(const float* ws, uint32_t splits, size_t JC, float cg, float cs, float* g_out, float* s_out,
                          hipStream_t stream) {
    hipLaunchKernelGGL(k_sqgrad_reduce, dim3((uint32_t)((JC + 255) / 256)), dim3(256), 0, stream, ws, splits, JC, cg, cs,
                       g_out, s_out);
}

template <int BM, int BN>
static void launch_conv_bf16(uint32_t nblk, hipStream_t stream, const void* X, const void* D, uint32_t B, uint32_t P,
                             uint32_t J, uint32_t C, uint32_t zper, uint32_t splits, float cg, float cs,
                             float* g_out, float* s_out, float* ws) {
    constexpr int NT = (BM / 64) * (BN / 64) * 64;
    if (g_out)
        hipLaunchKernelGGL((k_conv_bf16<BM, BN, true>), dim3(nblk), dim3(NT), 0, stream, (const uint16_t*)X,
                           (const uint16_t*)D, B, P, J, C, zper, splits, cg, cs, g_out, s_out, ws);
    else
        hipLaunchKernelGGL((k_conv_bf16<BM, BN, false>), dim3(nblk), dim3(NT), 0, stream, (const uint16_t*)X,
                           (const uint16_t*)D, B, P, J, C, zper, splits, cg, cs, g_out, s_out, ws);
}

int launch_conv_tiled(int dtype, const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                      float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    (void)dtype;
    const ConvTile t = conv_tile(J, C);
    uint32_t splits = conv_splits(B, J, C);
    if (splits > 1 && (!workspace || workspace_bytes < (size_t)splits * 2 * J * C * sizeof(float))) splits = 1;
    const uint32_t zper = (B + splits - 1) / splits;
    splits = (B + zper - 1) / zper;
    const uint64_t nblk = (uint64_t)((C + t.bn - 1) / t.bn) * ((J + t.bm - 1) / t.bm) * splits;
    if (nblk > 0x7FFFFFFFull) { set_error("vgc_sqgrad: shape exceeds the launch limit"); return VGC_ERR_SIZE; }
    const float cg = c, cs = c * c;
    float* ws = static_cast<float*>(workspace);
    if (t.bm == 256 && t.bn == 128) launch_conv_bf16<256, 128>((uint32_t)nblk, stream, X, D, B, P, J, C, zper, splits, cg, cs, g_out, s_out, ws);
    else if (t.bm == 256 && t.bn == 64) launch_conv_bf16<256, 64>((uint32_t)nblk, stream, X, D, B, P, J, C, zper, splits, cg, cs, g_out, s_out, ws);
    else if (t.bm == 128 && t.bn == 128) launch_conv_bf16<128, 128>((uint32_t)nblk, stream, X, D, B, P, J, C, zper, splits, cg, cs, g_out, s_out, ws);
    else launch_conv_bf16<128, 64>((uint32_t)nblk, stream, X, D, B, P, J, C, zper, splits, cg, cs, g_out, s_out, ws);
    if (splits > 1) launch_sqgrad_reduce(ws, splits, (size_t)J * C, cg, cs, g_out, s_out, stream);
    return hip_check(hipGetLastError(), "launch k_conv_bf16");
}

}  // namespace vgc

