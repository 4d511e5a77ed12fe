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

constexpr int kBM = 128, kBN = 128;      // block tile of [J, C]
constexpr int kKC = 32;                  // positions per LDS stage
constexpr int kPitch = 160;              // bf16 elements per staged row: 128 + 32 so that 4 rows x 2 halves hit distinct banks

__device__ __forceinline__ bf8v lds_frag_bf16(const uint16_t* tile, int ks, int mbase, uint32_t lane) {
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

// One staged chunk of an operand: rows p0 .. p0+31 of a [P, W] bf16 matrix, columns w0 .. w0+127.
struct ChunkRegs { u4v v[2]; };

__device__ __forceinline__ ChunkRegs load_chunk_bf16(const uint16_t* __restrict__ M, uint32_t P, uint32_t W,
                                                     uint32_t p0, uint32_t w0, uint32_t tid) {
    ChunkRegs R;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t idx = tid + 256u * i, row = idx >> 4, col = w0 + (idx & 15u) * 8u;
        R.v[i] = (u4v){0u, 0u, 0u, 0u};
        if (p0 + row < P && col < W) R.v[i] = *reinterpret_cast<const u4v*>(M + (size_t)(p0 + row) * W + col);
    }
    return R;
}

__device__ __forceinline__ void store_chunk_bf16(uint16_t* tile, const ChunkRegs& R, uint32_t tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const uint32_t idx = tid + 256u * i, row = idx >> 4, col = (idx & 15u) * 8u;
        *reinterpret_cast<u4v*>(tile + row * kPitch + col) = R.v[i];
    }
}

template <bool kWantG>
__global__ __launch_bounds__(256) void k_conv_bf16(const uint16_t* __restrict__ U, const uint16_t* __restrict__ D,
                                                   uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                                                   uint32_t z_per_split, float cg, float cs,
                                                   float* __restrict__ g_out, float* __restrict__ s_out,
                                                   float* __restrict__ ws) {
    __shared__ __attribute__((aligned(16))) uint16_t shA[2][kKC * kPitch];
    __shared__ __attribute__((aligned(16))) uint16_t shB[2][kKC * kPitch];

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1u;
    const uint32_t j0 = blockIdx.y * kBM, c0 = blockIdx.x * kBN;
    const uint32_t z_begin = blockIdx.z * z_per_split;
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

    // prologue: first chunk of the first sample
    {
        const uint16_t* Uz = U + (size_t)z_begin * P * J;
        const uint16_t* Dz = D + (size_t)z_begin * P * C;
        const ChunkRegs ra = load_chunk_bf16(Uz, P, J, 0, j0, tid);
        const ChunkRegs rb = load_chunk_bf16(Dz, P, C, 0, c0, tid);
        store_chunk_bf16(shA[0], ra, tid);
        store_chunk_bf16(shB[0], rb, tid);
    }
    __syncthreads();

    uint32_t z = z_begin, pc = 0;
    for (uint32_t q = 0; q < total; ++q) {
        const uint32_t buf = q & 1u;
        // next chunk: global -> registers while this one is multiplied
        uint32_t zn = z, pcn = pc + 1;
        if (pcn == n_chunks) { pcn = 0; ++zn; }
        const bool have_next = (q + 1 < total);
        ChunkRegs ra, rb;
        if (have_next) {
            ra = load_chunk_bf16(U + (size_t)zn * P * J, P, J, pcn * kKC, j0, tid);
            rb = load_chunk_bf16(D + (size_t)zn * P * C, P, C, pcn * kKC, c0, tid);
        }
#pragma unroll
        for (int ks = 0; ks < kKC / 16; ++ks) {
            bf8v a[2], b[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                a[t] = lds_frag_bf16(shA[buf], ks, wm * 64 + t * 32, lane);
                b[t] = lds_frag_bf16(shB[buf], ks, wn * 64 + t * 32, lane);
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
        }
        if (have_next) {
            store_chunk_bf16(shA[buf ^ 1u], ra, tid);
            store_chunk_bf16(shB[buf ^ 1u], rb, tid);
        }
        if (pc + 1 == n_chunks) {                      // sample finished: G_z is complete in acc
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
        z = zn; pc = pcn;
    }

    // ---- epilogue: scaled result, or unscaled partial sums for the fixed-order reduction ----
    const bool direct = (gridDim.z == 1);
    const size_t JC = (size_t)J * C;
    float* so = direct ? s_out : ws + (size_t)blockIdx.z * 2 * JC;
    float* go = direct ? g_out : ws + (size_t)blockIdx.z * 2 * JC + JC;
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

size_t sqgrad_workspace_bytes(int kind, int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    (void)P;
    if (kind != VGC_CONV || dtype != VGC_BF16) return 0;
    const uint32_t splits = conv_splits(B, J, C);
    return splits > 1 ? (size_t)splits * 2 * J * C * sizeof(float) : 0;
}

uint32_t conv_splits(uint32_t B, uint32_t J, uint32_t C) {
    const uint64_t tiles = (uint64_t)((J + kBM - 1) / kBM) * ((C + kBN - 1) / kBN);
    uint64_t want = (1024 + tiles - 1) / tiles;          // aim for about four workgroups per compute unit
    if (want > B) want = B;
    if (want < 1) want = 1;
    return (uint32_t)want;
}

bool conv_tiled_supported(int dtype, uint32_t J, uint32_t C) {
    return dtype == VGC_BF16 && (J % 8 == 0) && (C % 8 == 0);
}

int launch_conv_tiled(int dtype, const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                      float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    (void)dtype;
    uint32_t splits = conv_splits(B, J, C);
    if (splits > 1 && (!workspace || workspace_bytes < (size_t)splits * 2 * J * C * sizeof(float))) splits = 1;
    const uint32_t zper = (B + splits - 1) / splits;
    splits = (B + zper - 1) / zper;
    dim3 grid((C + kBN - 1) / kBN, (J + kBM - 1) / kBM, splits);
    if (grid.y > 65535u || grid.z > 65535u) { set_error("vgc_sqgrad: shape exceeds the launch limit"); return VGC_ERR_SIZE; }
    const float cg = c, cs = c * c;
    float* ws = static_cast<float*>(workspace);
    if (g_out)
        hipLaunchKernelGGL(k_conv_bf16<true>, grid, dim3(256), 0, stream, (const uint16_t*)X, (const uint16_t*)D, B, P, J, C,
                           zper, cg, cs, g_out, s_out, ws);
    else
        hipLaunchKernelGGL(k_conv_bf16<false>, grid, dim3(256), 0, stream, (const uint16_t*)X, (const uint16_t*)D, B, P, J, C,
                           zper, cg, cs, g_out, s_out, ws);
    if (splits > 1) {
        const size_t JC = (size_t)J * C;
        hipLaunchKernelGGL(k_sqgrad_reduce, dim3((uint32_t)((JC + 255) / 256)), dim3(256), 0, stream, ws, splits, JC, cg, cs,
                           g_out, s_out);
    }
    return hip_check(hipGetLastError(), "launch k_conv_bf16");
}

}  // namespace vgc
