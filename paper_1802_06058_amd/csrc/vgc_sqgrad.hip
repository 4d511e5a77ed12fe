// Per-parameter sums over the mini-batch (Alg. 1, first two lines of the loop body):
//   g = c * sum_z G_z,   s = c^2 * sum_z G_z . G_z,   G_z = gradient of sample z's loss (Section 4.1).
//
// FC form:   G_z = x_z d_z^T, so g = c X^T D and s = c^2 (X.X)^T (D.D): two MFMA chains over K = B.
// Conv form: G_z = U_z^T D_z (K = P positions); the per-sample product stays in the accumulator
//            registers, is squared and added to s (and added to g) when the sample is finished.
//
// float32 MFMA (v_mfma_f32_32x32x2_f32) with float32 accumulators.  Operand layout of that
// instruction: lane l supplies A[m = l%32][k = l/32] and B[k = l/32][n = l%32]; the 16 results a
// lane holds are D[m = 8*(i/4) + 4*(l/32) + i%4][n = l%32], i = 0..15.
#include "vgc_internal.h"

namespace vgc {

typedef float f16v __attribute__((ext_vector_type(16)));

template <typename T> __device__ __forceinline__ float ld(const T* p);
template <> __device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld<uint16_t>(const uint16_t* p) {   // bfloat16 bits, widened exactly
    return __uint_as_float((uint32_t)(*p) << 16);
}

// Each wave owns a 32 x 32 tile of [J, C]; a workgroup is 2 x 2 waves (64 x 64).
template <typename T, bool kConv>
__global__ __launch_bounds__(256) void k_sqgrad_simple(const T* __restrict__ X, const T* __restrict__ D,
                                                       uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                                                       float c, float* __restrict__ g_out, float* __restrict__ s_out) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t j0 = blockIdx.y * 64 + (wave >> 1) * 32;
    const uint32_t c0 = blockIdx.x * 64 + (wave & 1u) * 32;
    if (j0 >= J || c0 >= C) return;                       // wave-uniform
    const uint32_t col = lane & 31u, kh = lane >> 5;
    const uint32_t ja = j0 + col, cb = c0 + col;
    const bool va = ja < J, vb = cb < C;

    f16v acc_g = {0}, acc_s = {0};
    if (!kConv) {
        for (uint32_t z0 = 0; z0 < B; z0 += 2) {
            const uint32_t z = z0 + kh;
            float a = 0.f, b = 0.f;
            if (z < B) {
                if (va) a = ld<T>(X + (size_t)z * J + ja);
                if (vb) b = ld<T>(D + (size_t)z * C + cb);
            }
            acc_g = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc_g, 0, 0, 0);
            acc_s = __builtin_amdgcn_mfma_f32_32x32x2f32(a * a, b * b, acc_s, 0, 0, 0);
        }
    } else {
        for (uint32_t z = 0; z < B; ++z) {
            f16v acc = {0};
            const T* Xz = X + (size_t)z * P * J;
            const T* Dz = D + (size_t)z * P * C;
            for (uint32_t p0 = 0; p0 < P; p0 += 2) {
                const uint32_t p = p0 + kh;
                float a = 0.f, b = 0.f;
                if (p < P) {
                    if (va) a = ld<T>(Xz + (size_t)p * J + ja);
                    if (vb) b = ld<T>(Dz + (size_t)p * C + cb);
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                acc_g[i] += acc[i];
                acc_s[i] += acc[i] * acc[i];
            }
        }
    }
    const float c2 = c * c;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t row = j0 + 8 * (i >> 2) + 4 * kh + (i & 3);
        if (row < J && vb) {
            const size_t o = (size_t)row * C + cb;
            if (g_out) g_out[o] = c * acc_g[i];
            s_out[o] = c2 * acc_s[i];
        }
    }
}

int launch_sqgrad(int kind, int dtype, const void* X, const void* D, uint32_t B, uint32_t P,
                  uint32_t J, uint32_t C, float c, float* g_out, float* s_out,
                  void* workspace, size_t workspace_bytes, hipStream_t stream) {
    if (kind == VGC_CONV && conv_tiled_supported(dtype, P, J, C))
        return launch_conv_tiled(dtype, X, D, B, P, J, C, c, g_out, s_out, workspace, workspace_bytes, stream);
    if (kind == VGC_CONV && dtype == VGC_F32 && conv_f32_tiled_supported(P, J, C))
        return launch_conv_f32_tiled(X, D, B, P, J, C, c, g_out, s_out, workspace, workspace_bytes, stream);
    if (kind == VGC_FC && fc_tiled_supported(dtype, B, J, C))
        return launch_fc_tiled(dtype, X, D, B, J, C, c, g_out, s_out, stream);
    // shapes the tiled kernels do not take (row lengths that are not a multiple of 16 bytes)
    return launch_sqgrad_simple(kind, dtype, X, D, B, P, J, C, c, g_out, s_out, stream);
}

int launch_sqgrad_simple(int kind, int dtype, const void* X, const void* D, uint32_t B, uint32_t P,
                         uint32_t J, uint32_t C, float c, float* g_out, float* s_out, hipStream_t stream) {
    dim3 grid((C + 63) / 64, (J + 63) / 64), block(256);
    if (grid.y > 65535u) {
        set_error("vgc_sqgrad: J = %u exceeds the launch limit", J);
        return VGC_ERR_SIZE;
    }
#define VGC_LAUNCH(T, CONV) hipLaunchKernelGGL((k_sqgrad_simple<T, CONV>), grid, block, 0, stream, \
        (const T*)X, (const T*)D, B, P, J, C, c, g_out, s_out)
    if (kind == VGC_FC) {
        if (dtype == VGC_F32) VGC_LAUNCH(float, false); else VGC_LAUNCH(uint16_t, false);
    } else {
        if (dtype == VGC_F32) VGC_LAUNCH(float, true); else VGC_LAUNCH(uint16_t, true);
    }
#undef VGC_LAUNCH
    return hip_check(hipGetLastError(), "launch k_sqgrad");
}

}  // namespace vgc
