// Native driver of the squared-gradient statistic (Sec. 4.2: s = sum over the batch of the squared
// per-sample gradient, for fully connected and convolutional layers) for profiling without a Python
// process: fills the operands with seeded synthetic values on the device, runs one untimed call and
// then `reps` timed calls through the C ABI, and prints the average duration from HIP events.
//
//   vgc_sqgrad_bench fc     <f32|bf16> B J C             [want_g = 1] [reps = 20]
//   vgc_sqgrad_bench patch  <f32|bf16> B P J C           [want_g = 1] [reps = 20]
//   vgc_sqgrad_bench conv2d <f32|bf16> B H W Cin C k stride pad [want_g = 1] [reps = 20]
//
// fc:     a[B, J], d[B, C]                      (one position per sample)
// patch:  patch matrix a[B, P, J], d[B, P, C]   (convolution lowered by the caller)
// conv2d: NHWC activations a[B, H, W, Cin], d[B, Ho, Wo, C]; square kernel, equal strides and pads
//
// Values are uniform in [-1, 1) from a counter-based hash; their distribution does not affect the
// duration of a dense contraction.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "vgc.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1); } } while (0)
#define VK(x) do { int r_ = (x); if (r_ != 0) { fprintf(stderr, "vgc error %d (%s) at %s:%d\n", r_, vgc_last_error(), __FILE__, __LINE__); exit(1); } } while (0)

__device__ __forceinline__ float hash_uniform(uint64_t i, uint32_t seed) {
    uint32_t x = (uint32_t)i * 2654435761u + (uint32_t)(i >> 32) * 40503u + seed;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    return ((int)(x & 0xFFFF) - 32768) * (1.0f / 32768.0f);
}

__global__ void k_fill_bf16(uint16_t* p, uint64_t n, uint32_t seed) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (uint16_t)(__float_as_uint(hash_uniform(i, seed)) >> 16);   // 16 significant bits: exact in bf16
}

__global__ void k_fill_f32(float* p, uint64_t n, uint32_t seed) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = hash_uniform(i, seed);
}

static void* filled(uint64_t n, int dtype, uint32_t seed) {
    void* p;
    CK(hipMalloc(&p, n * (dtype == VGC_BF16 ? 2 : 4)));
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (dtype == VGC_BF16) k_fill_bf16<<<blocks, 256>>>((uint16_t*)p, n, seed);
    else k_fill_f32<<<blocks, 256>>>((float*)p, n, seed);
    CK(hipGetLastError());
    return p;
}

static int usage() {
    fprintf(stderr,
            "usage: vgc_sqgrad_bench fc     <f32|bf16> B J C [want_g] [reps]\n"
            "       vgc_sqgrad_bench patch  <f32|bf16> B P J C [want_g] [reps]\n"
            "       vgc_sqgrad_bench conv2d <f32|bf16> B H W Cin C k stride pad [want_g] [reps]\n");
    return 2;
}

int main(int argc, char** argv) {
    if (argc < 3) return usage();
    const char* form = argv[1];
    int dtype;
    if (!strcmp(argv[2], "bf16")) dtype = VGC_BF16;
    else if (!strcmp(argv[2], "f32")) dtype = VGC_F32;
    else return usage();
    const bool is_fc = !strcmp(form, "fc"), is_patch = !strcmp(form, "patch"), is_conv = !strcmp(form, "conv2d");
    const int n_dims = is_fc ? 3 : is_patch ? 4 : is_conv ? 8 : -1;
    if (n_dims < 0 || argc < 3 + n_dims) return usage();
    uint32_t v[8];
    for (int i = 0; i < n_dims; ++i) v[i] = (uint32_t)strtoul(argv[3 + i], 0, 10);
    const int want_g = argc > 3 + n_dims ? atoi(argv[3 + n_dims]) : 1;
    const int reps = argc > 4 + n_dims ? atoi(argv[4 + n_dims]) : 20;
    if (reps < 1) return usage();

    uint32_t B = v[0], P = 1, J, C, H = 0, W = 0, Cin = 0, k = 0, st = 0, pd = 0, Ho = 0, Wo = 0;
    uint64_t n_act, n_delta;
    size_t ws_bytes;
    if (is_conv) {
        H = v[1]; W = v[2]; Cin = v[3]; C = v[4]; k = v[5]; st = v[6]; pd = v[7];
        if (!st || H + 2 * pd < k || W + 2 * pd < k) return usage();
        Ho = (H + 2 * pd - k) / st + 1; Wo = (W + 2 * pd - k) / st + 1;
        J = k * k * Cin; P = Ho * Wo;
        n_act = (uint64_t)B * H * W * Cin; n_delta = (uint64_t)B * P * C;
        ws_bytes = vgc_sqgrad_conv2d_workspace_bytes(dtype, B, H, W, Cin, C, k, k, st, st, pd, pd);
    } else {
        if (is_patch) { P = v[1]; J = v[2]; C = v[3]; } else { J = v[1]; C = v[2]; }
        n_act = (uint64_t)B * P * J; n_delta = (uint64_t)B * P * C;
        ws_bytes = vgc_sqgrad_workspace_bytes(is_fc ? VGC_FC : VGC_CONV, dtype, B, P, J, C);
    }

    void* act = filled(n_act, dtype, 1);
    void* delta = filled(n_delta, dtype, 2);
    float *g = nullptr, *s;
    void* ws = nullptr;
    if (want_g) CK(hipMalloc(&g, (size_t)J * C * 4));
    CK(hipMalloc(&s, (size_t)J * C * 4));
    if (ws_bytes) CK(hipMalloc(&ws, ws_bytes));
    const float c = 1.0f / B;

    auto call = [&]() {
        if (is_conv) VK(vgc_sqgrad_conv2d(dtype, act, delta, B, H, W, Cin, C, k, k, st, st, pd, pd, c, g, s, ws, ws_bytes, 0));
        else VK(vgc_sqgrad(is_fc ? VGC_FC : VGC_CONV, dtype, act, delta, B, P, J, C, c, g, s, ws, ws_bytes, 0));
    };
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    call();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) call();
    CK(hipEventRecord(e1, 0));
    CK(hipDeviceSynchronize());
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    ms /= reps;
    // contraction flops of the statistic; the fully connected form with the mean also does the B-deep product for g
    const double flops = ((is_fc && want_g) ? 4.0 : 2.0) * B * P * (double)J * C;
    if (is_conv) printf("conv2d %s B=%u %ux%ux%u -> %ux%ux%u k=%u stride=%u pad=%u", argv[2], B, H, W, Cin, Ho, Wo, C, k, st, pd);
    else printf("%s %s B=%u P=%u J=%u C=%u", form, argv[2], B, P, J, C);
    printf(" want_g=%d workspace=%zu B: %.4f ms per call over %d calls, %.1f TFLOP/s\n", want_g, ws_bytes, ms, reps, flops / ms / 1e9);
    return 0;
}
