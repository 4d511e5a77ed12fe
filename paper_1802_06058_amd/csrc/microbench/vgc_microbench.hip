// Native driver of the C ABI for profiling without a Python process: builds a plan, fills g and s
// with seeded synthetic values on the device, then runs a plain copy of known size (the calibration
// dispatch for HBM-traffic counters) followed by accumulate/select, pack and the batched decode.
//
//   vgc_microbench [n = 1000000000] [reps = 2] [alpha = 1.0] [group = 16777216]
//
// Every step draws a fresh mini-batch (so the (r, v) state evolves as in training) and prints event
// timings of the three calls.
//
// Synthetic inputs: per parameter, a batch of 16 i.i.d. N(0,1) per-sample gradients reduced to
// g = mean and s = sum (y/16)^2, drawn as g = z/4, s = (chi2_15 + z^2)/256 from a counter-based hash.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "vgc.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1); } } while (0)
#define VK(x) do { int r_ = (x); if (r_ != 0) { fprintf(stderr, "vgc error %d (%s) at %s:%d\n", r_, vgc_last_error(), __FILE__, __LINE__); exit(1); } } while (0)

typedef float f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t mix(uint64_t x) {          // splitmix64 finaliser, high half
    x += 0x9E3779B97F4A7C15ull; x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull; x ^= x >> 31;
    return (uint32_t)(x >> 32);
}

__global__ void k_fill(float* __restrict__ g, float* __restrict__ s, uint64_t n, uint64_t seed) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float z0 = 0.f, chi = 0.f;
    for (int k = 0; k < 8; ++k) {                                // 8 Box-Muller pairs = 16 normals
        const uint32_t a = mix(seed + i * 16 + 2 * k), b = mix(seed + i * 16 + 2 * k + 1);
        const float u1 = ((a >> 8) + 1) * (1.0f / 16777216.0f), u2 = (b >> 8) * (1.0f / 16777216.0f);
        const float rad = sqrtf(-2.0f * __logf(u1));
        const float n0 = rad * __cosf(6.2831853f * u2), n1 = rad * __sinf(6.2831853f * u2);
        if (k == 0) { z0 = n0; chi += n1 * n1; } else { chi += n0 * n0 + n1 * n1; }
    }
    g[i] = 0.25f * z0;
    s[i] = (chi + z0 * z0) * (1.0f / 256.0f);
}

__global__ void k_copy(const f4* __restrict__ a, f4* __restrict__ b, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(a + i), b + i);
}

int main(int argc, char** argv) {
    const uint64_t n = argc > 1 ? strtoull(argv[1], 0, 10) : 1000000000ull;
    const int reps = argc > 2 ? atoi(argv[2]) : 2;
    const float alpha = argc > 3 ? (float)atof(argv[3]) : 1.0f;
    const uint64_t gsz = argc > 4 ? strtoull(argv[4], 0, 10) : (1ull << 24);

    std::vector<vgc_group> groups;
    for (uint64_t off = 0; off < n; off += gsz) groups.push_back(vgc_group{off, (uint32_t)((n - off < gsz) ? n - off : gsz), 0});
    const uint32_t ng = (uint32_t)groups.size();
    const size_t plan_bytes = vgc_plan_bytes(groups.data(), ng, n), scratch_bytes = vgc_scratch_bytes(groups.data(), ng, n);
    if (!plan_bytes) { fprintf(stderr, "%s\n", vgc_last_error()); return 1; }
    std::vector<char> plan_host(plan_bytes);
    VK(vgc_plan_build(groups.data(), ng, n, plan_host.data(), plan_bytes));

    void *plan, *scratch; float *g, *s, *r, *v, *dense; uint32_t* words; vgc_group_hdr* hdrs; vgc_pack_status* status;
    CK(hipMalloc(&plan, plan_bytes)); CK(hipMalloc(&scratch, scratch_bytes));
    CK(hipMalloc(&g, n * 4)); CK(hipMalloc(&s, n * 4)); CK(hipMalloc(&r, n * 4)); CK(hipMalloc(&v, n * 4));
    CK(hipMalloc(&dense, n * 4)); CK(hipMalloc(&words, n * 4)); CK(hipMalloc(&hdrs, ng * sizeof(vgc_group_hdr)));
    CK(hipMalloc(&status, sizeof(vgc_pack_status)));
    CK(hipMemcpy(plan, plan_host.data(), plan_bytes, hipMemcpyHostToDevice));
    CK(hipMemset(r, 0, n * 4)); CK(hipMemset(v, 0, n * 4));
    k_fill<<<(unsigned)((n + 255) / 256), 256>>>(g, s, n, 12345);
    CK(hipDeviceSynchronize());

    hipEvent_t e[5]; for (auto& x : e) CK(hipEventCreate(&x));
    printf("n=%llu groups=%u tiles=%llu tile=%u alpha=%g\n", (unsigned long long)n, ng,
           (unsigned long long)vgc_tile_count(groups.data(), ng, n), vgc_tile_size(), alpha);
    for (int it = 0; it < reps; ++it) {
        k_fill<<<(unsigned)((n + 255) / 256), 256>>>(g, s, n, 12345 + 7919ull * it);       // fresh mini-batch every step
        k_copy<<<(unsigned)((n / 4 + 255) / 256), 256>>>((const f4*)g, (f4*)dense, n / 4);   // calibration: 4n read, 4n written
        CK(hipEventRecord(e[0]));
        VK(vgc_accumulate_select(g, s, r, v, n, groups.data(), ng, plan, alpha, 0.999f, scratch, 0));
        CK(hipEventRecord(e[1]));
        VK(vgc_pack(n, groups.data(), ng, plan, scratch, words, n, hdrs, status, 0));
        CK(hipEventRecord(e[2]));
        CK(hipDeviceSynchronize());
        vgc_pack_status st; CK(hipMemcpy(&st, status, sizeof(st), hipMemcpyDeviceToHost));
        const uint32_t* wp[1] = {words}; const vgc_group_hdr* hp[1] = {hdrs}; uint64_t nw[1] = {st.total_words};
        CK(hipEventRecord(e[3]));
        VK(vgc_unpack_add_batch(wp, nw, hp, 1, groups.data(), ng, plan, 1.0f, 1, dense, n, 0));
        CK(hipEventRecord(e[4]));
        CK(hipDeviceSynchronize());
        float t_sel, t_pack, t_dec;
        CK(hipEventElapsedTime(&t_sel, e[0], e[1])); CK(hipEventElapsedTime(&t_pack, e[1], e[2])); CK(hipEventElapsedTime(&t_dec, e[3], e[4]));
        const double rho = (double)st.total_words / n;
        printf("iter %d: words=%llu (rho=%.4f) select %.3f ms  pack %.3f ms  decode(1 msg) %.3f ms  select+pack %.1f GB/s on %.2f B/param\n",
               it, (unsigned long long)st.total_words, rho, t_sel, t_pack, t_dec,
               (24.0 + 4.0 * rho) * n / ((t_sel + t_pack) * 1e-3) / 1e9, 24.0 + 4.0 * rho);
    }
    return 0;
}
