// Native driver of the C ABI for profiling without a Python process: the flat-stream workload of the benchmark
// (per parameter and step a batch of 16 Student-t(3) per-sample gradients, several simulated workers with a state
// of their own, groups of 2^24).  Per step it runs a plain copy of known size (the calibration dispatch for the
// HBM-traffic counters), then for every worker accumulate/select + pack, then the decode of all the workers'
// messages in one pass (vgc_unpack_add_batch, overwrite) and the same decode fused with a Momentum SGD and an
// Adam step (vgc_unpack_apply).
//
//   vgc_microbench [n = 1000000000] [steps = 2] [alpha = 1.0] [group = 16777216] [workers = 8]
//
// Synthetic inputs: y_z = z / sqrt(chi2_3 / 3) for 16 samples z per parameter, normals from Box-Muller on a
// counter-based hash (splitmix64); g = sum y_z / 16, s = sum (y_z / 16)^2, float32.
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
    float gsum = 0.f, ssum = 0.f;
    for (int z = 0; z < 16; ++z) {                               // one sample: 4 normals = 2 Box-Muller pairs
        float nrm[4];
        for (int k = 0; k < 2; ++k) {
            const uint32_t a = mix(seed + (i * 16 + z) * 4 + 2 * k), b = mix(seed + (i * 16 + z) * 4 + 2 * k + 1);
            const float u1 = ((a >> 8) + 1) * (1.0f / 16777216.0f), u2 = (b >> 8) * (1.0f / 16777216.0f);
            const float rad = sqrtf(-2.0f * __logf(u1));
            nrm[2 * k] = rad * __cosf(6.2831853f * u2);
            nrm[2 * k + 1] = rad * __sinf(6.2831853f * u2);
        }
        const float chi = nrm[1] * nrm[1] + nrm[2] * nrm[2] + nrm[3] * nrm[3];
        const float y = nrm[0] / sqrtf(chi * (1.0f / 3.0f)) * (1.0f / 16.0f);
        gsum += y;
        ssum += y * y;
    }
    g[i] = gsum;
    s[i] = ssum;
}

__global__ void k_copy(const f4* __restrict__ a, f4* __restrict__ b, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(a + i), b + i);
}

int main(int argc, char** argv) {
    const uint64_t n = argc > 1 ? strtoull(argv[1], 0, 10) : 1000000000ull;
    const int steps = argc > 2 ? atoi(argv[2]) : 2;
    const float alpha = argc > 3 ? (float)atof(argv[3]) : 1.0f;
    const uint64_t gsz = argc > 4 ? strtoull(argv[4], 0, 10) : (1ull << 24);
    const int P = argc > 5 ? atoi(argv[5]) : 8;
    if (P < 1 || P > VGC_MAX_UPDATE_MESSAGES) { fprintf(stderr, "workers: 1 .. %d\n", VGC_MAX_UPDATE_MESSAGES); return 1; }

    std::vector<vgc_group> groups;
    for (uint64_t off = 0; off < n; off += gsz) groups.push_back(vgc_group{off, (uint32_t)((n - off < gsz) ? n - off : gsz), 0});
    const uint32_t ng = (uint32_t)groups.size();
    const size_t plan_bytes = vgc_plan_bytes(groups.data(), ng, n), scratch_bytes = vgc_scratch_bytes(groups.data(), ng, n);
    if (!plan_bytes) { fprintf(stderr, "%s\n", vgc_last_error()); return 1; }
    std::vector<char> plan_host(plan_bytes);
    VK(vgc_plan_build(groups.data(), ng, n, plan_host.data(), plan_bytes));

    void *plan, *scratch; float *g, *s, *dense, *param, *m1, *m2;
    std::vector<float*> r(P), v(P); std::vector<uint32_t*> words(P); std::vector<vgc_group_hdr*> hdrs(P); std::vector<vgc_pack_status*> status(P);
    const uint64_t cap = n / 2 + 1024;
    CK(hipMalloc(&plan, plan_bytes)); CK(hipMalloc(&scratch, scratch_bytes));
    CK(hipMalloc(&g, n * 4)); CK(hipMalloc(&s, n * 4)); CK(hipMalloc(&dense, n * 4));
    CK(hipMalloc(&param, n * 4)); CK(hipMalloc(&m1, n * 4)); CK(hipMalloc(&m2, n * 4));
    CK(hipMemset(param, 0, n * 4)); CK(hipMemset(m1, 0, n * 4)); CK(hipMemset(m2, 0, n * 4));
    for (int w = 0; w < P; ++w) {
        CK(hipMalloc(&r[w], n * 4)); CK(hipMalloc(&v[w], n * 4)); CK(hipMalloc(&words[w], cap * 4));
        CK(hipMalloc(&hdrs[w], ng * sizeof(vgc_group_hdr))); CK(hipMalloc(&status[w], sizeof(vgc_pack_status)));
        CK(hipMemset(r[w], 0, n * 4)); CK(hipMemset(v[w], 0, n * 4));
    }
    CK(hipMemcpy(plan, plan_host.data(), plan_bytes, hipMemcpyHostToDevice));
    CK(hipDeviceSynchronize());

    hipEvent_t e[8]; for (auto& x : e) CK(hipEventCreate(&x));
    printf("n=%llu groups=%u tiles=%llu tile=%u alpha=%g workers=%d\n", (unsigned long long)n, ng,
           (unsigned long long)vgc_tile_count(groups.data(), ng, n), vgc_tile_size(), alpha, P);
    for (int it = 0; it < steps; ++it) {
        k_fill<<<(unsigned)((n + 255) / 256), 256>>>(g, s, n, 12345 + 7919ull * it);
        k_copy<<<(unsigned)((n / 4 + 255) / 256), 256>>>((const f4*)g, (f4*)dense, n / 4);   // calibration: 4n read, 4n written
        float t_sel = 0.f, t_pack = 0.f;
        std::vector<uint64_t> nw(P);
        for (int w = 0; w < P; ++w) {
            // every worker draws its own mini-batch every step, so its (r, v) state evolves as in training
            k_fill<<<(unsigned)((n + 255) / 256), 256>>>(g, s, n, 12345 + 7919ull * it + 104729ull * (w + 1));
            CK(hipEventRecord(e[0]));
            VK(vgc_accumulate_select(g, s, r[w], v[w], n, groups.data(), ng, plan, alpha, 0.999f, scratch, 0));
            CK(hipEventRecord(e[1]));
            VK(vgc_pack(n, groups.data(), ng, plan, scratch, words[w], cap, hdrs[w], status[w], 0));
            CK(hipEventRecord(e[2]));
            CK(hipDeviceSynchronize());
            vgc_pack_status st; CK(hipMemcpy(&st, status[w], sizeof(st), hipMemcpyDeviceToHost));
            if (st.overflow || st.plan_mismatch) { fprintf(stderr, "pack: overflow %u mismatch %u\n", st.overflow, st.plan_mismatch); return 1; }
            nw[w] = st.total_words;
            float a, b; CK(hipEventElapsedTime(&a, e[0], e[1])); CK(hipEventElapsedTime(&b, e[1], e[2]));
            t_sel += a / P; t_pack += b / P;
        }
        uint64_t total = 0; for (int w = 0; w < P; ++w) total += nw[w];
        std::vector<const uint32_t*> wp(words.begin(), words.end()); std::vector<const vgc_group_hdr*> hp(hdrs.begin(), hdrs.end());
        CK(hipEventRecord(e[3]));
        VK(vgc_unpack_add_batch(wp.data(), nw.data(), hp.data(), (uint32_t)P, groups.data(), ng, plan, 1.0f / P, 1, dense, n, 0));
        CK(hipEventRecord(e[4]));
        vgc_optimizer opt; opt.kind = VGC_OPT_MOMENTUM_SGD; opt.lr = 1e-3f; opt.momentum = 0.9f; opt.beta1 = 0.9f; opt.beta2 = 0.999f; opt.eps = 1e-8f; opt.step = (uint32_t)it + 1;
        VK(vgc_unpack_apply(wp.data(), nw.data(), hp.data(), (uint32_t)P, groups.data(), ng, plan, 1.0f / P, &opt, param, m1, nullptr, n, 0));
        CK(hipEventRecord(e[5]));
        opt.kind = VGC_OPT_ADAM;
        VK(vgc_unpack_apply(wp.data(), nw.data(), hp.data(), (uint32_t)P, groups.data(), ng, plan, 1.0f / P, &opt, param, m1, m2, n, 0));
        CK(hipEventRecord(e[6]));
        CK(hipDeviceSynchronize());
        float t_dec, t_sgd, t_adam;
        CK(hipEventElapsedTime(&t_dec, e[3], e[4])); CK(hipEventElapsedTime(&t_sgd, e[4], e[5])); CK(hipEventElapsedTime(&t_adam, e[5], e[6]));
        const double rho = (double)total / P / n;
        printf("step %d: words per worker %.0f (rho=%.4f)  select %.3f ms  pack %.3f ms  select+pack %.1f GB/s on %.2f B/param  |  "
               "%d messages: decode %.3f ms (%.1f GB/s on 4 B/word + 4 B/param)  +momentum-sgd %.3f ms (%.1f GB/s)  +adam %.3f ms (%.1f GB/s)\n",
               it, (double)total / P, rho, t_sel, t_pack, (24.0 + 4.0 * rho) * n / ((t_sel + t_pack) * 1e-3) / 1e9, 24.0 + 4.0 * rho, P,
               t_dec, (4.0 * total + 4.0 * n) / (t_dec * 1e-3) / 1e9, t_sgd, (4.0 * total + 16.0 * n) / (t_sgd * 1e-3) / 1e9,
               t_adam, (4.0 * total + 24.0 * n) / (t_adam * 1e-3) / 1e9);
    }
    return 0;
}
