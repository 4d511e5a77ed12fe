// Host-only exerciser of libvgc's C ABI, meant to be linked against a build of vgc_api.hip whose host code
// is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer.  It walks the pure-host entry points
// (group validation, plan construction, size queries) over group lists of every shape the plan builder
// distinguishes, re-derives each plan table from its definition and compares, and drives every compute entry
// point into each of its argument errors.  Nothing here launches a kernel or dereferences a device pointer:
// the "device" pointers are fabricated addresses that must never be touched before an error is returned.
// Exit status 0 = every check held (the sanitizers abort the process on their own findings).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "vgc.h"

static int g_failed = 0;
#define CHECK(cond)                                                                      \
    do {                                                                                 \
        if (!(cond)) { std::fprintf(stderr, "hostcheck: %s:%d: %s\n", __FILE__, __LINE__, #cond); ++g_failed; } \
    } while (0)

static std::vector<vgc_group> tiling(const std::vector<uint32_t>& sizes) {
    std::vector<vgc_group> g(sizes.size());
    uint64_t off = 0;
    for (size_t k = 0; k < sizes.size(); ++k) { g[k].offset = off; g[k].size = sizes[k]; g[k].reserved = 0; off += sizes[k]; }
    return g;
}

static uint64_t total(const std::vector<uint32_t>& sizes) {
    uint64_t n = 0;
    for (uint32_t s : sizes) n += s;
    return n;
}

// The plan blob as documented for its readers: header words, then group, tile, run and segment tables at the
// byte offsets the header names.  Only what the header itself states is assumed here.
struct Header { uint64_t magic, n, n_tiles; uint32_t n_groups, tile; uint64_t groups_off, tiles_off, runs_off, n_runs, segs_off, n_segs; };
struct PGroup { uint64_t offset; uint32_t size, first_tile; };
struct PTile { uint32_t group, start, seg, run; };
struct PRun { uint32_t group, first_tile; };
struct PSeg { uint32_t group, first_tile, seg_in_group, group_first_seg; };

static void check_plan(const std::vector<uint32_t>& sizes) {
    const std::vector<vgc_group> g = tiling(sizes);
    const uint64_t n = total(sizes);
    const uint32_t T = vgc_tile_size();
    const size_t bytes = vgc_plan_bytes(g.data(), (uint32_t)g.size(), n);
    CHECK(bytes > 0);
    uint64_t tiles = 0;
    for (uint32_t s : sizes) tiles += (s + T - 1) / T;
    CHECK(vgc_tile_count(g.data(), (uint32_t)g.size(), n) == tiles);
    uint64_t n_runs = 0;
    for (uint32_t s : sizes) n_runs += ((s + T - 1) / T + 63) / 64;
    CHECK(vgc_run_count(g.data(), (uint32_t)g.size(), n) == n_runs);
    CHECK(vgc_scratch_bytes(g.data(), (uint32_t)g.size(), n) >= tiles * (T * 2 + T / 8 + 32));
    CHECK(vgc_scratch_bitmap_offset(g.data(), (uint32_t)g.size(), n) < vgc_scratch_bytes(g.data(), (uint32_t)g.size(), n));
    // the builder must stay inside exactly `bytes`: the buffer is allocated to the byte, so that the
    // address sanitizer sees any overrun, and a buffer one byte short must be refused
    std::vector<char> buf(bytes);
    CHECK(vgc_plan_build(g.data(), (uint32_t)g.size(), n, buf.data(), bytes) == VGC_OK);
    std::vector<char> small(bytes - 1);
    CHECK(vgc_plan_build(g.data(), (uint32_t)g.size(), n, small.data(), bytes - 1) == VGC_ERR_SIZE);
    Header h;
    std::memcpy(&h, buf.data(), sizeof(h));
    CHECK(h.n == n && h.n_tiles == tiles && h.n_groups == g.size() && h.tile == T);
    CHECK(h.groups_off + h.n_groups * sizeof(PGroup) <= h.tiles_off);
    CHECK(h.tiles_off + h.n_tiles * sizeof(PTile) <= h.runs_off);
    CHECK(h.runs_off + h.n_runs * sizeof(PRun) <= h.segs_off);
    CHECK(h.segs_off + h.n_segs * sizeof(PSeg) <= bytes);
    const PGroup* G = reinterpret_cast<const PGroup*>(buf.data() + h.groups_off);
    const PTile* Tl = reinterpret_cast<const PTile*>(buf.data() + h.tiles_off);
    const PRun* R = reinterpret_cast<const PRun*>(buf.data() + h.runs_off);
    const PSeg* S = reinterpret_cast<const PSeg*>(buf.data() + h.segs_off);
    uint64_t t = 0, run = 0, seg = 0;
    for (size_t k = 0; k < g.size(); ++k) {
        CHECK(G[k].offset == g[k].offset && G[k].size == g[k].size && G[k].first_tile == t);
        const uint32_t nt = (g[k].size + T - 1) / T;
        const uint64_t first_seg = seg;
        for (uint32_t i = 0; i < nt; ++i, ++t) {
            if (i % 64 == 0) { CHECK(run < h.n_runs && R[run].group == k && R[run].first_tile == i); ++run; }
            if (i % 8192 == 0) {
                CHECK(seg < h.n_segs && S[seg].group == k && S[seg].first_tile == i && S[seg].seg_in_group == seg - first_seg &&
                      S[seg].group_first_seg == first_seg);
                ++seg;
            }
            CHECK(Tl[t].group == k && Tl[t].start == (uint64_t)i * T && Tl[t].seg == seg - 1 && Tl[t].run == run - 1);
        }
    }
    CHECK(t == tiles && run == h.n_runs && run == n_runs && seg == h.n_segs);
}

static void check_group_errors() {
    std::vector<vgc_group> g = tiling({100, 200});
    CHECK(vgc_tile_count(nullptr, 2, 300) == 0);
    CHECK(vgc_tile_count(g.data(), 0, 300) == 0);
    CHECK(vgc_tile_count(g.data(), 2, 0) == 0);
    CHECK(vgc_tile_count(g.data(), 2, 301) == 0 && std::strstr(vgc_last_error(), "cover") != nullptr);
    g[1].offset = 101;
    CHECK(vgc_plan_bytes(g.data(), 2, 300) == 0);
    g[1].offset = 100; g[1].reserved = 1;
    CHECK(vgc_plan_bytes(g.data(), 2, 300) == 0);
    g[1].reserved = 0; g[0].size = 0;
    CHECK(vgc_scratch_bytes(g.data(), 2, 300) == 0);
    std::vector<vgc_group> big = tiling({(1u << 28) + 1});
    char dummy[8];
    CHECK(vgc_plan_build(big.data(), 1, (1ull << 28) + 1, dummy, sizeof(dummy)) == VGC_ERR_GROUP_TOO_LARGE);
    std::vector<vgc_group> ok = tiling({100, 200});
    CHECK(vgc_plan_build(ok.data(), 2, 300, nullptr, 4096) == VGC_ERR_NULL);
}

// Fabricated "device" addresses with the alignment each argument asks for; no call below may get as far as using them.
static void* fake(uintptr_t a) { return reinterpret_cast<void*>(a); }

static void check_compute_errors() {
    const std::vector<vgc_group> g = tiling({5000, 3000});
    const uint64_t n = 8000;
    float* f = static_cast<float*>(fake(0x10000));
    void* plan = fake(0x20000);
    void* scratch = fake(0x30000);
    uint32_t* words = static_cast<uint32_t*>(fake(0x40000));
    vgc_group_hdr* hdrs = static_cast<vgc_group_hdr*>(fake(0x50000));
    vgc_pack_status* st = static_cast<vgc_pack_status*>(fake(0x60000));
    // (a)
    CHECK(vgc_sqgrad(7, VGC_F32, f, f, 4, 1, 8, 8, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_DTYPE);
    CHECK(vgc_sqgrad(VGC_FC, 7, f, f, 4, 1, 8, 8, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_DTYPE);
    CHECK(vgc_sqgrad(VGC_FC, VGC_F32, nullptr, f, 4, 1, 8, 8, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_sqgrad(VGC_FC, VGC_F32, f, f, 4, 2, 8, 8, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_sqgrad(VGC_CONV, VGC_F32, f, f, 4, 0, 8, 8, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_sqgrad(VGC_FC, VGC_F32, fake(0x10004), f, 4, 1, 8, 8, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_ALIGN);
    CHECK(vgc_sqgrad(VGC_FC, VGC_F32, f, f, 4, 1, 8, 8, 1.f / 0.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_PARAM);
    CHECK(vgc_sqgrad(VGC_FC, VGC_F32, f, f, 4, 1, 8, 8, 1.f, nullptr, f, fake(0x70004), 64, nullptr) == VGC_ERR_ALIGN);
    CHECK(vgc_sqgrad_noalloc(VGC_CONV, VGC_F32, f, f, 8, 49, 9216, 1024, 1.f, nullptr, f, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_sqgrad_noalloc(VGC_CONV, 3, f, f, 8, 49, 64, 64, 1.f, nullptr, f, nullptr) == VGC_ERR_DTYPE);
    for (uint32_t B : {1u, 7u, 32u, 64u})
        for (uint32_t P : {1u, 49u, 3136u})
            for (uint32_t J : {27u, 576u, 4608u})
                for (uint32_t C : {16u, 64u, 512u}) {
                    (void)vgc_sqgrad_workspace_bytes(VGC_CONV, VGC_F32, B, P, J, C);
                    (void)vgc_sqgrad_workspace_bytes(VGC_CONV, VGC_BF16, B, P, J, C);
                    CHECK(vgc_sqgrad_workspace_bytes(VGC_FC, VGC_BF16, B, 1, J, C) == 0);
                }
    CHECK(vgc_sqgrad_conv2d(VGC_BF16, f, f, 2, 8, 8, 4, 8, 3, 3, 1, 1, 1, 1, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_sqgrad_conv2d(VGC_BF16, f, f, 2, 8, 8, 8, 8, 3, 3, 1, 1, 3, 1, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_sqgrad_conv2d(VGC_BF16, f, f, 2, 8, 8, 8, 8, 3, 3, 0, 1, 1, 1, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_sqgrad_conv2d(9, f, f, 2, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_DTYPE);
    CHECK(vgc_sqgrad_conv2d(VGC_F32, nullptr, f, 2, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_sqgrad_conv2d_workspace_bytes(VGC_F32, 2, 8, 8, 6, 8, 7, 7, 1, 1, 3, 3) == 0);       // 6 channels under 7 x 7: not a first layer's shape
    CHECK(vgc_sqgrad_conv2d_workspace_bytes(VGC_F32, 2, 8, 8, 6, 8, 3, 3, 1, 1, 1, 1) == 2u * 54 * 8 * 4);   // the first-layer kernel: one part per sample
    CHECK(vgc_sqgrad_conv2d(VGC_BF16, f, f, 2, 8, 8, 4, 8, 7, 7, 1, 1, 3, 3, 1.f, nullptr, f, nullptr, 0, nullptr) == VGC_ERR_SIZE);
    (void)vgc_sqgrad_conv2d_workspace_bytes(VGC_BF16, 64, 224, 224, 64, 64, 3, 3, 1, 1, 1, 1);
    // (b)
    CHECK(vgc_accumulate_select(nullptr, f, f, f, n, g.data(), 2, plan, 1.f, 0.999f, scratch, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_accumulate_select(f, f, f, f, n + 1, g.data(), 2, plan, 1.f, 0.999f, scratch, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_accumulate_select(f, f, f, f, n, g.data(), 2, fake(0x20010), 1.f, 0.999f, scratch, nullptr) == VGC_ERR_ALIGN);
    CHECK(vgc_accumulate_select(f, f, static_cast<float*>(fake(0x10002)), f, n, g.data(), 2, plan, 1.f, 0.999f, scratch, nullptr) == VGC_ERR_ALIGN);
    CHECK(vgc_accumulate_select(f, f, f, f, n, g.data(), 2, plan, -1.f, 0.999f, scratch, nullptr) == VGC_ERR_PARAM);
    CHECK(vgc_accumulate_select(f, f, f, f, n, g.data(), 2, plan, 1.f, 0.f, scratch, nullptr) == VGC_ERR_PARAM);
    CHECK(vgc_accumulate_select(f, f, f, f, n, g.data(), 2, plan, 1.f, 1.5f, scratch, nullptr) == VGC_ERR_PARAM);
    CHECK(vgc_accumulate_select_hybrid(f, f, f, f, n, g.data(), 2, plan, 1.f, 0.999f, -0.5f, scratch, nullptr) == VGC_ERR_PARAM);
    // (c)
    CHECK(vgc_pack(n, g.data(), 2, plan, scratch, words, 100, nullptr, st, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_pack(n, g.data(), 2, plan, scratch, nullptr, 100, hdrs, st, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_pack(n, g.data(), 1, plan, scratch, words, 100, hdrs, st, nullptr) == VGC_ERR_SIZE);
    CHECK(vgc_pack(n, g.data(), 2, plan, scratch, words, 100, static_cast<vgc_group_hdr*>(fake(0x50004)), st, nullptr) == VGC_ERR_ALIGN);
    CHECK(vgc_pack_compact(n, g.data(), 2, plan, scratch, nullptr, 100, static_cast<uint16_t*>(fake(0x70000)), static_cast<uint64_t*>(fake(0x80000)), hdrs, st, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_pack_compact(n, g.data(), 2, plan, scratch, static_cast<uint8_t*>(fake(0x90001)), 100, static_cast<uint16_t*>(fake(0x70001)), static_cast<uint64_t*>(fake(0x80000)), hdrs, st, nullptr) == VGC_ERR_ALIGN);
    // (d)
    CHECK(vgc_unpack_add(words, 10, nullptr, g.data(), 2, plan, 1.f, f, n, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_unpack_add(words, 10, hdrs, g.data(), 2, plan, 0.f / 0.f, f, n, nullptr) == VGC_ERR_PARAM);
    CHECK(vgc_unpack_add(words, 10, hdrs, g.data(), 2, plan, 1.f, f, n - 1, nullptr) == VGC_ERR_SIZE);
    const uint32_t* wl[2] = {words, nullptr};
    const vgc_group_hdr* hl[2] = {hdrs, hdrs};
    const uint64_t nl[2] = {10, 10};
    CHECK(vgc_unpack_add_batch(wl, nl, hl, 2, g.data(), 2, plan, 1.f, 0, f, n, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_unpack_add_batch(nullptr, nullptr, nullptr, 0, g.data(), 2, plan, 1.f, 0, f, n, nullptr) == VGC_OK);   // nothing to do
    vgc_optimizer opt;
    std::memset(&opt, 0, sizeof(opt));
    opt.kind = VGC_OPT_MOMENTUM_SGD; opt.lr = 0.1f; opt.momentum = 1.0f;
    CHECK(vgc_unpack_apply(nullptr, nullptr, nullptr, 0, g.data(), 2, plan, 1.f, &opt, f, f, nullptr, n, nullptr) == VGC_ERR_PARAM);
    opt.kind = VGC_OPT_ADAM; opt.beta1 = 0.9f; opt.beta2 = 0.999f; opt.eps = 1e-8f; opt.step = 1;
    CHECK(vgc_unpack_apply(nullptr, nullptr, nullptr, 0, g.data(), 2, plan, 1.f, &opt, f, f, nullptr, n, nullptr) == VGC_ERR_NULL);
    opt.step = 0;
    CHECK(vgc_unpack_apply(nullptr, nullptr, nullptr, 0, g.data(), 2, plan, 1.f, &opt, f, f, f, n, nullptr) == VGC_ERR_PARAM);
    opt.step = 1;
    CHECK(vgc_unpack_apply(nullptr, nullptr, nullptr, VGC_MAX_UPDATE_MESSAGES + 1, g.data(), 2, plan, 1.f, &opt, f, f, f, n, nullptr) == VGC_ERR_NULL);
    CHECK(vgc_unpack_apply(wl, nl, hl, VGC_MAX_UPDATE_MESSAGES + 1, g.data(), 2, plan, 1.f, &opt, f, f, f, n, nullptr) == VGC_ERR_SIZE);
}

int main() {
    const uint32_t T = vgc_tile_size();
    check_plan({1});
    check_plan({T});
    check_plan({T + 1});
    check_plan({1000, 1, 37, 5000, 64, T, 2 * T + 3, 3, 3 * T, 10});
    check_plan({64 * T, 64 * T + 1, 63 * T});                       // run boundaries
    check_plan({8192 * T, 5, 8192 * T + 1, 1u << 28, 700});         // segment boundaries, the largest group
    std::vector<uint32_t> many(5000);
    for (size_t k = 0; k < many.size(); ++k) many[k] = (uint32_t)(1 + (k * 2654435761u) % 9000);
    check_plan(many);
    check_group_errors();
    check_compute_errors();
    if (g_failed) { std::fprintf(stderr, "hostcheck: %d check(s) failed\n", g_failed); return 1; }
    std::printf("hostcheck ok\n");
    return 0;
}
