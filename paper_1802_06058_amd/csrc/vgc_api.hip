// C-ABI entry points of libvgc: argument checking, plan construction, kernel dispatch.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "vgc_internal.h"

namespace vgc {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_check(hipError_t e, const char* what) {
    if (e == hipSuccess) return VGC_OK;
    set_error("%s: %s", what, hipGetErrorString(e));
    return VGC_ERR_HIP;
}

// Validates the group list and counts tiles.  Returns a vgc_status.
struct GroupStats { uint64_t n_runs; uint32_t n_segs; bool multi_seg; uint64_t hash; };

static int check_groups(const vgc_group* groups, uint32_t n_groups, uint64_t n, uint64_t* n_tiles_out,
                        GroupStats* stats_out = nullptr) {
    if (!groups) { set_error("groups is NULL"); return VGC_ERR_NULL; }
    if (n == 0 || n_groups == 0) { set_error("n and n_groups must be positive"); return VGC_ERR_SIZE; }
    uint64_t off = 0, tiles = 0, runs = 0, segs = 0;
    uint64_t hash = 0xCBF29CE484222325ull ^ n_groups;       // FNV-1a over the sizes (offsets follow from them)
    bool multi = false;
    for (uint32_t k = 0; k < n_groups; ++k) {
        hash = (hash ^ groups[k].size) * 0x100000001B3ull;
        if (groups[k].size == 0) { set_error("group %u is empty", k); return VGC_ERR_SIZE; }
        if (groups[k].size > VGC_MAX_GROUP_SIZE) {
            set_error("group %u has %u elements; a 28-bit index holds at most 2^28", k, groups[k].size);
            return VGC_ERR_GROUP_TOO_LARGE;
        }
        if (groups[k].offset != off || groups[k].reserved != 0) {
            set_error("group %u starts at %llu, expected %llu: groups must tile [0, n) in order", k,
                      (unsigned long long)groups[k].offset, (unsigned long long)off);
            return VGC_ERR_SIZE;
        }
        off += groups[k].size;
        const uint64_t nt = (groups[k].size + kTile - 1) / kTile;
        tiles += nt;
        runs += (nt + kRunTiles - 1) / kRunTiles;
        segs += (nt + kSegTiles - 1) / kSegTiles;
        multi = multi || nt > kSegTiles;
    }
    if (off != n) {
        set_error("groups cover %llu elements, n = %llu", (unsigned long long)off, (unsigned long long)n);
        return VGC_ERR_SIZE;
    }
    if (tiles > 0x7FFFFFFFull) { set_error("too many tiles (%llu)", (unsigned long long)tiles); return VGC_ERR_SIZE; }
    if (n_tiles_out) *n_tiles_out = tiles;
    if (stats_out) { stats_out->n_runs = runs; stats_out->n_segs = (uint32_t)segs; stats_out->multi_seg = multi; stats_out->hash = hash; }
    return VGC_OK;
}

// The run and segment tables sit after the tile table; their sizes are bounded through the tile and
// group counts, so the layout reserves the bound and the offsets depend on (n_tiles, n_groups) only.
static size_t plan_bytes_for(uint64_t n_tiles, uint32_t n_groups, size_t* groups_off, size_t* tiles_off,
                             size_t* runs_off = nullptr, size_t* segs_off = nullptr) {
    size_t off = sizeof(PlanHeader);
    if (groups_off) *groups_off = off;
    off = align_up(off + (size_t)n_groups * sizeof(PlanGroup), 256);
    if (tiles_off) *tiles_off = off;
    off = align_up(off + n_tiles * sizeof(PlanTile), 256);
    if (runs_off) *runs_off = off;
    off = align_up(off + (n_tiles / kRunTiles + n_groups) * sizeof(PlanRun), 256);
    if (segs_off) *segs_off = off;
    off = align_up(off + (n_tiles / kSegTiles + n_groups) * sizeof(PlanSeg), 256);
    return off;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

struct PlanView { const PlanGroup* groups; const PlanTile* tiles; const PlanRun* runs; const PlanSeg* segs; };

static PlanCheck plan_check(const void* plan_dev, const GroupStats& gs) {
    return PlanCheck{static_cast<const PlanHeader*>(plan_dev), gs.hash};
}

static PlanView plan_view(const void* plan_dev, uint64_t n_tiles, uint32_t n_groups) {
    size_t go, to, ro, so;
    plan_bytes_for(n_tiles, n_groups, &go, &to, &ro, &so);
    const char* b = static_cast<const char*>(plan_dev);
    return PlanView{reinterpret_cast<const PlanGroup*>(b + go), reinterpret_cast<const PlanTile*>(b + to),
                    reinterpret_cast<const PlanRun*>(b + ro), reinterpret_cast<const PlanSeg*>(b + so)};
}

// Working memory of vgc_sqgrad_noalloc: one copy per GPU the library's code object is loaded on, held until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels and copies get
// the device address that call returns.
static __device__ __align__(256) unsigned char scratch[VGC_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once looked up
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current GPU (looked up on the first call on that GPU).
static int static_scratch(void** out) {
    int dev = -1;
    int rc = hip_check(hipGetDevice(&dev), "hipGetDevice");
    if (rc != VGC_OK) return rc;
    if (dev < 0 || dev >= kMaxDevices) { set_error("vgc_sqgrad_noalloc: device ordinal %d out of range", dev); return VGC_ERR_HIP; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        rc = hip_check(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc != VGC_OK) return rc;
        if (!p) { set_error("vgc_sqgrad_noalloc: no device address for the static scratch"); return VGC_ERR_HIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return VGC_OK;
}

}  // namespace vgc

using namespace vgc;

extern "C" {

const char* vgc_last_error(void) { return g_err; }

uint32_t vgc_tile_size(void) { return kTile; }

uint64_t vgc_tile_count(const vgc_group* groups, uint32_t n_groups, uint64_t n) {
    uint64_t t = 0;
    return check_groups(groups, n_groups, n, &t) == VGC_OK ? t : 0;
}

size_t vgc_plan_bytes(const vgc_group* groups, uint32_t n_groups, uint64_t n) {
    uint64_t t = 0;
    if (check_groups(groups, n_groups, n, &t) != VGC_OK) return 0;
    return plan_bytes_for(t, n_groups, nullptr, nullptr);
}

size_t vgc_scratch_bytes(const vgc_group* groups, uint32_t n_groups, uint64_t n) {
    uint64_t t = 0;
    if (check_groups(groups, n_groups, n, &t) != VGC_OK) return 0;
    return scratch_layout(t, n_groups).total;
}

size_t vgc_scratch_bitmap_offset(const vgc_group* groups, uint32_t n_groups, uint64_t n) {
    uint64_t t = 0;
    if (check_groups(groups, n_groups, n, &t) != VGC_OK) return 0;
    return scratch_layout(t, n_groups).bitmap_off;
}

int vgc_plan_build(const vgc_group* groups, uint32_t n_groups, uint64_t n, void* plan_host, size_t plan_bytes) {
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    if (!plan_host) { set_error("plan_host is NULL"); return VGC_ERR_NULL; }
    size_t go, to, ro, so;
    const size_t need = plan_bytes_for(n_tiles, n_groups, &go, &to, &ro, &so);
    if (plan_bytes < need) { set_error("plan buffer has %zu bytes, %zu needed", plan_bytes, need); return VGC_ERR_SIZE; }
    char* b = static_cast<char*>(plan_host);
    memset(b, 0, need);
    PlanHeader* h = reinterpret_cast<PlanHeader*>(b);
    h->magic = kPlanMagic; h->n = n; h->n_tiles = n_tiles; h->n_groups = n_groups; h->tile = kTile;
    h->groups_off = go; h->tiles_off = to; h->runs_off = ro; h->n_runs = gs.n_runs;
    h->segs_off = so; h->n_segs = gs.n_segs; h->groups_hash = gs.hash;
    PlanGroup* G = reinterpret_cast<PlanGroup*>(b + go);
    PlanTile* T = reinterpret_cast<PlanTile*>(b + to);
    PlanRun* R = reinterpret_cast<PlanRun*>(b + ro);
    PlanSeg* S = reinterpret_cast<PlanSeg*>(b + so);
    uint64_t t = 0, rn = 0;
    uint32_t sn = 0;
    for (uint32_t k = 0; k < n_groups; ++k) {
        G[k].offset = groups[k].offset; G[k].size = groups[k].size; G[k].first_tile = (uint32_t)t;
        const uint32_t group_first_seg = sn;
        uint32_t in_group = 0;
        for (uint64_t start = 0; start < groups[k].size; start += kTile, ++t, ++in_group) {
            if (in_group % kSegTiles == 0) {
                S[sn].group = k; S[sn].first_tile = in_group; S[sn].seg_in_group = sn - group_first_seg;
                S[sn].group_first_seg = group_first_seg;
                ++sn;
            }
            if (in_group % kRunTiles == 0) { R[rn].group = k; R[rn].first_tile = in_group; ++rn; }
            T[t].group = k; T[t].start = (uint32_t)start; T[t].seg = sn - 1; T[t].run = (uint32_t)(rn - 1);
        }
    }
    return VGC_OK;
}

size_t vgc_sqgrad_workspace_bytes(int kind, int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    return sqgrad_workspace_bytes(kind, dtype, B, P, J, C);
}

int vgc_sqgrad(int kind, int dtype, const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C,
               float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (kind != VGC_FC && kind != VGC_CONV) { set_error("vgc_sqgrad: unknown kind %d", kind); return VGC_ERR_DTYPE; }
    if (dtype != VGC_F32 && dtype != VGC_BF16) { set_error("vgc_sqgrad: unknown dtype %d", dtype); return VGC_ERR_DTYPE; }
    if (!X || !D || !s_out) { set_error("vgc_sqgrad: X, D and s_out are required"); return VGC_ERR_NULL; }
    if (B == 0 || P == 0 || J == 0 || C == 0) { set_error("vgc_sqgrad: zero dimension"); return VGC_ERR_SIZE; }
    if (kind == VGC_FC && P != 1) { set_error("vgc_sqgrad: the FC form has P = 1"); return VGC_ERR_SIZE; }
    if (!aligned(X, 16) || !aligned(D, 16) || !aligned(s_out, 16) || (g_out && !aligned(g_out, 16))) {
        set_error("vgc_sqgrad: pointers must be 16-byte aligned");
        return VGC_ERR_ALIGN;
    }
    if (!std::isfinite(c)) { set_error("vgc_sqgrad: c is not finite"); return VGC_ERR_PARAM; }
    if (workspace && !aligned(workspace, 16)) { set_error("vgc_sqgrad: workspace must be 16-byte aligned"); return VGC_ERR_ALIGN; }
    return launch_sqgrad(kind, dtype, X, D, B, P, J, C, c, g_out, s_out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream));
}

int vgc_sqgrad_noalloc(int kind, int dtype, const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                       float c, float* g_out, float* s_out, void* stream) {
    if (kind != VGC_FC && kind != VGC_CONV) { set_error("vgc_sqgrad_noalloc: unknown kind %d", kind); return VGC_ERR_DTYPE; }
    if (dtype != VGC_F32 && dtype != VGC_BF16) { set_error("vgc_sqgrad_noalloc: unknown dtype %d", dtype); return VGC_ERR_DTYPE; }
    if (B == 0 || P == 0 || J == 0 || C == 0) { set_error("vgc_sqgrad_noalloc: zero dimension"); return VGC_ERR_SIZE; }
    const size_t need = sqgrad_workspace_bytes(kind, dtype, B, P, J, C);
    if (need > (size_t)VGC_NOALLOC_SCRATCH_BYTES) {
        set_error("vgc_sqgrad_noalloc: this shape wants %zu bytes of working memory, the static buffer has %zu; "
                  "call vgc_sqgrad with a workspace of the caller's", need, (size_t)VGC_NOALLOC_SCRATCH_BYTES);
        return VGC_ERR_SIZE;
    }
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != VGC_OK) return rc;
    return vgc_sqgrad(kind, dtype, X, D, B, P, J, C, c, g_out, s_out, ws, (size_t)VGC_NOALLOC_SCRATCH_BYTES, stream);
}

// Validates a convolution's geometry; on success the output extent.
static int conv2d_geometry(int dtype, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C, uint32_t kh, uint32_t kw,
                           uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw, uint32_t* Ho, uint32_t* Wo) {
    if (dtype != VGC_F32 && dtype != VGC_BF16) { set_error("vgc_sqgrad_conv2d: unknown dtype %d", dtype); return VGC_ERR_DTYPE; }
    if (B == 0 || H == 0 || W == 0 || Cin == 0 || C == 0 || kh == 0 || kw == 0 || sh == 0 || sw == 0) {
        set_error("vgc_sqgrad_conv2d: zero dimension");
        return VGC_ERR_SIZE;
    }
    if (ph >= kh || pw >= kw || (uint64_t)H + 2 * ph < kh || (uint64_t)W + 2 * pw < kw) {
        set_error("vgc_sqgrad_conv2d: need pad < kernel <= input + 2 pad");
        return VGC_ERR_SIZE;
    }
    if ((uint64_t)kh * kw * Cin > 0x7FFFFFFFull || (uint64_t)H * W > 0x7FFFFFFFull) { set_error("vgc_sqgrad_conv2d: shape too large"); return VGC_ERR_SIZE; }
    *Ho = (H + 2 * ph - kh) / sh + 1;
    *Wo = (W + 2 * pw - kw) / sw + 1;
    if (conv_stem_supported(dtype, Cin, C, kh, kw)) return VGC_OK;        // a first layer: few input channels, small kh kw Cin
    if (!conv2d_supported(dtype, H, W, Cin, C, *Ho * *Wo)) {
        set_error("vgc_sqgrad_conv2d: needs C a multiple of 16 bytes, Cin a multiple of 16 bytes or kh kw Cin <= 160, and "
                  "per-sample tensors below 2 GiB");
        return VGC_ERR_SIZE;
    }
    return VGC_OK;
}

size_t vgc_sqgrad_conv2d_workspace_bytes(int dtype, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C,
                                         uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw) {
    uint32_t Ho, Wo;
    if (conv2d_geometry(dtype, B, H, W, Cin, C, kh, kw, sh, sw, ph, pw, &Ho, &Wo) != VGC_OK) return 0;
    const uint32_t J = kh * kw * Cin;
    if (conv_stem_supported(dtype, Cin, C, kh, kw)) return conv_stem_workspace_bytes(dtype, B, Ho * Wo, J, C);
    if (dtype == VGC_BF16) {
        // the larger of what the two kernels that may serve the layer want (which one runs depends on whether g is asked for)
        size_t need = conv_workspace_bytes(B, Ho * Wo, J, C);
        if (conv_taps_supported(H, W, Cin, C, kh, kw, sh, sw, ph, pw)) {
            const size_t t = conv_taps_workspace_bytes(B, Ho * Wo, Cin, C);
            if (t > need) need = t;
        }
        return need;
    }
    return conv_f32_workspace_bytes(B, Ho * Wo, J, C);
}

// Argument checks of vgc_sqgrad_conv2d; the output size on success.
static int conv2d_check(int dtype, const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin,
                        uint32_t C, uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw,
                        float c, const float* g_out, const float* s_out, const void* workspace, size_t workspace_bytes,
                        uint32_t* Ho, uint32_t* Wo) {
    if (!act || !D || !s_out) { set_error("vgc_sqgrad_conv2d: act, D and s_out are required"); return VGC_ERR_NULL; }
    int rc = conv2d_geometry(dtype, B, H, W, Cin, C, kh, kw, sh, sw, ph, pw, Ho, Wo);
    if (rc != VGC_OK) return rc;
    if (!aligned(act, 16) || !aligned(D, 16) || !aligned(s_out, 16) || (g_out && !aligned(g_out, 16)) ||
        (workspace && !aligned(workspace, 16))) {
        set_error("vgc_sqgrad_conv2d: pointers must be 16-byte aligned");
        return VGC_ERR_ALIGN;
    }
    if (!std::isfinite(c)) { set_error("vgc_sqgrad_conv2d: c is not finite"); return VGC_ERR_PARAM; }
    if (conv_stem_supported(dtype, Cin, C, kh, kw) &&
        (!workspace || workspace_bytes < conv_stem_workspace_bytes(dtype, B, *Ho * *Wo, kh * kw * Cin, C))) {
        set_error("vgc_sqgrad_conv2d: a layer whose input channels are not a multiple of 16 bytes needs the workspace "
                  "vgc_sqgrad_conv2d_workspace_bytes() asks for");
        return VGC_ERR_SIZE;
    }
    return VGC_OK;
}

int vgc_sqgrad_conv2d(int dtype, const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin,
                      uint32_t C, uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw,
                      float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, void* stream) {
    uint32_t Ho, Wo;
    const int rc = conv2d_check(dtype, act, D, B, H, W, Cin, C, kh, kw, sh, sw, ph, pw, c, g_out, s_out, workspace, workspace_bytes, &Ho, &Wo);
    if (rc != VGC_OK) return rc;
    return launch_conv2d(dtype, act, D, B, H, W, Cin, C, kh, kw, sh, sw, ph, pw, Ho, Wo, c, g_out, s_out, workspace, workspace_bytes,
                         static_cast<hipStream_t>(stream));
}

// The library's own streams for vgc_sqgrad_conv2d_batch: one set per device, made on first use (default priority).
namespace {
constexpr int kSideStreams = 4;
struct SideStreams {
    bool ready = false;
    hipStream_t s[kSideStreams];
    hipEvent_t fork, join[kSideStreams];
};
std::mutex g_side_mutex;                                  // one batch call submits at a time per process
SideStreams g_side[64];
}  // namespace

int vgc_sqgrad_conv2d_batch(const vgc_conv2d_layer* layers, uint32_t n_layers, void* stream) {
    if (!layers && n_layers) { set_error("vgc_sqgrad_conv2d_batch: layers is NULL"); return VGC_ERR_NULL; }
    std::vector<uint32_t> Ho(n_layers), Wo(n_layers);
    for (uint32_t k = 0; k < n_layers; ++k) {             // every layer is checked before anything is launched
        const vgc_conv2d_layer& L = layers[k];
        const int rc = conv2d_check(L.dtype, L.act, L.D, L.B, L.H, L.W, L.Cin, L.C, L.kh, L.kw, L.stride_h, L.stride_w, L.pad_h,
                                    L.pad_w, L.c, L.g_out, L.s_out, L.workspace, L.workspace_bytes, &Ho[k], &Wo[k]);
        if (rc != VGC_OK) return rc;
    }
    hipStream_t user = static_cast<hipStream_t>(stream);
    int dev = 0;
    int rc = hip_check(hipGetDevice(&dev), "hipGetDevice");
    if (rc != VGC_OK) return rc;
    if (dev < 0 || dev >= 64) { set_error("vgc_sqgrad_conv2d_batch: device %d out of range", dev); return VGC_ERR_PARAM; }
    std::lock_guard<std::mutex> lock(g_side_mutex);
    SideStreams& S = g_side[dev];
    if (!S.ready) {
        for (int i = 0; i < kSideStreams; ++i) {
            if ((rc = hip_check(hipStreamCreateWithFlags(&S.s[i], hipStreamNonBlocking), "hipStreamCreate")) != VGC_OK) return rc;
            if ((rc = hip_check(hipEventCreateWithFlags(&S.join[i], hipEventDisableTiming), "hipEventCreate")) != VGC_OK) return rc;
        }
        if ((rc = hip_check(hipEventCreateWithFlags(&S.fork, hipEventDisableTiming), "hipEventCreate")) != VGC_OK) return rc;
        S.ready = true;
    }
    // Which stream takes which layer.  A layer of 2e10 multiply-adds or more fills the chip by itself (measured:
    // overlapping such layers costs time); it stays on the caller's stream.  Of the others each goes to the least
    // loaded side stream.
    std::vector<int> lane_of(n_layers, 0);
    double load[kSideStreams + 1] = {0.0};               // multiply-adds queued on each stream so far
    bool lane_used[kSideStreams + 1] = {false};
    uint32_t n_small = 0;
    for (uint32_t k = 0; k < n_layers; ++k) {
        const vgc_conv2d_layer& L = layers[k];
        const double macs = (double)L.B * Ho[k] * Wo[k] * L.kh * L.kw * L.Cin * L.C;
        if (macs < 2e10) ++n_small;
    }
    for (uint32_t k = 0; k < n_layers; ++k) {
        const vgc_conv2d_layer& L = layers[k];
        const double macs = (double)L.B * Ho[k] * Wo[k] * L.kh * L.kw * L.Cin * L.C;
        int lane = 0;
        if (n_small > 1 && macs < 2e10) {
            lane = 1;
            for (int i = 2; i <= kSideStreams; ++i)
                if (load[i] < load[lane]) lane = i;
        }
        load[lane] += macs + 2e8;                        // (+ a launch's worth)
        lane_of[k] = lane;
        lane_used[lane] = true;
    }
    // fork: the side streams that get work start after whatever the caller's stream holds so far
    bool forked = false;
    for (int i = 1; i <= kSideStreams; ++i) {
        if (!lane_used[i]) continue;
        if (!forked && (rc = hip_check(hipEventRecord(S.fork, user), "hipEventRecord")) != VGC_OK) return rc;
        forked = true;
        if ((rc = hip_check(hipStreamWaitEvent(S.s[i - 1], S.fork, 0), "hipStreamWaitEvent")) != VGC_OK) return rc;
    }
    int first_error = VGC_OK;
    for (uint32_t k = 0; k < n_layers; ++k) {
        const vgc_conv2d_layer& L = layers[k];
        hipStream_t st = lane_of[k] == 0 ? user : S.s[lane_of[k] - 1];
        const int r = launch_conv2d(L.dtype, L.act, L.D, L.B, L.H, L.W, L.Cin, L.C, L.kh, L.kw, L.stride_h, L.stride_w, L.pad_h,
                                    L.pad_w, Ho[k], Wo[k], L.c, L.g_out, L.s_out, L.workspace, L.workspace_bytes, st);
        if (r != VGC_OK && first_error == VGC_OK) first_error = r;
    }
    // join: the caller's stream continues when every side stream is done (also after a failed launch)
    for (int i = 1; i <= kSideStreams; ++i) {
        if (!lane_used[i]) continue;
        if ((rc = hip_check(hipEventRecord(S.join[i - 1], S.s[i - 1]), "hipEventRecord")) != VGC_OK) return rc;
        if ((rc = hip_check(hipStreamWaitEvent(user, S.join[i - 1], 0), "hipStreamWaitEvent")) != VGC_OK) return rc;
    }
    return first_error;
}

// first_group, group_count: the groups the launch covers (all of them for the whole-model calls)
static int accumulate_select_any(const float* g, const float* s, float* r, float* v, uint64_t n,
                                 const vgc_group* groups, uint32_t n_groups, const void* plan,
                                 uint32_t first_group, uint32_t group_count,
                                 float alpha, float zeta, float tau, bool hybrid, void* scratch, void* stream) {
    if (!g || !s || !r || !v || !plan || !scratch) { set_error("vgc_accumulate_select: NULL pointer"); return VGC_ERR_NULL; }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    if (first_group > n_groups || group_count > n_groups - first_group) {
        set_error("vgc_accumulate_select_range: groups %u .. %u + %u are not inside the list of %u", first_group, first_group, group_count, n_groups);
        return VGC_ERR_SIZE;
    }
    if (!aligned(g, 4) || !aligned(s, 4) || !aligned(r, 4) || !aligned(v, 4) || !aligned(plan, 256) || !aligned(scratch, 256)) {
        set_error("vgc_accumulate_select: g, s, r, v need 4-byte, plan and scratch 256-byte alignment");
        return VGC_ERR_ALIGN;
    }
    if (!(alpha >= 0.0f) || !std::isfinite(alpha) || !(zeta > 0.0f) || !(zeta <= 1.0f)) {
        set_error("vgc_accumulate_select: need alpha >= 0 finite and 0 < zeta <= 1 (got %g, %g)", alpha, zeta);
        return VGC_ERR_PARAM;
    }
    if (hybrid && (!(tau >= 0.0f) || !std::isfinite(tau))) {
        set_error("vgc_accumulate_select_hybrid: need tau >= 0 finite (got %g)", tau);
        return VGC_ERR_PARAM;
    }
    uint64_t tile0 = 0, tiles = 0;
    for (uint32_t k = 0; k < first_group + group_count; ++k) {
        const uint64_t nt = (groups[k].size + kTile - 1) / kTile;
        if (k < first_group) tile0 += nt; else tiles += nt;
    }
    const ScratchLayout L = scratch_layout(n_tiles, n_groups);
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    char* sc = static_cast<char*>(scratch);
    const bool vec = aligned(g, 16) && aligned(s, 16) && aligned(r, 16) && aligned(v, 16);
    return launch_accumulate_select(plan_check(plan, gs), reinterpret_cast<uint32_t*>(sc + L.flags_off), g, s, r, v, pv.groups, pv.tiles,
                                    tile0, tiles,
                                    reinterpret_cast<TileHdr*>(sc + L.tile_hdr_off),
                                    reinterpret_cast<uint32_t*>(sc + L.bitmap_off),
                                    reinterpret_cast<uint16_t*>(sc + L.staging_off),
                                    alpha, zeta, tau, hybrid, vec, static_cast<hipStream_t>(stream));
}

int vgc_accumulate_select(const float* g, const float* s, float* r, float* v, uint64_t n,
                          const vgc_group* groups, uint32_t n_groups, const void* plan,
                          float alpha, float zeta, void* scratch, void* stream) {
    return accumulate_select_any(g, s, r, v, n, groups, n_groups, plan, 0, n_groups, alpha, zeta, 0.0f, false, scratch, stream);
}

int vgc_accumulate_select_hybrid(const float* g, const float* s, float* r, float* v, uint64_t n,
                                 const vgc_group* groups, uint32_t n_groups, const void* plan,
                                 float alpha, float zeta, float tau, void* scratch, void* stream) {
    return accumulate_select_any(g, s, r, v, n, groups, n_groups, plan, 0, n_groups, alpha, zeta, tau, true, scratch, stream);
}

int vgc_accumulate_select_range(const float* g, const float* s, float* r, float* v, uint64_t n,
                                const vgc_group* groups, uint32_t n_groups, const void* plan,
                                uint32_t first_group, uint32_t group_count,
                                float alpha, float zeta, void* scratch, void* stream) {
    return accumulate_select_any(g, s, r, v, n, groups, n_groups, plan, first_group, group_count, alpha, zeta, 0.0f, false, scratch, stream);
}

size_t vgc_sqgrad_accumulate_select_workspace_bytes(int dtype, uint32_t B, uint32_t J, uint32_t C) {
    if (dtype != VGC_F32 && dtype != VGC_BF16) return 0;
    return fused_fc_workspace_bytes(dtype, B, J, C);
}

int vgc_sqgrad_accumulate_select(int dtype, const void* X, const void* D, uint32_t B, uint32_t J, uint32_t C, float c,
                                 float* r, float* v, uint64_t n, const vgc_group* groups, uint32_t n_groups, const void* plan,
                                 uint32_t group, float alpha, float zeta, void* scratch, void* workspace, size_t workspace_bytes,
                                 float* g_out, float* s_out, void* stream) {
    if (dtype != VGC_F32 && dtype != VGC_BF16) { set_error("vgc_sqgrad_accumulate_select: unknown dtype %d", dtype); return VGC_ERR_DTYPE; }
    if (!X || !D || !r || !v || !plan || !scratch || !workspace) { set_error("vgc_sqgrad_accumulate_select: NULL pointer"); return VGC_ERR_NULL; }
    if ((g_out == nullptr) != (s_out == nullptr)) { set_error("vgc_sqgrad_accumulate_select: g_out and s_out go together"); return VGC_ERR_NULL; }
    if (B == 0 || J == 0 || C == 0) { set_error("vgc_sqgrad_accumulate_select: zero dimension"); return VGC_ERR_SIZE; }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    if (group >= n_groups || (uint64_t)J * C != groups[group].size) {
        set_error("vgc_sqgrad_accumulate_select: group %u does not exist or does not have J x C = %llu elements", group,
                  (unsigned long long)J * C);
        return VGC_ERR_SIZE;
    }
    const size_t need = fused_fc_workspace_bytes(dtype, B, J, C);
    if (need == 0) {
        set_error("vgc_sqgrad_accumulate_select: C = %u is neither a multiple of 2048 nor 256, 512 or 1024 "
                  "(use vgc_sqgrad and vgc_accumulate_select)", C);
        return VGC_ERR_SIZE;
    }
    if (workspace_bytes < need) { set_error("vgc_sqgrad_accumulate_select: workspace has %zu bytes, %zu needed", workspace_bytes, need); return VGC_ERR_SIZE; }
    const size_t es = dtype == VGC_BF16 ? 2 : 4;
    if (!aligned(X, es) || !aligned(D, es) || !aligned(r, 4) || !aligned(v, 4) || !aligned(plan, 256) || !aligned(scratch, 256) ||
        !aligned(workspace, 16) || !aligned(g_out, 4) || !aligned(s_out, 4)) {
        set_error("vgc_sqgrad_accumulate_select: misaligned pointer");
        return VGC_ERR_ALIGN;
    }
    if (!std::isfinite(c) || !(alpha >= 0.0f) || !std::isfinite(alpha) || !(zeta > 0.0f) || !(zeta <= 1.0f)) {
        set_error("vgc_sqgrad_accumulate_select: need c finite, alpha >= 0 finite and 0 < zeta <= 1");
        return VGC_ERR_PARAM;
    }
    const ScratchLayout L = scratch_layout(n_tiles, n_groups);
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    char* sc = static_cast<char*>(scratch);
    return launch_fused_fc_select(plan_check(plan, gs), reinterpret_cast<uint32_t*>(sc + L.flags_off), dtype, X, D, B, J, C, c, r, v,
                                  pv.groups, group, reinterpret_cast<TileHdr*>(sc + L.tile_hdr_off),
                                  reinterpret_cast<uint32_t*>(sc + L.bitmap_off), reinterpret_cast<uint16_t*>(sc + L.staging_off),
                                  alpha, zeta, workspace, g_out, s_out, static_cast<hipStream_t>(stream));
}

int vgc_pack(uint64_t n, const vgc_group* groups, uint32_t n_groups, const void* plan, void* scratch,
             uint32_t* words_out, uint64_t words_cap, vgc_group_hdr* hdrs_out,
             vgc_pack_status* status_out, void* stream) {
    if (!plan || !scratch || !hdrs_out || !status_out || (!words_out && words_cap)) {
        set_error("vgc_pack: NULL pointer");
        return VGC_ERR_NULL;
    }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    if (!aligned(plan, 256) || !aligned(scratch, 256) || !aligned(words_out, 4) || !aligned(hdrs_out, 8) || !aligned(status_out, 8)) {
        set_error("vgc_pack: misaligned pointer");
        return VGC_ERR_ALIGN;
    }
    const ScratchLayout L = scratch_layout(n_tiles, n_groups);
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    char* sc = static_cast<char*>(scratch);
    return launch_pack(plan_check(plan, gs), reinterpret_cast<const uint32_t*>(sc + L.flags_off), pv.groups, pv.tiles, pv.segs, n_tiles, n_groups, gs.n_segs, gs.multi_seg,
                       reinterpret_cast<TileHdr*>(sc + L.tile_hdr_off),
                       reinterpret_cast<SegTmp*>(sc + L.seg_tmp_off),
                       reinterpret_cast<const uint16_t*>(sc + L.staging_off),
                       words_out, words_cap, hdrs_out, status_out, static_cast<hipStream_t>(stream));
}

uint64_t vgc_run_count(const vgc_group* groups, uint32_t n_groups, uint64_t n) {
    uint64_t t = 0;
    GroupStats gs;
    return check_groups(groups, n_groups, n, &t, &gs) == VGC_OK ? gs.n_runs : 0;
}

int vgc_pack_compact(uint64_t n, const vgc_group* groups, uint32_t n_groups, const void* plan, void* scratch,
                     uint8_t* stream_out, uint64_t stream_cap, uint16_t* tile_bytes_out, uint64_t* run_offsets_out,
                     vgc_group_hdr* hdrs_out, vgc_pack_status* status_out, void* stream) {
    if (!plan || !scratch || !hdrs_out || !status_out || !tile_bytes_out || !run_offsets_out || (!stream_out && stream_cap)) {
        set_error("vgc_pack_compact: NULL pointer");
        return VGC_ERR_NULL;
    }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    if (!aligned(plan, 256) || !aligned(scratch, 256) || !aligned(tile_bytes_out, 2) || !aligned(run_offsets_out, 8) ||
        !aligned(hdrs_out, 8) || !aligned(status_out, 8)) {
        set_error("vgc_pack_compact: misaligned pointer");
        return VGC_ERR_ALIGN;
    }
    const ScratchLayout L = scratch_layout(n_tiles, n_groups);
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    char* sc = static_cast<char*>(scratch);
    const PlanCheck pc = plan_check(plan, gs);
    TileHdr* th = reinterpret_cast<TileHdr*>(sc + L.tile_hdr_off);
    rc = launch_pack_scans(pc, reinterpret_cast<const uint32_t*>(sc + L.flags_off), pv.groups, pv.segs, n_groups, gs.n_segs, gs.multi_seg, th,
                           reinterpret_cast<SegTmp*>(sc + L.seg_tmp_off), hdrs_out, status_out, ~0ull, static_cast<hipStream_t>(stream));
    if (rc != VGC_OK) return rc;
    return launch_pack_compact(pc, pv.groups, pv.tiles, pv.runs, n_tiles, gs.n_runs, n_groups, th,
                               reinterpret_cast<const uint16_t*>(sc + L.staging_off), stream_out, stream_cap, tile_bytes_out,
                               run_offsets_out, hdrs_out, status_out, static_cast<hipStream_t>(stream));
}

int vgc_unpack_compact_add_batch(const uint8_t* const* streams, const uint64_t* stream_bytes, const uint16_t* const* tile_bytes,
                                 const uint64_t* const* run_offsets, const vgc_group_hdr* const* hdrs, uint32_t p,
                                 const vgc_group* groups, uint32_t n_groups, const void* plan, float scale, int overwrite,
                                 float* dense_out, uint64_t n, void* stream) {
    if (!plan || !dense_out || (p && (!streams || !stream_bytes || !tile_bytes || !run_offsets || !hdrs))) {
        set_error("vgc_unpack_compact_add_batch: NULL pointer");
        return VGC_ERR_NULL;
    }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    for (uint32_t w = 0; w < p; ++w) {
        if (!hdrs[w] || !tile_bytes[w] || !run_offsets[w] || (!streams[w] && stream_bytes[w])) {
            set_error("vgc_unpack_compact_add_batch: message %u has a NULL pointer", w);
            return VGC_ERR_NULL;
        }
        if (!aligned(tile_bytes[w], 2) || !aligned(run_offsets[w], 8) || !aligned(hdrs[w], 8)) {
            set_error("vgc_unpack_compact_add_batch: message %u is misaligned", w);
            return VGC_ERR_ALIGN;
        }
    }
    if (!aligned(plan, 256) || !aligned(dense_out, 4)) { set_error("vgc_unpack_compact_add_batch: misaligned pointer"); return VGC_ERR_ALIGN; }
    if (!std::isfinite(scale)) { set_error("vgc_unpack_compact_add_batch: scale is not finite"); return VGC_ERR_PARAM; }
    if (p == 0 && !overwrite) return VGC_OK;
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    return launch_unpack_compact_batch(plan_check(plan, gs), streams, stream_bytes, tile_bytes, run_offsets, hdrs, p, pv.groups, pv.runs,
                                       gs.n_runs, scale, overwrite, dense_out, static_cast<hipStream_t>(stream));
}

int vgc_unpack_add(const uint32_t* words, uint64_t n_words, const vgc_group_hdr* hdrs,
                   const vgc_group* groups, uint32_t n_groups, const void* plan,
                   float scale, float* dense_out, uint64_t n, void* stream) {
    if (!hdrs || !plan || !dense_out || (!words && n_words)) { set_error("vgc_unpack_add: NULL pointer"); return VGC_ERR_NULL; }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    if (!aligned(plan, 256) || !aligned(words, 4) || !aligned(hdrs, 8) || !aligned(dense_out, 4)) {
        set_error("vgc_unpack_add: misaligned pointer");
        return VGC_ERR_ALIGN;
    }
    if (!std::isfinite(scale)) { set_error("vgc_unpack_add: scale is not finite"); return VGC_ERR_PARAM; }
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    // A message that touches most cache lines of the buffer anyway (an eighth of the elements or more, going by
    // n_words) is decoded tile by tile like a batch of one: the same additions, the buffer streamed once instead of
    // read and written line by line under 64 scattered lanes (1.2 to 2.7 times faster from a sixth to two thirds sent).
    if (n_words && n_words >= n / 8) {
        const uint32_t* const wl[1] = {words};
        const uint64_t nl[1] = {n_words};
        const vgc_group_hdr* const hl[1] = {hdrs};
        return launch_unpack_add_batch(plan_check(plan, gs), wl, nl, hl, 1, pv.groups, pv.runs, gs.n_runs, scale, 0, dense_out,
                                       static_cast<hipStream_t>(stream));
    }
    return launch_unpack_add(plan_check(plan, gs), words, n_words, hdrs, pv.groups, n_groups, scale, dense_out, static_cast<hipStream_t>(stream));
}

int vgc_unpack_add_batch(const uint32_t* const* words, const uint64_t* n_words, const vgc_group_hdr* const* hdrs,
                         uint32_t p, const vgc_group* groups, uint32_t n_groups, const void* plan,
                         float scale, int overwrite, float* dense_out, uint64_t n, void* stream) {
    if (!plan || !dense_out || (p && (!words || !n_words || !hdrs))) { set_error("vgc_unpack_add_batch: NULL pointer"); return VGC_ERR_NULL; }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    for (uint32_t w = 0; w < p; ++w) {
        if (!hdrs[w] || (!words[w] && n_words[w])) { set_error("vgc_unpack_add_batch: message %u has a NULL pointer", w); return VGC_ERR_NULL; }
        if (!aligned(words[w], 4) || !aligned(hdrs[w], 8)) { set_error("vgc_unpack_add_batch: message %u is misaligned", w); return VGC_ERR_ALIGN; }
    }
    if (!aligned(plan, 256) || !aligned(dense_out, 4)) { set_error("vgc_unpack_add_batch: misaligned pointer"); return VGC_ERR_ALIGN; }
    if (!std::isfinite(scale)) { set_error("vgc_unpack_add_batch: scale is not finite"); return VGC_ERR_PARAM; }
    if (p == 0 && !overwrite) return VGC_OK;
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    return launch_unpack_add_batch(plan_check(plan, gs), words, n_words, hdrs, p, pv.groups, pv.runs, gs.n_runs, scale, overwrite, dense_out,
                                   static_cast<hipStream_t>(stream));
}

int vgc_unpack_apply(const uint32_t* const* words, const uint64_t* n_words, const vgc_group_hdr* const* hdrs,
                     uint32_t p, const vgc_group* groups, uint32_t n_groups, const void* plan, float scale,
                     const vgc_optimizer* opt, float* param, float* state1, float* state2, uint64_t n, void* stream) {
    if (!plan || !opt || !param || !state1 || (p && (!words || !n_words || !hdrs))) { set_error("vgc_unpack_apply: NULL pointer"); return VGC_ERR_NULL; }
    if (opt->kind != VGC_OPT_MOMENTUM_SGD && opt->kind != VGC_OPT_ADAM) { set_error("vgc_unpack_apply: unknown optimizer %d", opt->kind); return VGC_ERR_PARAM; }
    if (opt->kind == VGC_OPT_ADAM && !state2) { set_error("vgc_unpack_apply: Adam needs state2"); return VGC_ERR_NULL; }
    if (p > VGC_MAX_UPDATE_MESSAGES) { set_error("vgc_unpack_apply: %u messages, at most %d", p, VGC_MAX_UPDATE_MESSAGES); return VGC_ERR_SIZE; }
    uint64_t n_tiles = 0;
    GroupStats gs;
    int rc = check_groups(groups, n_groups, n, &n_tiles, &gs);
    if (rc != VGC_OK) return rc;
    for (uint32_t w = 0; w < p; ++w) {
        if (!hdrs[w] || (!words[w] && n_words[w])) { set_error("vgc_unpack_apply: message %u has a NULL pointer", w); return VGC_ERR_NULL; }
        if (!aligned(words[w], 4) || !aligned(hdrs[w], 8)) { set_error("vgc_unpack_apply: message %u is misaligned", w); return VGC_ERR_ALIGN; }
    }
    if (!aligned(plan, 256) || !aligned(param, 4) || !aligned(state1, 4) || !aligned(state2, 4)) { set_error("vgc_unpack_apply: misaligned pointer"); return VGC_ERR_ALIGN; }
    if (!std::isfinite(scale) || !std::isfinite(opt->lr)) { set_error("vgc_unpack_apply: scale or lr is not finite"); return VGC_ERR_PARAM; }
    float mu = 0.f, b1 = 0.f, b2 = 0.f, omb1 = 0.f, omb2 = 0.f, bias1 = 1.f, bias2 = 1.f, eps = 0.f;
    if (opt->kind == VGC_OPT_MOMENTUM_SGD) {
        if (!(opt->momentum >= 0.0f) || !(opt->momentum < 1.0f)) { set_error("vgc_unpack_apply: need 0 <= momentum < 1 (got %g)", opt->momentum); return VGC_ERR_PARAM; }
        mu = opt->momentum;
    } else {
        if (!(opt->beta1 >= 0.0f) || !(opt->beta1 < 1.0f) || !(opt->beta2 >= 0.0f) || !(opt->beta2 < 1.0f) || !(opt->eps >= 0.0f) ||
            !std::isfinite(opt->eps) || opt->step < 1) {
            set_error("vgc_unpack_apply: need 0 <= beta1, beta2 < 1, eps >= 0, step >= 1");
            return VGC_ERR_PARAM;
        }
        b1 = opt->beta1; b2 = opt->beta2; eps = opt->eps;
        omb1 = (float)(1.0 - (double)b1);
        omb2 = (float)(1.0 - (double)b2);
        bias1 = (float)(1.0 - std::pow((double)b1, (double)opt->step));
        bias2 = (float)(1.0 - std::pow((double)b2, (double)opt->step));
    }
    const PlanView pv = plan_view(plan, n_tiles, n_groups);
    return launch_unpack_apply(plan_check(plan, gs), words, n_words, hdrs, p, pv.groups, pv.runs, gs.n_runs, scale, opt->kind, opt->lr, mu, b1, b2,
                               omb1, omb2, bias1, bias2, eps, param, state1, state2, static_cast<hipStream_t>(stream));
}

}  // extern "C"
