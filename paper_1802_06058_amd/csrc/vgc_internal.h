// Internal layout shared by the host entry points and the kernels of libvgc.
#ifndef VGC_INTERNAL_H
#define VGC_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "vgc.h"

namespace vgc {

// A tile is the unit one workgroup of the accumulate kernel owns.  2048 elements lets a staged
// entry fit 16 bits: 4 bits exponent code, 1 bit sign, 11 bits position inside the tile.
constexpr uint32_t kTile = 2048;
constexpr uint32_t kTileShift = 11;
constexpr uint32_t kThreads = 256;
constexpr uint32_t kElemsPerThread = kTile / kThreads;   // 8
constexpr uint32_t kRelBins = 9;                          // staged exponent codes 0..8 (see StagedEntry)

constexpr uint64_t kPlanMagic = 0x34304E414C504756ull;    // "VGPLAN04"

struct PlanHeader {            // 128 bytes at the start of the plan blob
    uint64_t magic;
    uint64_t n;
    uint64_t n_tiles;
    uint32_t n_groups;
    uint32_t tile;
    uint64_t groups_off;       // byte offset of PlanGroup[n_groups]
    uint64_t tiles_off;        // byte offset of PlanTile[n_tiles]
    uint64_t runs_off;         // byte offset of PlanRun[n_runs]
    uint64_t n_runs;
    uint64_t segs_off;         // byte offset of PlanSeg[n_segs]
    uint64_t n_segs;
    uint64_t groups_hash;      // hash of the group list the plan was built from (see groups_hash())
    uint64_t reserved[5];
};

// Every compute call takes the host group list and the device plan built from it.  The host hashes the list it
// was given; every kernel that reads plan tables first compares that hash (and the magic) with the header's and
// does nothing when they differ: a plan that belongs to another group list is never used for addressing.
struct PlanCheck {
    const PlanHeader* header;  // device
    uint64_t hash;             // of the host group list of this call
};
__device__ __forceinline__ bool plan_ok(const PlanCheck& pc) {
    return pc.header->magic == kPlanMagic && pc.header->groups_hash == pc.hash;
}

struct PlanGroup {             // 16 bytes
    uint64_t offset;           // first element of the group in the flat parameter space
    uint32_t size;
    uint32_t first_tile;       // would overflow only beyond 2^43 parameters
};

struct PlanTile {              // 16 bytes
    uint32_t group;
    uint32_t start;            // element offset of the tile inside its group (multiple of kTile)
    uint32_t seg;              // index of the tile's segment in the segment table
    uint32_t run;              // index of the tile's run in the run table
};

// A segment is up to kSegTiles consecutive tiles of one group: the unit one workgroup of the scan
// kernel owns (8 tile records per thread, one pass).  A group of 2^28 elements has 16 of them.
constexpr uint32_t kSegTiles = 8192;
struct PlanSeg {               // 16 bytes
    uint32_t group;
    uint32_t first_tile;       // index of the segment's first tile inside its group
    uint32_t seg_in_group;
    uint32_t group_first_seg;  // index of the group's first segment in the table
};

// A run is up to kRunTiles consecutive tiles of one group: the unit one wave of the batched
// decoder owns.
constexpr uint32_t kRunTiles = 64;
struct PlanRun {               // 8 bytes
    uint32_t group;
    uint32_t first_tile;       // index of the run's first tile inside its group
};

// Per-tile record in the scratch.  Written by the accumulate kernel (w[0..4]) and completed by
// the first pack kernel (w[5..7]).
//   w[0..3]  : hist[0..7], two 16-bit counters per word (low half = even bin)
//   w[4]     : low half hist[8]; high half = largest truncated exponent field among the tile's sent elements
//   w[5]     : number of words the segment's earlier tiles produce (exclusive prefix inside the segment)
//   w[6]     : shift = E_k - tile exponent
//   w[7]     : words this tile produces
struct TileHdr { uint32_t w[8]; };

// Staged entry (uint16): rel << 12 | sign << 11 | position in tile, where
// rel = (tile exponent + 1) - rounded exponent field of the element, 0..8.
// With shift = E_k - tile exponent the final code is d = max(shift + rel - 1, 0)
// and the element is encoded iff rel <= 8 - shift.

struct SegTmp {                // 32 bytes, one per segment
    uint32_t max_e;            // largest tile exponent inside the segment (written only for groups of several segments)
    uint32_t exp_field;        // E_k of the segment's group
    uint32_t count;            // words the segment produces
    uint32_t reserved;
    uint64_t base;             // position of the segment's first word in the message
    uint64_t reserved2;
};

struct ScratchLayout {
    uint64_t n_tiles;
    size_t flags_off;          // uint32[64]; [0] = 1 if the accumulate kernel found the plan not to match the group list
    size_t tile_hdr_off;       // TileHdr[n_tiles]
    size_t seg_tmp_off;        // SegTmp[n_segs], sized for the bound n_tiles / kSegTiles + n_groups
    size_t bitmap_off;         // uint32[n_tiles * kTile / 32]
    size_t staging_off;        // uint16[n_tiles * kTile]
    size_t total;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline ScratchLayout scratch_layout(uint64_t n_tiles, uint32_t n_groups) {
    ScratchLayout L;
    L.n_tiles = n_tiles;
    size_t off = 0;
    L.flags_off = off;     off += 256;
    L.tile_hdr_off = off;  off = align_up(off + n_tiles * sizeof(TileHdr), 256);
    L.seg_tmp_off = off;   off = align_up(off + (size_t)(n_tiles / kSegTiles + n_groups) * sizeof(SegTmp), 256);
    L.bitmap_off = off;    off = align_up(off + n_tiles * (kTile / 8), 256);
    L.staging_off = off;   off = align_up(off + n_tiles * (size_t)kTile * 2, 256);
    L.total = off;
    return L;
}

// host-side helpers (vgc_api.hip)
void set_error(const char* fmt, ...);
int hip_check(hipError_t e, const char* what);

// kernel launchers
int launch_accumulate_select(PlanCheck pc, uint32_t* flags, const float* g, const float* s, float* r, float* v,
                             const PlanGroup* groups, const PlanTile* tiles, uint64_t tile0, uint64_t n_tiles,
                             TileHdr* hdrs, uint32_t* bitmap, uint16_t* staging,
                             float alpha, float zeta, float tau, bool hybrid, bool ptrs_vec_aligned,
                             hipStream_t stream);

// statistic of an FC layer fused into the accumulate pass (vgc_fused_fc.hip)
size_t fused_fc_workspace_bytes(int dtype, uint32_t B, uint32_t J, uint32_t C);
int launch_fused_fc_select(PlanCheck pc, uint32_t* flags, int dtype, const void* X, const void* D, uint32_t B, uint32_t J, uint32_t C,
                           float c, float* r, float* v, const PlanGroup* groups, uint32_t group, TileHdr* hdrs, uint32_t* bitmap,
                           uint16_t* staging, float alpha, float zeta, void* workspace, float* g_out, float* s_out, hipStream_t stream);

int launch_pack(PlanCheck pc, const uint32_t* flags, const PlanGroup* groups, const PlanTile* tiles, const PlanSeg* segs, uint64_t n_tiles,
                uint32_t n_groups, uint32_t n_segs, bool multi_seg,
                TileHdr* hdrs, SegTmp* stmp, const uint16_t* staging,
                uint32_t* words_out, uint64_t words_cap, vgc_group_hdr* hdrs_out,
                vgc_pack_status* status_out, hipStream_t stream);

// the scans of vgc_pack without the word emission (vgc_pack.hip), and the compressed index format (vgc_compact.hip)
int launch_pack_scans(PlanCheck pc, const uint32_t* flags, const PlanGroup* groups, const PlanSeg* segs, uint32_t n_groups,
                      uint32_t n_segs, bool multi_seg, TileHdr* hdrs, SegTmp* stmp, vgc_group_hdr* hdrs_out,
                      vgc_pack_status* status_out, uint64_t words_cap, hipStream_t stream);
int launch_pack_compact(PlanCheck pc, const PlanGroup* groups, const PlanTile* tiles, const PlanRun* runs, uint64_t n_tiles,
                        uint64_t n_runs, uint32_t n_groups, const TileHdr* hdrs, const uint16_t* staging, uint8_t* stream_out,
                        uint64_t stream_cap, uint16_t* tile_bytes_out, uint64_t* run_offsets_out, vgc_group_hdr* hdrs_out,
                        vgc_pack_status* status_out, hipStream_t stream);
int launch_unpack_compact_batch(PlanCheck pc, const uint8_t* const* streams, const uint64_t* stream_bytes, const uint16_t* const* tile_bytes,
                                const uint64_t* const* run_offsets, const vgc_group_hdr* const* hdrs, uint32_t p,
                                const PlanGroup* groups, const PlanRun* runs, uint64_t n_runs, float scale, int overwrite,
                                float* dense, hipStream_t stream);

int launch_unpack_add(PlanCheck pc, const uint32_t* words, uint64_t n_words, const vgc_group_hdr* hdrs,
                      const PlanGroup* groups, uint32_t n_groups, float scale, float* dense,
                      hipStream_t stream);

constexpr int kBatchMax = 8;   // messages one launch of the batched decoder takes
constexpr int kApplyMax = 64;  // messages the decoder fused with the parameter update takes (one launch; a lane per message)
int launch_unpack_add_batch(PlanCheck pc, const uint32_t* const* words, const uint64_t* n_words, const vgc_group_hdr* const* hdrs,
                            uint32_t p, const PlanGroup* groups, const PlanRun* runs, uint64_t n_runs,
                            float scale, int overwrite, float* dense, hipStream_t stream);

int launch_unpack_apply(PlanCheck pc, const uint32_t* const* words, const uint64_t* n_words, const vgc_group_hdr* const* hdrs,
                        uint32_t p, const PlanGroup* groups, const PlanRun* runs, uint64_t n_runs, float scale,
                        int kind, float lr, float mu, float b1, float b2, float omb1, float omb2, float bias1, float bias2,
                        float eps, float* param, float* state1, float* state2, hipStream_t stream);

int launch_sqgrad(int kind, int dtype, const void* X, const void* D, uint32_t B, uint32_t P,
                  uint32_t J, uint32_t C, float c, float* g_out, float* s_out,
                  void* workspace, size_t workspace_bytes, hipStream_t stream);
int launch_sqgrad_simple(int kind, int dtype, const void* X, const void* D, uint32_t B, uint32_t P,
                         uint32_t J, uint32_t C, float c, float* g_out, float* s_out, hipStream_t stream);

// LDS-tiled kernels (vgc_sqgrad_tiled.hip, vgc_sqgrad_fc.hip)
uint32_t conv_splits(uint32_t B, uint32_t J, uint32_t C);
size_t conv_workspace_bytes(uint32_t B, uint32_t P, uint32_t J, uint32_t C);
bool conv_taps_supported(uint32_t H, uint32_t W, uint32_t Cin, uint32_t C, uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw,
                         uint32_t ph, uint32_t pw);
size_t conv_taps_workspace_bytes(uint32_t B, uint32_t P, uint32_t Cin, uint32_t C);
bool conv_tiled_supported(int dtype, uint32_t P, uint32_t J, uint32_t C);
void launch_sqgrad_reduce(const float* ws, uint32_t splits, size_t JC, float cg, float cs, float* g_out, float* s_out,
                          hipStream_t stream);
bool fc_tiled_supported(int dtype, uint32_t B, uint32_t J, uint32_t C);
bool conv_f32_tiled_supported(uint32_t P, uint32_t J, uint32_t C);
uint32_t conv_f32_splits(uint32_t B, uint32_t J, uint32_t C);
size_t conv_f32_workspace_bytes(uint32_t B, uint32_t P, uint32_t J, uint32_t C);
void launch_sqgrad_reduce_parts(const float* ws, uint32_t B, uint32_t split_p, size_t JC, float cg, float cs, float* g_out,
                                float* s_out, hipStream_t stream);
int launch_fc_tiled(int dtype, const void* X, const void* D, uint32_t B, uint32_t J, uint32_t C, float c,
                    float* g_out, float* s_out, hipStream_t stream);
int launch_conv_f32_tiled(const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
                          float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t sqgrad_workspace_bytes(int kind, int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C);
// Geometry of a 2-d convolution whose patch matrix is never built: U[z, p, j] with p = y Wo + x and
// j = (ky kw + kx) Cin + i is the input element [z, y sh + ky - ph, x sw + kx - pw, i], or zero outside.
struct ConvGeom {
    uint32_t H, W, Cin, kw, sh, sw, ph, pw, Ho, Wo;
    uint32_t step_y, step_x; // one chunk of kKC positions further: kKC = step_y * Wo + step_x
    uint32_t period;         // bf16 kernel, unit strides and Wo = W: chunks after which the column pattern repeats (0: general path)
};

bool conv2d_supported(int dtype, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C, uint32_t P);
// first layers: input channels that are not a multiple of 16 bytes, small J (vgc_sqgrad_stem.hip)
bool conv_stem_supported(int dtype, uint32_t Cin, uint32_t C, uint32_t kh, uint32_t kw);
size_t conv_stem_workspace_bytes(int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C);
int launch_conv_stem(int dtype, const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C,
                     uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw, uint32_t Ho, uint32_t Wo,
                     float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream);
int launch_conv2d_f32(const void* act, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
                      float* g_out, float* s_out, void* workspace, size_t workspace_bytes, ConvGeom G, hipStream_t stream);
int launch_conv2d(int dtype, const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C,
                  uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw, uint32_t Ho, uint32_t Wo,
                  float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream);
int launch_conv_tiled(int dtype, const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                      float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream);

}  // namespace vgc
#endif
