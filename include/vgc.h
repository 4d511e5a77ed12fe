/*
 * vgc.h -- C ABI of the per-worker hot path of variance-based gradient compression
 * (Tsuzuku, Imachi, Akiba, "Variance-based Gradient Compression for Efficient
 * Distributed Deep Learning", arXiv 1802.06058) for AMD MI355X (gfx950).
 *
 * One training iteration of one worker (Alg. 1) maps onto the calls like this:
 *
 *   CalcGrad()                              the framework's forward/backward (not here)
 *   sum grad/B, sum (grad/B)^2  per param   vgc_sqgrad            (per layer)
 *   foreach parameter: accumulate, test,
 *     reset or decay                        vgc_accumulate_select (whole model, one launch)
 *     Encode()                              vgc_pack              (whole model)
 *   CommunicateAndUpdate(): decode + sum    vgc_unpack_add        (once per received message)
 *
 * Conventions
 *   - Pointers marked DEVICE point to GPU memory owned by the caller; pointers marked HOST
 *     to ordinary host memory.  The library never allocates, frees or keeps device memory.
 *   - Every compute call only enqueues kernels on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and returns without synchronising.
 *   - Return value: VGC_OK (0) or a negative vgc_status.  On an argument error nothing is
 *     launched and no buffer is touched.  vgc_last_error() gives a text for the calling thread.
 *   - A "group" is the set of elements of one weight matrix / weight tensor (Section 4.2):
 *     the unit that shares one floor(log2 M_k) and inside which the 28-bit index counts.
 */
#ifndef VGC_H
#define VGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VGC_OK = 0,
    VGC_ERR_NULL = -1,            /* a required pointer is NULL */
    VGC_ERR_SIZE = -2,            /* n == 0, a zero dimension, groups not tiling [0, n), buffer too small */
    VGC_ERR_GROUP_TOO_LARGE = -3, /* a group has more than 2^28 elements (28-bit index, Section 4.2) */
    VGC_ERR_DTYPE = -4,           /* unknown dtype / kind enum */
    VGC_ERR_ALIGN = -5,           /* pointer not aligned as documented */
    VGC_ERR_PARAM = -6,           /* alpha negative or non-finite, zeta outside (0, 1], scale non-finite */
    VGC_ERR_HIP = -7              /* a HIP runtime call failed; see vgc_last_error() */
} vgc_status;

enum { VGC_F32 = 0, VGC_BF16 = 1 };   /* element type of the activations / output-gradients */
enum { VGC_FC = 0, VGC_CONV = 1 };    /* fully-connected form / shared-weight (convolution) form */

/* One weight matrix: elements [offset, offset + size) of the flat parameter space. */
typedef struct {
    uint64_t offset;
    uint32_t size;        /* 1 .. 2^28 */
    uint32_t reserved;    /* must be 0 */
} vgc_group;

/* Header of one group inside a packed message (Section 4.2: floor(log2 M_k) "is also sent
 * for every weight matrix"; the count is what a variable-length gather needs, Section 5). */
typedef struct {
    uint32_t exp_field;   /* biased float32 exponent field of M_k, i.e. floor(log2 M_k) + 127; 0 if count == 0 */
    uint32_t count;       /* words of this group */
    uint64_t word_offset; /* index of the group's first word in the message's word array */
} vgc_group_hdr;

/* Result record of vgc_pack (DEVICE memory, written by the device). */
typedef struct {
    uint64_t total_words; /* words the message has (also when they did not all fit) */
    uint32_t overflow;    /* 1 if total_words > words_cap: words beyond the capacity were not written */
    uint32_t plan_mismatch; /* 1 if `plan` was not built from the `groups` of this call: nothing was computed, the
                               message is empty and r, v are untouched */
} vgc_pack_status;

/* Word layout (Section 4.2: 4-bit value, 28-bit index, one 32-bit word per sent element):
 *   bit 31      sign of the accumulated gradient
 *   bits 30..28 d = floor(log2 M_k) - log2 g'   (0..7; elements with d > 7 are not encoded)
 *   bits 27..0  index of the element inside its group, 0-based
 * Words of a group are in ascending index order; groups follow each other in order. */
#define VGC_WORD_SIGN(w)  ((uint32_t)(w) >> 31)
#define VGC_WORD_D(w)     (((uint32_t)(w) >> 28) & 7u)
#define VGC_WORD_INDEX(w) ((uint32_t)(w) & 0x0FFFFFFFu)
#define VGC_MAX_GROUP_SIZE (1u << 28)

/* ---- library information ------------------------------------------------------------------ */

const char* vgc_last_error(void);   /* text of the last error on this thread ("" if none) */
uint32_t    vgc_tile_size(void);    /* elements per tile of the accumulate/pack kernels (a tile never spans two groups) */

/* ---- plan and scratch ----------------------------------------------------------------------
 * The plan is a read-only device table derived from the group list (group table + tile table);
 * it can be shared by every worker state and by the decoder.  The scratch is per-worker working
 * memory that carries the staged result of vgc_accumulate_select to vgc_pack.
 */

/* Number of tiles the groups split into.  groups: HOST.  Returns 0 and sets the error text if the
 * groups are invalid (empty, zero-sized, larger than 2^28, or not tiling [0, n) in order). */
uint64_t vgc_tile_count(const vgc_group* groups, uint32_t n_groups, uint64_t n);

/* Bytes of the plan / of one scratch buffer for this group list (0 on invalid groups). */
size_t vgc_plan_bytes(const vgc_group* groups, uint32_t n_groups, uint64_t n);
size_t vgc_scratch_bytes(const vgc_group* groups, uint32_t n_groups, uint64_t n);

/* Build the plan on the host.  plan_host: HOST buffer of vgc_plan_bytes() bytes that the caller
 * then copies to device memory (256-byte aligned) and passes as `plan` below.  Pure host code. */
int vgc_plan_build(const vgc_group* groups, uint32_t n_groups, uint64_t n, void* plan_host, size_t plan_bytes);

/* Byte offset inside the scratch of the send bitmap that vgc_accumulate_select leaves behind:
 * one bit per element in tile order, i.e. bit (t * vgc_tile_size() + i) is element i of tile t
 * (tiles are numbered group after group, ceil(size / tile) per group); bit i lives in byte i/8,
 * bit position i%8.  1 = the element passed the test of Eq. 2 in this step. */
size_t vgc_scratch_bitmap_offset(const vgc_group* groups, uint32_t n_groups, uint64_t n);

/* ---- (a) per-parameter sums over the mini-batch ---------------------------------------------
 * Alg. 1, first two lines of the loop body: g_i = sum_z grad_i f_z * c and
 * s_i = sum_z (grad_i f_z * c)^2 with c = 1/B (or 1 if the output-gradients already carry it),
 * where grad f_z is the gradient of sample z's own loss (Section 4.1).  Section 5 counts
 * 2 N |B| multiply-adds for this statistic.
 *
 *   VGC_FC:   X [B, J], D [B, C] row-major; sample z's gradient of W[j, c] is X[z, j] * D[z, c]:
 *             g = c * X^T D,  s = c^2 * (X.X)^T (D.D).   P must be 1.
 *   VGC_CONV: X [B, P, J] (im2col patches), D [B, P, C]; sample z's gradient is
 *             G_z = sum_p X[z, p, :]^T D[z, p, :]:  g = c * sum_z G_z,  s = c^2 * sum_z G_z . G_z
 *             (the square is taken after the sum over the P positions).
 *
 * X, D: DEVICE, dtype VGC_F32 (float) or VGC_BF16 (bfloat16 bits), 16-byte aligned.
 * g_out (may be NULL), s_out: DEVICE float [J, C] row-major (the weight's own layout), 16-byte aligned.
 * Accumulation is in float32.  Errors: NULL, SIZE (a zero dimension, P != 1 for FC), DTYPE, ALIGN, PARAM.
 *
 * workspace: optional DEVICE buffer (16-byte aligned) of vgc_sqgrad_workspace_bytes() bytes.  When
 * [J, C] has too few tiles to fill the chip the samples are split over more workgroups and the
 * partial sums are added from the workspace in a fixed order (the result does not depend on
 * scheduling); when even one workgroup per (tile, sample) leaves a third or more of the chip idle, the
 * positions of a sample are split as well and the parts of each sample's gradient are added before the
 * square is taken.  With workspace == NULL or too small the call still works, without the splits.
 * Calls on different streams may overlap when each has a workspace of its own (a network's layers are
 * independent).  Non-finite inputs give unspecified sums, no fault.
 */
size_t vgc_sqgrad_workspace_bytes(int kind, int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C);
int vgc_sqgrad(int kind, int dtype, const void* X, const void* D,
               uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
               float* g_out, float* s_out, void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): vgc_sqgrad with the workspace taken from a buffer of VGC_NOALLOC_SCRATCH_BYTES that is
 * part of the library's own device image (each GPU the library runs on holds one copy until the process ends).
 * Same kernels, same splits, same results bit for bit as vgc_sqgrad given a workspace of
 * vgc_sqgrad_workspace_bytes() bytes; X, D, g_out, s_out, stream and errors as there.  A shape whose workspace
 * would exceed the buffer is refused with VGC_ERR_SIZE (nothing is launched).  The call allocates and frees
 * nothing and does not synchronise; on its first use on a GPU it looks the buffer's address up once.
 * Every call on one GPU shares that GPU's buffer: calls that may overlap there (different streams, different
 * threads) race; calls on one stream are ordered.  Nothing in the buffer needs clearing between calls (every
 * partial sum a call reads was written by that call). */
#define VGC_NOALLOC_SCRATCH_BYTES (128u << 20)
int vgc_sqgrad_noalloc(int kind, int dtype, const void* X, const void* D,
                       uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
                       float* g_out, float* s_out, void* stream);

/* The same sums for a 2-d convolution given as the layer stores it, without a patch matrix:
 *   act [B, H, W, Cin] (NHWC) the layer's input, D [B, Ho, Wo, C] (NHWC) the gradient of each sample's
 *   loss w.r.t. the layer's output, Ho = (H + 2 pad_h - kh) / stride_h + 1, Wo likewise.
 * Sample z's gradient of the weight W[ky, kx, i, o] is
 *   sum_{y, x} act[z, y stride_h + ky - pad_h, x stride_w + kx - pad_w, i] * D[z, y, x, o]
 * (positions outside the input count as zero); g and s come out as [kh * kw * Cin, C] row-major with
 * row (ky * kw + kx) * Cin + i, i.e. the weight in [kh, kw, Cin, C] layout.  It is VGC_CONV applied to
 * the im2col matrix of act, which is never materialised: the input is read directly, 1 / (kh kw) of
 * the bytes, and neighbouring filter taps find each other's lines in the cache.
 * dtype: VGC_F32 or VGC_BF16; C must be a multiple of 16 bytes (4 floats, 8 bfloat16), Cin as well or else
 * kh * kw * Cin at most 160 (a network's first layer: an RGB input under a 3 x 3 or 7 x 7 filter; such a layer needs
 * the workspace, VGC_ERR_SIZE without it), and a sample's tensors below 2 GiB, else VGC_ERR_SIZE (build the patch
 * matrix and call vgc_sqgrad).  Pointers, workspace and errors as for vgc_sqgrad.
 */
size_t vgc_sqgrad_conv2d_workspace_bytes(int dtype, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C,
                                         uint32_t kh, uint32_t kw, uint32_t stride_h, uint32_t stride_w,
                                         uint32_t pad_h, uint32_t pad_w);

int vgc_sqgrad_conv2d(int dtype, const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin,
                      uint32_t C, uint32_t kh, uint32_t kw, uint32_t stride_h, uint32_t stride_w,
                      uint32_t pad_h, uint32_t pad_w, float c, float* g_out, float* s_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/* The statistic of several convolution layers in one call.  The layers of a model are independent of each other
 * (Alg. 1 runs per parameter; a layer is one weight tensor, Section 4.2) and most of them are too small to fill the
 * chip alone, so the kernels of the small layers (below 2e10 multiply-adds) are spread over four streams of the
 * library's own, between a fork after what the caller's stream holds so far and a join back into it, while the large
 * ones run on the caller's stream: kernels of different layers fill each other's tails.  Every result is that of
 * vgc_sqgrad_conv2d on the same layer, bit for bit.
 *
 * layers: HOST array; the fields are the arguments of vgc_sqgrad_conv2d.  The layers run side by side, so each needs
 * outputs and a workspace of its own.  Every layer is checked before anything is launched; on an argument error
 * nothing is launched.  The side streams (default priority) and their events are created at the first call on a
 * device and kept; calls from several host threads are serialised while they submit.  Not for use under stream
 * capture on hosts where the first call has not been made yet (it creates streams).
 */
typedef struct {
    int dtype;
    const void* act;
    const void* D;
    uint32_t B, H, W, Cin, C, kh, kw, stride_h, stride_w, pad_h, pad_w;
    float c;
    float* g_out;          /* nullable */
    float* s_out;
    void* workspace;       /* nullable */
    size_t workspace_bytes;
} vgc_conv2d_layer;

int vgc_sqgrad_conv2d_batch(const vgc_conv2d_layer* layers, uint32_t n_layers, void* stream);

/* ---- (b) accumulate, test, reset or decay ---------------------------------------------------
 * The body of Alg. 1's parameter loop with the criterion of Eq. 2 and the decay of Section 4.4,
 * for all n parameters in one launch, in float32 with one rounding per operation:
 *     r' = r + g;  v' = v + s;  send = (r'*r' > alpha*v')        (strict)
 *     r  = send ? 0 : r';        v = send ? 0 : zeta*v'
 * For every element that is sent the kernel also takes the first half of Encode(): it rounds
 * |r'| to a power of two with the integer recipe of Section 4.4 and stages (sign, exponent,
 * position) in `scratch`, together with per-tile exponent statistics and the send bitmap, for
 * vgc_pack to finish.  After this call r and v hold Alg. 1's post-step state.
 *
 * g, s (read), r, v (read and written): DEVICE float[n], 4-byte aligned (16-byte alignment of
 * base + group offset enables the vector path).  groups: HOST, the list the plan was built from.
 * plan, scratch: DEVICE, 256-byte aligned.  alpha >= 0 finite, 0 < zeta <= 1.
 * Non-finite inputs give an unspecified mask but no fault.
 * The plan carries a hash of the group list it was built from; the kernels of this and of every other call
 * that takes a plan compare it with the hash of `groups` and do nothing when they differ (a plan of another
 * model is never used for addressing).  vgc_pack reports that case in vgc_pack_status.plan_mismatch.
 */
int vgc_accumulate_select(const float* g, const float* s, float* r, float* v, uint64_t n,
                          const vgc_group* groups, uint32_t n_groups, const void* plan,
                          float alpha, float zeta, void* scratch, void* stream);

/* Hybrid algorithm (Alg. 2, Section 4.5: the variance criterion combined with a threshold tau):
 *     r' = r + g;  v' = v + s;  send = (|r'| > tau) and (r'*r' > alpha*v')
 *     sent:   r = r' - sign(r')*tau;   v = max((v' - (2|r'|)*tau) + tau*tau, 0)      (|r'| before the subtraction)
 *     always: v = zeta * v
 * What is sent is Sign(r'), i.e. +-tau.  The staged result goes through the same vgc_pack: the message
 * has exp_field = 127 (2^0) in the header of every non-empty group and d = 0 in every word, and
 * vgc_unpack_add decodes it with scale = tau (times 1/p for the mean).  Same arguments as above, plus
 * tau >= 0 finite. */
int vgc_accumulate_select_hybrid(const float* g, const float* s, float* r, float* v, uint64_t n,
                                 const vgc_group* groups, uint32_t n_groups, const void* plan,
                                 float alpha, float zeta, float tau, void* scratch, void* stream);

/* The same pass over a range of consecutive groups only: [first_group, first_group + group_count) of the list.  The
 * other groups' r, v and staged results are left as they are.  For models some of whose layers go through
 * vgc_sqgrad_accumulate_select: the remaining groups are covered by one call per run of consecutive groups, and
 * vgc_pack then runs once over the whole model.  g, s, r, v are the whole-model arrays as above. */
int vgc_accumulate_select_range(const float* g, const float* s, float* r, float* v, uint64_t n,
                                const vgc_group* groups, uint32_t n_groups, const void* plan,
                                uint32_t first_group, uint32_t group_count,
                                float alpha, float zeta, void* scratch, void* stream);

/* ---- (a) + (b) for one fully-connected layer ---------------------------------------------------
 * Alg. 1's loop body from its first line on, for the weight matrix that is group `group` of the model:
 * g = c X^T D and s = c^2 (X.X)^T (D.D) (VGC_FC of vgc_sqgrad) are formed on the matrix cores and consumed in
 * place by r += g, v += s, the test of Eq. 2 and reset / decay, so that g and s of the layer never reach memory
 * (the layer moves 16 bytes per parameter instead of 32; Section 5 counts the statistic as the dominant added
 * cost, and for FC layers that cost is memory traffic).  r, v, scratch and the staged result are exactly what
 * vgc_accumulate_select would leave given this g and s; the other groups are untouched (see
 * vgc_accumulate_select_range), and vgc_pack finishes the whole model.
 *
 * X [B, J], D [B, C] row-major, dtype VGC_F32 or VGC_BF16 (accumulation in float32; bfloat16 squares are rounded to
 * bfloat16 before the contraction, 2^-9 relative per factor).  groups[group].size must be J * C, and C a multiple of
 * 2048 or one of 256, 512, 1024 (so that the 2048-element tiles of the pass are whole rows or whole pieces of
 * rows), else VGC_ERR_SIZE: use vgc_sqgrad + vgc_accumulate_select for such a layer.
 * workspace: DEVICE, 16-byte aligned, vgc_sqgrad_accumulate_select_workspace_bytes() bytes (transposed copies of X
 * and D; 0 from that function means the shape is not supported).
 * g_out, s_out: both NULL, or DEVICE float [J, C] that also receive the statistic (for inspection and tests).
 * r, v: the whole-model arrays (DEVICE float[n]); plan, scratch, alpha, zeta, errors as for vgc_accumulate_select. */
size_t vgc_sqgrad_accumulate_select_workspace_bytes(int dtype, uint32_t B, uint32_t J, uint32_t C);
int vgc_sqgrad_accumulate_select(int dtype, const void* X, const void* D, uint32_t B, uint32_t J, uint32_t C, float c,
                                 float* r, float* v, uint64_t n, const vgc_group* groups, uint32_t n_groups,
                                 const void* plan, uint32_t group, float alpha, float zeta, void* scratch,
                                 void* workspace, size_t workspace_bytes, float* g_out, float* s_out, void* stream);

/* ---- (c) quantise, compact, pack ------------------------------------------------------------
 * Encode() of Alg. 1 (Sections 4.2 and 4.4): per group, M_k = the largest magnitude among the
 * elements being sent, header = floor(log2 M_k); each sent element becomes one word (layout
 * above) unless its d exceeds 7, in which case it is rounded to zero and not encoded.
 * Consumes the scratch left by the preceding vgc_accumulate_select on the same stream.
 *
 * words_out: DEVICE uint32[words_cap]; never written past words_cap (words_cap >= n cannot overflow).
 * hdrs_out:  DEVICE vgc_group_hdr[n_groups].   status_out: DEVICE vgc_pack_status.
 */
int vgc_pack(uint64_t n, const vgc_group* groups, uint32_t n_groups, const void* plan, void* scratch,
             uint32_t* words_out, uint64_t words_cap, vgc_group_hdr* hdrs_out,
             vgc_pack_status* status_out, void* stream);

/* ---- (d) decode and sum ---------------------------------------------------------------------
 * The receiving half of CommunicateAndUpdate() (Section 4.3): decode one worker's message and
 * add it into the dense gradient buffer:
 *     dense_out[offset_k + index] += scale * (+-)2^(exp_field_k - d - 127)
 * with one float32 multiply and one float32 add per word.  Indices inside one message are
 * distinct, so the result is deterministic; several messages are applied by several calls on
 * the same stream, in call order.  scale = 1/p gives the mean over p workers.
 *
 * words, hdrs: DEVICE (as written by vgc_pack: indices ascending inside a group; n_words = the
 * message's total word count, known to the receiver from the transfer size; an upper bound is
 * allowed, the headers' counts decide).  plan: DEVICE.  dense_out: DEVICE float[n].
 * The kernel is chosen from n_words: one thread per word below n / 8, above it one pass over
 * dense_out tile by tile; the sums are the same bit for bit, so a loose upper bound costs time only.
 */
int vgc_unpack_add(const uint32_t* words, uint64_t n_words, const vgc_group_hdr* hdrs,
                   const vgc_group* groups, uint32_t n_groups, const void* plan,
                   float scale, float* dense_out, uint64_t n, void* stream);

/* Several messages in one pass over the dense buffer: the same result, bit for bit, as
 * (overwrite ? clear dense_out : nothing) followed by vgc_unpack_add(message 0), ..., (message p-1),
 * but dense_out is read and written once instead of p times.  Worth it when the messages together
 * touch most of the buffer (Section 4.3 expects few index collisions at high compression ratios;
 * there one launch per message moves less).
 *
 * words, hdrs: HOST arrays of p DEVICE pointers; n_words: HOST array of p counts (upper bounds
 * allowed).  overwrite != 0: dense_out = sum of messages instead of dense_out += sum (also with p == 0).
 * Messages must be well-formed (ascending indices inside a group, as vgc_pack writes them); a
 * malformed one gives unspecified sums but no out-of-range access.
 */
int vgc_unpack_add_batch(const uint32_t* const* words, const uint64_t* n_words,
                         const vgc_group_hdr* const* hdrs, uint32_t p,
                         const vgc_group* groups, uint32_t n_groups, const void* plan,
                         float scale, int overwrite, float* dense_out, uint64_t n, void* stream);

/* ---- compressed index encoding ----------------------------------------------------------------
 * Section 4.2 ends by noting that the bits spent on indexes can be reduced further by compressing them, without
 * giving an algorithm; this format is the library's own.  Elements are in ascending index order, so each is stored
 * as its distance from the previous element of its tile (vgc_tile_size() consecutive elements of a group):
 *     gap  = position in tile - position of the tile's previous element - 1      (the first element counts from -1)
 *     code = sign << 3 | d                                                      (the 4-bit value of Section 4.2)
 *     gap < 8:  one byte   gap << 4 | code
 *     else:     two bytes  0x80 | (gap & 7) << 4 | code,  gap >> 3              (gap <= 2047)
 * A message is: the group headers (exp_field and count as in the plain format; word_offset = BYTE offset of the
 * group's first tile in the stream), tile_bytes[t] (bytes of tile t, tiles numbered as for vgc_scratch_bitmap_offset),
 * run_offsets[r] (byte offset of the first tile of run r; a run is 64 consecutive tiles of one group, runs numbered
 * group after group) and the byte stream.  One or two bytes per element instead of four; with the directory
 * (2 bytes per tile, 8 per run) it is the smaller format once a message holds one element per tile on average.
 *
 * vgc_pack_compact consumes the scratch left by vgc_accumulate_select exactly as vgc_pack does (either or both may
 * follow one accumulate call).  stream_out: DEVICE uint8[stream_cap], never written past stream_cap (2 * n bytes
 * cannot overflow); tile_bytes_out: DEVICE uint16[vgc_tile_count()]; run_offsets_out: DEVICE uint64[vgc_run_count()];
 * status_out->total_words is the stream's length in BYTES, overflow and plan_mismatch as for vgc_pack.
 *
 * vgc_unpack_compact_add_batch is vgc_unpack_add_batch for such messages (HOST arrays of p DEVICE pointers;
 * stream_bytes: HOST array of the streams' lengths, beyond which nothing is read): same sums, bit for bit, as
 * decoding the messages in the plain format in message order. */
uint64_t vgc_run_count(const vgc_group* groups, uint32_t n_groups, uint64_t n);
int vgc_pack_compact(uint64_t n, const vgc_group* groups, uint32_t n_groups, const void* plan, void* scratch,
                     uint8_t* stream_out, uint64_t stream_cap, uint16_t* tile_bytes_out, uint64_t* run_offsets_out,
                     vgc_group_hdr* hdrs_out, vgc_pack_status* status_out, void* stream);
int vgc_unpack_compact_add_batch(const uint8_t* const* streams, const uint64_t* stream_bytes, const uint16_t* const* tile_bytes,
                                 const uint64_t* const* run_offsets, const vgc_group_hdr* const* hdrs, uint32_t p,
                                 const vgc_group* groups, uint32_t n_groups, const void* plan, float scale, int overwrite,
                                 float* dense_out, uint64_t n, void* stream);

/* ---- decode fused with the parameter update --------------------------------------------------
 * CommunicateAndUpdate() of Alg. 1 in one pass (Section 4.3; with Momentum SGD and the like,
 * elements that no worker sent enter the update as zero, Section 4.1): the p messages are decoded
 * and summed in message order into a zero gradient ghat, exactly as vgc_unpack_add_batch with
 * overwrite does, and instead of writing ghat out the optimizer step is applied to every parameter:
 *   VGC_OPT_MOMENTUM_SGD   m <- momentum m - lr ghat;   w <- w + m                  (state1 = m)
 *   VGC_OPT_ADAM           m <- beta1 m + (1 - beta1) ghat;  v <- beta2 v + (1 - beta2) ghat^2;
 *                          w <- w - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *                                                                               (state1 = m, state2 = v)
 * float32, one rounding per operation in the order written; 1 - beta and 1 - beta^step are formed in
 * double and rounded to float once.  The paper names the optimizers without printing them; these are
 * the classical forms.
 *
 * words, hdrs, n_words: HOST arrays as for vgc_unpack_add_batch, p <= VGC_MAX_UPDATE_MESSAGES.
 * opt: HOST.  param, state1, state2: DEVICE float[n], updated in place (state2 may be NULL for
 * Momentum SGD).  Moves 16 (Momentum SGD) or 24 (Adam) bytes per parameter plus 4 per word; no
 * dense gradient buffer exists.
 */
#define VGC_MAX_UPDATE_MESSAGES 64
enum { VGC_OPT_MOMENTUM_SGD = 0, VGC_OPT_ADAM = 1 };
typedef struct {
    int32_t kind;        /* VGC_OPT_* */
    float lr;
    float momentum;      /* Momentum SGD */
    float beta1, beta2, eps;   /* Adam */
    uint32_t step;       /* Adam: number of this step, >= 1 */
} vgc_optimizer;

int vgc_unpack_apply(const uint32_t* const* words, const uint64_t* n_words,
                     const vgc_group_hdr* const* hdrs, uint32_t p,
                     const vgc_group* groups, uint32_t n_groups, const void* plan, float scale,
                     const vgc_optimizer* opt, float* param, float* state1, float* state2,
                     uint64_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VGC_H */
