// LDS-tiled MFMA kernels for the per-parameter sums of Alg. 1 (g = c sum_z G_z, s = c^2 sum_z G_z.G_z,
// G_z the gradient of sample z's loss, Section 4.1), shared-weight form: G_z = U_z^T D_z with K = P.
//
// A workgroup owns a BM x BN tile of [J, C] (one wave per 64 x 64 sub-tile) and a range of samples.
// For every sample it runs the K loop over the P positions in chunks of 32 rows, keeping the
// per-sample product in MFMA accumulators; when the sample is finished the accumulators are squared
// into s (and added into g) and cleared, so a per-sample gradient never leaves registers.  The sample
// range can be split over workgroups to fill the chip when [J, C] has few tiles; the partial sums then
// go to a workspace and are added in fixed order by k_sqgrad_reduce.  For the few layers where that is
// still too little parallelism the positions of a sample are split as well: those workgroups leave
// their part of the sample's product in the workspace and k_sqgrad_reduce_parts completes it.
//
// Chunks travel from global memory straight into LDS (buffer loads with the LDS modifier: lane l of a
// wave-wide load deposits its 16 bytes at M0 + 16 l), several chunks ahead of the one being multiplied,
// in a ring of LDS buffers.  No staging registers, no LDS store instructions; the distance covers the
// HBM latency of the lines a workgroup is the first in its L2 to touch.
//
// bf16 operands: v_mfma_f32_32x32x16_bf16.  Lane l of that instruction holds, for row m = l % 32, the 8
// consecutive k = 8 * (l / 32) .. + 7.  Memory has the other order (k-major rows, m contiguous), so
// the operands are fetched with the LDS transposing read ds_read_b64_tr_b16: within 16 lanes, lane r
// supplies the address of 4 consecutive b16 and lane i receives element i % 4 from the addresses of
// lanes i / 4 + 4 j, j = 0..3.  With lane r pointing at row k0 + r / 4, columns m0 + 4 (r % 4) .. + 3,
// lane i receives k0 .. k0 + 3 for column m0 + i.
//
// A staged row is W * 2 bytes with no padding (a wave-wide load fills 1 KiB of consecutive LDS), so
// rows k0 .. k0+3 of one 64-byte column unit would share banks.  The unit index is therefore XORed
// with a function of the row (swizzle) on the way in, by choosing which global piece each lane
// fetches, and on the way out in the fragment addresses.
#include "vgc_internal.h"
#include <type_traits>

namespace vgc {

typedef short s4v __attribute__((ext_vector_type(4)));
typedef short s8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef int i4v __attribute__((ext_vector_type(4)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s4v* lds_s4v_ptr;

constexpr int kKC = 32;                  // positions per LDS stage

// XOR mask applied to the 64-byte unit index of row `row` in a staged tile W elements wide.  Four
// consecutive rows (row % 4 = 0..3) of one unit then start 16 banks apart.
template <int W> __device__ __forceinline__ uint32_t swizzle(uint32_t row) {
    return W >= 128 ? (row & 3u) : ((row >> 1) & 1u);
}

// One 16-byte piece per lane from the bounded buffer `rsrc` (byte offset voff) to LDS byte address
// lds_base + lds_off + 16 * lane (two scalar registers, added on the way into m0).  Lanes outside the range deposit zeros.  Counted by vmcnt.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"          // m0 is named as clobbered on purpose
__device__ __forceinline__ void load_to_lds(uint32_t lds_base, uint32_t lds_off, uint32_t voff, i4v rsrc) {
    asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds"
                 :: "s"(lds_base), "s"(lds_off), "v"(voff), "s"(rsrc) : "memory", "m0", "scc");
}
#pragma clang diagnostic pop
template <int N> __device__ __forceinline__ void wait_loads_but() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Buffer descriptor over the current sample of one operand ([B, rows, W] bf16), all in scalar registers.  Lanes
// address their pieces by byte offset inside the sample; rows past the sample's end read as zeros.  The window
// moves only when the chunk requests cross into the next sample, and closes (empty range: every lane reads
// zeros) once the workgroup's last chunk has been requested.
struct SampleWindow {
    uint32_t lo, hi, range;  // 48-bit address of the sample, its size in bytes
    uint32_t sample_bytes;
    uint32_t kind;           // the descriptor's fourth word, in a register of the window's own (a shared one gets copied around)
    __device__ __forceinline__ void init(const uint16_t* base, uint32_t z, uint32_t rows, uint32_t W) {
        sample_bytes = __builtin_amdgcn_readfirstlane(rows * W * 2u);
        const uint64_t addr = reinterpret_cast<uint64_t>(base) + (uint64_t)z * sample_bytes;
        // everything here is uniform over the workgroup; pin it to scalar registers
        lo = __builtin_amdgcn_readfirstlane((uint32_t)addr);
        hi = __builtin_amdgcn_readfirstlane((uint32_t)(addr >> 32) & 0xFFFFu);
        range = sample_bytes;
        asm volatile("s_mov_b32 %0, 0x00020000" : "=s"(kind));
    }
    __device__ __forceinline__ i4v rsrc() const {
        i4v r;
        r[0] = (int)__builtin_amdgcn_readfirstlane(lo);          // uniform values; the asm operand must be scalar registers
        r[1] = (int)__builtin_amdgcn_readfirstlane(hi);
        r[2] = (int)__builtin_amdgcn_readfirstlane(range);
        r[3] = (int)kind;
        return r;
    }
    __device__ __forceinline__ void next_sample() {
        lo += sample_bytes;
        hi += (lo < sample_bytes) ? 1u : 0u;
    }
    __device__ __forceinline__ void close() { range = 0u; }
};

// BM x BN block tile of [J, C]; one wave per 64 x 64 sub-tile.  kImplicit: U is the layer's NHWC input seen
// through the geometry G (J = kh kw Cin), otherwise a [B, P, J] matrix.  kLinear (with kImplicit): unit strides
// and an output as wide as the input (G.period > 0), where the input element of output position p and tap
// (ky, kx) is element p + (ky - ph) W + kx - pw of the sample: the lane's offset moves by a constant per chunk and
// what is left of the geometry is whether column x + kx - pw lies inside the row, which repeats every G.period
// chunks (x advances by kKC mod W per chunk) and is kept as one bit per chunk of the period.
template <int BM, int BN, bool kWantG, bool kImplicit, bool kLinear = false>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64, 2)
void k_conv_bf16(const uint16_t* __restrict__ U, const uint16_t* __restrict__ D,
                 uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                 uint32_t splits, uint32_t split_p, float cg, float cs,
                 float* __restrict__ g_out, float* __restrict__ s_out, float* __restrict__ ws, ConvGeom G) {
    constexpr int NW = (BM / 64) * (BN / 64);
    constexpr int kABytes = kKC * BM * 2, kBBytes = kKC * BN * 2, kBufBytes = kABytes + kBBytes;
    // ring of staged chunks = chunks in flight: as many as fit beside the other workgroups of the CU (at
    // most 6), the CU holding 8 waves of this kernel
    constexpr int kLdsBudget = 160 * 1024 / (8 / NW) - 1024;
    constexpr int kNB = kLdsBudget / kBufBytes < 6 ? kLdsBudget / kBufBytes : 6;
    static_assert(kNB >= 3, "the ring needs three buffers");
    constexpr int kInstrA = kABytes / 1024, kInstrB = kBBytes / 1024;          // wave-wide loads per chunk
    static_assert(kInstrA % NW == 0 && kInstrB % NW == 0, "every wave issues the same number of loads per chunk");
    constexpr int kPerA = kInstrA / NW, kPerB = kInstrB / NW, kPer = kPerA + kPerB;
    constexpr int kRingBytes = kNB * kBufBytes;
    __shared__ __attribute__((aligned(1024))) uint8_t sh[kRingBytes + 1024];

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    // split_p > 1: the workgroup owns part `part` of the positions of the single sample split / split_p and
    // leaves the unsquared partial product in the workspace (the sum over the parts has to precede the square)
    const uint32_t n_chunks = (P + kKC - 1) / kKC;
    const uint32_t part = split_p > 1 ? split % split_p : 0u;
    const uint32_t chunks_per_part = (n_chunks + split_p - 1) / split_p;
    const uint32_t c_begin = min(n_chunks, part * chunks_per_part);
    // sample ranges of the splits differ by at most one sample
    const uint32_t z_begin = split_p > 1 ? split / split_p : (uint32_t)((uint64_t)split * B / splits);
    const uint32_t z_end = split_p > 1 ? z_begin + 1u : (uint32_t)((uint64_t)(split + 1u) * B / splits);
    const uint32_t total = split_p > 1 ? min(n_chunks, c_begin + chunks_per_part) - c_begin : (z_end - z_begin) * n_chunks;

    // the compiler must see a store to the array: everything else arrives behind its back
    reinterpret_cast<uint32_t*>(sh + kRingBytes)[tid & 255u] = 0u;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)sh;

    // ---- global side: which piece each lane fetches, per wave-wide load ----
    // Load ii of an operand covers rows ii * rpi .. + rpi - 1 of the chunk (1 KiB of the staged tile);
    // lane l lands on row ii * rpi + l / npr, physical piece l % npr.  What is kept per load is the byte offset
    // of the lane's piece inside the sample for the chunk requested next; one chunk further is one add.
    // In the implicit form the lane's piece of 8 columns lies inside one filter tap (Cin is a multiple
    // of 8), and the offset is that of input element (y sh + ky - ph, x sw + kx - pw) for the lane's output
    // position (y, x); x sw and y are kept beside it, for the tests against the image's edges, and a chunk
    // of kKC positions further is (step_y rows, step_x columns) with at most one carry from x into y.
    const uint32_t strideA = kImplicit ? 0u : kKC * J * 2u, strideB = kKC * C * 2u;      // bytes from chunk to chunk
    uint32_t voffA[kPerA], voffB[kPerB];
    uint32_t xsA[kPerA], yA[kPerA], xs0A[kPerA], y0A[kPerA];    // implicit: x sw and y of the lane's row; the same in a sample's first chunk
    int32_t obA[kPerA], ob0A[kPerA], tapX[kPerA];               // implicit: byte offset of the tap's element; kx - pw
    uint32_t outA[kPerA];                                       // linear: bit k set = column outside the row in chunk k of the period
    uint32_t kph = __builtin_amdgcn_readfirstlane(kLinear ? c_begin % G.period : 0u);   // chunk of the period requested next
    const int32_t dLin = (int32_t)(kKC * G.Cin * 2u);
    const uint32_t sxw = G.step_x * G.sw, WoSw = G.Wo * G.sw;
    const int32_t dO = (int32_t)((G.step_y * G.sh * G.W + sxw) * G.Cin * 2u);            // offset change per chunk, no carry
    const int32_t dOC = dO + (int32_t)(G.sh * G.W - WoSw) * (int32_t)(G.Cin * 2u);       // ... with a carry into y
#pragma unroll
    for (int j = 0; j < kPerA; ++j) {
        constexpr uint32_t npr = BM / 8, rpi = 64 / npr;
        const uint32_t ii = wave + (uint32_t)NW * j, row = ii * rpi + lane / npr, p = lane % npr;
        const uint32_t piece = (((p >> 2) ^ swizzle<BM>(row)) << 2) | (p & 3u);
        if (kImplicit) {
            // A column past J (last row tile) lands on some other element of the sample or outside it: whatever
            // comes back only reaches rows of the tile that are never stored.
            const uint32_t col = j0 + piece * 8u, tap = col / G.Cin, ky = tap / G.kw;
            const uint32_t pos0 = c_begin * kKC + row;      // the lane's row in the workgroup's first chunk
            const uint32_t y0 = pos0 / G.Wo, x0 = pos0 - y0 * G.Wo;
            tapX[j] = (int32_t)(tap - ky * G.kw) - (int32_t)G.pw;
            const int32_t tapY = (int32_t)ky - (int32_t)G.ph;
            const int32_t tapOff = (tapY * (int32_t)G.W + tapX[j]) * (int32_t)G.Cin + (int32_t)(col - tap * G.Cin);
            if (kLinear) {
                ob0A[j] = ((int32_t)(row * G.Cin) + tapOff) * 2;
                obA[j] = ob0A[j] + (int32_t)(c_begin * kKC * G.Cin * 2u);
                uint32_t x = row % G.W, bits = 0;
                const uint32_t sx = kKC % G.W;
                for (uint32_t k = 0; k < G.period; ++k) {           // chunk k of the period: is the column outside?
                    bits |= ((uint32_t)((int32_t)x + tapX[j]) < G.W ? 0u : 1u) << k;
                    x += sx;
                    x = min(x, x - G.W);
                }
                outA[j] = bits;
            } else {
                xs0A[j] = xsA[j] = x0 * G.sw;
                y0A[j] = yA[j] = y0;
                ob0A[j] = obA[j] = ((int32_t)((y0 * G.sh * G.W + x0 * G.sw) * G.Cin) + tapOff) * 2;
            }
        } else {
            voffA[j] = (row * J + j0 + piece * 8u) * 2u + c_begin * strideA;
        }
    }
#pragma unroll
    for (int j = 0; j < kPerB; ++j) {
        constexpr uint32_t npr = BN / 8, rpi = 64 / npr;
        const uint32_t ii = wave + (uint32_t)NW * j, row = ii * rpi + lane / npr, p = lane % npr;
        const uint32_t piece = (((p >> 2) ^ swizzle<BN>(row)) << 2) | (p & 3u);
        voffB[j] = (row * C + c0 + piece * 8u) * 2u + c_begin * strideB;
    }

    // ---- LDS side: fragment addresses (bytes inside a buffer) for the two 32-wide tiles of each operand ----
    const uint32_t r = lane & 15u, grp = lane >> 4, mhalf = grp & 1u, khalf = grp >> 1;
    const uint32_t frow = khalf * 8u + (r >> 2);
    uint32_t fA[2], fB[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        fA[t] = frow * (BM * 2u) + (((wm * 2u + t) ^ swizzle<BM>(frow)) * 64u) + mhalf * 32u + (r & 3u) * 8u;
        fB[t] = kABytes + frow * (BN * 2u) + (((wn * 2u + t) ^ swizzle<BN>(frow)) * 64u) + mhalf * 32u + (r & 3u) * 8u;
    }
    // fragment (ks, t) of the chunk staged at byte offset `bo`: rows ks * 16 + {0, 4} keep row % 4 and (row / 2) % 2
    auto frag_a = [&](uint32_t bo, int ks, int t) -> bf8v {
        const uint8_t* p = sh + bo + fA[t] + ks * 16 * BM * 2;
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p + 4 * BM * 2));
        s8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf8v, v);
    };
    auto frag_b = [&](uint32_t bo, int ks, int t) -> bf8v {
        const uint8_t* p = sh + bo + fB[t] + ks * 16 * BN * 2;
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p + 4 * BN * 2));
        s8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf8v, v);
    };

    f16v acc[2][2], s_acc[2][2], g_acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            acc[a][b] = (f16v){0};
            s_acc[a][b] = (f16v){0};
            if (kWantG) g_acc[a][b] = (f16v){0};
        }

    // ---- the stream of chunk requests ----
    SampleWindow wa, wb;
    if (kImplicit) wa.init(U, z_begin, G.H * G.W, G.Cin);       // the whole input of the sample
    else wa.init(U, z_begin, P, J);
    wb.init(D, z_begin, P, C);
    // where this wave's loads land inside a staged chunk
    uint32_t ldsA[kPerA], ldsB[kPerB];
#pragma unroll
    for (int j = 0; j < kPerA; ++j) ldsA[j] = __builtin_amdgcn_readfirstlane((wave + (uint32_t)NW * j) * 1024u);
#pragma unroll
    for (int j = 0; j < kPerB; ++j) ldsB[j] = __builtin_amdgcn_readfirstlane(kABytes + (wave + (uint32_t)NW * j) * 1024u);
    auto next_buf = [&](uint32_t bo) -> uint32_t { return bo + kBufBytes == (uint32_t)kRingBytes ? 0u : bo + kBufBytes; };
    // Load n (A loads first, then B loads) of the request for the next chunk, into the ring buffer at byte offset
    // bo; moves the lane's offset for that load on by one chunk.
    auto issue_one = [&](uint32_t bo, int n) {
        const uint32_t base = lds0 + bo;
        if (n < kPerA) {
            const int j = n;
            uint32_t voff;
            if (kLinear) {
                // (a position past P aliases into a valid element, but the rows of D past P read as zeros)
                voff = (uint32_t)(obA[j] | __builtin_amdgcn_sbfe((int32_t)outA[j], kph, 1u));
                obA[j] += dLin;
            } else if (kImplicit) {
                // Rows of the input above or below the image need no test: their offset is negative or past the
                // sample's range, which the buffer load answers with zeros; a column outside would alias into the
                // neighbouring row, and a position past P into a valid one, so those two are masked.
                const bool inside = ((uint32_t)((int32_t)xsA[j] + tapX[j]) < G.W) & (yA[j] < G.Ho);
                voff = (uint32_t)obA[j] | (inside ? 0u : 0xFFFFFFFFu);
                const uint32_t t = xsA[j] + sxw;
                const bool carry = t >= WoSw;
                xsA[j] = min(t, t - WoSw);
                yA[j] += G.step_y + (carry ? 1u : 0u);
                obA[j] += carry ? dOC : dO;
            } else {
                voff = voffA[j];
                voffA[j] += strideA;
            }
            load_to_lds(base, ldsA[j], voff, wa.rsrc());
        } else {
            const int j = n - kPerA;
            load_to_lds(base, ldsB[j], voffB[j], wb.rsrc());
            voffB[j] += strideB;
        }
    };
    auto request_done = [&]() {                          // after the last load of a request
        if (kLinear) kph = (kph + 1u == G.period) ? 0u : kph + 1u;
    };
    auto issue = [&](uint32_t bo) {                      // the whole request
#pragma unroll
        for (int n = 0; n < kPer; ++n) issue_one(bo, n);
        request_done();
    };
    // The rare steps, kept out of the per-chunk code: the requests cross into the next sample ...
    auto wrap = [&]() {
        wa.next_sample();
        wb.next_sample();
        kph = 0u;
#pragma unroll
        for (int j = 0; j < kPerA; ++j) {
            if (kLinear) obA[j] = ob0A[j];
            else if (kImplicit) { xsA[j] = xs0A[j]; yA[j] = y0A[j]; obA[j] = ob0A[j]; }
            else voffA[j] -= n_chunks * strideA;
        }
#pragma unroll
        for (int j = 0; j < kPerB; ++j) voffB[j] -= n_chunks * strideB;
    };
    // ... the last chunk has been requested: whatever is requested after it is zeros ...
    auto close = [&]() { wa.close(); wb.close(); };
    // ... and the per-sample product G_z is complete in acc: square into s, add into g, clear.
    auto sample_end = [&]() {
        // acc is cleared by the matrix pipe (a product of zero operands onto a zero constant) rather than by 16 moves
        // per tile: while one wave of a SIMD squares, the other one's clearing MFMAs run beside it
        const bf8v zf = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float x = acc[mt][nt][i];
                    s_acc[mt][nt][i] = __builtin_fmaf(x, x, s_acc[mt][nt][i]);
                    if (kWantG) g_acc[mt][nt][i] += x;
                }
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zf, zf, (f16v){0}, 0, 0, 0);
            }
    };
    // Ring: chunk c lives in buffer c % kNB; kNB - 1 chunks are requested up front and one more per iteration:
    // chunk q + kNB - 1 goes into the buffer of chunk q - 1, one chunk after that was consumed (the loop is
    // pipelined across its barrier, below).  A wave's loads complete in order, so once all but the loads of its
    // last kNB - 3 requests are back, its pieces of the chunk needed next are in LDS.
    constexpr int kAhead = kNB - 1;                      // requests ahead of the chunk being consumed
    constexpr int kInFlight = (kAhead - 2) * kPer;
    constexpr uint32_t kNever = 0x3FFFFFFFu;
    // chunks until: the requests reach the end of a sample, the last request, the consumed sample is complete
    uint32_t to_wrap = __builtin_amdgcn_readfirstlane(n_chunks - c_begin);
    uint32_t todo = __builtin_amdgcn_readfirstlane(total);
    {
        uint32_t bo = 0;
#pragma unroll 1
        for (int i = 0; i < kAhead; ++i) {
            issue(bo);
            bo = next_buf(bo);
            if (--to_wrap == 0) { to_wrap = n_chunks; wrap(); }
            if (--todo == 0) { todo = kNever; close(); }
        }
    }
    uint32_t left = split_p > 1 ? kNever : n_chunks;     // (with the positions split the product is stored unsquared)
    // One countdown serves the three: `span` chunks from the last rare step to the next one.
    uint32_t span = min(left, min(to_wrap, todo)), ev = span;
    auto tick = [&]() {                                  // after chunk q is consumed and chunk q + kNB requested
        if (--ev == 0) {
            left -= span; to_wrap -= span; todo -= span;
            // (a surplus chunk may complete a "sample" of zeros when P fits one chunk: it adds nothing)
            if (left == 0) { left = n_chunks; sample_end(); }
            if (to_wrap == 0) { to_wrap = n_chunks; wrap(); }
            if (todo == 0) { todo = kNever; close(); }
            span = ev = min(left, min(to_wrap, todo));
        }
    };
    {
        // One k-step (16 positions: one MFMA per 32 x 32 tile) is a phase.  While the MFMAs of a phase run, the
        // operand fragments of the next phase are read from LDS: the A fragments into the other of two register
        // sets, a B fragment into the registers of the one it replaces as soon as the two MFMAs that use it are
        // issued (MFMA order: B-major).  The workgroup meets once per chunk, between the two phases of chunk q:
        // by then every wave has its pieces of chunk q + 1 in LDS (it waits for its own loads before the barrier)
        // and has issued every MFMA of chunk q - 1, so has received every fragment of that chunk: its buffer is
        // free for the next request.  No wave waits for LDS reads still in flight at the barrier.
        wait_loads_but<kInFlight + kPer>();              // chunk 0 has landed (this wave's pieces)
        __syncthreads();
        bf8v FA[2][2], FB[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            FA[0][t] = frag_a(0, 0, t);
            FB[t] = frag_b(0, 0, t);
        }
        // The ring is unrolled: the loop body exists once per buffer, so that buffer offsets are constants and LDS
        // addresses are a lane's fragment offset plus an immediate.
        for (uint32_t q0 = 0; q0 < total; q0 += kNB) {
#pragma unroll
            for (int b = 0; b < kNB; ++b) {
            if (q0 + (uint32_t)b >= total) break;
            const uint32_t bo_cur = (uint32_t)b * kBufBytes, bo_next = (uint32_t)((b + 1) % kNB) * kBufBytes;
            const uint32_t bo_prev = (uint32_t)((b + kNB - 1) % kNB) * kBufBytes;
            // phase 0: k-step 0 of chunk q; fragments of its k-step 1
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[0][mt], FB[nt], acc[mt][nt], 0, 0, 0);
                    if (nt == 0) FA[1][mt] = frag_a(bo_cur, 1, mt);
                }
                FB[nt] = frag_b(bo_cur, 1, nt);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // MFMA, A', MFMA, A' B', MFMA, MFMA, B'
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            wait_loads_but<kInFlight>();                 // chunk q + 1 has landed (this wave's pieces)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // phase 1: k-step 1 of chunk q; fragments of k-step 0 of chunk q + 1; the request for chunk
            // q + kNB - 1, spread over the phase
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[1][mt], FB[nt], acc[mt][nt], 0, 0, 0);
                    if (nt == 0) FA[0][mt] = frag_a(bo_next, 0, mt);
                    const int i = nt * 2 + mt;
#pragma unroll
                    for (int n = 0; n < kPer; ++n)
                        if (i == (n * 4) / kPer) issue_one(bo_prev, n);
                }
                FB[nt] = frag_b(bo_next, 0, nt);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            request_done();
            tick();
            }
        }
    }
    wait_loads_but<0>();                                 // nothing may still be landing when the workgroup ends

    // ---- epilogue: scaled result, or unscaled partial sums for the fixed-order reduction, or (split_p > 1) the
    // partial per-sample product ----
    const bool direct = (splits == 1);
    const size_t JC = (size_t)J * C;
    float* so = direct ? s_out : ws + (size_t)split * 2 * JC;
    float* go = direct ? g_out : ws + (size_t)split * 2 * JC + JC;
    if (split_p > 1) so = ws + (size_t)split * JC;
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
                    if (split_p > 1) {
                        __builtin_nontemporal_store(acc[mt][nt][i], so + o);
                    } else if (direct) {
                        __builtin_nontemporal_store(fs * s_acc[mt][nt][i], so + o);
                        if (kWantG) __builtin_nontemporal_store(fg * g_acc[mt][nt][i], go + o);
                    } else {                             // read again at once by the reduction: leave it in the caches
                        so[o] = s_acc[mt][nt][i];
                        if (kWantG) go[o] = g_acc[mt][nt][i];
                    }
                }
            }
        }
}

// kV consecutive floats (kV = 1 or 4) as one load or store.
template <int kV> struct FloatVec { float v[kV]; };
template <int kV> __device__ __forceinline__ FloatVec<kV> load_vec(const float* p) {
    FloatVec<kV> r;
    if constexpr (kV == 4) { const f4v t = *reinterpret_cast<const f4v*>(p); r.v[0] = t[0]; r.v[1] = t[1]; r.v[2] = t[2]; r.v[3] = t[3]; }
    else r.v[0] = *p;
    return r;
}
template <int kV> __device__ __forceinline__ void store_vec(float* p, const FloatVec<kV>& r) {
    if constexpr (kV == 4) *reinterpret_cast<f4v*>(p) = (f4v){r.v[0], r.v[1], r.v[2], r.v[3]};
    else *p = r.v[0];
}

// Adds the per-split partial sums in a fixed order and applies the scale factors.  `lanes` (1 or 4) threads
// share kV consecutive outputs: thread (outputs, lane q) takes splits q, q + lanes, ..., and the lanes' sums are
// added in lane order.  A workgroup owns 256 / lanes * kV consecutive outputs; JC is a multiple of kV.
template <int kV>
__global__ __launch_bounds__(256) void k_sqgrad_reduce(const float* __restrict__ ws, uint32_t splits, size_t JC,
                                                       float cg, float cs, float* __restrict__ g_out,
                                                       float* __restrict__ s_out, uint32_t lanes) {
    __shared__ FloatVec<kV> sh_s[256], sh_g[256];
    const uint32_t opb = 256u / lanes, il = threadIdx.x % opb, q = threadIdx.x / opb;
    const size_t i = ((size_t)blockIdx.x * opb + il) * kV;
    FloatVec<kV> s = {}, g = {};
    if (i < JC) {
        for (uint32_t k = q; k < splits; k += lanes) {
            const FloatVec<kV> ps = load_vec<kV>(ws + (size_t)k * 2 * JC + i);
            for (int e = 0; e < kV; ++e) s.v[e] += ps.v[e];
            if (g_out) {
                const FloatVec<kV> pg = load_vec<kV>(ws + (size_t)k * 2 * JC + JC + i);
                for (int e = 0; e < kV; ++e) g.v[e] += pg.v[e];
            }
        }
    }
    sh_s[threadIdx.x] = s;
    sh_g[threadIdx.x] = g;
    __syncthreads();
    if (q == 0 && i < JC) {
        FloatVec<kV> st = {}, gt = {};
        for (uint32_t k = 0; k < lanes; ++k)
            for (int e = 0; e < kV; ++e) { st.v[e] += sh_s[k * opb + il].v[e]; gt.v[e] += sh_g[k * opb + il].v[e]; }
        for (int e = 0; e < kV; ++e) { st.v[e] *= cs; gt.v[e] *= cg; }
        store_vec<kV>(s_out + i, st);
        if (g_out) store_vec<kV>(g_out + i, gt);
    }
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

// Sums the parts of every sample's product, then squares and sums over the samples, in a fixed order: a
// workgroup owns 16 kV consecutive outputs; thread (outputs, lane q) takes samples q, q + 16, ..., and the 16
// lanes' sums are added in lane order.  JC is a multiple of kV.
template <int kV>
__global__ __launch_bounds__(256) void k_sqgrad_reduce_parts(const float* __restrict__ ws, uint32_t B, uint32_t split_p, size_t JC,
                                                             float cg, float cs, float* __restrict__ g_out,
                                                             float* __restrict__ s_out) {
    __shared__ FloatVec<kV> sh_s[16][17], sh_g[16][17];
    const uint32_t il = threadIdx.x & 15u, q = threadIdx.x >> 4;
    const size_t i = ((size_t)blockIdx.x * 16 + il) * kV;
    FloatVec<kV> s = {}, g = {};
    if (i < JC) {
        for (uint32_t z = q; z < B; z += 16) {
            FloatVec<kV> G = {};
#pragma unroll 4                                     // (the loads of four parts in flight; the additions keep their order)
            for (uint32_t k = 0; k < split_p; ++k) {
                const FloatVec<kV> part = load_vec<kV>(ws + ((size_t)z * split_p + k) * JC + i);
                for (int e = 0; e < kV; ++e) G.v[e] += part.v[e];
            }
            for (int e = 0; e < kV; ++e) { s.v[e] = __builtin_fmaf(G.v[e], G.v[e], s.v[e]); g.v[e] += G.v[e]; }
        }
    }
    sh_s[q][il] = s;
    sh_g[q][il] = g;
    __syncthreads();
    if (q == 0 && i < JC) {
        FloatVec<kV> st = {}, gt = {};
        for (int k = 0; k < 16; ++k)
            for (int e = 0; e < kV; ++e) { st.v[e] += sh_s[k][il].v[e]; gt.v[e] += sh_g[k][il].v[e]; }
        for (int e = 0; e < kV; ++e) { st.v[e] *= cs; gt.v[e] *= cg; }
        store_vec<kV>(s_out + i, st);
        if (g_out) store_vec<kV>(g_out + i, gt);
    }
}

static uint64_t conv_slots(const ConvTile& t) {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n_cu = v;
        else n_cu = 256;
    }
    const uint64_t waves_per_wg = (uint64_t)(t.bm / 64) * (t.bn / 64);
    return (uint64_t)n_cu * (8 / waves_per_wg);
}

// How many ways to split the samples.  Workgroups run in rounds of `slots` (compute units x resident
// workgroups); the cost of a choice is rounds x samples per workgroup, plus one pass over the partial
// sums per split for the reduction (weighted as a fraction of one sample's work on a tile).
uint32_t conv_splits(uint32_t B, uint32_t J, uint32_t C) {
    const ConvTile t = conv_tile(J, C);
    const uint64_t tiles = (uint64_t)((J + t.bm - 1) / t.bm) * ((C + t.bn - 1) / t.bn);
    const uint64_t slots = conv_slots(t);
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

// When [J, C] has so few tiles that one workgroup per (tile, sample) fills at most two thirds of the chip's
// workgroup slots, the positions of a sample are split as well (at least eight chunks per part): up to half a
// round into as many parts as fill one round, beyond that into two or three parts, just under two rounds
// (measured on the box; above two thirds of a round the split does not pay).  1 = no split over positions.
uint32_t conv_split_p(uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    const ConvTile t = conv_tile(J, C);
    const uint64_t tiles = (uint64_t)((J + t.bm - 1) / t.bm) * ((C + t.bn - 1) / t.bn);
    const uint64_t slots = conv_slots(t);
    const uint32_t n_chunks = (P + kKC - 1) / kKC;
    if (tiles * B * 3 > slots * 2 || n_chunks < 16) return 1;
    // up to half a round: as many parts as fill one round; up to two thirds: just under two rounds
    const uint64_t sp = tiles * B * 2 <= slots ? slots / (tiles * B) : 2 * slots / (tiles * B);
    return (uint32_t)(sp < n_chunks / 8 ? sp : n_chunks / 8);
}

// Workspace the tiled bf16 conv kernel wants for a shape (0: none).
size_t conv_workspace_bytes(uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    const uint32_t sp = conv_split_p(B, P, J, C);
    if (sp > 1) return (size_t)B * sp * J * C * sizeof(float);
    const uint32_t splits = conv_splits(B, J, C);
    return splits > 1 ? (size_t)splits * 2 * J * C * sizeof(float) : 0;
}

size_t sqgrad_workspace_bytes(int kind, int dtype, uint32_t B, uint32_t P, uint32_t J, uint32_t C) {
    if (kind != VGC_CONV) return 0;
    if (conv_tiled_supported(dtype, P, J, C)) return conv_workspace_bytes(B, P, J, C);
    if (dtype == VGC_F32 && conv_f32_tiled_supported(P, J, C)) return conv_f32_workspace_bytes(B, P, J, C);
    return 0;
}

bool conv_tiled_supported(int dtype, uint32_t P, uint32_t J, uint32_t C) {
    const uint64_t limit = 0x7FFFFFFFull;               // buffer ranges and offsets are 32-bit
    return dtype == VGC_BF16 && (J % 8 == 0) && (C % 8 == 0) && (uint64_t)(P + 64) * J * 2 < limit &&
           (uint64_t)(P + 64) * C * 2 < limit;
}

// Four outputs per thread when the planes and the outputs allow 16-byte accesses.
static bool reduce_vec4(const float* ws, size_t JC, const float* g_out, const float* s_out) {
    return JC % 4 == 0 && (((uintptr_t)ws | (uintptr_t)g_out | (uintptr_t)s_out) & 15u) == 0;
}

void launch_sqgrad_reduce_parts(const float* ws, uint32_t B, uint32_t split_p, size_t JC, float cg, float cs, float* g_out,
                                float* s_out, hipStream_t stream) {
    if (reduce_vec4(ws, JC, g_out, s_out))
        hipLaunchKernelGGL(k_sqgrad_reduce_parts<4>, dim3((uint32_t)((JC / 4 + 15) / 16)), dim3(256), 0, stream, ws, B, split_p, JC,
                           cg, cs, g_out, s_out);
    else
        hipLaunchKernelGGL(k_sqgrad_reduce_parts<1>, dim3((uint32_t)((JC + 15) / 16)), dim3(256), 0, stream, ws, B, split_p, JC, cg,
                           cs, g_out, s_out);
}

void launch_sqgrad_reduce(const float* ws, uint32_t splits, size_t JC, float cg, float cs, float* g_out, float* s_out,
                          hipStream_t stream) {
    const uint32_t lanes = splits <= 4 ? 1u : 4u;        // (16 lanes for more than 16 splits read 256-byte runs: 15 against 12.5 us on 32 planes of 1 MB)
    const uint32_t opb = 256u / lanes;
    if (reduce_vec4(ws, JC, g_out, s_out))
        hipLaunchKernelGGL(k_sqgrad_reduce<4>, dim3((uint32_t)((JC / 4 + opb - 1) / opb)), dim3(256), 0, stream, ws, splits, JC, cg,
                           cs, g_out, s_out, lanes);
    else
        hipLaunchKernelGGL(k_sqgrad_reduce<1>, dim3((uint32_t)((JC + opb - 1) / opb)), dim3(256), 0, stream, ws, splits, JC, cg, cs,
                           g_out, s_out, lanes);
}

// ------------------------------------------------------------------------------------------------
// 3 x 3 filters with unit stride and padding 1 on few input channels (the first layers of a VGG-like
// network: 64 or 128 channels at 224^2 and 112^2 positions).  In the kernel above such a layer is bound by
// the feed: its block tile is small (J = 9 Cin has few 128-column tiles and C is narrow), and the nine
// taps of the filter fetch the same input elements nine times through the load path.  Here a workgroup
// owns ALL nine taps of a block of 64 input channels, times 64 output channels (a 576 x 64 tile of
// [J, C]), and stages the distinct input block of a chunk once: for 16 consecutive output positions of one
// output row that is 3 input rows x 18 columns x 64 channels, and the fragment of tap (ky, kx) is read
// from it at a constant offset, (ky 18 + kx) staged pixels further.  A chunk is two such halves of 16
// positions (one k-step each; W is a multiple of 16, so a half never crosses an output row): 2 x (54
// pixels x 128 bytes) of input and 2 x (16 x 128 bytes) of output gradient = 18 KiB for 576 x 64 x 32
// multiply-adds, against 40 KiB through the generic path.
//
// Twelve waves, three per SIMD: wave w takes column half cb = w % 2 of the 64 output channels and the
// three 32-row blocks jb = 3 (w / 2) + {0, 1, 2} of the 18 (tap, channel half) blocks: three MFMAs per
// k-step from three U fragments and one D fragment.  The 14 + 4 wave-wide loads of a chunk are dealt to
// the waves in order: waves 0..5 issue two, waves 6..11 one (the loop exists once per count, since a
// wave waits for its own loads by their number).  Pipeline, ring, sample bookkeeping, splits and the
// reduction kernels are those of the kernel above.  s only: the variant with g stays with that kernel.
// Staged layout of one chunk: [half 0: 56 pixel slots x 128 B][half 1][D half 0: 16 rows x 128 B][D half 1];
// slot = 18 ry + rx for input row y - 1 + ry and column x0 - 1 + rx, slots 54 and 55 unused.  The 64-byte
// halves of a slot (channels 0..31, 32..63) are swapped in slots with (slot / 2) odd, so that the four
// consecutive slots a transposing read touches fall on different banks.
constexpr int kTapHalfA = 56 * 128, kTapHalfB = 16 * 128, kTapBuf = 2 * kTapHalfA + 2 * kTapHalfB;
constexpr int kTapNB = 6, kTapWaves = 12;

__global__ __launch_bounds__(kTapWaves * 64, 3)
void k_conv_taps_bf16(const uint16_t* __restrict__ U, const uint16_t* __restrict__ D, uint32_t B, uint32_t H, uint32_t W,
                      uint32_t Cin, uint32_t C, uint32_t period, uint32_t splits, uint32_t split_p, float cs,
                      float* __restrict__ s_out, float* __restrict__ ws) {
    constexpr int kNB = kTapNB, kBufBytes = kTapBuf, kRingBytes = kNB * kBufBytes;
    __shared__ __attribute__((aligned(1024))) uint8_t sh[kRingBytes + 1024];
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t P = H * W, J = 9u * Cin;
    const uint32_t tiles_c = C / 64u, tiles_cb = Cin / 64u;
    // every XCD a contiguous range of (split, channel block, column tile): see the kernel above
    const uint32_t nblk = gridDim.x, per = nblk / 8u, rem = nblk % 8u;
    const uint32_t xcd = blockIdx.x % 8u, slot_x = blockIdx.x / 8u;
    const uint32_t logical = xcd * per + min(xcd, rem) + slot_x;
    const uint32_t tile_c = logical % tiles_c, tile_cb = (logical / tiles_c) % tiles_cb, split = logical / (tiles_c * tiles_cb);
    const uint32_t n_chunks = (P + kKC - 1) / kKC;
    const uint32_t part = split_p > 1 ? split % split_p : 0u;
    const uint32_t chunks_per_part = (n_chunks + split_p - 1) / split_p;
    const uint32_t c_begin = min(n_chunks, part * chunks_per_part);
    const uint32_t z_begin = split_p > 1 ? split / split_p : (uint32_t)((uint64_t)split * B / splits);
    const uint32_t z_end = split_p > 1 ? z_begin + 1u : (uint32_t)((uint64_t)(split + 1u) * B / splits);
    const uint32_t total = split_p > 1 ? min(n_chunks, c_begin + chunks_per_part) - c_begin : (z_end - z_begin) * n_chunks;

    reinterpret_cast<uint32_t*>(sh + kRingBytes)[tid & 255u] = 0u;      // the compiler must see a store to the array
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)sh;

    // ---- LDS side: fragment addresses inside a staged chunk ----
    const uint32_t r = lane & 15u, grp = lane >> 4, mhalf = grp & 1u, khalf = grp >> 1;
    const uint32_t frow = khalf * 8u + (r >> 2);                 // position inside the half (second read: + 4)
    const uint32_t cb = wave & 1u, jgrp = wave >> 1;
    uint32_t fA[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        const uint32_t jb = 3u * jgrp + (uint32_t)t, tap = jb >> 1, chb = jb & 1u, ky = tap / 3u, kx = tap - 3u * ky;
        const uint32_t s0 = ky * 18u + kx + frow;                // staged slot of the fragment's first row
        fA[t] = s0 * 128u + ((chb ^ ((s0 >> 1) & 1u)) * 64u) + mhalf * 32u + (r & 3u) * 8u;
    }
    const uint32_t fB = 2u * kTapHalfA + frow * 128u + ((cb ^ ((frow >> 1) & 1u)) * 64u) + mhalf * 32u + (r & 3u) * 8u;
    auto frag_a = [&](uint32_t bo, int ks, int t) -> bf8v {      // slots s and s + 4 share the swizzle
        const uint8_t* p = sh + bo + fA[t] + ks * kTapHalfA;
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p + 4 * 128));
        s8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf8v, v);
    };
    auto frag_b = [&](uint32_t bo, int ks) -> bf8v {
        const uint8_t* p = sh + bo + fB + ks * kTapHalfB;
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(p + 4 * 128));
        s8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf8v, v);
    };

    f16v acc[3], s_acc[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) { acc[t] = (f16v){0}; s_acc[t] = (f16v){0}; }

    SampleWindow wa, wb;
    wa.init(U, z_begin, P, Cin);                                 // the whole input of the sample
    wb.init(D, z_begin, P, C);

    auto run = [&](auto per_tag) __attribute__((always_inline)) {
        constexpr int kPer = decltype(per_tag)::value;
        // ---- global side: load n of this wave is load L = wave + 12 n of the chunk's 18; L < 14: input pixels of
        // half L / 7, slots 8 (L % 7) .. + 7; else output-gradient rows 8 ((L - 14) % 2) .. + 7 of half (L - 14) / 2.
        // Per load the lane keeps the byte offset of its 16-byte piece inside the sample for the chunk requested
        // next (it advances by a constant per chunk), the offset in a sample's first chunk, and for input pixels
        // one bit per chunk of the period saying that the pixel's column lies outside the row.
        uint32_t ob[kPer], ob0[kPer], step[kPer], outside[kPer], ldsoff[kPer];
        bool is_a[kPer];
        uint32_t kph = __builtin_amdgcn_readfirstlane(c_begin % period);
#pragma unroll
        for (int n = 0; n < kPer; ++n) {
            const uint32_t L = wave + (uint32_t)kTapWaves * n, p = lane & 7u;
            is_a[n] = L < 14u;
            if (is_a[n]) {
                const uint32_t h = L / 7u, i = L - 7u * h, slot = i * 8u + (lane >> 3);
                const uint32_t piece = (((p >> 2) ^ ((slot >> 1) & 1u)) << 2) | (p & 3u);
                const uint32_t ry = slot / 18u, rx = slot - 18u * ry;
                const int32_t pix = (int32_t)(16u * h) + ((int32_t)ry - 1) * (int32_t)W + (int32_t)rx - 1;
                ob0[n] = (uint32_t)((pix * (int32_t)Cin + (int32_t)(tile_cb * 64u + piece * 8u)) * 2);
                step[n] = kKC * Cin * 2u;
                uint32_t bits = 0, x0 = (16u * h) % W;
                for (uint32_t k = 0; k < period; ++k) {          // chunk k of the period: is the column outside?
                    bits |= ((uint32_t)((int32_t)x0 + (int32_t)rx - 1) < W ? 0u : 1u) << k;
                    x0 = (x0 + kKC) % W;
                }
                outside[n] = slot < 54u ? bits : 0xFFFFFFFFu;
                ldsoff[n] = __builtin_amdgcn_readfirstlane(h * kTapHalfA + i * 1024u);
            } else {
                const uint32_t q = L - 14u, h = q >> 1, row = (q & 1u) * 8u + (lane >> 3);
                const uint32_t piece = (((p >> 2) ^ ((row >> 1) & 1u)) << 2) | (p & 3u);
                ob0[n] = ((16u * h + row) * C + tile_c * 64u + piece * 8u) * 2u;
                step[n] = kKC * C * 2u;
                outside[n] = 0u;
                ldsoff[n] = __builtin_amdgcn_readfirstlane(2u * kTapHalfA + h * kTapHalfB + (q & 1u) * 1024u);
            }
            ob[n] = ob0[n] + c_begin * step[n];
        }
        auto issue_one = [&](uint32_t bo, int n) {
            // rows of the input above or below the image need no test: their offset is negative or past the sample's
            // range and reads as zeros; a column outside would alias into the neighbouring row and is masked; a
            // position past P aliases into a valid pixel, but the rows of D past P read as zeros
            const uint32_t voff = ob[n] | (uint32_t)__builtin_amdgcn_sbfe((int32_t)outside[n], kph, 1u);
            ob[n] += step[n];
            const i4v ra = wa.rsrc(), rb = wb.rsrc();
            i4v rs;
#pragma unroll
            for (int e = 0; e < 4; ++e) rs[e] = is_a[n] ? ra[e] : rb[e];
            load_to_lds(lds0 + bo, ldsoff[n], voff, rs);
        };
        auto request_done = [&]() { kph = (kph + 1u == period) ? 0u : kph + 1u; };
        auto issue = [&](uint32_t bo) {
#pragma unroll
            for (int n = 0; n < kPer; ++n) issue_one(bo, n);
            request_done();
        };
        auto wrap = [&]() {
            wa.next_sample();
            wb.next_sample();
            kph = 0u;
#pragma unroll
            for (int n = 0; n < kPer; ++n) ob[n] = ob0[n];
        };
        auto close = [&]() { wa.close(); wb.close(); };
        auto sample_end = [&]() {
            const bf8v zf = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int t = 0; t < 3; ++t) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float x = acc[t][i];
                    s_acc[t][i] = __builtin_fmaf(x, x, s_acc[t][i]);
                }
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zf, zf, (f16v){0}, 0, 0, 0);
            }
        };
        constexpr int kAhead = kNB - 1;
        constexpr int kInFlight = (kAhead - 2) * kPer;
        constexpr uint32_t kNever = 0x3FFFFFFFu;
        auto next_buf = [&](uint32_t bo) -> uint32_t { return bo + kBufBytes == (uint32_t)kRingBytes ? 0u : bo + kBufBytes; };
        uint32_t to_wrap = __builtin_amdgcn_readfirstlane(n_chunks - c_begin);
        uint32_t todo = __builtin_amdgcn_readfirstlane(total);
        {
            uint32_t bo = 0;
#pragma unroll 1
            for (int i = 0; i < kAhead; ++i) {
                issue(bo);
                bo = next_buf(bo);
                if (--to_wrap == 0) { to_wrap = n_chunks; wrap(); }
                if (--todo == 0) { todo = kNever; close(); }
            }
        }
        uint32_t left = split_p > 1 ? kNever : n_chunks;
        uint32_t span = min(left, min(to_wrap, todo)), ev = span;
        auto tick = [&]() {
            if (--ev == 0) {
                left -= span; to_wrap -= span; todo -= span;
                if (left == 0) { left = n_chunks; sample_end(); }
                if (to_wrap == 0) { to_wrap = n_chunks; wrap(); }
                if (todo == 0) { todo = kNever; close(); }
                span = ev = min(left, min(to_wrap, todo));
            }
        };
        wait_loads_but<kInFlight + kPer>();                      // chunk 0 has landed (this wave's pieces)
        __syncthreads();
        bf8v FA[2][3], FB[2];
#pragma unroll
        for (int t = 0; t < 3; ++t) FA[0][t] = frag_a(0, 0, t);
        FB[0] = frag_b(0, 0);
        for (uint32_t q0 = 0; q0 < total; q0 += kNB) {
#pragma unroll
            for (int b = 0; b < kNB; ++b) {
            if (q0 + (uint32_t)b >= total) break;
            const uint32_t bo_cur = (uint32_t)b * kBufBytes, bo_next = (uint32_t)((b + 1) % kNB) * kBufBytes;
            const uint32_t bo_prev = (uint32_t)((b + kNB - 1) % kNB) * kBufBytes;
            // phase 0: half 0 of chunk q; fragments of its half 1
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[0][t], FB[0], acc[t], 0, 0, 0);
                FA[1][t] = frag_a(bo_cur, 1, t);
                if (t == 2) FB[1] = frag_b(bo_cur, 1);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            wait_loads_but<kInFlight>();                         // chunk q + 1 has landed (this wave's pieces)
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // phase 1: half 1 of chunk q; fragments of half 0 of chunk q + 1; the request for chunk q + kNB - 1
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[1][t], FB[1], acc[t], 0, 0, 0);
                FA[0][t] = frag_a(bo_next, 0, t);
                if (t == 2) FB[0] = frag_b(bo_next, 0);
#pragma unroll
                for (int n = 0; n < kPer; ++n)
                    if (t == (n * 3) / kPer) issue_one(bo_prev, n);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            request_done();
            tick();
            }
        }
        wait_loads_but<0>();                                     // nothing may still be landing when the workgroup ends
    };
    if (wave < 6u) run(std::integral_constant<int, 2>{});
    else run(std::integral_constant<int, 1>{});

    // ---- epilogue: scaled result, unscaled partial sums for the fixed-order reduction, or (split_p > 1) the partial
    // per-sample product ----
    const bool direct = (splits == 1);
    const size_t JC = (size_t)J * C;
    float* so = direct ? s_out : ws + (size_t)split * 2 * JC;
    if (split_p > 1) so = ws + (size_t)split * JC;
    const float fs = direct ? cs : 1.0f;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        const uint32_t jb = 3u * jgrp + (uint32_t)t, tap = jb >> 1, chb = jb & 1u;
        const uint32_t col = tile_c * 64u + cb * 32u + (lane & 31u);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t row = tap * Cin + tile_cb * 64u + chb * 32u + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
            const size_t o = (size_t)row * C + col;
            if (split_p > 1) __builtin_nontemporal_store(acc[t][i], so + o);
            else if (direct) __builtin_nontemporal_store(fs * s_acc[t][i], so + o);
            else so[o] = s_acc[t][i];
        }
    }
}

template <int BM, int BN, bool kImplicit, bool kLinear = false>
static void launch_conv_bf16(uint32_t nblk, hipStream_t stream, const void* X, const void* D, uint32_t B, uint32_t P,
                             uint32_t J, uint32_t C, uint32_t splits, uint32_t split_p, float cg, float cs,
                             float* g_out, float* s_out, float* ws, const ConvGeom& G) {
    constexpr int NT = (BM / 64) * (BN / 64) * 64;
    // with the positions split the partial products are unsquared: the variant without g serves both
    if (g_out && split_p == 1)
        hipLaunchKernelGGL((k_conv_bf16<BM, BN, true, kImplicit, kLinear>), dim3(nblk), dim3(NT), 0, stream, (const uint16_t*)X,
                           (const uint16_t*)D, B, P, J, C, splits, split_p, cg, cs, g_out, s_out, ws, G);
    else
        hipLaunchKernelGGL((k_conv_bf16<BM, BN, false, kImplicit, kLinear>), dim3(nblk), dim3(NT), 0, stream, (const uint16_t*)X,
                           (const uint16_t*)D, B, P, J, C, splits, split_p, cg, cs, g_out, s_out, ws, G);
}

template <bool kImplicit>
static int launch_conv_any(const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C, float c,
                           float* g_out, float* s_out, void* workspace, size_t workspace_bytes, const ConvGeom& G,
                           hipStream_t stream) {
    const ConvTile t = conv_tile(J, C);
    const size_t JC = (size_t)J * C;
    uint32_t split_p = conv_split_p(B, P, J, C);
    if (split_p > 1 && (!workspace || workspace_bytes < (size_t)B * split_p * JC * sizeof(float))) split_p = 1;
    uint32_t splits = split_p > 1 ? B * split_p : conv_splits(B, J, C);
    if (split_p == 1 && splits > 1 && (!workspace || workspace_bytes < (size_t)splits * 2 * JC * sizeof(float))) splits = 1;
    const uint64_t nblk = (uint64_t)((C + t.bn - 1) / t.bn) * ((J + t.bm - 1) / t.bm) * splits;
    if (nblk > 0x7FFFFFFFull) { set_error("vgc_sqgrad: shape exceeds the launch limit"); return VGC_ERR_SIZE; }
    const float cg = c, cs = c * c;
    float* ws = static_cast<float*>(workspace);
#define VGC_LAUNCH_BF16(BM_, BN_)                                                                                          \
    do {                                                                                                                   \
        if (kImplicit && G.period > 0)                                                                                     \
            launch_conv_bf16<BM_, BN_, kImplicit, kImplicit>((uint32_t)nblk, stream, X, D, B, P, J, C, splits, split_p, cg, \
                                                             cs, g_out, s_out, ws, G);                                     \
        else                                                                                                               \
            launch_conv_bf16<BM_, BN_, kImplicit, false>((uint32_t)nblk, stream, X, D, B, P, J, C, splits, split_p, cg, cs, \
                                                         g_out, s_out, ws, G);                                             \
    } while (0)
    if (t.bm == 256 && t.bn == 128) VGC_LAUNCH_BF16(256, 128);
    else if (t.bm == 256 && t.bn == 64) VGC_LAUNCH_BF16(256, 64);
    else if (t.bm == 128 && t.bn == 128) VGC_LAUNCH_BF16(128, 128);
    else VGC_LAUNCH_BF16(128, 64);
#undef VGC_LAUNCH_BF16
    if (split_p > 1) {
        launch_sqgrad_reduce_parts(ws, B, split_p, JC, cg, cs, g_out, s_out, stream);
        return hip_check(hipGetLastError(), "launch k_conv_bf16");
    }
    if (splits > 1) launch_sqgrad_reduce(ws, splits, (size_t)J * C, cg, cs, g_out, s_out, stream);
    return hip_check(hipGetLastError(), "launch k_conv_bf16");
}

// ---- the 3 x 3 kernel for few input channels: when it applies, how it splits, what workspace it wants ----
static uint32_t taps_period(uint32_t W) {
    uint32_t a = W, b = kKC % W;
    while (b) { const uint32_t t = a % b; a = b; b = t; }
    return W / a;
}

bool conv_taps_supported(uint32_t H, uint32_t W, uint32_t Cin, uint32_t C, uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw,
                         uint32_t ph, uint32_t pw) {
    (void)H;
    return kh == 3 && kw == 3 && sh == 1 && sw == 1 && ph == 1 && pw == 1 && (Cin == 64 || Cin == 128) && C % 64 == 0 &&
           W % 16 == 0 && taps_period(W) <= 32;
}

struct TapsSplit { uint32_t splits, split_p; };
static TapsSplit taps_split(uint32_t B, uint32_t P, uint32_t Cin, uint32_t C) {
    const uint64_t tiles = (uint64_t)(Cin / 64) * (C / 64);
    ConvTile one_per_cu; one_per_cu.bm = 256; one_per_cu.bn = 128;      // eight waves' worth of slots: one workgroup per compute unit
    const uint64_t slots = conv_slots(one_per_cu);
    const uint32_t n_chunks = (P + kKC - 1) / kKC;
    TapsSplit r; r.splits = 1; r.split_p = 1;
    if (tiles * B * 3 <= slots * 2 && n_chunks >= 16) {                 // the same rule as conv_split_p
        const uint64_t sp = tiles * B * 2 <= slots ? slots / (tiles * B) : 2 * slots / (tiles * B);
        r.split_p = (uint32_t)(sp < n_chunks / 8 ? sp : n_chunks / 8);
    }
    if (r.split_p > 1) { r.splits = B * r.split_p; return r; }
    double best = 1e300;                                                // the same cost as conv_splits
    for (uint32_t s = 1; s <= B; ++s) {
        const uint32_t zper = (B + s - 1) / s, s2 = (B + zper - 1) / zper;
        if (s2 != s) continue;
        const uint64_t rounds = (tiles * s2 + slots - 1) / slots;
        const double cost = (double)rounds * zper + (s2 > 1 ? 0.5 * s2 * (double)tiles / slots + 0.5 : 0.0);
        if (cost < best - 1e-9) { best = cost; r.splits = s2; }
    }
    return r;
}

size_t conv_taps_workspace_bytes(uint32_t B, uint32_t P, uint32_t Cin, uint32_t C) {
    const TapsSplit t = taps_split(B, P, Cin, C);
    const size_t JC = (size_t)9 * Cin * C;
    if (t.split_p > 1) return (size_t)B * t.split_p * JC * sizeof(float);
    return t.splits > 1 ? (size_t)t.splits * 2 * JC * sizeof(float) : 0;
}

// false: the workspace is too small for this kernel's split (the caller takes the generic path)
static bool launch_conv_taps(const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C,
                             float c, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    const uint32_t P = H * W;
    const TapsSplit t = taps_split(B, P, Cin, C);
    if (conv_taps_workspace_bytes(B, P, Cin, C) > (workspace ? workspace_bytes : 0)) return false;
    const size_t JC = (size_t)9 * Cin * C;
    const uint64_t nblk = (uint64_t)(Cin / 64) * (C / 64) * t.splits;
    if (nblk > 0x7FFFFFFFull) return false;
    float* ws = static_cast<float*>(workspace);
    const float cs = c * c;
    hipLaunchKernelGGL(k_conv_taps_bf16, dim3((uint32_t)nblk), dim3(kTapWaves * 64), 0, stream, (const uint16_t*)act,
                       (const uint16_t*)D, B, H, W, Cin, C, taps_period(W), t.splits, t.split_p, cs, s_out, ws);
    if (t.split_p > 1) launch_sqgrad_reduce_parts(ws, B, t.split_p, JC, c, cs, nullptr, s_out, stream);
    else if (t.splits > 1) launch_sqgrad_reduce(ws, t.splits, JC, c, cs, nullptr, s_out, stream);
    return true;
}

int launch_conv_tiled(int dtype, const void* X, const void* D, uint32_t B, uint32_t P, uint32_t J, uint32_t C,
                      float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    (void)dtype;
    return launch_conv_any<false>(X, D, B, P, J, C, c, g_out, s_out, workspace, workspace_bytes, ConvGeom{}, stream);
}

bool conv2d_supported(int dtype, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C, uint32_t P) {
    const uint64_t limit = 0x7FFFFFFFull;               // buffer ranges and offsets are 32-bit
    // the fp32 kernel's address arithmetic multiplies (y sh W + x sw) by Cin with 24-bit multiplies; the same
    // limits keep the bf16 kernel's incremental offsets inside 32 bits
    const uint64_t m24 = 1u << 23;
    const uint64_t es = dtype == VGC_BF16 ? 2 : 4, piece = 16 / es;
    return (dtype == VGC_BF16 || dtype == VGC_F32) && (Cin % piece == 0) && (C % piece == 0) &&
           (uint64_t)H * W * Cin * es < limit && (uint64_t)(P + 64) * C * es < limit &&
           (uint64_t)(H + 64) * (W + 64) < m24 && Cin < m24;
}

int launch_conv2d(int dtype, const void* act, const void* D, uint32_t B, uint32_t H, uint32_t W, uint32_t Cin, uint32_t C,
                  uint32_t kh, uint32_t kw, uint32_t sh, uint32_t sw, uint32_t ph, uint32_t pw, uint32_t Ho, uint32_t Wo,
                  float c, float* g_out, float* s_out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    if (conv_stem_supported(dtype, Cin, C, kh, kw))
        return launch_conv_stem(dtype, act, D, B, H, W, Cin, C, kh, kw, sh, sw, ph, pw, Ho, Wo, c, g_out, s_out, workspace,
                                workspace_bytes, stream);
    ConvGeom G{};
    G.H = H; G.W = W; G.Cin = Cin; G.kw = kw; G.sh = sh; G.sw = sw; G.ph = ph; G.pw = pw; G.Ho = Ho; G.Wo = Wo;
    if (dtype == VGC_F32) return launch_conv2d_f32(act, D, B, Ho * Wo, kh * kw * Cin, C, c, g_out, s_out, workspace, workspace_bytes, G, stream);
    // s alone of a 3 x 3 layer on 64 or 128 channels: the kernel that stages the input block once for all nine taps
    if (!g_out && conv_taps_supported(H, W, Cin, C, kh, kw, sh, sw, ph, pw) &&
        launch_conv_taps(act, D, B, H, W, Cin, C, c, s_out, workspace, workspace_bytes, stream))
        return hip_check(hipGetLastError(), "launch k_conv_taps_bf16");
    G.step_y = kKC / Wo;
    G.step_x = kKC % Wo;
    // unit strides and an output as wide as the input: offsets are linear in the output position and the column
    // test repeats every W / gcd(W, kKC) chunks; the kernel keeps it in a 32-bit mask
    G.period = 0;
    if (sh == 1 && sw == 1 && Wo == W) {
        uint32_t a = W, b = kKC % W;
        while (b) { const uint32_t t = a % b; a = b; b = t; }
        if (W / a <= 32) G.period = W / a;
    }
    return launch_conv_any<true>(act, D, B, Ho * Wo, kh * kw * Cin, C, c, g_out, s_out, workspace, workspace_bytes, G, stream);
}

}  // namespace vgc

