// Register-tiled PCONV kernel for gfx950 (stride 1; stride 2 as stride 1 with every other output stored).
//
// Work decomposition.  A workgroup of NW waves owns 64 "patches" (a patch = a 4x4 block of output
// pixels of one image; one patch per lane) and 4 * NW filters (4 per wave, its "slots").  Two shapes
// are built: 16 waves with 8-channel chunks (one workgroup fills a compute unit), and 8 waves with
// 4-channel chunks (two workgroups share a compute unit; used for layers with at most 4 input
// channels, where one workgroup's output stores overlap with the other's loads).  Either way a SIMD
// runs 4 waves: a single wave issues a vector instruction only about every 6.5 cycles, so it takes
// three to four of them to keep a SIMD busy.
//
// The input channels are walked in chunks of CH through two LDS buffers.  For a chunk, the 6x6 input
// neighbourhood of every patch is staged into LDS (zero outside the image, so the inner loops have
// no bounds tests) while the previous chunk is being computed, and every wave copies the weights
// of its records for the chunk into its own LDS block.  Then each wave walks its records: a
// record is one (kernel, code) pair, i.e. up to four kept taps of one 3x3 kernel of one of the
// wave's filters.  When a record starts a new input channel the lane reloads its 6x6 neighbourhood
// from LDS (nine 128-bit reads) and keeps it in registers for all of the wave's filters connected
// to that channel; the record itself costs 16 FMAs per kept tap on the slot's 16 accumulators.
//
// The record loop is generated assembly (gen_tiled_compute.py): the pattern of a kernel selects
// straight-line code with compile-time register indices (paper: per-pattern generated code, one
// branch per kernel instead of per weight), reached by one computed jump per record.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <atomic>
#include <cstdlib>

#include "pconv_internal.h"
#include "pconv_tiled_codes.h"

// Hand-over words for callers that cannot let the library allocate (pconv_conv2d_static): one row
// of kFlagWords words per device, in the code object itself.  Host code never uses this name as an
// address; it asks the runtime for the array's device address once per device (static_flags()).
static __device__ __align__(256) uint32_t scratch[pconv::kFlagWords];

namespace pconv {

namespace {

struct bf16_t { uint16_t bits; };

constexpr int FB = kTileFB, BATCH = kTileBatch;
// A staged channel is nine blocks of one 16-byte quad per patch: blocks 0-5 hold columns x0..x0+3
// of input rows y0-1..y0+4; blocks 6-8 hold the patch's twelve halo values e = 0..11 (quad e / 4,
// element e % 4): e < 6 is column x0-1 of row e, e >= 6 is column x0+4 of row e - 6.  A lane reads its
// whole 6x6 neighbourhood with nine 128-bit LDS reads.
constexpr int QUAD_FLOATS = 64 * 4;
constexpr int CHAN_FLOATS = 9 * QUAD_FLOATS;  // 2304
constexpr int INV_FLOATS = 2 * 64;            // per-lane invariants {offset, mask}
constexpr int SYNC_WORDS = 8;                 // counters that order the waves
constexpr int HALO_TAB_WORDS = 12 * 64;       // source offsets of the halo loads (VEC)

template <int NW, int CH> struct Shape {
    static constexpr int BUF_FLOATS = CH * CHAN_FLOATS;        // one chunk
    static constexpr int WLDS_FLOATS = NW * BATCH * 4;         // weight blocks of the waves
    static constexpr int OFF_W = 2 * BUF_FLOATS;
    static constexpr int OFF_INV = OFF_W + WLDS_FLOATS;
    static constexpr int OFF_SYNC = OFF_INV + INV_FLOATS;
    static constexpr int OFF_HALO = OFF_SYNC + SYNC_WORDS;
    // 16 waves x 8 channels: 159776 of the compute unit's 163840 bytes; 8 x 4: 81696 (two fit)
    static constexpr int OFF_OUT = OFF_HALO + HALO_TAB_WORDS;   // per wave: {filter, bias} of its four slots
    static constexpr size_t LDS_BYTES = size_t(OFF_OUT + NW * 2 * FB) * 4;
    static constexpr int UNITS = 2 * CH;                       // staging units of half a channel per chunk
    static constexpr int SEGS = CH * 6 / NW;                   // (channel, row) segments per wave (register path)
    static_assert(CH * 6 % NW == 0 && UNITS % 8 == 0 && CH <= kTileCH && kTileCH % CH == 0, "unsupported shape");
};

static_assert(FB == 4 && BATCH == 32 && kTileCH == 8,
              "gen_tiled_compute.py is written for 4 slots, 32-record batches, channel field of 3 bits");

__device__ __forceinline__ float ld_act(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_act(const bf16_t *p, size_t i) { return __uint_as_float(uint32_t(p[i].bits) << 16); }
__device__ __forceinline__ void st_act(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_act(bf16_t *p, size_t i, float v)
{
    const uint32_t u = __float_as_uint(v);
    const uint32_t r = ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u) : ((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    p[i].bits = uint16_t(r);
}

typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
// Byte offset that lies beyond any tensor the VEC kernel accepts (at most 2^31 - 1 bytes): a buffer
// load at such an offset touches no memory and returns zero.
constexpr uint32_t kOutOfRange = 0x80000000u;

struct TiledArgs {
    const void *x; void *y; const float *bias;
    const int32_t *slot_filter; const uint32_t *chan_ptr; const uint32_t *meta; const float4 *w4;
    int n_img, c_in, row_len, h, w, c_out;
    int py, px;                 // patches per image column / row
    int n_patches, n_tiles, n_groups, n_blocks;
    int relu;
    int pool;                   // 1: y is the 2x2 / stride-2 max-pooled output (VEC kernel, whole units only)
    int sub2;                   // 1: stride 2: y holds the outputs at even rows and columns only
    int ks_log2;                // log2 of the channel split inside a workgroup (0, 1 or 2)
    int n_units;                // n_tiles * n_groups: (tile, filter group) pairs
    int n_chunks;               // chunks of CH input channels
    int split_units;            // 1: a workgroup's share of the work may begin and end inside a unit
    int one_set;                // 1 (with split_units): the iterations are dealt over all workgroups as one set
    uint32_t *flags;            // [gridDim.x] hand-over words of this call (split_units only)
    uint32_t epoch;             // value that marks a hand-over word as set by this call (never 0)
    uint32_t x_bytes;           // size of the input tensor (VEC kernel: below 2^31)
    uint32_t y_bytes;           // size of the output tensor (shared units only: below 2^31)
    uint32_t *err;              // sticky error word of the handle (host memory the device can write)
    int spin_limit;             // iterations after which a wait inside the kernel gives up
};

// Error codes a kernel leaves in the handle's error word.
constexpr uint32_t kErrChunkWait = 1u, kErrHandOverWait = 2u;

template <typename T, int LAYOUT>
__device__ __forceinline__ size_t act_at(int n, int c, int y, int x, int C, int H, int W)
{
    if (LAYOUT == PCONV_NCHW) return ((size_t(n) * C + c) * H + y) * W + x;
    return ((size_t(n) * H + y) * W + x) * C + c;
}

// How the work is spread over the workgroups.  A unit is one (tile of 64 patches, group of 4 * FW
// filters) pair walked over all chunks of input channels; one unit step ("iteration") is one chunk
// of one unit.  The workgroups whose ids are equal mod 8 run on one XCD (one L2); set s gets one
// contiguous eighth of the tiles with all their filter groups, tile-major, so that the filter
// groups of a tile, and neighbouring tiles (which share input rows and columns), read their input
// through the same L2 at about the same time.  Inside a set the iterations are dealt out evenly:
//   split_units == 0   in whole units (a workgroup gets zero or more of them);
//   split_units == 1   as equal contiguous ranges of iterations, so a unit may be shared by two
//                      or more consecutive workgroups of the set, each taking a range of its chunks
//                      (with one_set: over all workgroups as a single set, whatever their XCD).
// The workgroups that share a unit add their partial sums through the output tensor itself, in
// order of their ids: each one adds what its predecessor left there, and either leaves the new
// sum for its successor (raw, no bias) or, if it holds the unit's last chunk, finishes the
// outputs.  A workgroup runs the piece it must hand on first and the piece it takes over last;
// the hardware starts workgroups in order of their ids, so whatever a workgroup waits for
// belongs to a workgroup that has already started and handed over at its very beginning.
//
// VEC: fp32 NCHW tensors at least 4 wide move the four centre columns of a patch row (and the four
// outputs of a row) with one 128-bit access; the inputs go from global memory straight to LDS.
template <typename T, int LAYOUT, bool VEC, int NW, int CH, bool SPLIT>
__global__ void __launch_bounds__(NW * 64, 4)   // 4 waves per SIMD: at most 128 VGPRs
conv_tiled_kernel(const TiledArgs a)
{
    using S = Shape<NW, CH>;
    constexpr int BUF_FLOATS = S::BUF_FLOATS;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    // Everything outside the record loop (staging, the counters other waves wait for, the
    // epilogue) runs at the highest issue priority; the record loop drops to the lowest.
    __builtin_amdgcn_s_setprio(3);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // The waves are FW filter blocks x KS channel splits (KS = 1 for large layers).  With KS > 1
    // the waves of one filter block share its filters, each takes CH / KS of the channels of every
    // chunk, and the partial sums are added through LDS at the end in a fixed order.
    const int ks_log2 = a.ks_log2;
    const int fw = NW >> ks_log2;                        // filter blocks per workgroup
    const int ksplit = wave / fw;                        // this wave's channel split
    const int chs = CH >> ks_log2;                       // channels of a chunk per split
    const int sub_lo = ksplit * chs, sub_hi = sub_lo + chs;

    const T *__restrict__ x = static_cast<const T *>(a.x);
    T *__restrict__ y = static_cast<T *>(a.y);
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
    // buffer resource of the input tensor (VEC staging): base, stride 0, size in bytes, raw 32-bit data
    v4u rsrc;
    {
        const uint64_t xa = reinterpret_cast<uint64_t>(a.x);
        rsrc.x = __builtin_amdgcn_readfirstlane(uint32_t(xa));
        rsrc.y = __builtin_amdgcn_readfirstlane(uint32_t(xa >> 32) & 0xFFFFu);
        rsrc.z = __builtin_amdgcn_readfirstlane(a.x_bytes);
        rsrc.w = 0x00020000u;
    }
    // (Per-lane values are deliberately recomputed where they are used, from a lane id the
    // compiler cannot see through: only a few vector registers may stay live across the record
    // loop, and a spill reload there would wait for the loads in flight for the next chunk.)
    auto fresh_lane = [&]() { int l = threadIdx.x & 63; asm volatile("" : "+v"(l)); return l; };
    float *wlds = lds + S::OFF_W + wave * (BATCH * 4);   // this wave's weight block
    const uint32_t wa = lds_base + uint32_t(S::OFF_W + wave * (BATCH * 4)) * 4u;
    int *inv = reinterpret_cast<int *>(lds + S::OFF_INV);
    unsigned *sync_words = reinterpret_cast<unsigned *>(lds + S::OFF_SYNC);
    int *halo_tab = reinterpret_cast<int *>(lds + S::OFF_HALO);
    const int per_img = a.py * a.px;
    const int hw = a.h * a.w;
    const int n_chunks = a.n_chunks;

    // ---- this workgroup's range of iterations ----
    // (one_set: no XCD sets - the shares of all workgroups are then equal whatever the number of tiles,
    // and the workgroup that a piece waits for is simply the one before it)
    const bool one_set = SPLIT && a.one_set;
    const int set = one_set ? 0 : int(blockIdx.x & 7), j_in_set = one_set ? int(blockIdx.x) : int(blockIdx.x >> 3);
    const int set_stride = one_set ? 1 : 8;
    // set s: the contiguous block of tiles [s * tps, (s + 1) * tps): neighbouring tiles (which share
    // input rows and columns) then run next to each other in time on one XCD and find them in its L2
    // (with tiles s, s + 8, ... in a set, conv2 of VGG-16 fetched 699 MB for its 411 MB input; now 444)
    const int tps = (a.n_tiles + 7) >> 3;
    const int set_tile0 = set * tps;
    const int set_units = one_set ? a.n_units : max(0, min(a.n_tiles, set_tile0 + tps) - set_tile0) * a.n_groups;
    // SPLIT: iteration = (unit of the set) * n_chunks + chunk; otherwise one whole unit per workgroup
    int ua = j_in_set, ub = j_in_set, head_c0 = 0, tail_c1 = n_chunks;
    if constexpr (SPLIT) {
        const int wgs_in_set = one_set ? int(gridDim.x) : (int(gridDim.x) - set + 7) >> 3;
        const int64_t iters = int64_t(set_units) * n_chunks;
        const int64_t takers = iters < wgs_in_set ? iters : wgs_in_set;       // nobody gets an empty range in between
        if (j_in_set >= takers) return;
        int64_t it0 = iters * j_in_set / takers, it1 = iters * (j_in_set + 1) / takers;
        // When every unit is shared by the same number P of workgroups, those finish their chunks at
        // the same time and then pass the sums on one after the other, each link of that chain taking
        // about as long as 2.5 chunks.  Their shares are therefore graded, the first the smallest and
        // 2.5 chunks more for each successor (boundary k at k n / P - 2.5 k (P - k) / 2), so that a
        // workgroup finishes about when its predecessor's sums arrive.
        const int P = int(takers / set_units);
        if (set_units * P == takers && P >= 2 && 4 * n_chunks >= P * (16 + 5 * (P - 1))) {
            const int u = j_in_set / P, kk = j_in_set - u * P;
            auto bound = [&](int q) { return (4 * q * n_chunks / P - 5 * q * (P - q)) / 4; };
            it0 = int64_t(u) * n_chunks + bound(kk);
            it1 = int64_t(u) * n_chunks + bound(kk + 1);
        }
        ua = int(it0 / n_chunks); ub = int((it1 - 1) / n_chunks);            // first and last unit touched
        head_c0 = int(it0 - int64_t(ua) * n_chunks);                         // > 0: unit ua begins elsewhere
        tail_c1 = int(it1 - int64_t(ub) * n_chunks);                         // < n_chunks: unit ub ends elsewhere
    } else {
        if (j_in_set >= set_units) return;
    }
    const bool has_head = head_c0 > 0, has_tail = tail_c1 < n_chunks;
    const bool one_piece = ua == ub;
    // order: the piece to hand on, whole units, the piece taken over
    const int first_whole = has_head ? ua + 1 : ua, last_whole = has_tail ? ub - 1 : ub;
    const int n_whole = last_whole >= first_whole ? last_whole - first_whole + 1 : 0;
    const int n_pieces = SPLIT ? (has_tail ? 1 : 0) + n_whole + ((has_head && !(one_piece && has_tail)) ? 1 : 0) : 1;

    for (int piece = 0; piece < n_pieces; ++piece) {
        int unit, c_begin = 0, c_end = n_chunks;
        if (has_tail && piece == 0) { unit = ub; c_end = tail_c1; if (one_piece) c_begin = head_c0; }
        else if (piece - (has_tail ? 1 : 0) < n_whole) unit = first_whole + piece - (has_tail ? 1 : 0);
        else { unit = ua; c_begin = head_c0; }
        const bool takes_over = SPLIT && c_begin > 0, hands_on = SPLIT && c_end < n_chunks;
        const int tile = one_set ? unit / a.n_groups : set_tile0 + unit / a.n_groups, group = unit % a.n_groups;
        const int fblk = group * fw + (wave - ksplit * fw);
        const bool active = fblk < a.n_blocks;

        if (SPLIT) __syncthreads();                      // every wave has left the previous piece: LDS is free

        // The records of a (filter block, chunk) are contiguous and ordered by channel, so this wave's
        // share of a chunk is the range between two entries of chan_ptr.  The range bounds of up to
        // 64 consecutive chunks sit one per lane in ptr_pk and are read with v_readlane.
        // (Loaded first: they are on the way while the tables below are set up.)
        const int ptr_max = a.row_len - 1;               // last entry of a row: end of the block's records
        const uint32_t *__restrict__ ptr_row = a.chan_ptr + size_t(active ? fblk : 0) * a.row_len;
        int win_base = c_begin;
        // one register holds both bounds: first record (24 bits) and number of records (8 bits)
        auto load_bounds = [&]() {
            const uint32_t lo = ptr_row[min((win_base + lane) * CH + sub_lo, ptr_max)];
            const uint32_t hi = ptr_row[min((win_base + lane) * CH + sub_hi, ptr_max)];
            return lo << 8 | (hi - lo);
        };
        uint32_t ptr_pk = load_bounds();
        // The epilogue needs each slot's filter index and bias: two dependent loads, started here and
        // parked in LDS so that they cost the epilogue nothing (and no registers in between).
        float *out_tab = lds + S::OFF_OUT + wave * (2 * FB);
        if (lane < FB) {
            const int f = active ? a.slot_filter[fblk * FB + lane] : -1;
            const float b = (a.bias && f >= 0) ? a.bias[f] : 0.0f;
            out_tab[2 * lane] = __int_as_float(f);
            out_tab[2 * lane + 1] = b;
        }


        // this lane's patch
        const int pidx = tile * 64 + lane;
        const bool pvalid = pidx < a.n_patches;
        const int n = pvalid ? pidx / per_img : 0;
        const int prem = pvalid ? pidx - n * per_img : 0;
        // VEC: the last patch of a row is shifted left so that it ends at the image edge (it then
        // overlaps its neighbour and both compute identical values for the shared columns): the four
        // centre columns of a patch row are then always inside the image.
        const int y0 = (prem / a.px) * 4;
        const int x0 = VEC ? min((prem % a.px) * 4, a.w - 4) : (prem % a.px) * 4;

        // accumulators: slot s, output (row i, column k) of the patch = acc[s][4 * i + k].  The record
        // loop is assembly with a fixed register map, so each vector is pinned to its registers there.
        v16f acc[FB];
#pragma unroll
        for (int s = 0; s < FB; ++s) acc[s] = 0.0f;

        // ---- staging ----
        // Loads are branch-free: an out-of-image element is not loaded (VEC) or reads element 0 of the
        // tensor and is replaced by zero when the segment is written to LDS.  What is valid for this
        // lane does not change from chunk to chunk and is kept as one bit mask: bits 0-5 input rows
        // y0-1 .. y0+4, bits 8-13 input columns x0-1 .. x0+4.
        uint32_t vmask0 = 0;
#pragma unroll
        for (int r = 0; r < 6; ++r) {
            const int iy = y0 - 1 + r, ix = x0 - 1 + r;
            if (pvalid && iy >= 0 && iy < a.h) vmask0 |= 1u << r;
            if (ix >= 0 && ix < a.w) vmask0 |= 0x100u << r;
        }
        // element offset of (channel 0 of the chunk, row y0-1, column x0) follows from c0; tensors have
        // fewer than 2^31 elements, so 32-bit offsets suffice (they are only used where valid)
        const int lane_off0 = LAYOUT == PCONV_NCHW ? (n * a.c_in * a.h + (y0 - 1)) * a.w + x0
                                                  : ((n * a.h + (y0 - 1)) * a.w + x0) * a.c_in;
        // all waves work on the same 64 patches: the per-lane invariants live in LDS, one copy
        if (threadIdx.x < SYNC_WORDS) sync_words[threadIdx.x] = 0;
        if (wave == 0) { inv[2 * lane] = lane_off0; inv[2 * lane + 1] = int(vmask0); }
        // VEC path: the twelve halo values of a patch are fetched by twelve one-word loads per channel,
        // each of which fills 64 consecutive words of the halo blocks: word i of load j belongs to patch
        // 16 * (j % 4) + i / 4 and is its halo value e = 4 * (j / 4) + i % 4.  The element offset of that
        // value in channel 0, in bytes (or kOutOfRange outside the image), is the same for every chunk: tabulated once.
        if (VEC) {
            for (int t = threadIdx.x; t < HALO_TAB_WORDS; t += NW * 64) {
                const int j = t >> 6, i = t & 63;
                const int e = 4 * (j >> 2) + (i & 3);
                const int pidx_h = tile * 64 + 16 * (j & 3) + (i >> 2);
                const int n_h = pidx_h / per_img, prem_h = pidx_h - n_h * per_img;
                const int iy = (prem_h / a.px) * 4 - 1 + (e < 6 ? e : e - 6);
                const int xh = min((prem_h % a.px) * 4, a.w - 4);
                const int ix = e < 6 ? xh - 1 : xh + 4;
                const bool ok = pidx_h < a.n_patches && iy >= 0 && iy < a.h && ix >= 0 && ix < a.w;
                halo_tab[t] = ok ? ((n_h * a.c_in * a.h + iy) * a.w + ix) * 4 : int(kOutOfRange);
            }
        }
        // VEC path: global -> LDS directly, no registers and next to no vector ALU work.  The LDS
        // words of rows and halo values outside the image are zeroed once per piece and never get
        // anything but zero, so they stay zero for every chunk.
        // One unit of staging work = half a channel: three rows and six halo loads.
        auto stage_direct = [&](int c0, float *buf, int sunit) {
            const int ln = fresh_lane();
            const int ch = sunit >> 1, half = sunit & 1;
            if (c0 + ch >= a.c_in) return;                               // (uniform)

            const uint32_t soff = __builtin_amdgcn_readfirstlane(uint32_t(c0 + ch) * uint32_t(hw) * 4u);
            float *cbuf = buf + ch * CHAN_FLOATS;
            // everything the lane needs from the tables first, so that there is one wait for LDS
            const int lane_off_now = inv[2 * ln];
            const uint32_t vmask = uint32_t(inv[2 * ln + 1]);
            uint32_t off[6];
#pragma unroll
            for (int k = 0; k < 6; ++k) off[k] = uint32_t(halo_tab[(6 * half + k) * 64 + ln]);
            // Buffer loads: address = tensor + soff (channel, uniform) + per-lane byte offset; a lane
            // whose row or halo value lies outside the image has an offset beyond the buffer's size,
            // for which the hardware reads nothing and delivers zero.  The LDS address of lane 0's
            // element goes to M0 and every lane adds lane * size.  Written as assembly so that the
            // compiler does not track these loads: it would otherwise wait for them before the record
            // loop (they are waited for explicitly before they are published).
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const int r = 3 * half + k;
                const uint32_t voff = ((vmask >> r) & 1u) ? uint32_t(lane_off_now + r * a.w) * 4u : kOutOfRange;
                const uint32_t dst_b = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(cbuf + r * QUAD_FLOATS));
                asm volatile("s_mov_b32 m0, %1\n s_nop 0\n buffer_load_dwordx4 %0, %2, %3 offen lds"
                             ::"v"(voff), "s"(dst_b), "s"(rsrc), "s"(soff));
            }
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const int j = 6 * half + k;
                const uint32_t dst_b = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(cbuf + 6 * QUAD_FLOATS + j * 64));
                asm volatile("s_mov_b32 m0, %1\n s_nop 0\n buffer_load_dword %0, %2, %3 offen lds"
                             ::"v"(off[k]), "s"(dst_b), "s"(rsrc), "s"(soff));
            }
        };
        // generic path (any layout / dtype / width): through registers, with conversion to fp32;
        // every thread owns SEGS (channel, row) segments of its lane's patch
        constexpr int SEGS = S::SEGS;
        auto stage_load = [&](int c0, float (&t)[SEGS][6]) {
            const int ln = fresh_lane();
            const int lane_off_now = inv[2 * ln];
            const uint32_t vmask = uint32_t(inv[2 * ln + 1]);
#pragma unroll
            for (int kk = 0; kk < SEGS; ++kk) {
                const int seg = wave + NW * kk;
                const int ch = seg / 6, r = seg - ch * 6;
                const bool rv = ((vmask >> r) & 1u) && (c0 + ch < a.c_in);
                const int off = LAYOUT == PCONV_NCHW ? lane_off_now + (c0 + ch) * hw + r * a.w
                                                     : lane_off_now + r * a.w * a.c_in + (c0 + ch);
#pragma unroll
                for (int cc = 0; cc < 6; ++cc) {
                    const bool ok = rv && ((vmask >> (8 + cc)) & 1u);
                    const int e = LAYOUT == PCONV_NCHW ? off + (cc - 1) : off + (cc - 1) * a.c_in;
                    t[kk][cc] = ld_act(x, size_t(ok ? e : 0));
                }
            }
        };
        auto stage_store = [&](int c0, float *buf, const float (&t)[SEGS][6]) {
            const int ln = fresh_lane();
            const uint32_t vmask = uint32_t(inv[2 * ln + 1]);
#pragma unroll
            for (int kk = 0; kk < SEGS; ++kk) {
                const int seg = wave + NW * kk;
                const int ch = seg / 6, r = seg - ch * 6;
                const bool rv = ((vmask >> r) & 1u) && (c0 + ch < a.c_in);
                float v[6];
#pragma unroll
                for (int cc = 0; cc < 6; ++cc) v[cc] = (rv && ((vmask >> (8 + cc)) & 1u)) ? t[kk][cc] : 0.0f;
                float *cbuf = buf + ch * CHAN_FLOATS;
                *reinterpret_cast<float4 *>(cbuf + r * QUAD_FLOATS + ln * 4) = make_float4(v[1], v[2], v[3], v[4]);
                cbuf[(6 + r / 4) * QUAD_FLOATS + ln * 4 + r % 4] = v[0];                    // halo value e = r
                cbuf[(6 + (6 + r) / 4) * QUAD_FLOATS + ln * 4 + (6 + r) % 4] = v[5];        // halo value e = 6 + r
            }
        };
        // (rel = chunk index relative to the piece; it selects the LDS buffer)
        auto stage = [&](int rel) {
            float t[SEGS][6];
            stage_load((c_begin + rel) * CH, t);
            stage_store((c_begin + rel) * CH, lds + (rel & 1) * BUF_FLOATS, t);
        };

        if (VEC) {
            // zero both staged buffers (see stage_direct)
#pragma unroll
            for (int j = 0; j < 2 * BUF_FLOATS / (NW * 64 * 4); ++j)
                *reinterpret_cast<float4 *>(lds + (j * NW * 64 + threadIdx.x) * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        __syncthreads();                                 // zeroed buffers, tables and counters are visible

        // record range of this wave for a chunk, and the fetch of its first batch: lane j gets record
        // j (k0 + k_cnt is the next record or the padding record, always readable)
        auto fetch_records = [&](int chunk, uint32_t &k0, uint32_t &k_cnt, uint32_t &rec_m, float4 &rec_w) {
            if (chunk - win_base > 63) {                 // every 64 chunks: next window of bounds
                win_base = chunk;
                ptr_pk = load_bounds();
                __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0) here, so that the common path needs no wait
            }
            const uint32_t pk = __builtin_amdgcn_readlane(ptr_pk, chunk - win_base);
            k0 = pk >> 8;
            k_cnt = active ? pk & 0xFFu : 0u;

            const uint32_t ridx = k0 + min(uint32_t(lane), k_cnt);
            rec_m = a.meta[ridx];
            rec_w = a.w4[ridx];
        };

        // ---- the records of one chunk: generated assembly, in batches of up to BATCH records ----
        auto compute = [&](int rel, uint32_t k0, uint32_t k_cnt, uint32_t rec_m) {
            const uint32_t buf_bytes = uint32_t(rel & 1) * uint32_t(BUF_FLOATS * 4);
            // (one loop around a single copy of the assembly: the refill of a further batch sits behind it)
            uint32_t base = 0;
            while (base < k_cnt) {
                const uint32_t nb = __builtin_amdgcn_readfirstlane(min(uint32_t(BATCH), k_cnt - base));
                // lane j = record j of the batch; the lanes behind the last record end the list
                const uint32_t rm = uint32_t(fresh_lane()) < nb ? rec_m : kMetaEndOfList;
                const uint32_t koff = __builtin_amdgcn_readfirstlane((k0 + base) * 4u);
                asm volatile(
#include "pconv_tiled_compute.inc"
                    : "+{v[64:79]}"(acc[0]), "+{v[80:95]}"(acc[1]), "+{v[96:111]}"(acc[2]), "+{v[112:127]}"(acc[3])
                    : [recm] "v"(rm), [va] "v"(lds_base + buf_bytes + uint32_t(fresh_lane()) * 16u),
                      [wa] "s"(wa), [mp] "s"(a.meta), [koff] "s"(koff), [nb] "s"(nb), [chmask] "n"(CH - 1)
                    : "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33",
                      "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v44", "v45",
                      "v46", "v47", "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "v56", "v57",
                      "v58", "v59", "v60", "v61", "v62", "v63",
                      "s84", "s85", "s86", "s90", "s91", "s92", "s93", "s94", "s95", "scc");
                // No "memory" clobber on purpose: it would make the compiler wait for the
                // global->LDS loads of the next chunk, which may be in flight here and go to the
                // other buffer.  What the loop reads was published before (barrier / counters), or
                // written by the volatile stores below.
                base += BATCH;
                if (base < k_cnt) {
                    // more than BATCH records in this chunk (rare): next batch (the wave's weight
                    // block is private, and LDS accesses of one wave execute in order)
                    const uint32_t ridx = k0 + min(base + uint32_t(fresh_lane()), k_cnt);
                    rec_m = a.meta[ridx];
                    const float4 rec_w = a.w4[ridx];
                    // waiting here, in the rare path, keeps the common path free of a wait for all
                    // vector-memory loads (which would include the next chunk's staging)
                    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
                    if (fresh_lane() == 0) rec_m |= kMetaFirstOfChannel;   // input registers do not survive between batches
                    if (fresh_lane() < BATCH) {
                        volatile float *wv = wlds + fresh_lane() * 4;
                        wv[0] = rec_w.x; wv[1] = rec_w.y; wv[2] = rec_w.z; wv[3] = rec_w.w;
                    }
                }
            }
        };

        uint32_t k0, k_cnt, rec_m;
        const int n_rel = c_end - c_begin;

        if constexpr (VEC) {
            // ---- no barrier in this loop: three counters per LDS buffer order the waves ----
            //   tickets  staging work asked for           (a chunk has UNITS units of half a channel)
            //   staged   staging units whose data landed  chunk r is readable when staged == UNITS * (r/2 + 1)
            //   done     waves that finished a chunk      chunk r's buffer may be refilled (with chunk
            //                                             r + 2) when done == NW * (r/2 + 1)
            // All counters only grow.  A wave that has finished chunk r stages what is left of chunk
            // r + 1 (once every wave is done with chunk r - 1, whose buffer it takes), then computes it:
            // waves may be one chunk apart, so a chunk costs a wave its own records, not the records of
            // the busiest wave, and the staging falls to the waves with the least to do.  The slowest
            // wave never waits for a faster one: whatever it needs has been, or can be, produced by
            // itself.  Waits are bounded (TiledArgs::spin_limit polls) so that a mistake here ends in an
            // error code and poisoned outputs, not in a hang.
            unsigned *tickets = sync_words, *staged = sync_words + 2, *done = sync_words + 4;
            // A wait that runs out marks the workgroup (every wave poisons its outputs with NaN in
            // the epilogue) and leaves a code in the handle's error word, which the next call on
            // the handle reports.
            auto wait_ge = [&](unsigned *p, unsigned target) {
                bool reached = false;
                for (int guard = 0; guard < a.spin_limit; ++guard) {
                    const unsigned v = __builtin_amdgcn_readfirstlane(
                        __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
                    if (v >= target) { reached = true; break; }
                    __builtin_amdgcn_s_sleep(4);
                }
                if (!reached && fresh_lane() == 0) {
                    __hip_atomic_store(&sync_words[6], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __hip_atomic_store(a.err, kErrChunkWait, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                }
            };
            // A wave asks for staging work once per chunk, with one atomic add of kClaim: the counter
            // of a buffer therefore advances by exactly NW * kClaim per chunk, and the first
            // UNITS / kClaim askers (eight) get kClaim units each.  The add for chunk r is issued before the
            // wave reports chunk r - 1 as done, and LDS operations of a wave execute in order: once
            // every wave is done with r - 1, all adds for r have been applied, so a fast wave's add
            // for r + 2 (same counter) cannot get in between.
            constexpr unsigned kClaim = S::UNITS / 8;
            auto help_stage = [&](int rel, bool report_done) {
                const int p = rel & 1;
                unsigned got = 0;
                if (fresh_lane() == 0) {
                    got = __hip_atomic_fetch_add(&tickets[p], kClaim, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (report_done)                                   // chunk rel - 1 used the other buffer
                        __hip_atomic_fetch_add(&done[p ^ 1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                const unsigned unit0 = __builtin_amdgcn_readfirstlane(got) - unsigned(rel >> 1) * (NW * kClaim);
                if (unit0 < unsigned(S::UNITS)) {
                    wait_ge(&done[p], unsigned(rel >> 1) * NW);        // chunk rel - 2 is finished: the buffer is free
                    for (unsigned u = 0; u < kClaim; ++u)
                        stage_direct((c_begin + rel) * CH, lds + p * BUF_FLOATS, int(unit0 + u));
                    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): the data is in LDS
                    if (fresh_lane() == 0)
                        __hip_atomic_fetch_add(&staged[p], kClaim, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            };

            {
                float4 rec_w;
                fetch_records(c_begin, k0, k_cnt, rec_m, rec_w);       // on the way while chunk 0 is staged
                help_stage(0, false);
                if (lane < BATCH) *reinterpret_cast<float4 *>(wlds + lane * 4) = rec_w;
            }
            for (int rel = 0; rel < n_rel; ++rel) {
                const bool more = rel + 1 < n_rel;
                uint32_t nk0 = 0, nk_cnt = 0, nrec_m = 0;
                float4 nrec_w = make_float4(0.f, 0.f, 0.f, 0.f);
                if (more) fetch_records(c_begin + rel + 1, nk0, nk_cnt, nrec_m, nrec_w);   // lands during the records below
                wait_ge(&staged[rel & 1], unsigned((rel >> 1) + 1) * S::UNITS);
                compute(rel, k0, k_cnt, rec_m);
                // every LDS read of this chunk has returned (the record loop waits for its loads)
                if (more) {
                    { const int lw = fresh_lane(); if (lw < BATCH) *reinterpret_cast<float4 *>(wlds + lw * 4) = nrec_w; }
                    k0 = nk0; k_cnt = nk_cnt; rec_m = nrec_m;
                    help_stage(rel + 1, true);
                }
            }
        } else {
            // ---- register staging path: fixed assignment, one barrier per chunk ----
            {
                float4 rec_w;
                stage(0);
                fetch_records(c_begin, k0, k_cnt, rec_m, rec_w);
                if (lane < BATCH) *reinterpret_cast<float4 *>(wlds + lane * 4) = rec_w;
                __syncthreads();
            }
            for (int rel = 0; rel < n_rel; ++rel) {
                // The next chunk goes to the other LDS buffer, which every wave has finished reading
                // (they all passed the barrier at the end of the previous iteration).
                const bool more = rel + 1 < n_rel;
                uint32_t nk0 = 0, nk_cnt = 0, nrec_m = 0;
                float4 nrec_w = make_float4(0.f, 0.f, 0.f, 0.f);
                if (more) {
                    stage(rel + 1);
                    fetch_records(c_begin + rel + 1, nk0, nk_cnt, nrec_m, nrec_w);
                }
                compute(rel, k0, k_cnt, rec_m);
                if (more) {
                    { const int lw = fresh_lane(); if (lw < BATCH) *reinterpret_cast<float4 *>(wlds + lw * 4) = nrec_w; }
                    k0 = nk0; k_cnt = nk_cnt; rec_m = nrec_m;
                    __syncthreads();
                }
            }
        }

        // ---- channel splits: add the partial sums through LDS, split 2s+1 into 2s, then 2 into 0 ----
        if (ks_log2 > 0) {
            __syncthreads();                             // the staging buffers are free now
            float4 *red = reinterpret_cast<float4 *>(lds);
            for (int step = (1 << ks_log2) >> 1; step >= 1; step >>= 1) {
                const bool sender = ksplit >= step && ksplit < 2 * step;
                const bool receiver = ksplit < step;
                // slot of (filter block fbw, split): 16 float4 per lane
                const int fbw = wave - ksplit * fw;
                const int slot = ((sender ? ksplit - step : ksplit) * fw + fbw) * (16 * 64);
                if (sender) {
#pragma unroll
                    for (int s = 0; s < FB; ++s)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd)
                            red[slot + (s * 4 + qd) * 64 + lane] =
                                make_float4(acc[s][4 * qd], acc[s][4 * qd + 1], acc[s][4 * qd + 2], acc[s][4 * qd + 3]);
                }
                __syncthreads();
                if (receiver) {
#pragma unroll
                    for (int s = 0; s < FB; ++s)
#pragma unroll
                        for (int qd = 0; qd < 4; ++qd) {
                            const float4 p = red[slot + (s * 4 + qd) * 64 + lane];
                            acc[s][4 * qd] += p.x; acc[s][4 * qd + 1] += p.y; acc[s][4 * qd + 2] += p.z; acc[s][4 * qd + 3] += p.w;
                        }
                }
                __syncthreads();
            }
        }

        // ---- epilogue ----
        // Whole unit, or its last chunks: bias, ReLU, store (filters go back to their original
        // index).  A piece that takes over first adds what the previous workgroup left in the
        // output tensor; a piece that hands on stores the raw sums there instead.
        // the patch coordinates are recomputed here instead of being kept in registers across the loop
        int pidx_e = tile * 64 + lane;
        asm volatile("" : "+v"(pidx_e));
        const bool writer = active && ksplit == 0 && pidx_e < a.n_patches;
        if constexpr (VEC && SPLIT) {
            if (takes_over) {
                // The predecessor (id - 8: same set, previous range) started before this workgroup
                // and ran the shared unit first, so this wait is normally over before it begins.
                // It is bounded all the same; if it ever expires the outputs are poisoned with NaN.
                // One wave polls, and only its successful read is followed by the (costly)
                // device-wide acquire; the barrier passes it on to the other waves.
                if (wave == 0) {
                    bool there = false;
                    for (int guard = 0; guard < (a.spin_limit >> 2) && !there; ++guard) {
                        there = __hip_atomic_load(a.flags + (blockIdx.x - set_stride), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.epoch;
                        if (!there) __builtin_amdgcn_s_sleep(8);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                    if (!there && lane == 0) {
                        sync_words[6] = 1u;
                        __hip_atomic_store(a.err, kErrHandOverWait, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    }
                }
                __syncthreads();
                // Add what the predecessor left in the output tensor: generated assembly, all loads of
                // two slots in flight at once (the workgroups that share a unit wait for one another
                // here, one after the other, so this is on the critical path of the layer).  A lane
                // without a patch, a row below the image and an empty slot read nothing or something
                // that is never stored.
                {
                    const int lt = fresh_lane();
                    const int pidx_t = tile * 64 + lt;
                    const bool pv = pidx_t < a.n_patches;
                    const int n_t = pv ? pidx_t / per_img : 0, prem_t = pv ? pidx_t - n_t * per_img : 0;
                    const int ye_t = (prem_t / a.px) * 4, xe_t = min((prem_t % a.px) * 4, a.w - 4);
                    uint32_t voff[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        voff[i] = (pv && ye_t + i < a.h) ? uint32_t(((n_t * a.c_out * a.h + ye_t + i) * a.w) + xe_t) * 4u : kOutOfRange;
                    uint32_t so[FB];
#pragma unroll
                    for (int s = 0; s < FB; ++s) {
                        const int f = __builtin_amdgcn_readfirstlane(__float_as_int(out_tab[2 * s]));
                        so[s] = uint32_t(max(f, 0)) * uint32_t(hw) * 4u;
                    }
                    v4u yrsrc;
                    {
                        const uint64_t ya = reinterpret_cast<uint64_t>(a.y);
                        yrsrc.x = __builtin_amdgcn_readfirstlane(uint32_t(ya));
                        yrsrc.y = __builtin_amdgcn_readfirstlane(uint32_t(ya >> 32) & 0xFFFFu);
                        yrsrc.z = __builtin_amdgcn_readfirstlane(a.y_bytes);
                        yrsrc.w = 0x00020000u;
                    }
                    asm volatile(
#include "pconv_tiled_takeover.inc"
                        : "+{v[64:79]}"(acc[0]), "+{v[80:95]}"(acc[1]), "+{v[96:111]}"(acc[2]), "+{v[112:127]}"(acc[3])
                        : [voff0] "v"(voff[0]), [voff1] "v"(voff[1]), [voff2] "v"(voff[2]), [voff3] "v"(voff[3]),
                          [rsrc] "s"(yrsrc), [so0] "s"(so[0]), [so1] "s"(so[1]), [so2] "s"(so[2]), [so3] "s"(so[3])
                        : "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33", "v34", "v35",
                          "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v44", "v45", "v46", "v47",
                          "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "memory");
                }
            }
        }
        if constexpr (VEC) {
            // a wait of this workgroup ran out: its sums cannot be trusted
            if (__hip_atomic_load(&sync_words[6], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) {
#pragma unroll
                for (int s = 0; s < FB; ++s) acc[s] = __builtin_nanf("");
            }
        }
        if (writer) {
            const int n_e = pidx_e / per_img, prem_e = pidx_e - n_e * per_img;
            const int ye = (prem_e / a.px) * 4;
            const int xe = VEC ? min((prem_e % a.px) * 4, a.w - 4) : (prem_e % a.px) * 4;
            const int ho = a.h, wo = a.w;
#pragma unroll
            for (int s = 0; s < FB; ++s) {
                const int f = __float_as_int(out_tab[2 * s]);
                if (f < 0) continue;
                const float b = hands_on ? 0.0f : out_tab[2 * s + 1];
                if constexpr (VEC) {
                    if (a.pool) {
                        // 2x2 / stride-2 max-pool of the lane's 4x4 outputs (the patch is aligned to the
                        // pooling grid: rows at multiples of 4, columns at a multiple of 4 or at W - 4
                        // with W even): two rows of two pooled values.  Bias and ReLU first.
                        const int hp = ho >> 1, wp = wo >> 1;
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            if ((ye >> 1) + i >= hp) continue;
                            float m[2];
#pragma unroll
                            for (int k = 0; k < 2; ++k) {
                                float v = fmaxf(fmaxf(acc[s][(2 * i) * 4 + 2 * k], acc[s][(2 * i) * 4 + 2 * k + 1]),
                                                fmaxf(acc[s][(2 * i + 1) * 4 + 2 * k], acc[s][(2 * i + 1) * 4 + 2 * k + 1])) + b;
                                m[k] = a.relu ? fmaxf(v, 0.0f) : v;
                            }
                            float *dst = reinterpret_cast<float *>(y) + ((size_t(n_e) * a.c_out + f) * hp + (ye >> 1) + i) * wp + (xe >> 1);
                            *reinterpret_cast<float2 *>(dst) = make_float2(m[0], m[1]);
                        }
                        continue;
                    }
                    if (a.sub2) {
                        // stride 2: of the lane's 4x4 outputs the two even rows, and of each the two even
                        // columns (the patch starts at a multiple of 4, or at W - 4 in the last patch of a row)
                        const int h2 = (ho + 1) >> 1, w2 = (wo + 1) >> 1, k0 = xe & 1;
#pragma unroll
                        for (int i = 0; i < 4; i += 2) {
                            if (ye + i >= ho) continue;
                            float o[2];
#pragma unroll
                            for (int kk = 0; kk < 2; ++kk) {
                                float v = (k0 ? acc[s][i * 4 + 2 * kk + 1] : acc[s][i * 4 + 2 * kk]) + b;
                                o[kk] = a.relu ? fmaxf(v, 0.0f) : v;
                            }
                            float *dst = reinterpret_cast<float *>(y) + ((size_t(n_e) * a.c_out + f) * h2 + ((ye + i) >> 1)) * w2 + ((xe + k0) >> 1);
                            dst[0] = o[0];
                            if (((xe + k0) >> 1) + 1 < w2) dst[1] = o[1];
                        }
                        continue;
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (ye + i >= ho) continue;
                        float *dst = reinterpret_cast<float *>(y) + ((size_t(n_e) * a.c_out + f) * ho + ye + i) * wo + xe;
                        float o[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) o[k] = acc[s][i * 4 + k];
                        if (!hands_on) {
#pragma unroll
                            for (int k = 0; k < 4; ++k) { o[k] += b; if (a.relu) o[k] = fmaxf(o[k], 0.0f); }
                        }
                        *reinterpret_cast<float4 *>(dst) = make_float4(o[0], o[1], o[2], o[3]);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int oy = ye + i;
                        if (oy >= ho || (a.sub2 && (oy & 1))) continue;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            float v = acc[s][i * 4 + k] + b;
                            if (a.relu) v = fmaxf(v, 0.0f);
                            const int ox = xe + k;
                            if (ox >= wo) continue;
                            if (!a.sub2) st_act(y, act_at<T, LAYOUT>(n_e, f, oy, ox, a.c_out, ho, wo), v);
                            else if (!(ox & 1))
                                st_act(y, act_at<T, LAYOUT>(n_e, f, oy >> 1, ox >> 1, a.c_out, (ho + 1) >> 1, (wo + 1) >> 1), v);
                        }
                    }
                }
            }
        }
        if constexpr (VEC && SPLIT) {
            if (hands_on) {
                // the barrier orders every thread's stores before the release below, which makes
                // them visible to the whole device before the successor is told
                __syncthreads();
                if (threadIdx.x == 0)
                    __hip_atomic_store(a.flags + blockIdx.x, a.epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

template <typename T, int LAYOUT, bool VEC, int NW, int CH, bool SPLIT>
hipError_t launch_shape(const TiledArgs &a, int64_t wgs, hipStream_t st, int dev)
{
    // The kernel needs more dynamic LDS than the default limit: raised once per device (the flag is
    // set to the same value by every thread that gets here first).
    static std::atomic<bool> attr_done[64];
    constexpr size_t lds_bytes = Shape<NW, CH>::LDS_BYTES;
    if (dev < 0 || dev >= 64 || !attr_done[dev].load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_tiled_kernel<T, LAYOUT, VEC, NW, CH, SPLIT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) attr_done[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((conv_tiled_kernel<T, LAYOUT, VEC, NW, CH, SPLIT>), dim3(unsigned(wgs)), dim3(NW * 64), lds_bytes, st, a);
    return hipGetLastError();
}

template <int NW, int CH>
hipError_t launch_any(const TiledArgs &a, int64_t wgs, hipStream_t st, bool vec, int layout, int dtype, int dev)
{
    if (vec)
        return a.split_units ? launch_shape<float, PCONV_NCHW, true, NW, CH, true>(a, wgs, st, dev)
                             : launch_shape<float, PCONV_NCHW, true, NW, CH, false>(a, wgs, st, dev);
    if (dtype == PCONV_F32)
        return layout == PCONV_NCHW ? launch_shape<float, PCONV_NCHW, false, NW, CH, false>(a, wgs, st, dev)
                                    : launch_shape<float, PCONV_NHWC, false, NW, CH, false>(a, wgs, st, dev);
    return layout == PCONV_NCHW ? launch_shape<bf16_t, PCONV_NCHW, false, NW, CH, false>(a, wgs, st, dev)
                                : launch_shape<bf16_t, PCONV_NHWC, false, NW, CH, false>(a, wgs, st, dev);
}

// test overrides, see set_tiled_tuning / set_tiled_spin_limit
std::atomic<int> g_force_waves{0}, g_force_ks{-1}, g_force_split{-1};
constexpr double kShareGain = 0.97;
constexpr int kDefaultSpinLimit = 1 << 22;
std::atomic<int> g_spin_limit{kDefaultSpinLimit};

}  // namespace

void set_tiled_tuning(int waves, int ks_log2, int split_units)
{
    g_force_waves.store((waves == 8 || waves == 16) ? waves : 0);
    g_force_ks.store((ks_log2 >= 0 && ks_log2 <= 2) ? ks_log2 : -1);
    g_force_split.store((split_units >= 0 && split_units <= 2) ? split_units : -1);
}

void set_tiled_spin_limit(int limit) { g_spin_limit.store(limit > 0 ? limit : kDefaultSpinLimit); }

bool tiled_supported(const pconv_handle *h, int n, int hin, int win, int stride, int layout, int dtype)
{
    (void)layout; (void)dtype;
    // (stride 2 runs at full resolution and stores every other output)
    if (!h->d_meta || (stride != 1 && stride != 2)) return false;
    const int64_t patches = int64_t(n) * ((hin + 3) / 4) * ((win + 3) / 4);
    return patches < (int64_t(1) << 30);
}

bool tiled_preferred(int hin, int win, int stride)
{
    // Stride 2 through this kernel computes four times the outputs it stores; measured 1.6 to 3.4
    // times faster than the gather kernel all the same (ResNet-50 shapes, batch 32, inputs of 56x56,
    // 28x28 and 14x14).  Smaller images are left to the gather kernel.
    return stride == 1 || int64_t(hin) * win >= 12 * 12;
}

bool tiled_pool_supported(const pconv_handle *h, int n, int hin, int win, int layout, int dtype)
{
    return tiled_supported(h, n, hin, win, 1, layout, dtype) && dtype == PCONV_F32 && layout == PCONV_NCHW &&
           win >= 4 && win % 2 == 0 && hin >= 2 && int64_t(n) * h->c_in * hin * win * 4 < (int64_t(1) << 31);
}

namespace {

__global__ void fill_words_kernel(uint32_t *p, int count, uint32_t value)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = value;
}

// Device address of `scratch` on the handle's device (which is the current one), looked up on the
// first call per device and kept; nullptr (message set) if the runtime refuses.
uint32_t *static_flags(int dev)
{
    static std::atomic<uint32_t *> ptrs[64];
    if (dev < 0 || dev >= 64) { set_error("pconv_conv2d_static: device index out of range"); return nullptr; }
    uint32_t *p = ptrs[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *sym = nullptr;
    const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !sym) {
        set_error(std::string("pconv_conv2d_static: hipGetSymbolAddress: ") + hipGetErrorName(e));
        return nullptr;
    }
    p = static_cast<uint32_t *>(sym);
    ptrs[dev].store(p, std::memory_order_release);   // (every thread gets the same address)
    return p;
}

std::atomic<uint32_t> g_static_calls{0};             // epochs of the calls that use `scratch`

}  // namespace

bool tiled_shares_units(const pconv_handle *h, int n, int hin, int win)
{
    // the automatic choice of launch_conv_tiled for an fp32 NCHW call with stride 1 and no fused pool
    const int py = (hin + 3) / 4, px = (win + 3) / 4;
    const int64_t n_tiles = (int64_t(n) * py * px + 63) / 64;
    const int64_t x_bytes = int64_t(n) * h->c_in * hin * win * 4, y_bytes = int64_t(n) * h->c_out * hin * win * 4;
    const bool vec = win >= 4 && x_bytes < (int64_t(1) << 31);
    const int nw = h->c_in <= 4 ? 8 : 16;
    const int slots = (h->cus > 0 ? h->cus : 256) * (16 / nw);
    const bool rows_whole = win % 4 == 0 || n_tiles == 1 || 64 % px == 0;
    return vec && y_bytes < (int64_t(1) << 31) && rows_whole &&
           n_tiles * ((h->tiled.num_blocks + nw - 1) / nw) <= slots / 2;
}

int launch_conv_tiled(const pconv_handle *h, const void *x, void *y, const float *bias, int n,
                      int hin, int win, int stride, int layout, int dtype, int relu, int pool, void *stream,
                      bool static_scratch)
{
    TiledArgs a;
    a.sub2 = stride == 2;
    a.x = x; a.y = y; a.bias = bias;
    a.slot_filter = h->d_slot_filter; a.chan_ptr = h->d_chan_ptr; a.meta = h->d_meta;
    a.w4 = reinterpret_cast<const float4 *>(h->d_w4);
    a.n_img = n; a.c_in = h->c_in; a.row_len = h->tiled.row_len; a.h = hin; a.w = win; a.c_out = h->c_out;
    a.py = (hin + 3) / 4; a.px = (win + 3) / 4;
    a.n_patches = n * a.py * a.px;
    a.n_tiles = (a.n_patches + 63) / 64;
    a.n_blocks = h->tiled.num_blocks;
    a.relu = relu; a.pool = pool;
    const int64_t x_bytes = int64_t(n) * h->c_in * hin * win * 4;
    const bool vec = dtype == PCONV_F32 && layout == PCONV_NCHW && win >= 4 && x_bytes < (int64_t(1) << 31);
    a.x_bytes = uint32_t(std::min<int64_t>(x_bytes, 0x7FFFFFFF));
    // Shape: 16-wave workgroups, one per compute unit.  A layer whose input channels fit one 4-channel
    // chunk is all staging and output stores: there two 8-wave workgroups per compute unit overlap
    // one's stores with the other's loads.
    const int force_waves = g_force_waves.load(), force_ks = g_force_ks.load(), force_split = g_force_split.load();
    a.err = h->h_err; a.spin_limit = g_spin_limit.load();
    const int nw = force_waves ? force_waves : (h->c_in <= 4 ? 8 : 16);
    const int ch = nw == 16 ? 8 : 4;
    a.n_chunks = (h->c_in + ch - 1) / ch;
    // Few units: share them between workgroups (needs fp32 outputs written 128 bits at a time, the
    // VEC kernel), else split the channels inside the workgroups.
    const int cus = h->cus > 0 ? h->cus : 256;
    const int slots = cus * (16 / nw);                   // workgroups that can run at once
    // Sharing units costs every workgroup a second start-up and a pass of the partial sums through
    // memory: it pays where whole units would leave half of the compute units or more without work.
    // (Not with a fused max-pool: the partial sums need the full-size output tensor.)
    // (and needs an output below 2 GiB: the partial sums are read back with range-checked buffer loads)
    const int64_t y_bytes = int64_t(n) * h->c_out * hin * win * 4;
    // (and tiles whose borders fall between patch rows: where the image width is no multiple of 4
    // the last patch of a row overlaps its neighbour, and both write the columns they share; if the
    // two lay in different tiles, their workgroups would read and overwrite each other's partial sums)
    const bool rows_whole = win % 4 == 0 || a.n_tiles == 1 || 64 % a.px == 0;
    const bool can_split = vec && !pool && !a.sub2 && y_bytes < (int64_t(1) << 31) && rows_whole;
    a.y_bytes = uint32_t(std::min<int64_t>(y_bytes, 0x7FFFFFFF));
    const int64_t whole_units = int64_t(a.n_tiles) * ((a.n_blocks + nw - 1) / nw);
    a.split_units = can_split && whole_units <= slots / 2;
    a.one_set = 0;
    if (can_split && !a.split_units && nw == 16) {
        // Many units, but not a multiple of the number of compute units: whole units leave part of
        // the chip idle in the last round.  Dealing the chunks of all units evenly (every workgroup
        // one contiguous share, over all workgroups as one set) was measured to cost each workgroup
        // the time of about ten chunks (further start-ups, the partial sums through memory with a
        // device-wide release and acquire); a last round with few units runs faster than a full
        // one (measured: 0.87 of it at 53 % busy).  So it pays for few, long units only (VGG
        // conv9: 200 units of 64 chunks, -4 %).
        constexpr double kShareOverhead = 10.0;
        const double full = double(whole_units / slots), rest = double(whole_units % slots) / slots;
        const double t_whole = a.n_chunks * (full + (rest > 0.0 ? 0.72 + 0.28 * rest : 0.0));
        const double t_share = double(whole_units) * a.n_chunks / slots + kShareOverhead;
        if (t_share < kShareGain * t_whole) { a.split_units = 1; a.one_set = 1; }
    }
    if (force_split >= 0) { a.split_units = can_split ? (force_split != 0) : 0; a.one_set = a.split_units && force_split == 2; }
    a.ks_log2 = 0;
    if (!a.split_units)
        while (a.ks_log2 < 2 && int64_t(a.n_tiles) * ((a.n_blocks + (nw >> a.ks_log2) - 1) / (nw >> a.ks_log2)) <= slots / 2)
            ++a.ks_log2;
    if (force_ks >= 0) a.ks_log2 = force_ks;
    const int fw = nw >> a.ks_log2;
    a.n_groups = (a.n_blocks + fw - 1) / fw;
    const int64_t units = int64_t(a.n_tiles) * a.n_groups;
    if (units > 0x3FFFFFFF) { set_error("pconv_conv2d: too many workgroups"); return PCONV_UNSUPPORTED; }
    a.n_units = int(units);
    int64_t wgs;
    a.flags = nullptr; a.epoch = 0;
    if (a.split_units) {
        // one workgroup per slot, but no fewer than two chunks each
        const int64_t iters = units * a.n_chunks;
        wgs = std::min<int64_t>(std::min<int>(slots, kFlagWords), std::max<int64_t>(8, iters / 2));
        if (static_scratch) {
            // the one row of the device's static array, cleared by a small kernel ahead of the
            // convolution on the same stream (calls that overlap on one device would race here)
            if (wgs > kFlagWords) { set_error("pconv_conv2d_static: more workgroups than hand-over words"); return PCONV_UNSUPPORTED; }
            uint32_t *row = static_flags(h->device);
            if (!row) return PCONV_HIP_ERROR;
            hipLaunchKernelGGL(fill_words_kernel, dim3((kFlagWords + 255) / 256), dim3(256), 0,
                               static_cast<hipStream_t>(stream), row, kFlagWords, 0u);
            if (hipGetLastError() != hipSuccess) { set_error("pconv_conv2d_static: clearing the hand-over words failed"); return PCONV_HIP_ERROR; }
            const uint32_t call = g_static_calls.fetch_add(1u);
            a.flags = row;
            a.epoch = call + 1u ? call + 1u : 1u;
        } else {
            const uint32_t call = h->calls.fetch_add(1u);
            a.flags = h->d_flags + size_t(call % kFlagSlots) * kFlagWords;
            a.epoch = call + 1u ? call + 1u : 1u;
        }
    } else {
        wgs = int64_t((a.n_tiles + 7) / 8) * 8 * a.n_groups;   // one per unit of the largest set, in every set
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const hipError_t e = nw == 16 ? launch_any<16, 8>(a, wgs, st, vec, layout, dtype, h->device)
                                  : launch_any<8, 4>(a, wgs, st, vec, layout, dtype, h->device);
    if (e != hipSuccess) {
        set_error(std::string("pconv_conv2d (tiled kernel): ") + hipGetErrorName(e));
        return PCONV_HIP_ERROR;
    }
    return PCONV_OK;
}

}  // namespace pconv
