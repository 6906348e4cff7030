// Register-tiled PCONV kernel for gfx950 (stride 1).
//
// Work decomposition.  A workgroup of 8 waves owns 64 "patches" (each a 4x4 block of output
// pixels of one image, one patch per lane) and 64 filters (8 per wave).  The input channels are
// walked in chunks of 8: all 512 threads stage the 6x6 input neighbourhood of every patch of the
// chunk's channels into LDS (zero-filled outside the image, so the inner loops have no bounds
// tests), then every wave walks the records of its 8 filters for those channels.  For one input
// channel a lane reads its 6x6 neighbourhood from LDS once (six b128 + six b64 reads) and keeps it
// in registers for all of the wave's filters that are connected to that channel; each record then
// costs 16 FMAs per kept tap on 128 accumulator registers, with the weights in scalar registers.
//
// The pattern of a kernel selects straight-line code: the switch below has one case per
// (slot, code), all register indices are compile-time constants (paper: per-pattern generated
// code, branch per kernel instead of per weight; here by template instantiation).
#include <hip/hip_runtime.h>
#include <cstdlib>

#include "pconv_internal.h"
#include "pconv_tiled_codes.h"

namespace pconv {

namespace {

struct bf16_t { uint16_t bits; };

constexpr int FB = kTileFB, NWAVE = kTileWaves, CH = kTileCH;
constexpr int ROW_FLOATS = 64 * 6;            // one input row of all 64 patches: [64][4] then [64][2]
constexpr int CHAN_FLOATS = 6 * ROW_FLOATS;   // 2304
constexpr int BUF_FLOATS = CH * CHAN_FLOATS;  // 18432 floats = 72 KiB; two buffers

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

static_assert(kNumCodes == 24 && FB == 8 && CH == 8, "gen_tiled_compute.py is written for 24 codes, 8 slots, 8-channel chunks");

struct TiledArgs {
    const void *x; void *y; const float *bias;
    const int32_t *slot_filter; const uint32_t *chan_ptr; const uint32_t *meta; const float4 *w4;
    int n_img, c_in, row_len, h, w, c_out;
    int py, px;                 // patches per image column / row
    int n_patches, n_tiles, n_groups, n_blocks;
    int relu, dbg;
};

template <typename T, int LAYOUT>
__device__ __forceinline__ size_t act_at(int n, int c, int y, int x, int C, int H, int W)
{
    if (LAYOUT == PCONV_NCHW) return ((size_t(n) * C + c) * H + y) * W + x;
    return ((size_t(n) * H + y) * W + x) * C + c;
}

// VEC: fp32 NCHW tensors whose width is a multiple of 4 and whose base is 16-byte aligned move
// the four centre columns of a row (and the four outputs of a row) with one 128-bit access.
template <typename T, int LAYOUT, bool VEC>
__global__ void __launch_bounds__(512)
conv_tiled_kernel(const TiledArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];

    // workgroup id -> (tile, filter group); the groups of one tile share an XCD (ids equal mod 8)
    const int id = blockIdx.x;
    const int xcd = id & 7, q = id >> 3;
    const int tile = (q / a.n_groups) * 8 + xcd, group = q % a.n_groups;
    if (tile >= a.n_tiles) return;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int fblk = group * NWAVE + wave;
    const bool active = fblk < a.n_blocks;

    const T *__restrict__ x = static_cast<const T *>(a.x);
    T *__restrict__ y = static_cast<T *>(a.y);

    // this lane's patch
    const int pidx = tile * 64 + lane;
    const bool pvalid = pidx < a.n_patches;
    const int per_img = a.py * a.px;
    const int n = pvalid ? pidx / per_img : 0;
    const int prem = pvalid ? pidx - n * per_img : 0;
    const int y0 = (prem / a.px) * 4, x0 = (prem % a.px) * 4;

    // accumulators: slot s, output (row i, column k) of the patch = acc[s][4 * i + k].  The record
    // loop below is assembly with a fixed register map, so each vector is pinned to its registers.
    v16f acc[FB];
#pragma unroll
    for (int s = 0; s < FB; ++s) acc[s] = 0.0f;
    // per-lane LDS byte addresses of this lane's patch inside a staged buffer (128-bit / 64-bit part)
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));
    const uint32_t lane_a = lds_base + uint32_t(lane) * 16u;
    const uint32_t lane_b = lds_base + 1024u + uint32_t(lane) * 8u;

    // ---- staging helpers: every thread owns 6 (channel, row) segments of its lane's patch ----
    // Loads are branch-free: an out-of-image element reads element 0 of the tensor instead and
    // is replaced by zero when the segment is written to LDS, so all loads of a chunk are in
    // flight together (and stay in flight while the previous chunk is being computed).
    auto seg_row_valid = [&](int c0, int kk, int &ch, int &r, int &c, int &iy) -> bool {
        const int seg = wave + NWAVE * kk;              // 0..47, uniform per wave
        ch = seg / 6; r = seg - ch * 6;
        c = c0 + ch; iy = y0 - 1 + r;
        return pvalid && c < a.c_in && iy >= 0 && iy < a.h;
    };
    auto stage_load = [&](int c0, float (&t)[6][6]) {
#pragma unroll
        for (int kk = 0; kk < 6; ++kk) {
            int ch, r, c, iy;
            const bool rv = seg_row_valid(c0, kk, ch, r, c, iy);
            if (VEC) {
                const size_t row_off = rv ? ((size_t(n) * a.c_in + c) * a.h + iy) * a.w + x0 : 0;
                const float *rowp = reinterpret_cast<const float *>(x) + row_off;
                const float4 mid = *reinterpret_cast<const float4 *>(rowp);
                const bool lv = rv && x0 > 0, hv = rv && x0 + 4 < a.w;
                t[kk][0] = *(lv ? rowp - 1 : rowp);
                t[kk][1] = mid.x; t[kk][2] = mid.y; t[kk][3] = mid.z; t[kk][4] = mid.w;
                t[kk][5] = *(hv ? rowp + 4 : rowp);
            } else {
#pragma unroll
                for (int cc = 0; cc < 6; ++cc) {
                    const int ix = x0 - 1 + cc;
                    const bool ok = rv && ix >= 0 && ix < a.w;
                    t[kk][cc] = ld_act(x, ok ? act_at<T, LAYOUT>(n, c, iy, ix, a.c_in, a.h, a.w) : size_t(0));
                }
            }
        }
    };
    auto stage_store = [&](int c0, float *buf, const float (&t)[6][6]) {
#pragma unroll
        for (int kk = 0; kk < 6; ++kk) {
            int ch, r, c, iy;
            const bool rv = seg_row_valid(c0, kk, ch, r, c, iy);
            float v[6];
#pragma unroll
            for (int cc = 0; cc < 6; ++cc) {
                const int ix = x0 - 1 + cc;
                v[cc] = (rv && ix >= 0 && ix < a.w) ? t[kk][cc] : 0.0f;
            }
            float *dst = buf + (ch * 6 + r) * ROW_FLOATS;
            *reinterpret_cast<float4 *>(dst + lane * 4) = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float2 *>(dst + 256 + lane * 2) = make_float2(v[4], v[5]);
        }
    };
    // This wave's records of a chunk are contiguous; each lane fetches one of them.  The chunk
    // boundaries (chan_ptr at multiples of CH) of up to 64 consecutive chunks sit one per lane in
    // chunk_ptrs and are read with v_readlane, so that no load has to be waited for here.
    const int n_chunks = (a.c_in + CH - 1) / CH;
    const uint32_t *__restrict__ ptr_row = a.chan_ptr + size_t(active ? fblk : 0) * a.row_len;
    int win_base = 0;
    uint32_t chunk_ptrs = ptr_row[min(lane, n_chunks) * CH];
    auto fetch_records = [&](int chunk, uint32_t &k0, uint32_t &k_cnt, uint32_t &rec_m, float4 &rec_w) {
        if (chunk + 1 - win_base > 63) {                 // every 63 chunks: next window
            win_base = chunk;
            chunk_ptrs = ptr_row[min(win_base + lane, n_chunks) * CH];
            __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0), see the note in the record loop
        }
        k0 = __builtin_amdgcn_readlane(chunk_ptrs, chunk - win_base);
        k_cnt = active ? __builtin_amdgcn_readlane(chunk_ptrs, chunk + 1 - win_base) - k0 : 0u;
        const uint32_t idx = k0 + min(uint32_t(lane), k_cnt);   // k0 + k_cnt is the next record or the pad
        rec_m = a.meta[idx];
        rec_w = a.w4[idx];
    };

    float t[6][6];
    uint32_t k0, k_cnt, rec_m;
    float4 rec_w;
    fetch_records(0, k0, k_cnt, rec_m, rec_w);
    stage_load(0, t);
    stage_store(0, lds, t);
    __syncthreads();

    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int c0 = chunk * CH;
        const bool more = chunk + 1 < n_chunks;
        const bool do_stage = more && !((a.dbg & 1) && chunk >= 2);
        uint32_t nk0 = 0, nk_cnt = 0, nrec_m = 0;
        float4 nrec_w = make_float4(0.f, 0.f, 0.f, 0.f);
        // next chunk: global loads are issued now and land while this chunk is computed (the
        // record fetch comes first: it waits for its two pointers, which must not be behind the
        // staging loads in the in-order load counter)
        if (more) fetch_records(chunk + 1, nk0, nk_cnt, nrec_m, nrec_w);
        if (do_stage) stage_load(c0 + CH, t);

        // ---- compute: records of this wave's filter block for channels c0 .. c0+7 ----
        // Record j is broadcast from lane j with v_readlane; a record either starts a new channel
        // (the lane reloads its 6x6 input neighbourhood from LDS) or reuses the registers; then
        // its (slot, code) body runs: 16 FMAs per kept tap, weights in scalar registers.
        if (active && !(a.dbg & 2)) {
            const uint32_t buf_bytes = uint32_t(chunk & 1) * uint32_t(BUF_FLOATS * sizeof(float));
            const uint32_t va = lane_a + buf_bytes, vb = lane_b + buf_bytes;
            for (uint32_t base = 0; base < k_cnt; base += 64) {
                if (base > 0) {
                    const uint32_t idx = k0 + min(base + uint32_t(lane), k_cnt - 1);
                    rec_m = a.meta[idx];
                    rec_w = a.w4[idx];
                    // Rare path (more than 64 records in one chunk).  Waiting here keeps the
                    // record loop free of any wait on vector-memory loads, which would also wait
                    // for the next chunk's staging loads issued above.
                    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
                    if (lane == 0) rec_m |= kMetaFirstOfChannel;   // input registers do not survive between batches
                }
                const uint32_t nb = __builtin_amdgcn_readfirstlane(min(64u, k_cnt - base));
                asm volatile(
#include "pconv_tiled_compute.inc"
                    : "+{v[128:143]}"(acc[0]), "+{v[144:159]}"(acc[1]), "+{v[160:175]}"(acc[2]),
                      "+{v[176:191]}"(acc[3]), "+{v[192:207]}"(acc[4]), "+{v[208:223]}"(acc[5]),
                      "+{v[224:239]}"(acc[6]), "+{v[240:255]}"(acc[7])
                    : [recm] "v"(rec_m), [rw0] "v"(rec_w.x), [rw1] "v"(rec_w.y), [rw2] "v"(rec_w.z),
                      [rw3] "v"(rec_w.w), [va] "v"(va), [vb] "v"(vb), [cnt] "s"(nb)
                    : "v86", "v87", "v88", "v89", "v90", "v91", "v92", "v93", "v94", "v95", "v96", "v97", "v98", "v99", "v100", "v101",
                      "v102", "v103", "v104", "v105", "v106", "v107", "v108", "v109", "v110", "v111",
                      "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121",
                      "v122", "v123", "v124", "v125", "v126", "v127",
                      "s84", "s85", "s86", "s87", "s88", "s89", "s90", "s91", "s92", "s93", "s94", "s95",
                      "scc", "memory");
            }
        }

        // next chunk goes to the other buffer: nobody reads it any more (all waves passed the
        // previous barrier after finishing the chunk before this one)
        if (do_stage) stage_store(c0 + CH, lds + ((chunk + 1) & 1) * BUF_FLOATS, t);
        k0 = nk0; k_cnt = nk_cnt; rec_m = nrec_m; rec_w = nrec_w;
        __syncthreads();
    }

    // ---- epilogue: bias, ReLU, store (filters go back to their original index) ----
    if (!active || !pvalid) return;
    const int ho = a.h, wo = a.w;
#pragma unroll
    for (int s = 0; s < FB; ++s) {
        const int f = a.slot_filter[fblk * FB + s];
        if (f < 0) continue;
        const float b = a.bias ? a.bias[f] : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int oy = y0 + i;
            if (oy >= ho) continue;
            float o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                o[k] = acc[s][i * 4 + k] + b;
                if (a.relu) o[k] = fmaxf(o[k], 0.0f);
            }
            if (VEC) {
                float *dst = reinterpret_cast<float *>(y) + ((size_t(n) * a.c_out + f) * ho + oy) * wo + x0;
                *reinterpret_cast<float4 *>(dst) = make_float4(o[0], o[1], o[2], o[3]);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (x0 + k < wo) st_act(y, act_at<T, LAYOUT>(n, f, oy, x0 + k, a.c_out, ho, wo), o[k]);
            }
        }
    }
}

}  // namespace

bool tiled_supported(const pconv_handle *h, int n, int hin, int win, int stride, int layout, int dtype)
{
    (void)n; (void)layout; (void)dtype;
    if (!h->d_meta || stride != 1) return false;
    const int64_t patches = int64_t(n) * ((hin + 3) / 4) * ((win + 3) / 4);
    return patches < (int64_t(1) << 30);
}

int launch_conv_tiled(const pconv_handle *h, const void *x, void *y, const float *bias, int n,
                      int hin, int win, int stride, int layout, int dtype, int relu, void *stream)
{
    (void)stride;
    TiledArgs a;
    a.x = x; a.y = y; a.bias = bias;
    a.slot_filter = h->d_slot_filter; a.chan_ptr = h->d_chan_ptr; a.meta = h->d_meta;
    a.w4 = reinterpret_cast<const float4 *>(h->d_w4);
    a.n_img = n; a.c_in = h->c_in; a.row_len = h->tiled.row_len; a.h = hin; a.w = win; a.c_out = h->c_out;
    a.py = (hin + 3) / 4; a.px = (win + 3) / 4;
    a.n_patches = n * a.py * a.px;
    a.n_tiles = (a.n_patches + 63) / 64;
    a.n_blocks = h->tiled.num_blocks;
    a.n_groups = (a.n_blocks + NWAVE - 1) / NWAVE;
    a.relu = relu;
    { const char *e = getenv("PCONV_DEBUG_FLAGS"); a.dbg = e ? atoi(e) : 0; }
    const bool vec = dtype == PCONV_F32 && layout == PCONV_NCHW && (win % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (reinterpret_cast<uintptr_t>(y) % 16 == 0);
    const int64_t wgs = int64_t((a.n_tiles + 7) / 8) * 8 * a.n_groups;
    if (wgs > 0x7FFFFFFF) { set_error("pconv_conv2d: too many workgroups"); return PCONV_UNSUPPORTED; }
    const size_t lds_bytes = size_t(2) * BUF_FLOATS * sizeof(float);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
#define PCONV_LAUNCH(T, L, V)                                                                          \
    do {                                                                                              \
        static bool attr_done = false;                                                                \
        if (!attr_done) {                                                                             \
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_tiled_kernel<T, L, V>),         \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));      \
            attr_done = (e == hipSuccess);                                                            \
        }                                                                                             \
        if (e == hipSuccess)                                                                          \
            hipLaunchKernelGGL((conv_tiled_kernel<T, L, V>), dim3(unsigned(wgs)), dim3(512), lds_bytes, st, a); \
    } while (0)
    if (vec) PCONV_LAUNCH(float, PCONV_NCHW, true);
    else if (dtype == PCONV_F32) {
        if (layout == PCONV_NCHW) PCONV_LAUNCH(float, PCONV_NCHW, false); else PCONV_LAUNCH(float, PCONV_NHWC, false);
    } else {
        if (layout == PCONV_NCHW) PCONV_LAUNCH(bf16_t, PCONV_NCHW, false); else PCONV_LAUNCH(bf16_t, PCONV_NHWC, false);
    }
#undef PCONV_LAUNCH
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(std::string("pconv_conv2d (tiled kernel): ") + hipGetErrorName(e));
        return PCONV_HIP_ERROR;
    }
    return PCONV_OK;
}

}  // namespace pconv
