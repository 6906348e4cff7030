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

// 16 FMAs per kept tap of MASK on the 4x4 outputs of one slot.  in[] is the 6x6 neighbourhood
// (row-major, in[(i+r)*6 + (k+s)] is the input under tap (r,s) of output (i,k)).
template <unsigned MASK>
__device__ __forceinline__ void mac_code(float (&acc)[16], const float (&in)[36], const float4 &wv)
{
    const float w[4] = {wv.x, wv.y, wv.z, wv.w};
    int j = 0;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        if (MASK & (1u << t)) {
            const int r = t / 3, s = t % 3;
            const float wt = w[j];
            ++j;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    acc[i * 4 + k] = fmaf(wt, in[(i + r) * 6 + (k + s)], acc[i * 4 + k]);
        }
    }
}

#define PCONV_CODE_CASE(S, C) \
    case (S) * kNumCodes + (C): mac_code<kCodeMask[C]>(acc[S], in, wv); break;
#define PCONV_SLOT_CASES(S)                                                                        \
    PCONV_CODE_CASE(S, 0) PCONV_CODE_CASE(S, 1) PCONV_CODE_CASE(S, 2) PCONV_CODE_CASE(S, 3)        \
    PCONV_CODE_CASE(S, 4) PCONV_CODE_CASE(S, 5) PCONV_CODE_CASE(S, 6) PCONV_CODE_CASE(S, 7)        \
    PCONV_CODE_CASE(S, 8) PCONV_CODE_CASE(S, 9) PCONV_CODE_CASE(S, 10) PCONV_CODE_CASE(S, 11)      \
    PCONV_CODE_CASE(S, 12) PCONV_CODE_CASE(S, 13) PCONV_CODE_CASE(S, 14) PCONV_CODE_CASE(S, 15)    \
    PCONV_CODE_CASE(S, 16) PCONV_CODE_CASE(S, 17) PCONV_CODE_CASE(S, 18) PCONV_CODE_CASE(S, 19)    \
    PCONV_CODE_CASE(S, 20) PCONV_CODE_CASE(S, 21) PCONV_CODE_CASE(S, 22) PCONV_CODE_CASE(S, 23)
static_assert(kNumCodes == 24 && FB == 8, "the case list below is written for 24 codes x 8 slots");

struct TiledArgs {
    const void *x; void *y; const float *bias;
    const int32_t *slot_filter; const uint32_t *chan_ptr; const uint32_t *meta; const float4 *w4;
    int n_img, c_in, row_len, h, w, c_out;
    int py, px;                 // patches per image column / row
    int n_patches, n_tiles, n_groups, n_blocks;
    int relu;
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

    float acc[FB][16];
#pragma unroll
    for (int s = 0; s < FB; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[s][i] = 0.0f;

    const int n_chunks = (a.c_in + CH - 1) / CH;
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int c0 = chunk * CH;
        float *buf = lds + (chunk & 1) * BUF_FLOATS;

        // ---- stage: every thread fills 6 (channel, row) segments of its lane's patch ----
        // Branch-free: out-of-image reads are redirected to element 0 of the tensor and the value
        // is replaced by zero afterwards, so that all loads of a thread are in flight together.
        float v[6][6];
#pragma unroll
        for (int kk = 0; kk < 6; ++kk) {
            const int seg = wave + NWAVE * kk;          // 0..47, uniform per wave
            const int ch = seg / 6, r = seg - ch * 6;
            const int c = c0 + ch, iy = y0 - 1 + r;
            const bool rv = pvalid && c < a.c_in && iy >= 0 && iy < a.h;
            if (VEC) {
                // width is a multiple of 4 and the tensor 16-byte aligned: columns x0..x0+3 in one load
                const size_t row_off = rv ? ((size_t(n) * a.c_in + c) * a.h + iy) * a.w + x0 : 0;
                const float *rowp = reinterpret_cast<const float *>(x) + row_off;
                const float4 mid = *reinterpret_cast<const float4 *>(rowp);
                const bool lv = rv && x0 > 0, hv = rv && x0 + 4 < a.w;
                const float lo = *(lv ? rowp - 1 : rowp);
                const float hi = *(hv ? rowp + 4 : rowp);
                v[kk][0] = lv ? lo : 0.0f;
                v[kk][1] = rv ? mid.x : 0.0f; v[kk][2] = rv ? mid.y : 0.0f;
                v[kk][3] = rv ? mid.z : 0.0f; v[kk][4] = rv ? mid.w : 0.0f;
                v[kk][5] = hv ? hi : 0.0f;
            } else {
#pragma unroll
                for (int cc = 0; cc < 6; ++cc) {
                    const int ix = x0 - 1 + cc;
                    const bool ok = rv && ix >= 0 && ix < a.w;
                    const float t = ld_act(x, ok ? act_at<T, LAYOUT>(n, c, iy, ix, a.c_in, a.h, a.w) : size_t(0));
                    v[kk][cc] = ok ? t : 0.0f;
                }
            }
        }
#pragma unroll
        for (int kk = 0; kk < 6; ++kk) {
            const int seg = wave + NWAVE * kk;
            const int ch = seg / 6, r = seg - ch * 6;
            float *dst = buf + (ch * 6 + r) * ROW_FLOATS;
            *reinterpret_cast<float4 *>(dst + lane * 4) = make_float4(v[kk][0], v[kk][1], v[kk][2], v[kk][3]);
            *reinterpret_cast<float2 *>(dst + 256 + lane * 2) = make_float2(v[kk][4], v[kk][5]);
        }
        __syncthreads();

        // ---- compute: records of this wave's filter block for channels c0 .. c0+7 ----
        if (active) {
            const uint32_t *__restrict__ cp = a.chan_ptr + size_t(fblk) * a.row_len + c0;
            for (int ch = 0; ch < CH; ++ch) {
                const uint32_t beg = cp[ch], end = cp[ch + 1];
                if (beg == end) continue;
                float in[36];
                const float *src = buf + ch * CHAN_FLOATS;
#pragma unroll
                for (int r = 0; r < 6; ++r) {
                    const float4 va = *reinterpret_cast<const float4 *>(src + r * ROW_FLOATS + lane * 4);
                    const float2 vb = *reinterpret_cast<const float2 *>(src + r * ROW_FLOATS + 256 + lane * 2);
                    in[r * 6 + 0] = va.x; in[r * 6 + 1] = va.y; in[r * 6 + 2] = va.z; in[r * 6 + 3] = va.w;
                    in[r * 6 + 4] = vb.x; in[r * 6 + 5] = vb.y;
                }
                for (uint32_t k = beg; k < end; ++k) {
                    const uint32_t m = a.meta[k];
                    const float4 wv = a.w4[k];
                    switch (m) {
                        PCONV_SLOT_CASES(0) PCONV_SLOT_CASES(1) PCONV_SLOT_CASES(2) PCONV_SLOT_CASES(3)
                        PCONV_SLOT_CASES(4) PCONV_SLOT_CASES(5) PCONV_SLOT_CASES(6) PCONV_SLOT_CASES(7)
                        default: break;
                    }
                }
            }
        }
        // The next chunk is staged into the other buffer; the barrier after that staging also
        // orders this chunk's reads before the buffer is overwritten two chunks from now.
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
