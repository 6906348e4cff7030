// bf16 PCONV on the matrix cores of gfx950: Eq. (1) as nine shifted contractions.
//
// For every tap (r, s) of the 3x3 kernel the layer is a matrix product over the input channels,
//     Y[f, p] += sum_c  W_rs[f, c] * X[c, p shifted by (r, s)],
// with W_rs the masked weights of that tap (zero where the kernel is removed or the pattern does not
// keep the tap).  Nothing is unfolded in memory: the shifted operand is read from one staged input
// tile in LDS at nine different offsets.  The pattern / connectivity sparsity enters twice: a
// (tap, 16 channels, 32 filters) block of W_rs that holds no kept weight at all is skipped (found at
// pack time), and everything else runs dense on v_mfma_f32_32x32x16_bf16 with fp32 accumulation.
// At the kept fractions of the ResNet-50 workload (1 / 2.5 of the kernels, 4 of 9 taps) the matrix
// cores' rate more than pays for the multiplications by zero; very sparse layers stay on the
// vector kernel (see mfma_preferred).
//
// Work decomposition.  A workgroup of 4 waves owns a tile of output pixels, TN images x TH rows x TW
// columns (at most 256 pixels, taken in blocks of 32 = the N dimension of the instruction), and
// MT blocks of 32 filters (the M dimension).  Wave w works on filter block w % MT and on the pixel
// blocks w / MT, w / MT + 4 / MT, ...  The input channels are walked in blocks of 32: the input tile
// of the block (with its one-pixel halo, zero outside the image) is staged into LDS as
// [pixel][channel] so that a lane finds the 8 consecutive channels of its pixel with one 128-bit
// read; the 18 weight fragments of the block (9 taps x 2 halves of 16 channels) come straight from
// global memory, 16 bytes per lane, while the tile is being staged.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>

#include "pconv_internal.h"

namespace pconv {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPitch = 40;          // bf16 per staged pixel: 32 channels + 8 of padding (bank spread)
constexpr int kMaxNBW = 8;          // pixel blocks of 32 per wave

struct MfmaArgs {
    const uint16_t *x; uint16_t *y; const float *bias;
    const uint16_t *wd;             // [9][cb16][fpad][16] bf16 bit patterns
    const uint32_t *nz;             // [cb32][fpad / 32]: bit (2 * tap + half) = block holds a kept weight
    int n, c_in, h, w, c_out, ho, wo, stride, relu;
    int cb32, fpad;
    int tn, th, tw;                 // tile: images, output rows, output columns
    int tiles_n, tiles_y, tiles_x, fgroups;
    int nb;                         // pixel blocks per tile
    int mt;                         // filter blocks per workgroup: 1, 2 or 4
    int in_h, in_w;                 // rows and columns of the staged input tile
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float v)
{
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x40u);
    return uint16_t((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

template <int LAYOUT>
__global__ void __launch_bounds__(256, 2)
conv_mfma_kernel(const MfmaArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t tile[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % a.mt, wn = wave / a.mt, wn_count = 4 / a.mt;

    // workgroup -> (tile, filter group); the filter groups of a tile are neighbours in the grid
    const int fg = blockIdx.x % a.fgroups;
    int t = blockIdx.x / a.fgroups;
    const int tx = t % a.tiles_x; t /= a.tiles_x;
    const int ty = t % a.tiles_y;
    const int tnn = t / a.tiles_y;
    const int img0 = tnn * a.tn, oy0 = ty * a.th, ox0 = tx * a.tw;
    const int iy0 = oy0 * a.stride - 1, ix0 = ox0 * a.stride - 1;     // input coordinates of tile element (0, 0)
    const int fb = fg * a.mt + wm;                                     // this wave's block of 32 filters
    const bool fb_ok = fb * 32 < a.fpad;
    const int npix = a.tn * a.th * a.tw;
    const int tile_pix = a.in_h * a.in_w;                              // staged pixels per image

    // the pixel of this lane in each of the wave's pixel blocks, as an element offset into the staged tile
    const int col = lane & 31, kg = lane >> 5;
    int poff[kMaxNBW];
    int nbw = 0;
#pragma unroll
    for (int j = 0; j < kMaxNBW; ++j) {
        const int blk = wn + j * wn_count;
        if (blk < a.nb) nbw = j + 1;
        const int p = min(blk * 32 + col, npix - 1);
        const int pi = p / (a.th * a.tw), pr = p - pi * (a.th * a.tw);
        const int py = pr / a.tw, px = pr - py * a.tw;
        poff[j] = ((pi * a.in_h + py * a.stride) * a.in_w + px * a.stride) * kPitch + kg * 8;
    }
    nbw = __builtin_amdgcn_readfirstlane(nbw);

    f32x16 acc[kMaxNBW];
#pragma unroll
    for (int j = 0; j < kMaxNBW; ++j) acc[j] = 0.0f;

    const int cb16n = a.cb32 * 2;
    const int items = a.tn * tile_pix * 8;            // (pixel, 4-channel group) pairs of a staged block
    for (int cb = 0; cb < a.cb32; ++cb) {
        // ---- weight fragments of this channel block: 16 bytes per lane each, straight from memory ----
        const uint32_t nzbits = fb_ok ? a.nz[cb * (a.fpad / 32) + fb] : 0u;
        u32x4 wf[18];
#pragma unroll
        for (int q = 0; q < 18; ++q) {
            const int tap = q >> 1, half = q & 1;
            if ((nzbits >> q) & 1u) {
                const size_t e = ((size_t(tap) * cb16n + cb * 2 + half) * a.fpad + fb * 32 + col) * 16 + kg * 8;
                wf[q] = *reinterpret_cast<const u32x4 *>(a.wd + e);
            } else {
                wf[q] = u32x4{0u, 0u, 0u, 0u};
            }
        }
        // ---- stage the input tile of the block: [image][row][column][channel], zero outside the image ----
        __syncthreads();                               // everybody has finished reading the previous block
        for (int it = threadIdx.x; it < items; it += 256) {
            int q, pix;
            if (LAYOUT == PCONV_NCHW) { q = it / (a.tn * tile_pix); pix = it - q * (a.tn * tile_pix); }   // pixels fastest: coalesced rows
            else { pix = it >> 3; q = it & 7; }                                                             // channels fastest
            const int pi = pix / tile_pix, pr = pix - pi * tile_pix;
            const int ry = pr / a.in_w, rx = pr - ry * a.in_w;
            const int img = img0 + pi, iy = iy0 + ry, ix = ix0 + rx;
            const bool ok = img < a.n && iy >= 0 && iy < a.h && ix >= 0 && ix < a.w;
            const int c = cb * 32 + q * 4;
            uint16_t v[4] = {0, 0, 0, 0};
            if (ok) {
                if (LAYOUT == PCONV_NCHW) {
                    const size_t base = ((size_t(img) * a.c_in + c) * a.h + iy) * a.w + ix;
                    const size_t plane = size_t(a.h) * a.w;
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (c + k < a.c_in) v[k] = a.x[base + k * plane];
                } else {
                    const size_t base = ((size_t(img) * a.h + iy) * a.w + ix) * a.c_in + c;
                    if ((a.c_in & 3) == 0 && c + 3 < a.c_in) {
                        const uint2 u = *reinterpret_cast<const uint2 *>(a.x + base);
                        v[0] = uint16_t(u.x); v[1] = uint16_t(u.x >> 16); v[2] = uint16_t(u.y); v[3] = uint16_t(u.y >> 16);
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (c + k < a.c_in) v[k] = a.x[base + k];
                    }
                }
            }
            uint2 packed;
            packed.x = uint32_t(v[0]) | (uint32_t(v[1]) << 16);
            packed.y = uint32_t(v[2]) | (uint32_t(v[3]) << 16);
            *reinterpret_cast<uint2 *>(tile + size_t(pix) * kPitch + q * 4) = packed;
        }
        __syncthreads();

        // ---- nine taps x two halves of 16 channels ----
#pragma unroll
        for (int q = 0; q < 18; ++q) {
            if (!((nzbits >> q) & 1u)) continue;       // (wave-uniform) no kept weight in this block
            const int tap = q >> 1, half = q & 1;
            const int toff = ((tap / 3) * a.in_w + (tap % 3)) * kPitch + half * 16;
            const bf16x8 wa = __builtin_bit_cast(bf16x8, wf[q]);
#pragma unroll
            for (int j = 0; j < kMaxNBW; ++j) {
                if (j < nbw) {
                    const bf16x8 xb = *reinterpret_cast<const bf16x8 *>(tile + poff[j] + toff);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xb, acc[j], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue: bias, ReLU, round to bf16, store ----
    // register v of a lane holds filter 8 * (v / 4) + 4 * (lane / 32) + v % 4 of the block, pixel lane % 32
    if (!fb_ok) return;
#pragma unroll
    for (int j = 0; j < kMaxNBW; ++j) {
        if (j >= nbw) continue;
        const int p = (wn + j * wn_count) * 32 + col;
        if (p >= npix) continue;
        const int pi = p / (a.th * a.tw), pr = p - pi * (a.th * a.tw);
        const int py = pr / a.tw, px = pr - py * a.tw;
        const int img = img0 + pi, oy = oy0 + py, ox = ox0 + px;
        if (img >= a.n || oy >= a.ho || ox >= a.wo) continue;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int f0 = fb * 32 + 8 * g + 4 * kg;
            uint16_t o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float v = acc[j][4 * g + k];
                if (f0 + k < a.c_out && a.bias) v += a.bias[f0 + k];
                if (a.relu) v = fmaxf(v, 0.0f);
                o[k] = f32_to_bf16_rne(v);
            }
            if (LAYOUT == PCONV_NCHW) {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (f0 + k < a.c_out)
                        a.y[((size_t(img) * a.c_out + f0 + k) * a.ho + oy) * a.wo + ox] = o[k];
            } else {
                const size_t base = ((size_t(img) * a.ho + oy) * a.wo + ox) * a.c_out + f0;
                if ((a.c_out & 3) == 0 && f0 + 3 < a.c_out) {
                    uint2 u;
                    u.x = uint32_t(o[0]) | (uint32_t(o[1]) << 16);
                    u.y = uint32_t(o[2]) | (uint32_t(o[3]) << 16);
                    *reinterpret_cast<uint2 *>(a.y + base) = u;
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (f0 + k < a.c_out) a.y[base + k] = o[k];
                }
            }
        }
    }
}

constexpr int kLdsLimit = 64 * 1024;    // two workgroups per compute unit

}  // namespace

bool mfma_supported(const pconv_handle *h, int dtype)
{
    return dtype == PCONV_BF16 && h->wdtype == PCONV_BF16 && h->d_wdense != nullptr;
}

bool mfma_preferred(const pconv_handle *h)
{
    // Dense contraction of masked weights: pays when enough of the 9 * c_in * c_out weights are kept.
    // The vector kernel runs bf16 layers at some 30 effective TFLOP/s, this one at several hundred
    // dense TFLOP/s: the break-even lies near 1 kept weight in 20.
    return h->nnz * 20 >= int64_t(9) * h->c_in * h->c_out;
}

int launch_conv_mfma(const pconv_handle *h, const void *x, void *y, const float *bias, int n,
                     int hin, int win, int stride, int layout, int relu, void *stream)
{
    MfmaArgs a;
    a.x = static_cast<const uint16_t *>(x); a.y = static_cast<uint16_t *>(y); a.bias = bias;
    a.wd = h->d_wdense; a.nz = h->d_wnz;
    a.n = n; a.c_in = h->c_in; a.h = hin; a.w = win; a.c_out = h->c_out;
    a.ho = (hin - 1) / stride + 1; a.wo = (win - 1) / stride + 1;
    a.stride = stride; a.relu = relu;
    a.cb32 = (h->c_in + 31) / 32; a.fpad = (h->c_out + 31) / 32 * 32;
    const int cus = h->cus > 0 ? h->cus : 256;
    // Tile: whole rows where a row fits 256 pixels, as many rows as fit, then as many images as fit;
    // the staged input tile must stay within kLdsLimit.  Fewer pixels per tile when the layer would
    // otherwise give fewer workgroups than two per compute unit.
    auto lds_bytes = [&](int tn, int th, int tw) {
        return size_t(tn) * ((th - 1) * stride + 3) * ((tw - 1) * stride + 3) * kPitch * 2;
    };
    int best_tn = 1, best_th = 1, best_tw = std::min(a.wo, 32), best_mt = 1;
    double best_cost = 1e300;
    for (int mt = 1; mt <= 4; mt *= 2) {
        if (mt > 1 && (mt / 2) * 32 >= a.fpad) break;        // no more filter blocks than the layer has
        const int fgroups = (a.fpad / 32 + mt - 1) / mt;
        for (int tw = std::min(a.wo, 256); tw >= 1; tw = (tw > 32 ? (tw + 1) / 2 : 0)) {
            for (int th = 1; th <= a.ho && th * tw <= 256; ++th) {
                for (int tn = 1; tn <= n && tn * th * tw <= 256; ++tn) {
                    if (tn > 1 && (th < a.ho || tw < a.wo)) break;            // several images only as whole images
                    if (lds_bytes(tn, th, tw) > size_t(kLdsLimit)) break;
                    const int npix = tn * th * tw, nb = (npix + 31) / 32;
                    if ((nb + 4 / mt - 1) / (4 / mt) > kMaxNBW) continue;
                    const int64_t tiles = int64_t((n + tn - 1) / tn) * ((a.ho + th - 1) / th) * ((a.wo + tw - 1) / tw);
                    const int64_t wgs = tiles * fgroups;
                    // cost model: matrix work of all workgroups (padded pixel blocks x filter blocks), spread
                    // over the compute units in rounds of two workgroups each, plus the staging of the
                    // tile once per workgroup (its weight relative to the matrix work grows as MT shrinks)
                    const double per_wg = double(nb) * 32 * mt * 32 + 0.6 * double(tn) * ((th - 1) * stride + 3) * ((tw - 1) * stride + 3) * 32;
                    const double rounds = double((wgs + 2 * cus - 1) / (2 * cus));
                    const double cost = rounds * per_wg;
                    if (cost < best_cost) { best_cost = cost; best_tn = tn; best_th = th; best_tw = tw; best_mt = mt; }
                }
            }
            if (tw <= 32) break;
        }
    }
    a.tn = best_tn; a.th = best_th; a.tw = best_tw; a.mt = best_mt;
    a.tiles_n = (n + a.tn - 1) / a.tn; a.tiles_y = (a.ho + a.th - 1) / a.th; a.tiles_x = (a.wo + a.tw - 1) / a.tw;
    a.fgroups = (a.fpad / 32 + a.mt - 1) / a.mt;
    a.nb = (a.tn * a.th * a.tw + 31) / 32;
    a.in_h = (a.th - 1) * stride + 3; a.in_w = (a.tw - 1) * stride + 3;
    const size_t lds = lds_bytes(a.tn, a.th, a.tw);
    const int64_t wgs = int64_t(a.tiles_n) * a.tiles_y * a.tiles_x * a.fgroups;
    if (lds > size_t(kLdsLimit) || wgs > 0x7FFFFFFF || (a.nb + 4 / a.mt - 1) / (4 / a.mt) > kMaxNBW) {
        set_error("pconv_conv2d (matrix-core kernel): no tile fits this call");
        return PCONV_UNSUPPORTED;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (layout == PCONV_NCHW)
        hipLaunchKernelGGL(conv_mfma_kernel<PCONV_NCHW>, dim3(unsigned(wgs)), dim3(256), lds, st, a);
    else
        hipLaunchKernelGGL(conv_mfma_kernel<PCONV_NHWC>, dim3(unsigned(wgs)), dim3(256), lds, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(std::string("pconv_conv2d (matrix-core kernel): ") + hipGetErrorName(e));
        return PCONV_HIP_ERROR;
    }
    return PCONV_OK;
}

}  // namespace pconv
