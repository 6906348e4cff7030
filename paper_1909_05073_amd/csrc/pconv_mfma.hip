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
// columns (at most 128 / MT pixels, taken in blocks of 32 = the N dimension of the instruction), and
// MT blocks of 32 filters (the M dimension): wave w works on filter block w % MT and pixel block
// w / MT.  The input channels are walked in blocks of 32: the input tile of the block (with its
// one-pixel halo, zero outside the image) is staged into LDS as [pixel][channel], so that a lane
// finds the 8 consecutive channels of its pixel with one 128-bit read; the 18 weight fragments of a
// block (9 taps x 2 halves of 16 channels) come straight from global memory, 16 bytes per lane, a
// few fragments ahead of their use.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>
#include <type_traits>

#include "pconv_internal.h"

namespace pconv {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPitch = 40;          // bf16 per staged pixel: 32 channels + 8 of padding (bank spread)

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
    uint32_t x_bytes;               // size of the input tensor, below 2^31
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float v)
{
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x40u);
    return uint16_t((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// Staging goes through registers, one channel block ahead: the loads of block b + 1 are issued
// before the matrix instructions of block b and written to LDS after them.  A thread owns
// kPixPerThread staged pixels with the 32 channels of the block each.
constexpr int kPixPerThread = 2;
constexpr int kMaxTilePixels = kPixPerThread * 256;   // staged pixels (all images of the tile, halo included)

// PAIR (NCHW with an even image width): the staged tile starts at an even input column and a thread
// stages two neighbouring pixels, which one 32-bit load per channel brings in (a 16-bit load per
// pixel and channel keeps the memory pipeline busy for longer than everything else in this kernel).
template <int LAYOUT, bool PAIR>
__global__ void __launch_bounds__(256, 2)
conv_mfma_kernel(const MfmaArgs a)
{
    constexpr int NBW = 1;          // pixel blocks per wave
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
    // input coordinates of staged element (0, 0); with PAIR the column is rounded down to an even one
    // and the pixels' own columns are `shift` further right
    const int iy0 = oy0 * a.stride - 1;
    const int shift = PAIR ? ((ox0 * a.stride - 1) & 1) : 0;
    const int ix0 = ox0 * a.stride - 1 - shift;
    const int fb = fg * a.mt + wm;                                     // this wave's block of 32 filters
    const bool fb_ok = fb * 32 < a.fpad;
    const int npix = a.tn * a.th * a.tw;
    const int tile_pix = a.in_h * a.in_w;                              // staged pixels per image
    const int all_pix = a.tn * tile_pix;

    // the pixel of this lane in each of the wave's pixel blocks, as an element offset into the staged tile
    const int col = lane & 31, kg = lane >> 5;
    int poff[NBW];
    int nbw = 0;
#pragma unroll
    for (int j = 0; j < NBW; ++j) {
        const int blk = wn + j * wn_count;
        if (blk < a.nb) nbw = j + 1;
        const int p = min(blk * 32 + col, npix - 1);
        const int pi = p / (a.th * a.tw), pr = p - pi * (a.th * a.tw);
        const int py = pr / a.tw, px = pr - py * a.tw;
        poff[j] = ((pi * a.in_h + py * a.stride) * a.in_w + px * a.stride + shift) * kPitch + kg * 8;
    }
    nbw = __builtin_amdgcn_readfirstlane(nbw);

    f32x16 acc[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j) acc[j] = 0.0f;

    // ---- what this thread stages: the 32 channels of kPixPerThread staged pixels, the same for every block ----
    int src[kPixPerThread];         // element offset of (channel 0, pixel) in the input; -1 outside the image or the tile
    int dst[kPixPerThread];         // element offset of the pixel in the staged tile; -1 beyond the tile
#pragma unroll
    for (int i = 0; i < kPixPerThread; ++i) {
        // PAIR: one item of two pixels (the second array entries stay unused)
        if (PAIR && i > 0) { src[i] = -1; dst[i] = -1; continue; }
        const int pix = PAIR ? 2 * int(threadIdx.x) : int(threadIdx.x) + 256 * i;
        const int pi = pix / tile_pix, pr = pix - pi * tile_pix;
        const int ry = pr / a.in_w, rx = pr - ry * a.in_w;
        const int img = img0 + pi, iy = iy0 + ry, ix = ix0 + rx;
        const bool ok = pix < all_pix && img < a.n && iy >= 0 && iy < a.h && ix >= 0 && ix < a.w;
        // (the input holds fewer than 2^31 bytes: the launcher sends larger ones to the vector kernel)
        if (LAYOUT == PCONV_NCHW) src[i] = ok ? (img * a.c_in * a.h + iy) * a.w + ix : -1;
        else src[i] = ok ? ((img * a.h + iy) * a.w + ix) * a.c_in : -1;
        dst[i] = pix < all_pix ? pix * kPitch : -1;
    }
    const int plane = a.h * a.w;
    const bool vec8 = LAYOUT == PCONV_NHWC && (a.c_in & 7) == 0;
    // The input as a buffer resource: a load whose per-lane byte offset lies beyond the tensor reads
    // nothing and returns zero, which is what a staged pixel outside the image must hold (no branch);
    // the channel is a uniform offset on top (it is not part of the range check).
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(a.x), 0, int(a.x_bytes), 0x00020000);
    constexpr int kBeyond = int(0x80000000u);
    // registers of a staged pixel: 32 channels = 16 dwords
    auto load_block = [&](int cb, uint32_t (&xr)[kPixPerThread][16]) {
        const int c0 = cb * 32;
        const bool whole = c0 + 32 <= a.c_in;          // (uniform) all 32 channels exist
#pragma unroll
        for (int i = 0; i < kPixPerThread; ++i) {
            const int voff = src[i] >= 0 ? src[i] * 2 : kBeyond;
            if (PAIR) {
                // registers 0..15: pixel 0, channels in pairs; 16..31 would be pixel 1: xr[1]
                if (i > 0) continue;
                const int cstep = plane * 2;
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    // (a channel beyond c_in, in the last block only: nothing is read)
                    const int v0 = (whole || c0 + 2 * k < a.c_in) ? voff : kBeyond;
                    const int v1 = (whole || c0 + 2 * k + 1 < a.c_in) ? voff : kBeyond;
                    const uint32_t e = __builtin_amdgcn_raw_buffer_load_b32(xrs, v0, (c0 + 2 * k) * cstep, 0);
                    const uint32_t o = __builtin_amdgcn_raw_buffer_load_b32(xrs, v1, (c0 + 2 * k + 1) * cstep, 0);
                    xr[0][k] = __builtin_amdgcn_perm(o, e, 0x05040100u);      // low halves: the first pixel
                    xr[1][k] = __builtin_amdgcn_perm(o, e, 0x07060302u);      // high halves: its right neighbour
                }
            } else if (LAYOUT == PCONV_NHWC && vec8 && whole) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u32x4 u = __builtin_amdgcn_raw_buffer_load_b128(xrs, voff, (c0 + 8 * k) * 2, 0);
                    xr[i][4 * k] = u.x; xr[i][4 * k + 1] = u.y; xr[i][4 * k + 2] = u.z; xr[i][4 * k + 3] = u.w;
                }
            } else if (whole) {
                const int cstep = LAYOUT == PCONV_NCHW ? plane * 2 : 2;          // bytes from one channel to the next
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const uint32_t lo = __builtin_amdgcn_raw_buffer_load_b16(xrs, voff, (c0 + 2 * k) * cstep, 0);
                    const uint32_t hi = __builtin_amdgcn_raw_buffer_load_b16(xrs, voff, (c0 + 2 * k + 1) * cstep, 0);
                    xr[i][k] = lo | (hi << 16);
                }
            } else {
                // the last, partial block of channels: channels beyond c_in are staged as zero
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    uint32_t lo = 0, hi = 0;
                    if (src[i] >= 0) {
                        const size_t e = LAYOUT == PCONV_NCHW ? size_t(src[i]) + size_t(c0 + 2 * k) * plane
                                                              : size_t(src[i]) + c0 + 2 * k;
                        const size_t step = LAYOUT == PCONV_NCHW ? size_t(plane) : size_t(1);
                        if (c0 + 2 * k < a.c_in) lo = a.x[e];
                        if (c0 + 2 * k + 1 < a.c_in) hi = a.x[e + step];
                    }
                    xr[i][k] = lo | (hi << 16);
                }
            }
        }
    };
    auto store_block = [&](const uint32_t (&xr)[kPixPerThread][16]) {
#pragma unroll
        for (int i = 0; i < kPixPerThread; ++i)
            if (dst[PAIR ? 0 : i] >= 0) {
                u32x4 *lp = reinterpret_cast<u32x4 *>(tile + (PAIR ? dst[0] + i * kPitch : dst[i]));
#pragma unroll
                for (int k = 0; k < 4; ++k) lp[k] = u32x4{xr[i][4 * k], xr[i][4 * k + 1], xr[i][4 * k + 2], xr[i][4 * k + 3]};
            }
    };
    const int cb16n = a.cb32 * 2;
    auto weight_frag = [&](int cb, int q, uint32_t nzb) -> u32x4 {
        if (!((nzb >> q) & 1u)) return u32x4{0u, 0u, 0u, 0u};
        const int tap = q >> 1, half = q & 1;
        const size_t e = ((size_t(tap) * cb16n + cb * 2 + half) * a.fpad + fb * 32 + col) * 16 + kg * 8;
        return *reinterpret_cast<const u32x4 *>(a.wd + e);
    };
    auto block_map = [&](int cb) -> uint32_t { return fb_ok ? a.nz[cb * (a.fpad / 32) + fb] : 0u; };

    // Weight fragments: a window of kWin fragments ahead of the one in use (fragment = (block, tap,
    // half), in the order they are used); a fragment that has been used is replaced at once by the
    // one kWin places later, which may belong to the next block of channels.
    constexpr int kWin = 6;
    static_assert(18 % kWin == 0, "the window slot of a fragment must not depend on the block");
    u32x4 wf[kWin];
    uint32_t nzbits = block_map(0);
    uint32_t nz_n = a.cb32 > 1 ? block_map(1) : 0u;
    {
        uint32_t xr[kPixPerThread][16];
#pragma unroll
        for (int q = 0; q < kWin; ++q) wf[q] = weight_frag(0, q, nzbits);
        load_block(0, xr);
        store_block(xr);
    }
    __syncthreads();
    for (int cb = 0; cb < a.cb32; ++cb) {
        const bool more = cb + 1 < a.cb32;
        uint32_t xr[kPixPerThread][16];
        if (more) load_block(cb + 1, xr);              // on its way during the matrix instructions below
        // ---- nine taps x two halves of 16 channels ----
        // Two forms of the same loop: straight-line when every fragment of the block holds weights
        // (the usual case; the LDS reads then run ahead of the matrix instructions), and with a
        // (wave-uniform) test per fragment otherwise, which skips the empty ones.
        const bool all_present = nzbits == 0x3FFFFu && nbw == NBW;
        auto tap_offset = [&](int q) { return (((q >> 1) / 3) * a.in_w + ((q >> 1) % 3)) * kPitch + (q & 1) * 16; };
        auto next_weights = [&](int q) {
            if (q + kWin < 18) wf[q % kWin] = weight_frag(cb, q + kWin, nzbits);
            else if (more) wf[q % kWin] = weight_frag(cb + 1, q + kWin - 18, nz_n);
        };
        if (all_present) {
            // the pixel fragments of tap q + 1 are read while the matrix instructions of tap q run
            bf16x8 xb[2][NBW];
#pragma unroll
            for (int j = 0; j < NBW; ++j) xb[0][j] = *reinterpret_cast<const bf16x8 *>(tile + poff[j] + tap_offset(0));
#pragma unroll
            for (int q = 0; q < 18; ++q) {
                if (q + 1 < 18) {
#pragma unroll
                    for (int j = 0; j < NBW; ++j)
                        xb[(q + 1) & 1][j] = *reinterpret_cast<const bf16x8 *>(tile + poff[j] + tap_offset(q + 1));
                }
                const bf16x8 wa = __builtin_bit_cast(bf16x8, wf[q % kWin]);
#pragma unroll
                for (int j = 0; j < NBW; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xb[q & 1][j], acc[j], 0, 0, 0);
                next_weights(q);
                __builtin_amdgcn_sched_barrier(0);     // keep this order: no more reads in flight than two taps' worth
            }
        } else {
#pragma unroll
            for (int q = 0; q < 18; ++q) {
                if ((nzbits >> q) & 1u) {
                    const bf16x8 wa = __builtin_bit_cast(bf16x8, wf[q % kWin]);
#pragma unroll
                    for (int j = 0; j < NBW; ++j) {
                        if (j < nbw) {
                            const bf16x8 xb = *reinterpret_cast<const bf16x8 *>(tile + poff[j] + tap_offset(q));
                            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xb, acc[j], 0, 0, 0);
                        }
                    }
                }
                next_weights(q);
            }
        }
        if (more) {
            __syncthreads();                           // everybody has finished reading this block's tile
            store_block(xr);
            nzbits = nz_n;
            nz_n = cb + 2 < a.cb32 ? block_map(cb + 2) : 0u;
            __syncthreads();
        }
    }

    // ---- epilogue: bias, ReLU, round to bf16, store ----
    // register v of a lane holds filter 8 * (v / 4) + 4 * (lane / 32) + v % 4 of the block, pixel lane % 32
    if (!fb_ok) return;
#pragma unroll
    for (int j = 0; j < NBW; ++j) {
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

bool mfma_supported(const pconv_handle *h, int dtype, int n, int hin, int win)
{
    // (the kernel addresses its input through a buffer resource with 32-bit byte offsets)
    return dtype == PCONV_BF16 && h->wdtype == PCONV_BF16 && h->d_wdense != nullptr &&
           int64_t(n) * h->c_in * hin * win * 2 < (int64_t(1) << 31);
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
    a.x_bytes = uint32_t(int64_t(n) * h->c_in * hin * win * 2);
    a.cb32 = (h->c_in + 31) / 32; a.fpad = (h->c_out + 31) / 32 * 32;
    const bool pair = layout == PCONV_NCHW && win % 2 == 0;
    // rows and columns of the staged input tile (with PAIR one more column, rounded up to an even count)
    auto staged_h = [&](int th) { return (th - 1) * stride + 3; };
    auto staged_w = [&](int tw) { const int w0 = (tw - 1) * stride + 3; return pair ? (w0 + 2) & ~1 : w0; };
    auto lds_bytes = [&](int tn, int th, int tw) { return size_t(tn) * staged_h(th) * staged_w(tw) * kPitch * 2; };
    // Tile search.  Every wave holds exactly one block of 32 pixels (more blocks per wave were
    // measured slower: the register allocation of the larger kernels spills), so a tile has at
    // most 128 / MT pixels.  Measured on the ResNet-50 shapes, tiles that keep all four waves busy
    // take about the same time; what separates them is how much of the 32-pixel blocks and of the
    // tile grid holds real pixels, and how many staged pixels (halo included) a tile needs per
    // output pixel.  Score = product of those efficiencies; ties go to more filters per workgroup
    // (the tile is staged once for all of them).
    int best_tn = 1, best_th = 1, best_tw = std::min(a.wo, 8), best_mt = 1;
    double best_score = -1.0;
    for (int mt = 4; mt >= 1; mt /= 2) {
        if (mt > 1 && (mt / 2) * 32 >= a.fpad) continue;     // no more filter blocks than the layer has
        const int max_pix = 32 * (4 / mt);
        for (int tw = std::min(a.wo, max_pix); tw >= 1; --tw) {
            if (tw < a.wo && tw > 8 && (a.wo % tw) > 0 && (a.wo % tw) < tw / 2) continue;   // (prune very ragged splits)
            for (int th = 1; th <= a.ho && th * tw <= max_pix; ++th) {
                for (int tn = 1; tn <= n && tn * th * tw <= max_pix; ++tn) {
                    if (tn > 1 && (th < a.ho || tw < a.wo)) break;            // several images only as whole images
                    const int staged = tn * staged_h(th) * staged_w(tw);
                    if (staged > kMaxTilePixels || lds_bytes(tn, th, tw) > size_t(kLdsLimit)) break;
                    const int npix = tn * th * tw;
                    const double fill = double(npix) / max_pix;
                    const double grid = (double(n) / (double((n + tn - 1) / tn) * tn)) * (double(a.ho) / (double((a.ho + th - 1) / th) * th)) *
                                        (double(a.wo) / (double((a.wo + tw - 1) / tw) * tw));
                    const double score = fill * grid / (1.0 + 0.1 * (double(staged) / npix - 1.0));
                    if (score > best_score * 1.0001) { best_score = score; best_tn = tn; best_th = th; best_tw = tw; best_mt = mt; }
                }
            }
        }
    }
    a.tn = best_tn; a.th = best_th; a.tw = best_tw; a.mt = best_mt;
    a.tiles_n = (n + a.tn - 1) / a.tn; a.tiles_y = (a.ho + a.th - 1) / a.th; a.tiles_x = (a.wo + a.tw - 1) / a.tw;
    a.fgroups = (a.fpad / 32 + a.mt - 1) / a.mt;
    a.nb = (a.tn * a.th * a.tw + 31) / 32;
    a.in_h = staged_h(a.th); a.in_w = staged_w(a.tw);
    const size_t lds = lds_bytes(a.tn, a.th, a.tw);
    const int64_t wgs = int64_t(a.tiles_n) * a.tiles_y * a.tiles_x * a.fgroups;
    const int nbw = (a.nb + 4 / a.mt - 1) / (4 / a.mt);
    if (lds > size_t(kLdsLimit) || wgs > 0x7FFFFFFF || nbw > 1 || a.tn * a.in_h * a.in_w > kMaxTilePixels) {
        set_error("pconv_conv2d (matrix-core kernel): no tile fits this call");
        return PCONV_UNSUPPORTED;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid{unsigned(wgs)}, block{256};
    if (layout == PCONV_NHWC) hipLaunchKernelGGL((conv_mfma_kernel<PCONV_NHWC, false>), grid, block, lds, st, a);
    else if (pair) hipLaunchKernelGGL((conv_mfma_kernel<PCONV_NCHW, true>), grid, block, lds, st, a);
    else hipLaunchKernelGGL((conv_mfma_kernel<PCONV_NCHW, false>), grid, block, lds, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(std::string("pconv_conv2d (matrix-core kernel): ") + hipGetErrorName(e));
        return PCONV_HIP_ERROR;
    }
    return PCONV_OK;
}

}  // namespace pconv
