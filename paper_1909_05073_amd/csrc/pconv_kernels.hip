// gfx950 kernels of the PCONV library: the generic gather kernel (any mask, stride, layout,
// dtype), and the 2x2 max-pool helper.  The register-tiled fast kernel lives in
// pconv_tiled.hip.
#include <hip/hip_runtime.h>

#include "pconv_internal.h"

namespace pconv {

namespace {

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float load_act(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_act(const bf16_t *p, size_t i)
{
    return __uint_as_float(uint32_t(p[i].bits) << 16);
}
__device__ __forceinline__ void store_act(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_act(bf16_t *p, size_t i, float v)
{
    // round to nearest even; NaN kept quiet
    uint32_t u = __float_as_uint(v);
    uint32_t r = ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u)
                                                   : ((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    p[i].bits = uint16_t(r);
}

template <int LAYOUT>
__device__ __forceinline__ size_t act_at(int n, int c, int y, int x, int C, int H, int W)
{
    if (LAYOUT == PCONV_NCHW) return ((size_t(n) * C + c) * H + y) * W + x;
    return ((size_t(n) * H + y) * W + x) * C + c;
}

// One thread = one output pixel of one filter.  blockIdx.y walks the filters in reordered
// position order, so a block runs the branch-free kernel list of a single filter: the mask
// test below is uniform across the block (paper: kernels of one pattern grouped in a filter
// remove per-kernel branching).  Eq. (1), zero padding by bounds test.
template <typename T, int LAYOUT>
__global__ void __launch_bounds__(256)
conv_generic_kernel(const T *__restrict__ x, T *__restrict__ y, const float *__restrict__ bias,
                    const int32_t *__restrict__ perm, const uint32_t *__restrict__ row_ptr,
                    const uint32_t *__restrict__ kern, const uint32_t *__restrict__ val_ptr,
                    const float *__restrict__ vals, int n_img, int c_in, int h, int w, int c_out,
                    int ho, int wo, int stride, int relu)
{
    const int64_t pix = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t total = int64_t(n_img) * ho * wo;
    if (pix >= total) return;
    const int ox = int(pix % wo), oy = int((pix / wo) % ho), n = int(pix / (int64_t(wo) * ho));
    const int pos = blockIdx.y;
    const int f = perm[pos];
    float acc = bias ? bias[f] : 0.0f;
    const uint32_t k_end = row_ptr[pos + 1];
    for (uint32_t k = row_ptr[pos]; k < k_end; ++k) {
        const uint32_t km = kern[k];
        const int c = int(km & 0xFFFFu);
        const uint32_t mask = km >> 16;
        uint32_t v = val_ptr[k];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (mask & (1u << t)) {
                const int iy = oy * stride + t / 3 - 1, ix = ox * stride + t % 3 - 1;
                const float wv = vals[v++];
                if (iy >= 0 && iy < h && ix >= 0 && ix < w)
                    acc = fmaf(wv, load_act(x, act_at<LAYOUT>(n, c, iy, ix, c_in, h, w)), acc);
            }
        }
    }
    if (relu) acc = fmaxf(acc, 0.0f);
    store_act(y, act_at<LAYOUT>(n, f, oy, ox, c_out, ho, wo), acc);
}

template <typename T, int LAYOUT>
__global__ void __launch_bounds__(256)
maxpool2x2_kernel(const T *__restrict__ x, T *__restrict__ y, int n_img, int c, int h, int w)
{
    const int ho = h / 2, wo = w / 2;
    const int64_t total = int64_t(n_img) * c * ho * wo;
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int n, ch, oy, ox;
    if (LAYOUT == PCONV_NCHW) {
        ox = int(i % wo); oy = int((i / wo) % ho); ch = int((i / (int64_t(wo) * ho)) % c);
        n = int(i / (int64_t(wo) * ho * c));
    } else {
        ch = int(i % c); ox = int((i / c) % wo); oy = int((i / (int64_t(c) * wo)) % ho);
        n = int(i / (int64_t(c) * wo * ho));
    }
    float m = load_act(x, act_at<LAYOUT>(n, ch, 2 * oy, 2 * ox, c, h, w));
    m = fmaxf(m, load_act(x, act_at<LAYOUT>(n, ch, 2 * oy, 2 * ox + 1, c, h, w)));
    m = fmaxf(m, load_act(x, act_at<LAYOUT>(n, ch, 2 * oy + 1, 2 * ox, c, h, w)));
    m = fmaxf(m, load_act(x, act_at<LAYOUT>(n, ch, 2 * oy + 1, 2 * ox + 1, c, h, w)));
    store_act(y, act_at<LAYOUT>(n, ch, oy, ox, c, ho, wo), m);
}

int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(std::string(what) + ": launch failed: " + hipGetErrorName(e));
        return PCONV_HIP_ERROR;
    }
    return PCONV_OK;
}

}  // namespace

int launch_conv_generic(const pconv_handle *h, const void *x, void *y, const float *bias, int n,
                        int hin, int win, int stride, int layout, int dtype, int relu, void *stream)
{
    const int ho = (hin + 2 - 3) / stride + 1, wo = (win + 2 - 3) / stride + 1;
    const int64_t pixels = int64_t(n) * ho * wo;
    dim3 grid(unsigned((pixels + 255) / 256), unsigned(h->c_out));
    dim3 block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
#define PCONV_LAUNCH(T, L)                                                                         \
    hipLaunchKernelGGL((conv_generic_kernel<T, L>), grid, block, 0, st, static_cast<const T *>(x), \
                       static_cast<T *>(y), bias, h->d_perm, h->d_row_ptr, h->d_kern,              \
                       h->d_val_ptr, h->d_vals, n, h->c_in, hin, win, h->c_out, ho, wo, stride, relu)
    if (dtype == PCONV_F32) {
        if (layout == PCONV_NCHW) PCONV_LAUNCH(float, PCONV_NCHW); else PCONV_LAUNCH(float, PCONV_NHWC);
    } else {
        if (layout == PCONV_NCHW) PCONV_LAUNCH(bf16_t, PCONV_NCHW); else PCONV_LAUNCH(bf16_t, PCONV_NHWC);
    }
#undef PCONV_LAUNCH
    return check_launch("pconv_conv2d (generic kernel)");
}

int launch_maxpool2x2(const void *x, void *y, int n, int c, int h, int w, int layout, int dtype,
                      void *stream)
{
    const int64_t total = int64_t(n) * c * (h / 2) * (w / 2);
    if (total == 0) return PCONV_OK;
    dim3 grid(unsigned((total + 255) / 256)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
#define PCONV_LAUNCH(T, L)                                                                       \
    hipLaunchKernelGGL((maxpool2x2_kernel<T, L>), grid, block, 0, st, static_cast<const T *>(x), \
                       static_cast<T *>(y), n, c, h, w)
    if (dtype == PCONV_F32) {
        if (layout == PCONV_NCHW) PCONV_LAUNCH(float, PCONV_NCHW); else PCONV_LAUNCH(float, PCONV_NHWC);
    } else {
        if (layout == PCONV_NCHW) PCONV_LAUNCH(bf16_t, PCONV_NCHW); else PCONV_LAUNCH(bf16_t, PCONV_NHWC);
    }
#undef PCONV_LAUNCH
    return check_launch("pconv_maxpool2x2");
}

namespace {

// 64 independent accumulators per lane, all operands in vector registers (an FMA with a scalar
// operand issues at half the rate on this chip), 16 waves per compute unit: the rate the tiled
// kernel's inner loops could reach with nothing else to do.
__global__ void __launch_bounds__(1024) fma_peak_kernel(float *out, int iters)
{
    float acc[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] = float(threadIdx.x + i);
    float w0 = 1.0f + 1e-7f * float(threadIdx.x), w1 = 1.0f - 1e-7f * float(threadIdx.x);
    float x0 = 1e-3f * float(threadIdx.x & 7), x1 = x0 + 0.5f;
    asm volatile("" : "+v"(w0), "+v"(w1), "+v"(x0), "+v"(x1));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 64; i += 2) {
            acc[i] = fmaf(w0, x0, acc[i]);
            acc[i + 1] = fmaf(w1, x1, acc[i + 1]);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 64; ++i) s += acc[i];
    out[size_t(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

}  // namespace

int measure_fma_peak(double *tflops)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        set_error("pconv_debug_measure_fma_peak: no device");
        return PCONV_HIP_ERROR;
    }
    const int blocks = cus * 4, threads = 1024, iters = 4000;
    float *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&out), size_t(blocks) * threads * sizeof(float));
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    float best_ms = 0.0f;
    for (int rep = 0; e == hipSuccess && rep < 3; ++rep) {
        e = hipEventRecord(e0, nullptr);
        if (e != hipSuccess) break;
        hipLaunchKernelGGL(fma_peak_kernel, dim3(blocks), dim3(threads), 0, nullptr, out, iters);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess && rep > 0 && (best_ms == 0.0f || ms < best_ms)) best_ms = ms;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (out) (void)hipFree(out);
    if (e != hipSuccess || best_ms <= 0.0f) {
        set_error(std::string("pconv_debug_measure_fma_peak: ") + hipGetErrorName(e));
        return PCONV_HIP_ERROR;
    }
    *tflops = 2.0 * 64 * iters * double(blocks) * threads / (double(best_ms) * 1e-3) / 1e12;
    return PCONV_OK;
}

}  // namespace pconv
