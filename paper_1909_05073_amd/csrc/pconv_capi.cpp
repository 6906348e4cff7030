// extern "C" boundary of the PCONV library (see include/pconv.h for the contract).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstring>
#include <new>

#include "pconv_internal.h"
#include "pconv_tiled_codes.h"

namespace pconv {

static thread_local std::string g_error;
void set_error(const std::string &msg) { g_error = msg; }
const char *get_error() { return g_error.c_str(); }

static std::atomic<int> g_policy{0};

namespace {

int hip_fail(const char *what, hipError_t e)
{
    set_error(std::string(what) + ": " + hipGetErrorName(e) + " (" + hipGetErrorString(e) + ")");
    return e == hipErrorOutOfMemory ? PCONV_OOM : PCONV_HIP_ERROR;
}

template <typename T>
int upload(T *&dst, const T *src, size_t count, int64_t &bytes)
{
    dst = nullptr;
    const size_t sz = (count ? count : 1) * sizeof(T);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&dst), sz);
    if (e != hipSuccess) return hip_fail("pconv_pack: hipMalloc", e);
    bytes += int64_t(sz);
    if (count) {
        e = hipMemcpy(dst, src, count * sizeof(T), hipMemcpyHostToDevice);
        if (e != hipSuccess) return hip_fail("pconv_pack: hipMemcpy", e);
    }
    return PCONV_OK;
}

void release_device(pconv_handle *h)
{
    void *ptrs[] = {h->d_perm, h->d_row_ptr, h->d_kern, h->d_val_ptr, h->d_vals,
                    h->d_slot_filter, h->d_chan_ptr, h->d_meta, h->d_w4, h->d_flags, h->d_wdense, h->d_wnz};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (h->h_err) (void)hipHostFree(h->h_err);
    h->h_err = nullptr;
}

// Reports (once) that a kernel launched earlier on this handle gave up one of its bounded waits.
int take_async_error(const pconv_handle *h, const char *who)
{
    if (!h->h_err) return PCONV_OK;
    const uint32_t code = __atomic_load_n(h->h_err, __ATOMIC_ACQUIRE);
    if (code == 0) return PCONV_OK;
    __atomic_store_n(h->h_err, 0u, __ATOMIC_RELEASE);
    set_error(std::string(who) + ": an earlier kernel on this handle ran out of a bounded wait (code " +
              std::to_string(code) + "); the outputs of that call are invalid (NaN where the kernel noticed)");
    return PCONV_HIP_ERROR;
}

}  // namespace
}  // namespace pconv

using namespace pconv;

extern "C" {

const char *pconv_last_error(void) { return get_error(); }

int pconv_set_kernel_policy(int policy)
{
    if (policy < 0 || policy > 3) { set_error("pconv_set_kernel_policy: policy must be 0, 1, 2 or 3"); return PCONV_INVALID_ARG; }
    g_policy.store(policy);
    return PCONV_OK;
}

int pconv_debug_set_tiling(int waves, int ks_log2, int split_units)
{
    set_tiled_tuning(waves, ks_log2, split_units);
    return PCONV_OK;
}

int pconv_debug_set_spin_limit(int limit)
{
    set_tiled_spin_limit(limit);
    return PCONV_OK;
}

int pconv_get_async_error(const pconv_handle *h)
{
    if (!h) { set_error("pconv_get_async_error: null pointer argument"); return PCONV_INVALID_ARG; }
    return take_async_error(h, "pconv_get_async_error");
}

static int pack_impl(const float *w_dense, const uint8_t *pattern_id, const uint8_t *conn,
                     const uint16_t *table, int num_patterns, int c_out, int c_in,
                     pconv_dtype weight_dtype, pconv_handle **out, bool to_device)
{
    if (out) *out = nullptr;
    if (!w_dense || !pattern_id || !conn || !table || !out) { set_error("pconv_pack: null pointer argument"); return PCONV_INVALID_ARG; }
    if (num_patterns < 1 || num_patterns > PCONV_MAX_PATTERNS) { set_error("pconv_pack: num_patterns must be 1..16"); return PCONV_INVALID_ARG; }
    if (c_out < 1 || c_out > 65535 || c_in < 1 || c_in > 65535) { set_error("pconv_pack: c_out and c_in must be 1..65535"); return PCONV_INVALID_ARG; }
    if (weight_dtype != PCONV_F32 && weight_dtype != PCONV_BF16) { set_error("pconv_pack: unknown weight_dtype"); return PCONV_INVALID_ARG; }
    pconv_handle *h = nullptr;
    try {
        h = new pconv_handle();
        h->c_out = c_out; h->c_in = c_in; h->np = num_patterns; h->wdtype = int(weight_dtype);
        std::memcpy(h->table, table, sizeof(uint16_t) * size_t(num_patterns));
        int rc = build_canonical(w_dense, pattern_id, conn, table, num_patterns, c_out, c_in,
                                 int(weight_dtype), h->canon);
        if (rc != PCONV_OK) { delete h; return rc; }
        h->K = int64_t(h->canon.cin.size());
        h->nnz = int64_t(h->canon.vals_bits.size());

        build_tiled_stream(h->canon, table, num_patterns, c_out, c_in, h->tiled);
        if (!to_device) { *out = h; return PCONV_OK; }
        hipError_t e = hipGetDevice(&h->device);
        if (e != hipSuccess) { delete h; return hip_fail("pconv_pack: hipGetDevice", e); }

        std::vector<int32_t> perm32(h->canon.perm.begin(), h->canon.perm.end());
        std::vector<uint32_t> kern(size_t(h->K));
        for (int64_t k = 0; k < h->K; ++k)
            kern[size_t(k)] = uint32_t(h->canon.cin[size_t(k)]) | (uint32_t(table[h->canon.pat[size_t(k)]]) << 16);
        rc = upload(h->d_perm, perm32.data(), perm32.size(), h->device_bytes);
        if (rc == PCONV_OK) rc = upload(h->d_row_ptr, h->canon.row_ptr.data(), h->canon.row_ptr.size(), h->device_bytes);
        if (rc == PCONV_OK) rc = upload(h->d_kern, kern.data(), kern.size(), h->device_bytes);
        if (rc == PCONV_OK) rc = upload(h->d_val_ptr, h->canon.val_ptr.data(), size_t(h->K), h->device_bytes);
        if (rc == PCONV_OK)
            rc = upload(h->d_vals, reinterpret_cast<const float *>(h->canon.vals_bits.data()),
                        h->canon.vals_bits.size(), h->device_bytes);
        if (rc == PCONV_OK) rc = upload(h->d_slot_filter, h->tiled.slot_filter.data(), h->tiled.slot_filter.size(), h->device_bytes);
        if (rc == PCONV_OK) rc = upload(h->d_chan_ptr, h->tiled.chan_ptr.data(), h->tiled.chan_ptr.size(), h->device_bytes);
        // (the tiled kernel keeps a record index in 24 bits: a longer stream stays off the device,
        //  and the layer runs on the general kernels)
        if (rc == PCONV_OK && h->tiled.meta.size() < (size_t(1) << 24))
            rc = upload(h->d_meta, h->tiled.meta.data(), h->tiled.meta.size(), h->device_bytes);
        if (rc == PCONV_OK) rc = upload(h->d_w4, h->tiled.w4.data(), h->tiled.w4.size(), h->device_bytes);
        if (rc == PCONV_OK && weight_dtype == PCONV_BF16) {
            std::vector<uint16_t> wd; std::vector<uint32_t> nz;
            build_dense_taps(h->canon, table, c_out, c_in, wd, nz);
            rc = upload(h->d_wdense, wd.data(), wd.size(), h->device_bytes);
            if (rc == PCONV_OK) rc = upload(h->d_wnz, nz.data(), nz.size(), h->device_bytes);
        }
        if (rc == PCONV_OK) {
            const std::vector<uint32_t> zeros(size_t(kFlagSlots) * kFlagWords, 0u);
            rc = upload(h->d_flags, zeros.data(), zeros.size(), h->device_bytes);
        }
        if (rc == PCONV_OK) {
            e = hipHostMalloc(reinterpret_cast<void **>(&h->h_err), 64, hipHostMallocDefault);
            if (e != hipSuccess) { h->h_err = nullptr; rc = hip_fail("pconv_pack: hipHostMalloc", e); }
            else std::memset(h->h_err, 0, 64);
        }
        if (rc == PCONV_OK) {
            if (hipDeviceGetAttribute(&h->cus, hipDeviceAttributeMultiprocessorCount, h->device) != hipSuccess || h->cus <= 0)
                h->cus = 256;
        }
        if (rc != PCONV_OK) { release_device(h); delete h; return rc; }
    } catch (const std::bad_alloc &) {
        if (h) { release_device(h); delete h; }
        set_error("pconv_pack: out of host memory");
        return PCONV_OOM;
    } catch (const std::exception &ex) {
        if (h) { release_device(h); delete h; }
        set_error(std::string("pconv_pack: ") + ex.what());
        return PCONV_INVALID_ARG;
    }
    *out = h;
    return PCONV_OK;
}

int pconv_pack(const float *w_dense, const uint8_t *pattern_id, const uint8_t *conn,
               const uint16_t *table, int num_patterns, int c_out, int c_in,
               pconv_dtype weight_dtype, pconv_handle **out)
{
    return pack_impl(w_dense, pattern_id, conn, table, num_patterns, c_out, c_in, weight_dtype, out, true);
}

int pconv_project(const float *w_dense, const uint16_t *table, int num_patterns, int c_out, int c_in,
                  int64_t keep_kernels, uint8_t *pattern_id_out, uint8_t *conn_out)
{
    if (!w_dense || !table || !pattern_id_out || !conn_out) { set_error("pconv_project: null pointer argument"); return PCONV_INVALID_ARG; }
    if (num_patterns < 1 || num_patterns > PCONV_MAX_PATTERNS) { set_error("pconv_project: num_patterns must be 1..16"); return PCONV_INVALID_ARG; }
    if (c_out < 1 || c_out > 65535 || c_in < 1 || c_in > 65535) { set_error("pconv_project: c_out and c_in must be 1..65535"); return PCONV_INVALID_ARG; }
    if (keep_kernels < 0 || keep_kernels > int64_t(c_out) * c_in) { set_error("pconv_project: keep_kernels must be 0..c_out*c_in"); return PCONV_INVALID_ARG; }
    for (int p = 0; p < num_patterns; ++p)
        if (table[p] == 0 || table[p] > 0x1FF) { set_error("pconv_project: table entries must be non-zero 9-bit masks"); return PCONV_INVALID_ARG; }
    try {
        return project_weights(w_dense, table, num_patterns, c_out, c_in, keep_kernels, pattern_id_out, conn_out);
    } catch (const std::bad_alloc &) {
        set_error("pconv_project: out of host memory");
        return PCONV_OOM;
    }
}

int pconv_debug_pack_host(const float *w_dense, const uint8_t *pattern_id, const uint8_t *conn,
                          const uint16_t *table, int num_patterns, int c_out, int c_in,
                          pconv_dtype weight_dtype, pconv_handle **out)
{
    return pack_impl(w_dense, pattern_id, conn, table, num_patterns, c_out, c_in, weight_dtype, out, false);
}

void pconv_free(pconv_handle *h)
{
    if (!h) return;
    release_device(h);
    delete h;
}

int pconv_get_info(const pconv_handle *h, pconv_info *info)
{
    if (!h || !info) { set_error("pconv_get_info: null pointer argument"); return PCONV_INVALID_ARG; }
    info->c_out = h->c_out; info->c_in = h->c_in; info->num_patterns = h->np;
    info->weight_dtype = h->wdtype; info->kept_kernels = h->K; info->nnz = h->nnz;
    info->device_bytes = h->device_bytes; info->fast_path = h->d_meta ? 1 : 0; info->reserved = 0;
    return PCONV_OK;
}

static int conv2d_impl(const pconv_handle *h, const void *x_dev, void *y_dev, const float *bias_dev,
                       int n, int h_in, int w_in, int stride, int pad, pconv_layout layout,
                       pconv_dtype act_dtype, int fuse_relu, void *hip_stream, bool static_scratch)
{
    if (!h || !x_dev || !y_dev) { set_error("pconv_conv2d: null pointer argument"); return PCONV_INVALID_ARG; }
    if (x_dev == y_dev) { set_error("pconv_conv2d: y_dev must not alias x_dev"); return PCONV_INVALID_ARG; }
    if (n <= 0 || h_in <= 0 || w_in <= 0) { set_error("pconv_conv2d: n, h_in and w_in must be positive"); return PCONV_INVALID_ARG; }
    if (stride != 1 && stride != 2) { set_error("pconv_conv2d: stride must be 1 or 2"); return PCONV_INVALID_ARG; }
    if (pad != 1) { set_error("pconv_conv2d: pad must be 1"); return PCONV_INVALID_ARG; }
    if (layout != PCONV_NCHW && layout != PCONV_NHWC) { set_error("pconv_conv2d: unknown layout"); return PCONV_INVALID_ARG; }
    if (h->device < 0) { set_error("pconv_conv2d: handle was packed on the host only and holds no device data"); return PCONV_INVALID_ARG; }
    if (int(act_dtype) != h->wdtype) { set_error("pconv_conv2d: act_dtype differs from the handle's weight dtype"); return PCONV_INVALID_ARG; }
    { int dev = -1; if (hipGetDevice(&dev) == hipSuccess && dev != h->device) { set_error("pconv_conv2d: the handle was packed for another device than the current one"); return PCONV_INVALID_ARG; } }
    const int ho = (h_in - 1) / stride + 1, wo = (w_in - 1) / stride + 1;
    const int64_t lim = (int64_t(1) << 31) - 1;
    if (int64_t(n) * h->c_in * h_in * w_in > lim || int64_t(n) * h->c_out * ho * wo > lim) {
        set_error("pconv_conv2d: tensors of 2^31 elements or more are not supported");
        return PCONV_INVALID_ARG;
    }
    if (const int rc = take_async_error(h, "pconv_conv2d")) return rc;
    const int policy = g_policy.load();
    const bool can_mfma = mfma_supported(h, int(act_dtype), n, h_in, w_in);
    if (policy == 3 && !can_mfma) { set_error("pconv_conv2d: the matrix-core kernel serves bf16 handles with inputs below 2 GiB only"); return PCONV_UNSUPPORTED; }
    if (can_mfma && (policy == 3 || (policy == 0 && mfma_preferred(h))))
        return launch_conv_mfma(h, x_dev, y_dev, bias_dev, n, h_in, w_in, stride, int(layout), fuse_relu ? 1 : 0, hip_stream);
    const bool can_tile = tiled_supported(h, n, h_in, w_in, stride, int(layout), int(act_dtype));
    if (policy == 2 && !can_tile) { set_error("pconv_conv2d: register-tiled kernel not available for this call"); return PCONV_UNSUPPORTED; }
    if (can_tile && (policy == 2 || (policy == 0 && tiled_preferred(h_in, w_in, stride))))
        return launch_conv_tiled(h, x_dev, y_dev, bias_dev, n, h_in, w_in, stride, int(layout),
                                 int(act_dtype), fuse_relu ? 1 : 0, 0, hip_stream, static_scratch);
    return launch_conv_generic(h, x_dev, y_dev, bias_dev, n, h_in, w_in, stride, int(layout),
                               int(act_dtype), fuse_relu ? 1 : 0, hip_stream);
}

int pconv_conv2d(const pconv_handle *h, const void *x_dev, void *y_dev, const float *bias_dev,
                 int n, int h_in, int w_in, int stride, int pad, pconv_layout layout,
                 pconv_dtype act_dtype, int fuse_relu, void *hip_stream)
{
    return conv2d_impl(h, x_dev, y_dev, bias_dev, n, h_in, w_in, stride, pad, layout, act_dtype, fuse_relu,
                       hip_stream, false);
}

int pconv_conv2d_static(const pconv_handle *h, const void *x_dev, void *y_dev, const float *bias_dev,
                        int n, int h_in, int w_in, int stride, int pad, pconv_layout layout,
                        pconv_dtype act_dtype, int fuse_relu, void *hip_stream)
{
    return conv2d_impl(h, x_dev, y_dev, bias_dev, n, h_in, w_in, stride, pad, layout, act_dtype, fuse_relu,
                       hip_stream, true);
}

int pconv_conv2d_pool2x2(const pconv_handle *h, const void *x_dev, void *y_dev, const float *bias_dev,
                         int n, int h_in, int w_in, pconv_layout layout, pconv_dtype act_dtype,
                         int fuse_relu, void *hip_stream)
{
    if (!h || !x_dev || !y_dev) { set_error("pconv_conv2d_pool2x2: null pointer argument"); return PCONV_INVALID_ARG; }
    if (x_dev == y_dev) { set_error("pconv_conv2d_pool2x2: y_dev must not alias x_dev"); return PCONV_INVALID_ARG; }
    if (n <= 0 || h_in <= 0 || w_in <= 0) { set_error("pconv_conv2d_pool2x2: n, h_in and w_in must be positive"); return PCONV_INVALID_ARG; }
    if (layout != PCONV_NCHW && layout != PCONV_NHWC) { set_error("pconv_conv2d_pool2x2: unknown layout"); return PCONV_INVALID_ARG; }
    if (h->device < 0) { set_error("pconv_conv2d_pool2x2: handle was packed on the host only and holds no device data"); return PCONV_INVALID_ARG; }
    if (int(act_dtype) != h->wdtype) { set_error("pconv_conv2d_pool2x2: act_dtype differs from the handle's weight dtype"); return PCONV_INVALID_ARG; }
    { int dev = -1; if (hipGetDevice(&dev) == hipSuccess && dev != h->device) { set_error("pconv_conv2d_pool2x2: the handle was packed for another device than the current one"); return PCONV_INVALID_ARG; } }
    const int64_t lim = (int64_t(1) << 31) - 1;
    if (int64_t(n) * h->c_in * h_in * w_in > lim || int64_t(n) * h->c_out * h_in * w_in > lim) {
        set_error("pconv_conv2d_pool2x2: tensors of 2^31 elements or more are not supported");
        return PCONV_INVALID_ARG;
    }
    if (const int rc = take_async_error(h, "pconv_conv2d_pool2x2")) return rc;
    if (g_policy.load() == 1 || !tiled_pool_supported(h, n, h_in, w_in, int(layout), int(act_dtype))) {
        set_error("pconv_conv2d_pool2x2: needs the register-tiled kernel with fp32 NCHW tensors of even width >= 4 "
                  "and height >= 2; use pconv_conv2d and pconv_maxpool2x2");
        return PCONV_UNSUPPORTED;
    }
    return launch_conv_tiled(h, x_dev, y_dev, bias_dev, n, h_in, w_in, 1, int(layout), int(act_dtype),
                             fuse_relu ? 1 : 0, 1, hip_stream);
}

int pconv_pool2x2_fusion(const pconv_handle *h, int n, int h_in, int w_in, pconv_layout layout, pconv_dtype act_dtype)
{
    if (!h) { set_error("pconv_pool2x2_fusion: null pointer argument"); return PCONV_INVALID_ARG; }
    if (n <= 0 || h_in <= 0 || w_in <= 0) { set_error("pconv_pool2x2_fusion: n, h_in and w_in must be positive"); return PCONV_INVALID_ARG; }
    if (h->device < 0 || int(act_dtype) != h->wdtype || g_policy.load() == 1 ||
        !tiled_pool_supported(h, n, h_in, w_in, int(layout), int(act_dtype)))
        return 0;
    return tiled_shares_units(h, n, h_in, w_in) ? 1 : 2;
}

int pconv_debug_measure_fma_peak(double *tflops)
{
    if (!tflops) { set_error("pconv_debug_measure_fma_peak: null pointer argument"); return PCONV_INVALID_ARG; }
    return measure_fma_peak(tflops);
}

int pconv_maxpool2x2(const void *x_dev, void *y_dev, int n, int c, int h, int w,
                     pconv_layout layout, pconv_dtype dtype, void *hip_stream)
{
    if (!x_dev || !y_dev) { set_error("pconv_maxpool2x2: null pointer argument"); return PCONV_INVALID_ARG; }
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) { set_error("pconv_maxpool2x2: dimensions must be positive"); return PCONV_INVALID_ARG; }
    if ((layout != PCONV_NCHW && layout != PCONV_NHWC) || (dtype != PCONV_F32 && dtype != PCONV_BF16)) {
        set_error("pconv_maxpool2x2: unknown layout or dtype");
        return PCONV_INVALID_ARG;
    }
    return launch_maxpool2x2(x_dev, y_dev, n, c, h, w, int(layout), int(dtype), hip_stream);
}

int pconv_debug_export(const pconv_handle *h, uint16_t *perm, uint32_t *row_ptr, uint16_t *pat_cnt,
                       uint16_t *cin, void *vals)
{
    if (!h || !perm || !row_ptr || !pat_cnt || !cin || !vals) { set_error("pconv_debug_export: null pointer argument"); return PCONV_INVALID_ARG; }
    const Canonical &c = h->canon;
    std::memcpy(perm, c.perm.data(), c.perm.size() * 2);
    std::memcpy(row_ptr, c.row_ptr.data(), c.row_ptr.size() * 4);
    std::memcpy(pat_cnt, c.pat_cnt.data(), c.pat_cnt.size() * 2);
    std::memcpy(cin, c.cin.data(), c.cin.size() * 2);
    if (h->wdtype == PCONV_F32) {
        std::memcpy(vals, c.vals_bits.data(), c.vals_bits.size() * 4);
    } else {
        uint16_t *o = static_cast<uint16_t *>(vals);
        for (size_t i = 0; i < c.vals_bits.size(); ++i) o[i] = uint16_t(c.vals_bits[i] >> 16);
    }
    return PCONV_OK;
}

int pconv_debug_export_blocks(const pconv_handle *h, int32_t *slot_filter, uint32_t *records)
{
    if (!h || !slot_filter || !records) { set_error("pconv_debug_export_blocks: null pointer argument"); return PCONV_INVALID_ARG; }
    const int nb = h->tiled.num_blocks, row = h->tiled.row_len, chunks = (row - 1) / kTileCH;
    std::memcpy(slot_filter, h->tiled.slot_filter.data(), size_t(nb) * kTileFB * sizeof(int32_t));
    for (int b = 0; b < nb; ++b)
        for (int j = 0; j < chunks; ++j)
            records[size_t(b) * chunks + j] = h->tiled.chan_ptr[size_t(b) * row + (j + 1) * kTileCH] -
                                              h->tiled.chan_ptr[size_t(b) * row + j * kTileCH];
    return PCONV_OK;
}

int pconv_debug_unpack(const pconv_handle *h, float *w_dense_out)
{
    if (!h || !w_dense_out) { set_error("pconv_debug_unpack: null pointer argument"); return PCONV_INVALID_ARG; }
    if (h->device < 0) { set_error("pconv_debug_unpack: handle holds no device data"); return PCONV_INVALID_ARG; }
    try {
        const size_t F = size_t(h->c_out), K = size_t(h->K), NNZ = size_t(h->nnz);
        std::vector<int32_t> perm(F);
        std::vector<uint32_t> row_ptr(F + 1), kern(K), val_ptr(K);
        std::vector<float> vals(NNZ);
        hipError_t e = hipMemcpy(perm.data(), h->d_perm, F * 4, hipMemcpyDeviceToHost);
        if (e == hipSuccess) e = hipMemcpy(row_ptr.data(), h->d_row_ptr, (F + 1) * 4, hipMemcpyDeviceToHost);
        if (e == hipSuccess && K) e = hipMemcpy(kern.data(), h->d_kern, K * 4, hipMemcpyDeviceToHost);
        if (e == hipSuccess && K) e = hipMemcpy(val_ptr.data(), h->d_val_ptr, K * 4, hipMemcpyDeviceToHost);
        if (e == hipSuccess && NNZ) e = hipMemcpy(vals.data(), h->d_vals, NNZ * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) return hip_fail("pconv_debug_unpack: hipMemcpy", e);
        std::memset(w_dense_out, 0, F * size_t(h->c_in) * 9 * sizeof(float));
        for (size_t i = 0; i < F; ++i)
            for (uint32_t k = row_ptr[i]; k < row_ptr[i + 1]; ++k) {
                const uint32_t c = kern[k] & 0xFFFFu, mask = kern[k] >> 16;
                uint32_t v = val_ptr[k];
                for (int t = 0; t < 9; ++t)
                    if (mask & (1u << t)) w_dense_out[(size_t(perm[i]) * h->c_in + c) * 9 + t] = vals[v++];
            }
    } catch (const std::bad_alloc &) {
        set_error("pconv_debug_unpack: out of host memory");
        return PCONV_OOM;
    }
    return PCONV_OK;
}

}  // extern "C"
