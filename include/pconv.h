/*
 * pconv.h - C ABI of the MI355X (gfx950) PCONV sparse 3x3 convolution library.
 *
 * PCONV weights carry two kinds of sparsity (paper, "Theory of Sparse Convolution
 * Patterns"): every surviving 3x3 kernel keeps only the taps of one binary mask, its
 * Sparse Convolution Pattern, drawn from a small per-layer pattern table; and whole
 * kernels, i.e. (output filter f, input channel c) connections, are removed
 * (connectivity pruning).  The layer computes the ordinary un-flipped DNN convolution,
 * Eq. (1) of "The Convolution Operator", over those masked weights:
 *
 *   Y[n,f,y,x] = act( b[f] + sum_c sum_r sum_s  W[f,c,r,s] * P_{pid[f,c]}[r,s] * conn[f,c]
 *                                                * Xpad[n, c, y*stride + r - pad, x*stride + s - pad] )
 *
 * Xpad is X inside the image and 0 outside; act is ReLU or identity.
 *
 * All functions return PCONV_OK (0) or a negative pconv_status; no C++ exception crosses
 * this boundary.  A human-readable message for the last failing call of the calling thread
 * is available from pconv_last_error().  "host" / "device" below says where a pointer must
 * live; device pointers must belong to the HIP device that is current at the call.
 */
#ifndef PCONV_H
#define PCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pconv_handle pconv_handle;   /* opaque; owns its host and device buffers */

typedef enum { PCONV_F32 = 0, PCONV_BF16 = 1 } pconv_dtype;
typedef enum { PCONV_NCHW = 0, PCONV_NHWC = 1 } pconv_layout;

typedef enum {
    PCONV_OK = 0,
    PCONV_INVALID_ARG = -1,   /* null pointer, bad dimension, bad mask, bad pattern id, ... */
    PCONV_OOM = -2,           /* host or device allocation failed                            */
    PCONV_HIP_ERROR = -3,     /* a HIP runtime call failed (message has the HIP error name)  */
    PCONV_UNSUPPORTED = -4    /* valid request this build has no kernel for                  */
} pconv_status;

enum { PCONV_MAX_PATTERNS = 16 };

/*
 * pconv_pack - the offline compiler stage of the paper ("Compiler-assisted DNN Inference
 * Framework": layer-wise information extraction, filter kernel reorder, compact storage),
 * run on the host.  Synchronous.
 *
 *   w_dense      host, [c_out][c_in][3][3] fp32 (OIHW).  Values under a cleared mask bit or
 *                on a removed kernel are ignored; kept values are copied bit for bit
 *                (fp32) or rounded to nearest-even bf16 (weight_dtype == PCONV_BF16).
 *   pattern_id   host, [c_out][c_in]; index into table; ignored where conn == 0.
 *   conn         host, [c_out][c_in]; 0 = kernel removed, non-zero = kept.
 *   table        host, [num_patterns]; 9-bit masks, bit (3*r + s) keeps tap (r, s).
 *                Any non-zero mask <= 0x1FF is legal (0x1FF = dense kernel).
 *   num_patterns 1 .. PCONV_MAX_PATTERNS;  c_out, c_in in 1 .. 65535.
 *   out          receives a new handle (valid only when PCONV_OK is returned).
 *
 * The caller keeps ownership of every input; everything needed is copied.  The packed
 * weights are uploaded to the current HIP device.  Filters with no kept kernel are legal.
 * Errors: PCONV_INVALID_ARG (null pointers, sizes out of range, mask == 0 or > 0x1FF,
 * pattern_id >= num_patterns on a kept kernel), PCONV_OOM, PCONV_HIP_ERROR.
 */
int pconv_pack(const float *w_dense, const uint8_t *pattern_id, const uint8_t *conn,
               const uint16_t *table, int num_patterns, int c_out, int c_in,
               pconv_dtype weight_dtype, pconv_handle **out);

/*
 * pconv_project - the step before pconv_pack: gives dense 3x3 weights their PCONV form, as the
 * Euclidean projection that an ADMM pruner for the paper's two constraints repeats ("Accuracy
 * Analysis": the models are produced by an ADMM framework extended to pattern and connectivity
 * pruning; the paper's own algorithm text is in supplemental material).  Per kernel the table
 * pattern is chosen under which the kernel keeps the largest sum of squared weights (the first
 * such pattern among equals); then the keep_kernels kernels that keep the most under their
 * pattern survive (the smaller f * c_in + c among equals).  Sums are formed in double over the
 * taps in ascending order.  Host only, synchronous, no GPU needed.
 *
 *   w_dense          host, [c_out][c_in][3][3] fp32
 *   table            host, [num_patterns] 9-bit masks as for pconv_pack
 *   keep_kernels     0 .. c_out * c_in: number of kernels connectivity pruning leaves
 *   pattern_id_out   host, [c_out][c_in], written for every kernel
 *   conn_out         host, [c_out][c_in], 1 = kept, 0 = removed
 *
 * The outputs, with w_dense itself, are what pconv_pack takes (it ignores the weights under
 * cleared mask bits and on removed kernels).  Errors: PCONV_INVALID_ARG, PCONV_OOM.
 */
int pconv_project(const float *w_dense, const uint16_t *table, int num_patterns, int c_out, int c_in,
                  int64_t keep_kernels, uint8_t *pattern_id_out, uint8_t *conn_out);

/*
 * pconv_conv2d - the sparse convolution itself (Eq. (1) over the packed weights; the
 * "load redundancy elimination" stage of the paper: only inputs under kept taps of kept
 * kernels are touched).  Asynchronous on hip_stream; allocates nothing.  The packed weights in
 * the handle are only read.  A call does write two small things that belong to the handle: it
 * takes a ticket from a call counter, and, when the layer has so few tiles that workgroups share
 * them, its workgroups signal each other through one of 64 rows of hand-over words in device
 * memory (row = ticket mod 64).  Calls on one handle may therefore run concurrently on different
 * streams, as long as no more than 64 such calls are in flight at once.
 *
 * Every wait inside the kernels is bounded.  If one ever runs out, the affected outputs are set
 * to NaN and the handle remembers it: the next pconv_conv2d / pconv_conv2d_pool2x2 on the handle,
 * or pconv_get_async_error, returns PCONV_HIP_ERROR once (and launches nothing).
 *
 *   x_dev     device, activations [n][c_in][h_in][w_in] (NCHW) or [n][h_in][w_in][c_in]
 *             (NHWC), fp32 or bf16 as act_dtype says.
 *   y_dev     device, output in the same layout and dtype with c_out channels and
 *             h_out = (h_in + 2*pad - 3)/stride + 1 (same for w).  Must not alias x_dev.
 *   bias_dev  device, [c_out] fp32, or NULL for no bias.
 *   stride    1 or 2;  pad must be 1;  fuse_relu != 0 applies max(., 0) after the bias.
 *   act_dtype must equal the handle's weight dtype.  Products are accumulated in fp32;
 *             bf16 outputs are rounded to nearest even.
 *   hip_stream  a hipStream_t, or NULL for the default stream.
 *
 * Errors: PCONV_INVALID_ARG (null pointers, n/h/w <= 0, stride not in {1,2}, pad != 1,
 * dtype mismatch, tensors of 2^31 elements or more), PCONV_HIP_ERROR (launch failed, or an
 * earlier kernel on this handle gave up a wait: see above).
 */
int pconv_conv2d(const pconv_handle *h, const void *x_dev, void *y_dev, const float *bias_dev,
                 int n, int h_in, int w_in, int stride, int pad,
                 pconv_layout layout, pconv_dtype act_dtype, int fuse_relu, void *hip_stream);

/*
 * pconv_conv2d_static - pconv_conv2d for callers that must not cause, or depend on, any device
 * allocation of the library's: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same results.  The one difference: the
 * hand-over words that workgroups use when they share tiles come from a static array in the
 * library's code object (1024 words = 4 KiB per device, held until the process ends) instead of
 * from the handle; a small fill kernel clears them on hip_stream ahead of the convolution.  The
 * call itself allocates and frees nothing.  All calls on one device share that array: calls of
 * this entry point that overlap on one device (different streams) race and must be serialised by
 * the caller.  Errors: as pconv_conv2d; PCONV_UNSUPPORTED if a launch would need more hand-over
 * words than the array has; PCONV_HIP_ERROR if the array's address cannot be obtained.
 */
int pconv_conv2d_static(const pconv_handle *h, const void *x_dev, void *y_dev, const float *bias_dev,
                        int n, int h_in, int w_in, int stride, int pad,
                        pconv_layout layout, pconv_dtype act_dtype, int fuse_relu, void *hip_stream);

/*
 * pconv_get_async_error - PCONV_HIP_ERROR (once, with a message) if a kernel launched on this
 * handle gave up one of its bounded waits since the last report, else PCONV_OK.  Touches no
 * device; meaningful after the stream(s) of the calls in question have been synchronised.
 */
int pconv_get_async_error(const pconv_handle *h);

/*
 * pconv_conv2d_pool2x2 - pconv_conv2d (stride 1, pad 1) followed by a 2x2 / stride-2 max-pool,
 * in one kernel: y_dev receives [n][c_out][h_in/2][w_in/2] (floor), the full-size convolution
 * output is never written.  Max-pooling is not part of the paper's method; VGG-16 has one
 * after five of its thirteen 3x3 layers, and there this saves writing and re-reading the
 * largest tensors of the network.  Values are those of pconv_conv2d followed by
 * pconv_maxpool2x2 (bit for bit when both add the input channels in the same order; for layers
 * with few tiles pconv_conv2d may add them in a different order).  Arguments as for pconv_conv2d.
 *
 * Errors: as pconv_conv2d, and PCONV_UNSUPPORTED unless the tensors are fp32 NCHW with
 * w_in even and >= 4, h_in >= 2 and an input of less than 2 GiB (and the kernel policy is not 1).
 */
int pconv_conv2d_pool2x2(const pconv_handle *h, const void *x_dev, void *y_dev, const float *bias_dev,
                         int n, int h_in, int w_in, pconv_layout layout, pconv_dtype act_dtype,
                         int fuse_relu, void *hip_stream);

/*
 * pconv_pool2x2_fusion - what pconv_conv2d_pool2x2 would do with this call, without launching
 * anything: 0 = not supported (use pconv_conv2d + pconv_maxpool2x2), 1 = supported, but the layer has
 * so few tiles that pconv_conv2d would let workgroups share them, which the fused call cannot (the
 * two separate calls are expected to be faster), 2 = supported and recommended.  Negative = error.
 */
int pconv_pool2x2_fusion(const pconv_handle *h, int n, int h_in, int w_in, pconv_layout layout,
                         pconv_dtype act_dtype);

/* pconv_free - releases the handle's host and device memory.  NULL is allowed. */
void pconv_free(pconv_handle *h);

/*
 * pconv_maxpool2x2 - plain 2x2 / stride-2 max-pool used between VGG-16 blocks (not part of
 * the paper's method; a helper so a whole 3x3 stack can be chained on the device).
 *   x_dev [n][c][h][w] or [n][h][w][c] -> y_dev with h/2, w/2 (floor).  Asynchronous.
 */
int pconv_maxpool2x2(const void *x_dev, void *y_dev, int n, int c, int h, int w,
                     pconv_layout layout, pconv_dtype dtype, void *hip_stream);

/* ---- inspection of a handle (tests, benchmarks) --------------------------------------- */

typedef struct {
    int32_t c_out, c_in, num_patterns, weight_dtype;
    int64_t kept_kernels;      /* K   = number of kept (f, c) pairs                        */
    int64_t nnz;               /* sum over kept kernels of popcount(mask)                  */
    int64_t device_bytes;      /* device memory held by the handle                         */
    int32_t fast_path;         /* 1 if the register-tiled kernel can serve this handle     */
    int32_t reserved;
} pconv_info;

int pconv_get_info(const pconv_handle *h, pconv_info *info);

/*
 * pconv_debug_export - copies out the canonical logical layout produced by the filter
 * kernel reorder, for bit-exact comparison.  All outputs are caller-allocated host arrays:
 *   perm[c_out]            filter at each position; filters sorted by (kept-kernel count
 *                          descending, per-pattern counts descending in pattern order,
 *                          filter index ascending)
 *   row_ptr[c_out + 1]     first kernel of each position; row_ptr[c_out] = K
 *   pat_cnt[c_out][P]      kernels per pattern at each position
 *   cin[K]                 input channel of each kernel; inside a filter kernels are ordered
 *                          by (pattern id, input channel)
 *   vals[nnz]              kept weights of each kernel in ascending tap order; fp32 bit
 *                          copies, or uint16 bf16 bit patterns for a bf16 handle
 */
int pconv_debug_export(const pconv_handle *h, uint16_t *perm, uint32_t *row_ptr,
                       uint16_t *pat_cnt, uint16_t *cin, void *vals);

/* pconv_debug_pack_host - the host stages of pconv_pack only (analysis, reorder, compact
 * storage) with no upload, so the packing logic can be checked on a machine without a GPU.
 * The handle works with pconv_get_info, pconv_debug_export and pconv_free; pconv_conv2d and
 * pconv_debug_unpack reject it with PCONV_INVALID_ARG.  Arguments as for pconv_pack. */
int pconv_debug_pack_host(const float *w_dense, const uint8_t *pattern_id, const uint8_t *conn,
                          const uint16_t *table, int num_patterns, int c_out, int c_in,
                          pconv_dtype weight_dtype, pconv_handle **out);

/* pconv_debug_export_blocks - how the register-tiled kernel's work was dealt out by pconv_pack
 * (workload balance, the purpose of the paper's filter kernel reorder).  Filters are dealt to
 * blocks of 4 (one block per wave); 16 consecutive blocks are the filters of one workgroup; the
 * input channels are walked in chunks of 8.  Caller-allocated host arrays:
 *   slot_filter[4 * B]   filter in each slot of each block, -1 for an empty slot;  B = ceil(c_out / 4)
 *   records[B][J]        work items ("records": one per kept kernel for masks that are in the
 *                        kernel's code table, more for other masks) of block b in chunk j;
 *                        J = ceil(c_in / 8)
 * Works on handles from pconv_debug_pack_host as well. */
int pconv_debug_export_blocks(const pconv_handle *h, int32_t *slot_filter, uint32_t *records);

/* pconv_debug_unpack - rebuilds dense masked weights [c_out][c_in][3][3] fp32 on the host
 * from the DEVICE copy of the packed data (zeros where nothing is stored). */
int pconv_debug_unpack(const pconv_handle *h, float *w_dense_out);

/* Kernel selection, for tests and benchmarks: 0 = automatic (default: the register-tiled vector
 * kernel; for bf16 handles that keep at least 1 weight in 20, the matrix-core kernel, which runs
 * the nine taps of Eq. (1) as dense bf16 contractions over the masked weights with fp32
 * accumulation; the gather kernel for what neither serves), 1 = always the generic gather kernel,
 * 2 = require the register-tiled kernel, 3 = require the matrix-core kernel (bf16 handles, inputs
 * below 2 GiB).  2 and 3 give PCONV_UNSUPPORTED if the handle or the call cannot use the kernel.
 * Process-wide. */
int pconv_set_kernel_policy(int policy);

/* pconv_debug_set_tiling - for tests: pins launch choices the register-tiled kernel otherwise
 * makes per call.  waves = 8 or 16 (workgroup size in waves; 0 = automatic); ks_log2 = 0, 1 or 2
 * (the waves of a workgroup split the input channels 1, 2 or 4 ways; -1 = automatic);
 * split_units = 0, 1 or 2 (whether several workgroups may share one tile of outputs, each taking a
 * range of the input channels: 0 = never, 1 = yes, with the work dealt out per group of workgroups
 * that share a level-2 cache, 2 = yes, dealt out evenly over all workgroups; -1 = automatic).
 * Values out of range mean automatic.
 * Process-wide; results are the same for every choice up to the order of the fp32 additions. */
int pconv_debug_set_tiling(int waves, int ks_log2, int split_units);

/* pconv_debug_set_spin_limit - for tests of the error path: the number of polls after which a
 * wait inside the register-tiled kernel gives up (limit <= 0 restores the default, about half a
 * second).  With limit = 1 every such wait gives up at once: the kernels still run to their end,
 * their outputs are invalid, and the handle reports the error as described at pconv_conv2d.
 * Process-wide. */
int pconv_debug_set_spin_limit(int limit);

/* pconv_debug_measure_fma_peak - for benchmarks: runs a kernel of nothing but independent fp32
 * FMAs on vector-register operands (16 waves per compute unit) on the current device and reports
 * the rate in TFLOP/s: the measured counterpart of the datasheet's fp32 vector peak for the
 * instruction the convolution kernel is made of.  Synchronous; allocates and frees a scratch
 * buffer of its own. */
int pconv_debug_measure_fma_peak(double *tflops);

const char *pconv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PCONV_H */
