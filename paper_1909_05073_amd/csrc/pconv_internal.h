// Internal declarations shared by the host packer, the kernels' launchers and the C ABI.
#pragma once

#include <atomic>
#include <cstdint>
#include <string>
#include <vector>

#include "pconv.h"

namespace pconv {

constexpr int kFlagSlots = 64, kFlagWords = 1024;

// Thread-local message for pconv_last_error().
void set_error(const std::string &msg);
const char *get_error();

// Result of the host-side analysis + reorder (paper: layer-wise information extraction and
// filter kernel reorder).  "Position" i means the i-th filter in the sorted order.
struct Canonical {
    std::vector<uint16_t> perm;      // [F]     filter at position i
    std::vector<uint32_t> row_ptr;   // [F+1]   first kernel of position i
    std::vector<uint16_t> pat_cnt;   // [F][P]  kernels per pattern at position i
    std::vector<uint16_t> cin;       // [K]     input channel of kernel k
    std::vector<uint8_t>  pat;       // [K]     pattern id of kernel k (derivable from pat_cnt)
    std::vector<uint32_t> val_ptr;   // [K+1]   first stored weight of kernel k
    std::vector<uint32_t> vals_bits; // [nnz]   fp32 bit patterns (bf16 handles: value << 16)
};

// Device-side stream of the register-tiled kernel.  Filters are dealt into blocks of kTileFB
// filters ("slots"); for every (block, input channel) the records of that channel are stored
// contiguously, ordered by slot.  A record is one code (sub-mask with a specialised inner
// loop) of one kernel, with up to four weights in ascending tap order.
struct TiledStream {
    int num_blocks = 0;                 // ceil(F / kTileFB)
    int row_len = 0;                    // entries per chan_ptr row: round_up(C, kTileCH) + 1
    std::vector<int32_t>  slot_filter;  // [num_blocks * kTileFB] original filter index or -1
    std::vector<uint32_t> chan_ptr;     // [num_blocks][row_len]
    std::vector<uint32_t> meta;         // [R+1] record words (see pconv_tiled_codes.h), one pad
    std::vector<float>    w4;           // [R+1][4]
};

}  // namespace pconv

struct pconv_handle {
    int c_out = 0, c_in = 0, np = 0, wdtype = 0, device = -1;
    uint16_t table[PCONV_MAX_PATTERNS] = {0};
    int64_t K = 0, nnz = 0, device_bytes = 0;
    pconv::Canonical canon;
    pconv::TiledStream tiled;
    // device copies (generic gather kernel)
    int32_t  *d_perm = nullptr;
    uint32_t *d_row_ptr = nullptr;
    uint32_t *d_kern = nullptr;      // [K] cin | mask << 16
    uint32_t *d_val_ptr = nullptr;   // [K]
    float    *d_vals = nullptr;      // [nnz] fp32 (bf16 weights widened exactly)
    // device copies (register-tiled kernel)
    int32_t  *d_slot_filter = nullptr;
    uint32_t *d_chan_ptr = nullptr;
    uint32_t *d_meta = nullptr;
    float    *d_w4 = nullptr;
    // device copies (matrix-core kernel, bf16 handles only): the masked weights as nine dense
    // [filter][channel] matrices, tap-major, in blocks of 16 channels: [9][cb16][fpad][16] bf16, fpad
    // = c_out rounded up to 32, cb16 = c_in rounded up to 32, in sixteens; and per (block of 32
    // channels, block of 32 filters) a word whose bit 2 * tap + half says whether that
    // (tap, 16 channels, 32 filters) block holds any kept weight
    uint16_t *d_wdense = nullptr;
    uint32_t *d_wnz = nullptr;
    // Hand-over words of the tiled kernel: workgroups that share a unit of work signal each other
    // through kFlagWords words; every call takes the next of kFlagSlots such rows and a fresh
    // value, so calls that overlap on different streams do not see each other's signals.
    uint32_t *d_flags = nullptr;     // [kFlagSlots][kFlagWords], zero at start
    mutable std::atomic<uint32_t> calls{0};
    // Sticky error word of the kernels launched on this handle: pinned host memory that the device
    // writes (non-zero = a bounded wait inside a kernel ran out) and that the next call on the
    // handle reads without touching the device.
    uint32_t *h_err = nullptr;
    int cus = 0;                     // compute units of `device`, read once at pack time
};

namespace pconv {

// Host analysis + reorder.  Returns PCONV_OK or an error status (message set).
int build_canonical(const float *w, const uint8_t *pid, const uint8_t *conn, const uint16_t *table,
                    int np, int c_out, int c_in, int wdtype, Canonical &out);

int project_weights(const float *w, const uint16_t *table, int np, int c_out, int c_in, int64_t keep,
                    uint8_t *pattern_id, uint8_t *conn);

void build_tiled_stream(const Canonical &cn, const uint16_t *table, int np, int c_out, int c_in,
                        TiledStream &out);

// Kernel launchers (pconv_kernels.hip, pconv_tiled.hip).  All return a pconv_status.
int launch_conv_generic(const pconv_handle *h, const void *x, void *y, const float *bias, int n,
                        int hin, int win, int stride, int layout, int dtype, int relu, void *stream);
// static_scratch: take the hand-over words from the code object's static array instead of the handle.
int launch_conv_tiled(const pconv_handle *h, const void *x, void *y, const float *bias, int n,
                      int hin, int win, int stride, int layout, int dtype, int relu, int pool, void *stream,
                      bool static_scratch = false);
// whether the tiled kernel can write the 2x2 max-pooled output directly (pool = 1)
bool tiled_pool_supported(const pconv_handle *h, int n, int hin, int win, int layout, int dtype);
bool tiled_supported(const pconv_handle *h, int n, int hin, int win, int stride, int layout, int dtype);
// whether pconv_conv2d (fp32 NCHW, stride 1) would let workgroups share tiles of this call, which a
// fused max-pool rules out
bool tiled_shares_units(const pconv_handle *h, int n, int hin, int win);
// plain vector-FMA rate of the device (see pconv_debug_measure_fma_peak)
int measure_fma_peak(double *tflops);
// whether the automatic policy should take the tiled kernel for a call it supports
bool tiled_preferred(int hin, int win, int stride);
// Test override of the tiled kernel's launch choices: waves per workgroup (8 or 16, anything else =
// automatic), log2 of the channel split inside a workgroup (0..2, anything else = automatic), and
// whether workgroups may share a unit of work (0 / 1, anything else = automatic).
void set_tiled_tuning(int waves, int ks_log2, int split_units);
// Test override of the iteration limit of the kernels' bounded waits (<= 0 restores the default).
void set_tiled_spin_limit(int limit);
// bf16 layers on the matrix cores (pconv_mfma.hip)
bool mfma_supported(const pconv_handle *h, int dtype, int n, int hin, int win);
bool mfma_preferred(const pconv_handle *h);
int launch_conv_mfma(const pconv_handle *h, const void *x, void *y, const float *bias, int n,
                     int hin, int win, int stride, int layout, int relu, void *stream);
// masked weights of a bf16 handle in the matrix-core kernel's layout (see pconv_handle::d_wdense)
void build_dense_taps(const Canonical &cn, const uint16_t *table, int c_out, int c_in,
                      std::vector<uint16_t> &wd, std::vector<uint32_t> &nz);
int launch_maxpool2x2(const void *x, void *y, int n, int c, int h, int w, int layout, int dtype,
                      void *stream);

}  // namespace pconv
