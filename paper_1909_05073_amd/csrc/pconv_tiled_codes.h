// Sub-masks the register-tiled kernel has a specialised inner loop for ("codes").
// Every pattern of a layer's table is split at pack time into disjoint codes from this list (see
// gen_tiled_compute.py, which defines the list and generates the array below): every 4-tap mask
// that contains the centre is a code of its own, rows, pairs and single taps serve the rest.
// Bit (3*r + s) = tap (r, s).
#pragma once
#include <cstdint>

namespace pconv {

#include "pconv_tiled_code_masks.inc"   // kNumCodes, kBodyStrideLog2, kCodeMask[]

constexpr int kTileFB = 4;      // filters per wave ("slots")
constexpr int kTileWaves = 16;  // waves per workgroup
constexpr int kTileCH = 8;      // input channels staged per LDS chunk
constexpr int kTileBatch = 32;  // records a wave fetches at a time (one per lane)

// Record word of the tiled stream: bits 0-2 the channel within its chunk, bit 3 set on the first
// record of a channel (the lane then reloads its input patch), bits kBodyStrideLog2 and up the case
// slot * kNumCodes + code, so that the word masked to those bits is the byte offset of the
// record's inner loop in the kernel's table of bodies.  Case kTileFB * kNumCodes ends a list.
constexpr uint32_t kMetaChannelMask = 7u;
constexpr uint32_t kMetaFirstOfChannel = 8u;
constexpr int kMetaCaseShift = kBodyStrideLog2;
static_assert(kMetaCaseShift > 3 && kTileCH <= 8, "the case field must lie above the channel and first-of-channel bits");
constexpr uint32_t kMetaEndOfList = uint32_t(kTileFB * kNumCodes) << kMetaCaseShift;

}  // namespace pconv
