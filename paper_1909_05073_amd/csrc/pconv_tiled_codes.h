// Sub-masks the register-tiled kernel has a specialised inner loop for ("codes").
// Every pattern of a layer's table is split at pack time into disjoint codes from this list;
// the single-tap codes make that possible for any 9-bit mask.  Bit (3*r + s) = tap (r, s).
#pragma once
#include <cstdint>

namespace pconv {

constexpr int kNumCodes = 24;
constexpr uint16_t kCodeMask[kNumCodes] = {
    // the four Sparse Convolution Patterns (centre + three edge neighbours)
    0x03A, 0x09A, 0x0B8, 0x0B2,
    // 2x2 blocks around the centre
    0x01B, 0x036, 0x0D8, 0x1B0,
    // centre + diagonal pair + one edge tap
    0x113, 0x074, 0x191, 0x05C,
    // kernel rows (a dense 3x3 kernel is three of these)
    0x007, 0x038, 0x1C0,
    // single taps
    0x001, 0x002, 0x004, 0x008, 0x010, 0x020, 0x040, 0x080, 0x100,
};

// Record word of the tiled stream: bits 0-7 slot * kNumCodes + code, bits 8-10 channel within
// its chunk, bit 11 set on the first record of a channel (the lane then reloads its input patch).
constexpr uint32_t kMetaCaseMask = 0xFFu;
constexpr uint32_t kMetaFirstOfChannel = 0x800u;

constexpr int kTileFB = 4;      // filters per wave ("slots")
constexpr int kTileWaves = 16;  // waves per workgroup
constexpr int kTileCH = 8;      // input channels staged per LDS chunk
constexpr int kTileBatch = 32;  // records a wave fetches at a time (one per lane)

}  // namespace pconv
