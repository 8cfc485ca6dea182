// Packed device layout of the RSR index (internal to the library; shared by the host packer,
// the host decoder and the HIP kernels).
//
// Logical content, per part (B(1), B(2) of Proposition 2.1) and per k-column block
// (Definition 3.1): the row permutation sigma of Definition 3.2 and the full segmentation L of
// Section 3.3.  Physical layout: sigma itself, 16 bits per row, in sorted order, plus one bit per
// row that says "a new value starts here" (L in unary), arranged for 64-lane wavefronts and
// 16-byte coalesced loads:
//
//   * A row's value in a block is its k bits read with the first column most significant.  A
//     last block narrower than k is treated as if its missing columns were zero, i.e. its
//     values are shifted left by (k - width).  Rows with value 0 add nothing to the block
//     (row 0 of Bin_[k] is zero) and are not stored.
//   * The 2^k values of a block are cut into windows of 2^kw consecutive values
//     (kw = min(k, 9)).  One wavefront handles one work unit at a time: a run of consecutive
//     sorted rows of one window, whose segment sums u[j] live in that wavefront's private LDS
//     slice (slot = value - first value of the window), where the low kw levels of the RSR++
//     fold are taken; the remaining k - kw levels only need each window's total.  A window with
//     more rows than a unit holds is spread over several units: their results add up because the
//     fold is linear in u (a segment may be cut anywhere).
//   * A unit's entries are its sorted rows in order.  A value of the window that no row has,
//     lying between two values of the unit that do occur, is represented by one entry with the
//     null row index `rows` (which reads a zero kept behind the activation vector in LDS), so that
//     consecutive entries differ by at most one value.  Every entry carries a flag: 1 = its value
//     is the previous entry's value plus one, 0 = the same value.  The first entry's flag is 0 and
//     the unit's descriptor names its slot (`slot0`).
//   * The n entries are dealt out to the 64 lanes in consecutive runs of `npos` = ceil(n / 64)
//     (<= kMaxPositions): lane l holds entries l*npos .. (l+1)*npos-1; the tail is padded with null
//     entries (flag 0).  A lane walks its run with one running sum: at a flagged entry it stores
//     the sum to the current slot, moves to the next slot and restarts.  Its first slot follows
//     from the flags of the lanes before it (a prefix sum over the lanes' flag counts); the sum
//     it is left with at the end belongs to a segment that continues in the next lane and is
//     added to its slot afterwards.
//   * In memory, position p of the unit is the 64 uint16 entries (lane 0..63) at step p of the
//     lanes' runs.  A lane's uint16s of 8 consecutive positions are adjacent: positions
//     8g .. 8g+7 form a granule of 64 x 16 bytes (lane-major), read with one 16-byte load per
//     lane.  The positions behind the last full granule are stored as rows of dwords (two
//     positions per lane, 256 bytes per row) and, if npos is odd, a last row of uint16 (128
//     bytes).  Then the flags follow: one dword per lane for
//     positions 0..31 (position p = bit 31-p) and, if npos > 32, one uint16 per lane for positions
//     32..47 (position p = bit 47-p).  A unit's stream starts on a 128-byte boundary.
//
// Streams on the device:
//   stream    bytes   unit streams, back to back
//   units     Unit    32-byte descriptors, ordered by block
//   blk_unit  uint32  nblocks+1 offsets into `units`
#ifndef RSR_FORMAT_H_
#define RSR_FORMAT_H_

#include <stdint.h>

namespace rsr {

constexpr int kLanes = 64;             // wavefront width
constexpr int kMaxWindowBits = 9;      // window = 2^kw values, kw = min(k, 9)
constexpr int kWindow = 1 << kMaxWindowBits;   // LDS slots of a window (always allocated in full)
constexpr int kGranulePositions = 8;   // positions per 16-byte granule
constexpr int kMaxGranules = 6;        // full granules of a unit at most
constexpr int kMaxPositions = kMaxGranules * kGranulePositions;  // 48
constexpr int kMaxUnitEntries = kMaxPositions * kLanes;          // 3072
constexpr int kPositionBytes = kLanes * 2;    // 128
constexpr int kFlagBytes0 = kLanes * 4;       // flags of positions 0..31
constexpr int kFlagBytes1 = kLanes * 2;       // flags of positions 32..47 (only if npos > 32)
constexpr int kStreamAlign = 128;      // unit streams start on multiples of this
constexpr int kMaxK = 16;
constexpr int kMaxRows = 65534;        // 65535 values of uint16 minus the null index
constexpr int64_t kTileRows = 32768;   // a matrix with more rows is indexed in row tiles of at most this height
constexpr int kRecordWords = 16;       // per-unit result record in LDS: 9 low-bit sums, total, meta

// bytes of a unit's stream before alignment
constexpr uint32_t unit_stream_bytes(int npos) {
  return (uint32_t)npos * kPositionBytes + (npos > 0 ? kFlagBytes0 : 0) + (npos > 32 ? kFlagBytes1 : 0);
}

struct alignas(16) Unit {
  uint32_t stream_off;      // start of the unit's stream, in multiples of kStreamAlign bytes
  uint32_t block;           // column block
  uint16_t window;          // window index inside the block: value >> kw
  uint8_t part;             // 0: B(1) (or binary B), 1: B(2)
  uint8_t npos;             // positions in the stream, <= kMaxPositions; 0 = a unit without entries
  uint16_t units_in_block;  // units of this unit's column block (all parts and windows)
  uint16_t index_in_block;  // this unit's number among the units of its block
  uint16_t slot0;           // window slot of the first entry
  uint16_t reserved0;
  uint32_t nrows;           // real (non-null) row indices in the unit
  uint32_t nheads;          // flagged entries
  uint32_t nentries;        // entries before the padding of the last lanes (rows and nulls for absent values)
};
static_assert(sizeof(Unit) == 32, "unit descriptor must be 32 bytes");

}  // namespace rsr
#endif  // RSR_FORMAT_H_
