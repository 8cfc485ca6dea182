// Packed device layout of the RSR index (internal to the library; shared by the host packer,
// the host decoder and the HIP kernels).
//
// Logical content, per part (B(1), B(2) of Proposition 2.1) and per k-column block
// (Definition 3.1): the row permutation sigma of Definition 3.2 and the full segmentation L of
// Section 3.3.  Physical layout, chosen for 64-lane wavefronts and 16-byte coalesced loads:
//
//   * A row's value in a block is its k bits read with the first column most significant.  A
//     last block narrower than k is treated as if its missing columns were zero, i.e. its
//     values are shifted left by (k - width).  Rows with value 0 add nothing to the block
//     (row 0 of Bin_[k] is zero) and are not stored.
//   * The 2^k values of a block are cut into windows of 2^kw consecutive values
//     (kw = min(k, 9)).  One wavefront handles one work unit at a time: (part of) a window, whose
//     segment sums u[j] live in that wavefront's private LDS slice, where the low kw levels of
//     the RSR++ fold are taken; the remaining k - kw levels only need each window's total.  A
//     window may be spread over several units: their results add up because the fold is
//     linear in u.
//   * Every set of equal rows ("segment") of the window is cut into pieces of at most T rows (T is
//     chosen per window so that the stream gets shortest).  Pieces are ranked by descending
//     length; ranks 64i .. 64i+63 form group i, one piece per lane.  Inside a unit the first
//     piece of a segment delivers its sum to the segment's own slot of the window; every further
//     piece of that segment gets an overflow slot of its own, and the unit lists the segment
//     value ("parent") of each overflow slot: the fold adds an overflow sum wherever its parent's
//     bits say so, which is the same as adding it to the parent first.  Overflow slot x is folded
//     by lane x % 64, whose 16-lane row stands for the value bits 7 and 8: x is chosen so that
//     (x % 64) / 16 == parent >> 7.  Unused overflow slots below the highest one in use have the
//     null index as parent.
//   * The unit's stream is a sequence of positions; a position holds one uint16 per lane.  It
//     starts with 0 to 4 parent positions (lane x of parent position c: the parent of overflow
//     slot 64c + x).  Then the groups follow: a header position and n index positions (n = the
//     group's longest piece).  The header names, per lane, the window slot that receives the
//     lane's sum for the group; lanes without a piece name a dummy slot.  An index position holds
//     one row of each lane's piece, or the null row index `rows` (which reads a zero kept behind
//     the activation vector in LDS): a piece shorter than its group leaves some positions of its
//     lane empty, and which ones is the packer's choice (it places the rows so that the lanes of
//     a half wavefront read different LDS banks where possible).  A bit mask in the
//     descriptor marks the header positions.  The number of positions is even (a null position is
//     appended if needed) and at most kMaxPositions.
//   * In memory a lane's uint16s of 8 consecutive positions are adjacent: positions 8g .. 8g+7
//     form a granule of 64 x 16 bytes (lane-major), read with one 16-byte load per lane.  The
//     positions behind the last full granule are stored as rows of dwords (two positions per
//     lane, 256 bytes per row).  A unit's stream starts on a 256-byte boundary.
//   * Within a unit no two pieces deliver to the same slot (plain stores, no read-modify-write).
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
constexpr int kDummySlots = 8;         // slot ids kWindow .. kWindow+7 swallow lanes without a piece
constexpr int kMaxOverflow = 256;      // overflow slots per unit (ids kOverflowBase ..), a quarter per row class
constexpr int kOverflowBase = kWindow + kDummySlots;
constexpr int kWindowSlots = kOverflowBase + kMaxOverflow;  // 776 accumulators per wavefront
constexpr int kGranulePositions = 8;   // positions per 16-byte granule
constexpr int kMaxGranules = 6;        // full granules of a unit at most
constexpr int kMaxPositions = kMaxGranules * kGranulePositions;  // 48
constexpr int kPositionBytes = kLanes * 2;    // 128
constexpr int kStreamAlign = 256;      // unit streams start on multiples of this
constexpr int kMaxK = 16;
constexpr int kMaxRows = 65534;        // 65535 values of uint16 minus the null index
constexpr int kRecordWords = 16;       // per-unit result record in LDS: 9 low-bit sums, total, meta

struct alignas(16) Unit {
  uint32_t stream_off;      // start of the unit's stream, in multiples of kStreamAlign bytes
  uint32_t block;           // column block
  uint16_t window;          // window index inside the block: value >> kw
  uint8_t part;             // 0: B(1) (or binary B), 1: B(2)
  uint8_t npar;             // parent positions, 0 .. 4: the overflow slots 0 .. 64*npar-1 may be in use
  uint16_t units_in_block;  // units of this unit's column block (all parts and windows)
  uint8_t npos;             // positions in the stream: even, <= kMaxPositions
  uint8_t ngroups;          // groups = header positions
  uint32_t hdr_lo;          // bit p: position p is a header (positions 0..31)
  uint16_t hdr_hi;          // positions 32..47
  uint16_t index_in_block;  // this unit's number among the units of its block
  uint32_t nidx;            // real (non-null) row indices in the unit
  uint32_t npieces;         // pieces in the unit
};
static_assert(sizeof(Unit) == 32, "unit descriptor must be 32 bytes");

}  // namespace rsr
#endif  // RSR_FORMAT_H_
