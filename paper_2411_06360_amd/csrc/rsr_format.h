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
//     (kw = min(k, 9)).  One wavefront handles one window at a time: the segment sums u[j] of
//     the window live in that wavefront's private LDS slice, where the low kw levels of the
//     RSR++ fold are taken; the remaining k - kw levels only need each window's total.
//   * Inside a window every group of equal rows ("segment") is a piece.  Pieces are ranked by
//     descending length; lane l of the wavefront owns ranks 8l .. 8l+7 and keeps one
//     accumulator per rank.  Diagonal t of the window lists, for ranks 0 .. cnt_t-1 (the pieces
//     longer than t), the t-th row of each piece.  Diagonals come in two tiers:
//       - wide diagonals (t < nt_main): padded to a multiple of 8 with the null row index `rows`
//         (which reads a zero kept behind the activation vector in LDS).  A lane reads its 8
//         entries with one 16-byte load; a wavefront reads one contiguous KB.
//       - tail diagonals (t >= nt_main, the first diagonal with at most 64 pieces left): stored
//         back to back without padding; lane l reads the single entry of rank l and adds it to a
//         ninth accumulator, which is merged into the rank's slot afterwards.  This keeps the few
//         long segments from costing a full 8-gather step each.  The tail region as a whole is
//         padded to 16 bytes.
//   * A segment longer than kMaxDiag rows is cut into several pieces; the first keeps the
//     segment's slot in the window, the others get overflow slots whose parent value is listed
//     behind the unit's slot ids.  A window with more pieces than one unit can hold continues
//     in further units; unit results add up because the fold is linear in u.
//
// Streams on the device:
//   entries   uint16  row indices, unit after unit, diagonal after diagonal
//   slots     uint16  per unit: slot id of every rank (padded to 8 with the dummy slot), then the
//                     parent values of its overflow slots (padded to 8)
//   units     Unit    64-byte descriptors, ordered by block, then part, then window
//   blk_unit  uint32  nblocks+1 offsets into `units`
#ifndef RSR_FORMAT_H_
#define RSR_FORMAT_H_

#include <stdint.h>

namespace rsr {

constexpr int kLanes = 64;             // wavefront width
constexpr int kPerLane = 8;            // ranks (accumulators) per lane = uint16 entries per 16-byte load
constexpr int kTileRanks = kLanes * kPerLane;  // 512 pieces per unit
constexpr int kMaxWindowBits = 9;      // window = 2^kw values, kw = min(k, 9)
constexpr int kWindow = 1 << kMaxWindowBits;   // LDS slots of a window (always allocated in full)
constexpr int kDummySlots = 8;         // slot ids kWindow .. kWindow+7 swallow padding ranks
constexpr int kMaxOverflow = 64;       // overflow slots per unit (ids kWindow+8 .. kWindow+71)
constexpr int kOverflowBase = kWindow + kDummySlots;
constexpr int kWindowSlots = kOverflowBase + kMaxOverflow;  // 584 accumulators per wavefront
constexpr int kMaxDiag = 40;           // diagonals (rows per piece) per unit
constexpr int kMaxK = 16;
constexpr int kTailRanks = 64;         // a tail diagonal has at most one entry per lane
constexpr int kMaxRows = 65534;        // 65535 values of uint16 minus the null index
constexpr int kRecordWords = 16;       // per-unit result record in LDS: 9 low-bit sums, total, meta

struct alignas(16) Unit {
  uint32_t entry_off;  // start of the unit's entries, in 16-byte granules
  uint32_t slot_off;   // start of the unit's slot ids, in 16-byte granules
  uint32_t block;      // column block
  uint16_t window;     // window index inside the block: value >> kw
  uint16_t npieces;    // ranks in use, <= 512
  uint8_t nt;          // diagonals, <= kMaxDiag
  uint8_t part;        // 0: B(1) (or binary B), 1: B(2)
  uint8_t nov;         // overflow slots in use, <= kMaxOverflow
  uint8_t nt_main;     // wide diagonals; diagonals nt_main .. nt-1 form the tail
  uint16_t units_in_block;  // units of this unit's column block (all parts and windows)
  uint16_t main_granules;   // 16-byte granules of the wide diagonals = offset of the tail region
  uint8_t cnt8[kMaxDiag];   // wide diagonal: active lanes (16-byte granules); tail diagonal: entries
};
static_assert(sizeof(Unit) == 64, "unit descriptor must be 64 bytes");

}  // namespace rsr
#endif  // RSR_FORMAT_H_
