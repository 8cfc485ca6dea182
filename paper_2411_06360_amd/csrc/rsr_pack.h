// Host side of rsr_preprocess: Algorithm 1 (Section 3.4) plus the packing of its output
// (permutations and full segmentations) into the device layout of rsr_format.h, and the
// inverse used by rsr_export_block.
#ifndef RSR_PACK_H_
#define RSR_PACK_H_

#include <cstdint>
#include <string>
#include <vector>

#include "rsr_format.h"

namespace rsr {

struct Packed {
  int64_t rows = 0, cols = 0;
  int k = 0, kw = 0, parts = 0, last_width = 0;
  int64_t nblocks = 0;
  std::vector<uint16_t> stream;    // unit streams (row indices in sorted order, then their flags)
  std::vector<Unit> units;
  std::vector<uint32_t> blk_unit;  // nblocks + 1
  int64_t stored_rows = 0;         // real (non-null) row indices in `stream`
  int64_t segments = 0;            // runs of equal rows as stored (a run cut by a unit boundary counts twice)
  int64_t flag_bytes = 0;          // bytes of `stream` that hold flags rather than row indices
  uint32_t max_units_per_block = 0;
};

// Builds the packed index of A (row-major rows x cols, entries in {-1,0,1}).  Returns 0 or a
// negative rsr_status value; *err describes the failure.  `threads` <= 0 picks a default.
// `parts` = 0 infers the kind (any -1 makes the matrix ternary), 1 or 2 forces it (2 for a tile of
// a ternary matrix that happens to hold no -1).
int pack_matrix(const int8_t* A, int64_t rows, int64_t cols, int k, int threads, int parts, Packed* out, std::string* err);

// A matrix with more rows than kTileRows is indexed in row tiles of equal height (the product
// is linear in the rows: the tiles' products add up).  Every tile is a packed index of its own.
struct Index {
  int64_t rows = 0, cols = 0;
  std::vector<Packed> tiles;
  std::vector<int64_t> row0;   // first row of every tile
};
int pack_tiles(const int8_t* A, int64_t rows, int64_t cols, int k, int threads, Index* out, std::string* err);

// Recovers sigma (rows entries) and L (2^width + 1 entries) of one block from the packed tiles.
// Either output pointer may be null.
int decode_block(const Index& X, int part, int64_t block, int32_t* sigma, int32_t* L, std::string* err);

}  // namespace rsr
#endif  // RSR_PACK_H_
