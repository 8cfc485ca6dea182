// Shared between the translation units of the library (not part of the C ABI).
#ifndef RSR_INTERNAL_H_
#define RSR_INTERNAL_H_

#include <cstddef>
#include <cstdint>
#include <string>

namespace rsr_internal {

// the calling thread's message for rsr_last_error(); returns `code`
int set_error(int code, const std::string& msg);

// The packed tables of one row tile, built in device memory by device_build_tile (rsr_prep.hip).
// The three buffers are owned by the caller afterwards (hipFree).
struct BuiltTile {
  void* d_stream = nullptr;
  void* d_units = nullptr;
  void* d_blk_unit = nullptr;
  size_t stream_bytes = 0, unit_bytes = 0, blk_bytes = 0;
  uint32_t max_units_per_block = 0;
  int64_t nunits = 0, stored_rows = 0, segments = 0, flag_bytes = 0;
  int parts = 0;
  double ms_values = 0, ms_sort = 0, ms_emit = 0;  // where the time went (events around the kernels)
};

// Algorithm 1 on the device for the rows x cols tile at dA (DEVICE, row-major, `ld` elements between rows):
// row values, stable counting sort per column block and part, full segmentation, packing into the layout of
// rsr_format.h.  parts = 1 or 2 (decided by the caller for the whole matrix).  Returns 0 or a negative status.
int device_build_tile(const int8_t* dA, int64_t rows, int64_t cols, int64_t ld, int k, int parts, BuiltTile* out, std::string* err);

// Checks the entries of a device matrix: *kind = 0 if an entry lies outside {-1,0,1}, 2 if some entry is -1, else 1.
int device_matrix_kind(const int8_t* dA, int64_t count, int* kind, std::string* err);

}  // namespace rsr_internal
#endif  // RSR_INTERNAL_H_
