// q-bit matrices as weighted sums of binary matrices (include/rsr_qbit.h): host code on top of the
// C ABI of rsr.h; the products themselves are the binary kernel's.
#include <cstdint>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "../../include/rsr_qbit.h"
#include "rsr_internal.h"

struct rsr_qbit {
  uint64_t magic = 0;
  int q = 0;
  std::vector<rsr_handle*> planes;  // plane i: bit i of the two's complement entries
  int64_t table_bytes = 0;
};

namespace {
constexpr uint64_t kMagic = 0x7162697452535221ull;
bool valid(const rsr_qbit* h) { return h && h->magic == kMagic; }
int fail(int code, const std::string& msg) { return rsr_internal::set_error(code, msg); }
// weight of plane i: 2^i, and -2^(q-1) for the sign plane
int32_t weight(int i, int q) { return i == q - 1 ? -(1 << i) : (1 << i); }
}  // namespace

extern "C" {

rsr_qbit* rsr_qbit_preprocess(const int8_t* A, int64_t rows, int64_t cols, int k, int q) {
  if (!A) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_qbit_preprocess: null pointer"); return nullptr; }
  if (q < 2 || q > 8) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_qbit_preprocess: q must be in 2..8"); return nullptr; }
  if (rows < 1 || cols < 1) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_qbit_preprocess: rows and cols must be >= 1"); return nullptr; }
  const int lo = -(1 << (q - 1)), hi = (1 << (q - 1)) - 1;
  const int64_t count = rows * cols;
  for (int64_t i = 0; i < count; ++i)
    if (A[i] < lo || A[i] > hi) {
      fail(RSR_ERR_INVALID_ARGUMENT, "rsr_qbit_preprocess: entry " + std::to_string((int)A[i]) + " at flat index " + std::to_string(i) +
                                         " lies outside " + std::to_string(lo) + ".." + std::to_string(hi));
      return nullptr;
    }
  std::unique_ptr<rsr_qbit> h(new (std::nothrow) rsr_qbit());
  std::vector<int8_t> plane;
  try { plane.resize((size_t)count); } catch (const std::bad_alloc&) { h.reset(); }
  if (!h) { fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory"); return nullptr; }
  h->q = q;
  for (int i = 0; i < q; ++i) {
    for (int64_t j = 0; j < count; ++j) plane[(size_t)j] = (int8_t)(((uint8_t)A[j] >> i) & 1u);
    rsr_handle* p = rsr_preprocess(plane.data(), rows, cols, k);
    if (!p) {  // (the message of rsr_preprocess stands)
      for (rsr_handle* x : h->planes) rsr_destroy(x);
      return nullptr;
    }
    h->planes.push_back(p);
    rsr_info_t info;
    if (rsr_info(p, &info) == RSR_OK) h->table_bytes += info.table_bytes;
  }
  h->magic = kMagic;
  return h.release();
}

int rsr_qbit_matvec(rsr_qbit* h, const float* v, float* out, int batch, void* stream) {
  if (!valid(h)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid handle");
  int rc = rsr_matvec(h->planes[0], v, out, batch, stream);
  for (int i = 1; i < h->q && rc == RSR_OK; ++i) rc = rsr_matvec_acc(h->planes[(size_t)i], v, out, (float)weight(i, h->q), batch, stream);
  return rc;
}

int rsr_qbit_matvec_i8(rsr_qbit* h, const int8_t* v, int32_t* out, int batch, void* stream) {
  if (!valid(h)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid handle");
  int rc = rsr_matvec_i8(h->planes[0], v, out, batch, stream);
  for (int i = 1; i < h->q && rc == RSR_OK; ++i) rc = rsr_matvec_acc_i8(h->planes[(size_t)i], v, out, weight(i, h->q), batch, stream);
  return rc;
}

int rsr_qbit_planes(const rsr_qbit* h) { return valid(h) ? h->q : RSR_ERR_INVALID_ARGUMENT; }
int64_t rsr_qbit_table_bytes(const rsr_qbit* h) { return valid(h) ? h->table_bytes : (int64_t)RSR_ERR_INVALID_ARGUMENT; }

void rsr_qbit_destroy(rsr_qbit* h) {
  if (!valid(h)) return;
  for (rsr_handle* p : h->planes) rsr_destroy(p);
  h->magic = 0;
  delete h;
}

}  // extern "C"
