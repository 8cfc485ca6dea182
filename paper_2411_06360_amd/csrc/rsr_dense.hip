// Comparator (include/rsr_dense.h): out = v . A from the bit-packed matrix on the same GPU.
//
// Layout: one bit per entry and part ("plane": [A == 1], and [A == -1] for a ternary matrix).  The
// bits of 32 consecutive rows of one column are one dword; dwords are ordered plane, row chunk, column,
// so that the 64 lanes of a wavefront, one column each, read 256 consecutive bytes.
// Kernel 1: a workgroup takes 256 columns and a tile of 512 rows.  Every lane first requests the 16
// dwords of its column (per plane); the workgroup then tabulates, for every group of four rows of the
// tile, the 16 sums of subsets of their activations (8 KB of LDS per vector); a lane adds one table
// entry per four rows of its column (minus the entry of the second plane) and leaves the tile's
// partial sum in a scratch buffer.  Kernel 2 adds the tiles' partial sums in order.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/rsr_dense.h"

#include "rsr_internal.h"

// Buffer of partial sums for rsr_dense_matvec_static: part of the code object, so every GPU the library
// runs on holds its own copy at its own address from the moment the module is loaded there.  In host
// code the name below is only a handle for hipGetSymbolAddress; kernels get the resolved address.
static __device__ __align__(256) unsigned char scratch[RSR_DENSE_STATIC_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices];  // per device: address of `scratch` there (nullptr = not resolved yet)

// Address of the static buffer on the CURRENT device (resolved once per device, with that device
// current); nullptr and *err set on failure.
void* static_scratch_on_current_device(int* device, std::string* err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    *err = e != hipSuccess ? std::string("hipGetDevice: ") + hipGetErrorString(e) : "device ordinal out of range";
    return nullptr;
  }
  *device = dev;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      *err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
      return nullptr;
    }
    g_static_ptr[dev] = ptr;
  }
  return g_static_ptr[dev];
}

constexpr int kTileRows = 512;             // rows per workgroup: 128 groups of four, 16 dwords per column
constexpr int kTileChunks = kTileRows / 32;
constexpr int kColsPerWg = 256;
constexpr int kMaxBatch = 16;
constexpr uint64_t kDenseMagic = 0x52535264656e7331ull;  // "RSRdens1"

template <typename VT> struct DAcc;
template <> struct DAcc<float> { using type = float; };
template <> struct DAcc<int8_t> { using type = int32_t; };

template <typename VT, int PLANES>
__global__ void __launch_bounds__(kColsPerWg)
dense_partial_kernel(const uint32_t* __restrict__ bits, const VT* __restrict__ v, typename DAcc<VT>::type* __restrict__ partial,
                     int rows, int cols, int cols_pad, int nchunks, int batch) {
  using AT = typename DAcc<VT>::type;
  __shared__ __align__(16) AT lut[kTileRows / 4][16];
  const int tid = threadIdx.x;
  const int c = blockIdx.x * kColsPerWg + tid;
  const int tile = blockIdx.y;
  const int row0 = tile * kTileRows;
  const int chunk0 = tile * kTileChunks;
  // the column's bits of this tile: requested first, used after the table is built
  uint32_t wp[kTileChunks], wm[kTileChunks];
  const int cc = c < cols ? c : 0;  // (columns past the end read column 0 and store nothing)
#pragma unroll
  for (int ch = 0; ch < kTileChunks; ++ch) {
    const bool in = chunk0 + ch < nchunks;
    wp[ch] = in ? bits[((int64_t)(chunk0 + ch)) * cols_pad + cc] : 0u;
    wm[ch] = (PLANES == 2 && in) ? bits[((int64_t)(nchunks + chunk0 + ch)) * cols_pad + cc] : 0u;
  }
  for (int b = 0; b < batch; ++b) {
    const VT* vb = v + (int64_t)b * rows;
    __syncthreads();  // the table of the previous vector is no longer read
    if (tid < kTileRows / 4) {
      const int g = tid;
      AT x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = row0 + 4 * g + i;
        x[i] = r < rows ? (AT)vb[r] : (AT)0;
      }
      AT e[16];
      e[0] = (AT)0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int m = 0; m < (1 << i); ++m) e[(1 << i) + m] = e[m] + x[i];  // subsets that contain row i
#pragma unroll
      for (int m = 0; m < 16; ++m) lut[g][m] = e[m];
    }
    __syncthreads();
    // four running sums, so that the additions do not form one chain
    AT acc[4] = {(AT)0, (AT)0, (AT)0, (AT)0};
#pragma unroll
    for (int ch = 0; ch < kTileChunks; ++ch) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        acc[q & 3] += lut[ch * 8 + q][(wp[ch] >> (4 * q)) & 15u];
        if (PLANES == 2) acc[q & 3] -= lut[ch * 8 + q][(wm[ch] >> (4 * q)) & 15u];
      }
    }
    if (c < cols) partial[((int64_t)tile * batch + b) * cols + c] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  }
}

// Sum of the row tiles' partial results, in a fixed order: a workgroup of 256 threads owns 64
// outputs; thread (q, j) adds the tiles q, q+4, q+8, ... of output j (independent loads, all in
// flight together), and the four quarter sums are added in order through LDS.
template <typename AT>
__global__ void __launch_bounds__(256) dense_reduce_kernel(const AT* __restrict__ partial, AT* __restrict__ out, int ntiles, int64_t n) {
  __shared__ AT quarter[4][64];
  const int j = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int64_t i = (int64_t)blockIdx.x * 64 + j;
  AT s = (AT)0;
  if (i < n) {
    AT s0 = (AT)0, s1 = (AT)0;
    int t = q;
    for (; t + 4 < ntiles; t += 8) {
      s0 += partial[(int64_t)t * n + i];
      s1 += partial[(int64_t)(t + 4) * n + i];
    }
    if (t < ntiles) s0 += partial[(int64_t)t * n + i];
    s = s0 + s1;
  }
  quarter[q][j] = s;
  __syncthreads();
  if (q == 0 && i < n) out[i] = (quarter[0][j] + quarter[1][j]) + (quarter[2][j] + quarter[3][j]);
}

}  // namespace

struct rsr_dense {
  uint64_t magic = 0;
  int device = 0;
  int64_t rows = 0, cols = 0, cols_pad = 0, nchunks = 0;
  int planes = 0, ntiles = 0;
  size_t bits_bytes = 0, scratch_bytes = 0;
  void* d_bits = nullptr;
  void* d_scratch = nullptr;
};

namespace {

bool valid(const rsr_dense* h) { return h && h->magic == kDenseMagic; }

template <typename VT>
int dense_launch(rsr_dense* h, const VT* v, void* out, int batch, void* stream, void* scratch, size_t scratch_bytes) {
  using AT = typename DAcc<VT>::type;
  if (!valid(h)) return rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "invalid dense handle");
  if (!v || !out) return rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "null pointer");
  if (batch < 1 || batch > kMaxBatch) return rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "batch must be in 1..16");
  const size_t need = (size_t)h->ntiles * batch * h->cols * sizeof(AT);
  if (need > scratch_bytes)
    return rsr_internal::set_error(RSR_ERR_UNSUPPORTED, "partial sums of " + std::to_string(need) + " bytes (4 * ceil(rows/512) * batch * cols) exceed the buffer of " +
                                                           std::to_string(scratch_bytes) + " bytes");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)((h->cols + kColsPerWg - 1) / kColsPerWg), (unsigned)h->ntiles);
  auto kern = h->planes == 2 ? dense_partial_kernel<VT, 2> : dense_partial_kernel<VT, 1>;
  hipLaunchKernelGGL(kern, grid, dim3(kColsPerWg), 0, st, static_cast<const uint32_t*>(h->d_bits), v,
                     static_cast<AT*>(scratch), (int)h->rows, (int)h->cols, (int)h->cols_pad, (int)h->nchunks, batch);
  const int64_t n = (int64_t)batch * h->cols;
  hipLaunchKernelGGL(dense_reduce_kernel<AT>, dim3((unsigned)((n + 63) / 64)), dim3(256), 0, st, static_cast<const AT*>(scratch),
                     static_cast<AT*>(out), h->ntiles, n);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return rsr_internal::set_error(RSR_ERR_HIP, std::string("dense launch: ") + hipGetErrorString(e));
  return RSR_OK;
}

}  // namespace

extern "C" {

rsr_dense* rsr_dense_preprocess(const int8_t* A, int64_t rows, int64_t cols) {
  if (!A) { rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "null pointer"); return nullptr; }
  if (rows < 1 || cols < 1 || rows > (1 << 24) || cols > (1 << 24)) { rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "rows and cols must be in 1..2^24"); return nullptr; }
  std::unique_ptr<rsr_dense> h(new (std::nothrow) rsr_dense());
  if (!h) { rsr_internal::set_error(RSR_ERR_OUT_OF_MEMORY, "out of host memory"); return nullptr; }
  int planes = 1;
  for (int64_t i = 0; i < rows * cols; ++i) {
    const int x = A[i];
    if (x < -1 || x > 1) {
      rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "entry outside {-1,0,1} at row " + std::to_string(i / cols) + ", column " + std::to_string(i % cols));
      return nullptr;
    }
    if (x < 0) planes = 2;
  }
  h->rows = rows; h->cols = cols; h->planes = planes;
  h->cols_pad = (cols + 63) / 64 * 64;
  h->nchunks = (rows + 31) / 32;
  h->ntiles = (int)((rows + kTileRows - 1) / kTileRows);
  std::vector<uint32_t> bits;
  try {
    bits.assign((size_t)planes * h->nchunks * h->cols_pad, 0u);
  } catch (const std::bad_alloc&) {
    rsr_internal::set_error(RSR_ERR_OUT_OF_MEMORY, "out of host memory");
    return nullptr;
  }
  for (int64_t r = 0; r < rows; ++r) {
    const int8_t* a = A + r * cols;
    uint32_t* plus = &bits[(size_t)(r / 32) * h->cols_pad];
    uint32_t* minus = planes == 2 ? &bits[(size_t)(h->nchunks + r / 32) * h->cols_pad] : nullptr;
    const uint32_t bit = 1u << (r % 32);
    for (int64_t c = 0; c < cols; ++c) {
      if (a[c] == 1) plus[c] |= bit;
      else if (a[c] == -1) minus[c] |= bit;
    }
  }
  h->bits_bytes = bits.size() * sizeof(uint32_t);
  h->scratch_bytes = (size_t)h->ntiles * kMaxBatch * cols * 4;
  hipError_t e = hipGetDevice(&h->device);
  if (e == hipSuccess) e = hipMalloc(&h->d_bits, h->bits_bytes);
  if (e == hipSuccess) e = hipMalloc(&h->d_scratch, h->scratch_bytes);
  if (e == hipSuccess) e = hipMemcpy(h->d_bits, bits.data(), h->bits_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipGetLastError();
    if (h->d_bits) (void)hipFree(h->d_bits);
    if (h->d_scratch) (void)hipFree(h->d_scratch);
    rsr_internal::set_error(RSR_ERR_HIP, std::string("rsr_dense_preprocess: ") + hipGetErrorString(e));
    return nullptr;
  }
  {
    // set-up time is the right moment to find the static buffer of this device (the device is current and
    // nothing is being captured); a failure only matters to rsr_dense_matvec_static, which reports it
    int dev = 0;
    std::string ignored;
    (void)static_scratch_on_current_device(&dev, &ignored);
  }
  h->magic = kDenseMagic;
  return h.release();
}

int rsr_dense_matvec(rsr_dense* h, const float* v, float* out, int batch, void* stream) {
  if (!valid(h)) return rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "invalid dense handle");
  return dense_launch<float>(h, v, out, batch, stream, h->d_scratch, h->scratch_bytes);
}

int rsr_dense_matvec_static(rsr_dense* h, const float* v, float* out, int batch, void* stream) {
  if (!valid(h)) return rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "invalid dense handle");
  int dev = -1;
  std::string err;
  void* ptr = static_scratch_on_current_device(&dev, &err);
  if (!ptr) return rsr_internal::set_error(RSR_ERR_HIP, "rsr_dense_matvec_static: " + err);
  if (dev != h->device)
    return rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "rsr_dense_matvec_static: the handle belongs to device " + std::to_string(h->device) +
                                                                 " but device " + std::to_string(dev) + " is current");
  // (every partial sum that the second kernel reads is written by the first kernel of the same call:
  // what an earlier call left in the buffer is never read, nothing has to be cleared)
  return dense_launch<float>(h, v, out, batch, stream, ptr, (size_t)RSR_DENSE_STATIC_BYTES);
}

int rsr_dense_matvec_i8(rsr_dense* h, const int8_t* v, int32_t* out, int batch, void* stream) {
  if (!valid(h)) return rsr_internal::set_error(RSR_ERR_INVALID_ARGUMENT, "invalid dense handle");
  return dense_launch<int8_t>(h, v, out, batch, stream, h->d_scratch, h->scratch_bytes);
}

int64_t rsr_dense_table_bytes(const rsr_dense* h) { return valid(h) ? (int64_t)h->bits_bytes : -1; }

void rsr_dense_destroy(rsr_dense* h) {
  if (!valid(h)) return;
  (void)hipFree(h->d_bits);
  (void)hipFree(h->d_scratch);
  h->magic = 0;
  delete h;
}

}  // extern "C"
