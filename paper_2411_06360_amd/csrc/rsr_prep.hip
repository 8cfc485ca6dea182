// Algorithm 1 (Section 3.4) on the device: the index of a matrix that already sits in device memory
// is built there, in the packed layout of rsr_format.h.
//
//   1. values_kernel     the k-bit value of every row in every column block and part (Definition 3.2,
//                        first column most significant; a narrow last block is shifted left).
//   2. sort_kernel       per (block, part), by one wavefront: histogram of the values, its exclusive prefix
//                        (the full segmentation L of Section 3.3) and the stable counting sort that gives
//                        sigma ("bucket sort" in the proof of Theorem 3.6; equal rows stay in row order: the
//                        wavefront walks the rows in order, 64 at a time, and ranks equal values by lane).
//   3. window_kernel     per window of 2^kw values: how many entries its stream has (its rows, plus one
//                        null entry for every absent value between two present ones).
//   (host)               the unit descriptors and stream offsets from those counts: O(windows), no row data.
//   4. emit_kernel       per unit: the entries dealt out to the 64 lanes, row indices in granule order, flags.
//
// Inside emit_kernel the rows of a segment are then dealt out over the LDS banks (as the host packer does in
// rsr_pack.cpp, by the same exchange rule): that changes the speed of the product, not the index it encodes.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/rsr.h"
#include "rsr_format.h"
#include "rsr_internal.h"

namespace {

using rsr::Unit;

#define PREP_TRY(expr)                                                        \
  do {                                                                        \
    hipError_t e_ = (expr);                                                   \
    if (e_ != hipSuccess) {                                                   \
      (void)hipGetLastError();                                                \
      *err = std::string(#expr) + ": " + hipGetErrorString(e_);               \
      return RSR_ERR_HIP;                                                     \
    }                                                                         \
  } while (0)

__global__ void kind_kernel(const int8_t* __restrict__ A, int64_t count, unsigned* __restrict__ flags) {
  unsigned f = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
    const int x = A[i];
    if (x < -1 || x > 1) f |= 2u;
    if (x == -1) f |= 1u;
  }
  if (f) atomicOr(flags, f);
}

// val[(block * parts + part) * rows + r]
__global__ void values_kernel(const int8_t* __restrict__ A, int rows, int cols, int64_t ld, int k, int parts, int nblocks,
                              uint16_t* __restrict__ val) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  for (int b = blockIdx.y; b < nblocks; b += gridDim.y) {
    const int width = min(k, cols - b * k);
    const int8_t* a = A + (int64_t)r * ld + (int64_t)b * k;
    uint32_t plus = 0, minus = 0;
    for (int c = 0; c < width; ++c) {
      const int x = a[c];
      plus = (plus << 1) | (uint32_t)(x == 1);
      minus = (minus << 1) | (uint32_t)(x == -1);
    }
    const int shift = k - width;
    val[((int64_t)b * parts) * rows + r] = (uint16_t)(plus << shift);
    if (parts == 2) val[((int64_t)b * parts + 1) * rows + r] = (uint16_t)(minus << shift);
  }
}

// One wavefront per (block, part).  LDS: 2^k counters of 16 bits per wavefront (a tile has at most 32768 rows).
__global__ void sort_kernel(const uint16_t* __restrict__ val, int rows, int k, int nbp, int waves_per_wg,
                            uint32_t* __restrict__ off, uint16_t* __restrict__ sigma) {
  extern __shared__ uint32_t lds_hist[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int bp = blockIdx.x * waves_per_wg + wave;
  if (bp >= nbp) return;  // (no barriers below: the wavefronts are independent)
  const int nvals = 1 << k;
  const int ndw = max(1, nvals >> 1);
  volatile uint32_t* h = lds_hist + (size_t)wave * ndw;
  const uint16_t* v = val + (int64_t)bp * rows;
  for (int i = lane; i < ndw; i += 64) h[i] = 0;
  // histogram
  for (int r0 = 0; r0 < rows; r0 += 64) {
    const int r = r0 + lane;
    if (r < rows) {
      const uint32_t x = v[r];
      atomicAdd(const_cast<uint32_t*>(&h[x >> 1]), 1u << (16 * (x & 1)));
    }
  }
  // exclusive prefix: the full segmentation (kept in LDS as the next free position of every value)
  uint32_t carry = 0;
  uint32_t* o = off + (int64_t)bp * (nvals + 1);
  for (int i0 = 0; i0 < ndw; i0 += 64) {
    const int i = i0 + lane;
    const uint32_t w = i < ndw ? h[i] : 0u;
    const uint32_t c0 = w & 0xffffu, c1 = w >> 16;
    uint32_t s = c0 + c1;
    uint32_t incl = s;
#pragma unroll
    for (int d = 1; d < 64; d *= 2) {
      const uint32_t t = __shfl_up(incl, d);
      if (lane >= d) incl += t;
    }
    const uint32_t start0 = carry + incl - s, start1 = start0 + c0;
    if (i < ndw) {
      h[i] = start0 | (start1 << 16);
      o[2 * i] = start0;
      if (2 * i + 1 < nvals) o[2 * i + 1] = start1;
    }
    carry += __shfl(incl, 63);
  }
  if (lane == 0) o[nvals] = (uint32_t)rows;
  // stable placement: rows in order, 64 at a time; equal values of a chunk are ranked by lane
  uint16_t* sg = sigma + (int64_t)bp * rows;
  for (int r0 = 0; r0 < rows; r0 += 64) {
    const int r = r0 + lane;
    const bool active = r < rows;
    const uint32_t x = active ? (uint32_t)v[r] : 0xffffffffu;
    unsigned long long todo = __ballot(active);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const uint32_t s = (uint32_t)__shfl((int)x, leader);
      const unsigned long long m = __ballot(active && x == s);
      const uint32_t cur = (h[s >> 1] >> (16 * (s & 1))) & 0xffffu;
      if (active && x == s) {
        const int rank = __popcll(m & ((1ull << lane) - 1ull));
        sg[cur + rank] = (uint16_t)r;
      }
      if (lane == leader) h[s >> 1] = h[s >> 1] + ((uint32_t)__popcll(m) << (16 * (s & 1)));
      todo &= ~m;
    }
  }
}

// Per (block-part, window): entries of the window's stream (rows + nulls for absent values between present ones).
__global__ void window_kernel(const uint32_t* __restrict__ off, int k, int kw, int nbp, uint32_t* __restrict__ n_ext) {
  const int nwin = 1 << (k - kw);
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)nbp * nwin) return;
  const int bp = (int)(id / nwin), w = (int)(id % nwin);
  const int W = 1 << kw;
  const uint32_t* o = off + (int64_t)bp * ((1 << k) + 1) + (int64_t)w * W;
  int first = -1, last = -1;
  for (int j = (w == 0 ? 1 : 0); j < W; ++j)
    if (o[j + 1] != o[j]) { if (first < 0) first = j; last = j; }
  uint32_t n = 0;
  if (first >= 0)
    for (int j = first; j <= last; ++j) n += max(1u, o[j + 1] - o[j]);
  n_ext[id] = n;
}

struct UnitJob {
  uint32_t bp, window, entry_begin, n;
};

__global__ void __launch_bounds__(256)
emit_kernel(const UnitJob* __restrict__ jobs, Unit* __restrict__ units, const uint32_t* __restrict__ off,
            const uint16_t* __restrict__ sigma, int rows, int k, int kw, uint16_t* __restrict__ stream) {
  __shared__ uint32_t cnt[512], estart[513], f0[64], f1[64], wsum[4];
  __shared__ uint16_t ent[64 * rsr::kMaxPositions];            // the unit's entries, [lane][position]
  __shared__ uint32_t bank_load[2][rsr::kMaxPositions][32];    // rows per LDS bank, per half wavefront and position
  __shared__ int first_s, last_s;
  __shared__ uint32_t nrows_s, nheads_s;
  const int u = blockIdx.x, tid = threadIdx.x;
  const UnitJob J = jobs[u];
  const int npos = units[u].npos;
  if (npos == 0) return;  // a unit without entries (an all-zero block)
  const int W = 1 << kw;
  const uint32_t* o = off + (int64_t)J.bp * ((1 << k) + 1) + (int64_t)J.window * W;
  const uint16_t* sg = sigma + (int64_t)J.bp * rows;
  const uint16_t null_index = (uint16_t)rows;
  if (tid == 0) { first_s = W; last_s = -1; nrows_s = 0; nheads_s = 0; }
  if (tid < 64) { f0[tid] = 0; f1[tid] = 0; }
  __syncthreads();
  for (int j = tid; j < 512; j += 256) {
    uint32_t c = 0;
    if (j < W && !(J.window == 0 && j == 0)) c = o[j + 1] - o[j];
    cnt[j] = c;
    if (c) { atomicMin(&first_s, j); atomicMax(&last_s, j); }
  }
  __syncthreads();
  const int first = first_s, last = last_s;
  // exclusive prefix of the entries per value (two values per thread)
  const int j0 = 2 * tid, j1 = 2 * tid + 1;
  const uint32_t e0 = (j0 >= first && j0 <= last) ? max(1u, cnt[j0]) : 0u;
  const uint32_t e1 = (j1 >= first && j1 <= last) ? max(1u, cnt[j1]) : 0u;
  uint32_t incl = e0 + e1;
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int d = 1; d < 64; d *= 2) {
    const uint32_t t = __shfl_up(incl, d);
    if (lane >= d) incl += t;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += wsum[w];
  const uint32_t ex = base + incl - (e0 + e1);
  estart[j0] = ex;
  estart[j1] = ex + e0;
  if (tid == 255) estart[512] = ex + e0 + e1;
  __syncthreads();
  const int full = npos / 8;
  const int64_t sbase = (int64_t)units[u].stream_off * (rsr::kStreamAlign / 2);  // in uint16 elements
  uint32_t my_rows = 0, my_heads = 0;
  for (int idx = tid; idx < 64 * npos; idx += 256) {
    const int l = idx / npos, p = idx - l * npos;
    uint16_t row = null_index;
    int flag = 0;
    if ((uint32_t)idx < J.n) {
      const uint32_t i = J.entry_begin + (uint32_t)idx;
      int lo = 0, hi = 513;  // upper bound of i in estart[0..512]
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (estart[mid] <= i) lo = mid + 1; else hi = mid;
      }
      const int j = lo - 1;  // the value whose entries contain i
      if (cnt[j]) { row = sg[o[j] + (i - estart[j])]; ++my_rows; }
      flag = (i == estart[j]) && idx > 0;
      if (idx == 0) units[u].slot0 = (uint16_t)j;
    }
    ent[l * rsr::kMaxPositions + p] = row;
    if (flag) {
      ++my_heads;
      if (p < 32) atomicOr(&f0[l], 1u << (31 - p)); else atomicOr(&f1[l], 1u << (47 - p));
    }
  }
  if (my_rows) atomicAdd(&nrows_s, my_rows);
  if (my_heads) atomicAdd(&nheads_s, my_heads);
  for (int i = tid; i < 2 * rsr::kMaxPositions * 32; i += 256) (&bank_load[0][0][0])[i] = 0;
  __syncthreads();
  // The order of the rows inside a segment is free.  As in the host packer, two rows of a lane's run that
  // lies in one segment trade places while that lowers the squared loads of the LDS banks (row mod 32) at
  // their two positions, counted per half wavefront: the gathers of the product then meet in fewer banks.
  // One thread per lane; the loads are kept with atomics, a decision may see a neighbour's move late, which
  // only costs quality.
  if (tid < 64) {
    const int L = tid, h = L >> 5;
    for (int p = 0; p < npos; ++p) {
      const uint16_t r = ent[L * rsr::kMaxPositions + p];
      if (r != null_index) atomicAdd(&bank_load[h][p][r & 31], 1u);
    }
  }
  __syncthreads();
  for (int pass = 0; pass < 6; ++pass) {
    if (tid < 64) {
      const int L = tid, h = L >> 5;
      const uint32_t g0 = f0[L], g1 = f1[L];
      auto flagged = [&](int q) { return q < 32 ? (g0 >> (31 - q)) & 1u : (g1 >> (47 - q)) & 1u; };
      uint16_t* e = ent + L * rsr::kMaxPositions;
      int p0 = 0;
      while (p0 < npos) {
        int p1 = p0 + 1;
        while (p1 < npos && !flagged(p1)) ++p1;
        for (int pp = p0; pp < p1; ++pp)
          for (int q = pp + 1; q < p1; ++q) {
            const uint16_t rp = e[pp], rq = e[q];
            if (rp == null_index || rq == null_index) continue;
            const int bp = rp & 31, bq = rq & 31;
            if (bp == bq) continue;
            volatile uint32_t* lp = bank_load[h][pp];
            volatile uint32_t* lq = bank_load[h][q];
            const int delta = ((int)lp[bq] - (int)lp[bp] + 1) + ((int)lq[bp] - (int)lq[bq] + 1);
            if (delta < 0) {
              atomicSub(&bank_load[h][pp][bp], 1u); atomicAdd(&bank_load[h][pp][bq], 1u);
              atomicSub(&bank_load[h][q][bq], 1u); atomicAdd(&bank_load[h][q][bp], 1u);
              e[pp] = rq; e[q] = rp;
            }
          }
        p0 = p1;
      }
    }
    __syncthreads();
  }
  for (int idx = tid; idx < 64 * npos; idx += 256) {
    const int l = idx / npos, p = idx - l * npos;
    const uint16_t row = ent[l * rsr::kMaxPositions + p];
    int64_t at;
    if (p < full * 8) {
      at = ((int64_t)(p / 8) * 64 + l) * 8 + (p % 8);
    } else {
      const int q = p - full * 8;
      const int64_t rest = (int64_t)full * 8 * 64;
      at = ((npos & 1) && p == npos - 1) ? rest + (int64_t)(q / 2) * 2 * 64 + l : rest + ((int64_t)(q / 2) * 64 + l) * 2 + (q & 1);
    }
    stream[sbase + at] = row;
  }
  if (tid < 64) {
    const int64_t fb = sbase + (int64_t)npos * 64;
    stream[fb + 2 * tid] = (uint16_t)(f0[tid] & 0xffffu);
    stream[fb + 2 * tid + 1] = (uint16_t)(f0[tid] >> 16);
    if (npos > 32) stream[fb + 128 + tid] = (uint16_t)f1[tid];
  }
  if (tid == 0) { units[u].nrows = nrows_s; units[u].nheads = nheads_s; }
}

struct DevBuf {  // frees on scope exit
  void* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  void* release() { void* q = p; p = nullptr; return q; }
};

}  // namespace

namespace rsr_internal {

int device_matrix_kind(const int8_t* dA, int64_t count, int* kind, std::string* err) {
  DevBuf flags;
  PREP_TRY(hipMalloc(&flags.p, 4));
  PREP_TRY(hipMemset(flags.p, 0, 4));
  const int grid = (int)std::min<int64_t>(4096, (count + 255) / 256);
  hipLaunchKernelGGL(kind_kernel, dim3((unsigned)grid), dim3(256), 0, nullptr, dA, count, static_cast<unsigned*>(flags.p));
  PREP_TRY(hipGetLastError());
  unsigned f = 0;
  PREP_TRY(hipMemcpy(&f, flags.p, 4, hipMemcpyDeviceToHost));
  *kind = (f & 2u) ? 0 : ((f & 1u) ? 2 : 1);
  return 0;
}

int device_build_tile(const int8_t* dA, int64_t rows, int64_t cols, int64_t ld, int k, int parts, BuiltTile* out, std::string* err) {
  const int kw = std::min(k, rsr::kMaxWindowBits);
  const int64_t nblocks = (cols + k - 1) / k;
  const int64_t nbp = nblocks * parts;
  const int nvals = 1 << k, nwin = 1 << (k - kw);
  if (rows < 1 || rows > rsr::kTileRows) { *err = "tile height out of range"; return RSR_ERR_INVALID_ARGUMENT; }
  if (nbp * nwin > 0x7fffffff) { *err = "too many column blocks"; return RSR_ERR_UNSUPPORTED; }
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  struct EvGuard { hipEvent_t* e; ~EvGuard() { for (int i = 0; i < 4; ++i) if (e[i]) (void)hipEventDestroy(e[i]); } } evg{ev};
  for (auto& e : ev) PREP_TRY(hipEventCreate(&e));

  DevBuf val, sigma, off, next;
  PREP_TRY(hipMalloc(&val.p, (size_t)nbp * rows * 2));
  PREP_TRY(hipMalloc(&sigma.p, (size_t)nbp * rows * 2));
  PREP_TRY(hipMalloc(&off.p, (size_t)nbp * (nvals + 1) * 4));
  PREP_TRY(hipMalloc(&next.p, (size_t)nbp * nwin * 4));
  PREP_TRY(hipEventRecord(ev[0], nullptr));
  hipLaunchKernelGGL(values_kernel, dim3((unsigned)((rows + 255) / 256), (unsigned)std::min<int64_t>(nblocks, 32768)), dim3(256), 0, nullptr, dA, (int)rows,
                     (int)cols, ld, k, parts, (int)nblocks, static_cast<uint16_t*>(val.p));
  PREP_TRY(hipGetLastError());
  PREP_TRY(hipEventRecord(ev[1], nullptr));
  {
    const size_t per_wave = (size_t)std::max(1, nvals >> 1) * 4;
    int waves = (int)std::min<size_t>(4, (size_t)(128 * 1024) / per_wave);
    if (waves < 1) waves = 1;
    const void* kern = reinterpret_cast<const void*>(sort_kernel);
    PREP_TRY(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
    hipLaunchKernelGGL(sort_kernel, dim3((unsigned)((nbp + waves - 1) / waves)), dim3((unsigned)(64 * waves)), per_wave * waves, nullptr,
                       static_cast<const uint16_t*>(val.p), (int)rows, k, (int)nbp, waves, static_cast<uint32_t*>(off.p),
                       static_cast<uint16_t*>(sigma.p));
    PREP_TRY(hipGetLastError());
  }
  hipLaunchKernelGGL(window_kernel, dim3((unsigned)((nbp * nwin + 255) / 256)), dim3(256), 0, nullptr, static_cast<const uint32_t*>(off.p), k,
                     kw, (int)nbp, static_cast<uint32_t*>(next.p));
  PREP_TRY(hipGetLastError());
  PREP_TRY(hipEventRecord(ev[2], nullptr));
  std::vector<uint32_t> n_ext((size_t)nbp * nwin);
  PREP_TRY(hipMemcpy(n_ext.data(), next.p, n_ext.size() * 4, hipMemcpyDeviceToHost));

  // ---- descriptors and stream offsets (host; no row data involved) ----
  std::vector<Unit> units;
  std::vector<UnitJob> jobs;
  std::vector<uint32_t> blk_unit((size_t)nblocks + 1);
  uint64_t stream_units = 0;  // in multiples of kStreamAlign
  int64_t flag_bytes = 0;
  uint32_t max_units = 0;
  for (int64_t b = 0; b < nblocks; ++b) {
    blk_unit[(size_t)b] = (uint32_t)units.size();
    const size_t first_unit = units.size();
    for (int p = 0; p < parts; ++p)
      for (int w = 0; w < nwin; ++w) {
        const uint32_t total = n_ext[(size_t)((b * parts + p) * nwin + w)];
        if (!total) continue;
        const uint32_t nu = (total + rsr::kMaxUnitEntries - 1) / rsr::kMaxUnitEntries;
        for (uint32_t ui = 0; ui < nu; ++ui) {
          const uint32_t eb = (uint32_t)((uint64_t)total * ui / nu), ee = (uint32_t)((uint64_t)total * (ui + 1) / nu);
          Unit u;
          std::memset(&u, 0, sizeof(u));
          u.block = (uint32_t)b; u.window = (uint16_t)w; u.part = (uint8_t)p;
          u.npos = (uint8_t)((ee - eb + rsr::kLanes - 1) / rsr::kLanes);
          u.nentries = ee - eb;
          u.stream_off = (uint32_t)stream_units;
          const uint32_t bytes = rsr::unit_stream_bytes(u.npos);
          stream_units += (bytes + rsr::kStreamAlign - 1) / rsr::kStreamAlign;
          flag_bytes += rsr::kFlagBytes0 + (u.npos > 32 ? rsr::kFlagBytes1 : 0);
          units.push_back(u);
          jobs.push_back(UnitJob{(uint32_t)(b * parts + p), (uint32_t)w, eb, ee - eb});
        }
      }
    if (units.size() == first_unit) {  // an all-zero block still has to write its outputs
      Unit u;
      std::memset(&u, 0, sizeof(u));
      u.block = (uint32_t)b;
      u.stream_off = (uint32_t)stream_units;
      units.push_back(u);
      jobs.push_back(UnitJob{(uint32_t)(b * parts), 0, 0, 0});
    }
    const size_t nub = units.size() - first_unit;
    if (nub > 0xffffu) { *err = "too many work units in one column block"; return RSR_ERR_UNSUPPORTED; }
    for (size_t i = 0; i < nub; ++i) {
      units[first_unit + i].units_in_block = (uint16_t)nub;
      units[first_unit + i].index_in_block = (uint16_t)i;
    }
    max_units = std::max<uint32_t>(max_units, (uint32_t)nub);
    if (stream_units > 0xffffffffull) { *err = "index too large"; return RSR_ERR_UNSUPPORTED; }
  }
  blk_unit[(size_t)nblocks] = (uint32_t)units.size();

  DevBuf d_stream, d_units, d_blk, d_jobs;
  const size_t stream_bytes = (size_t)stream_units * rsr::kStreamAlign;
  PREP_TRY(hipMalloc(&d_stream.p, stream_bytes + 1024));
  PREP_TRY(hipMalloc(&d_units.p, units.size() * sizeof(Unit) + 32));
  PREP_TRY(hipMalloc(&d_blk.p, blk_unit.size() * 4 + 16));
  PREP_TRY(hipMalloc(&d_jobs.p, jobs.size() * sizeof(UnitJob)));
  PREP_TRY(hipMemset(d_stream.p, 0, stream_bytes + 1024));
  PREP_TRY(hipMemcpy(d_units.p, units.data(), units.size() * sizeof(Unit), hipMemcpyHostToDevice));
  PREP_TRY(hipMemcpy(d_blk.p, blk_unit.data(), blk_unit.size() * 4, hipMemcpyHostToDevice));
  PREP_TRY(hipMemcpy(d_jobs.p, jobs.data(), jobs.size() * sizeof(UnitJob), hipMemcpyHostToDevice));
  hipLaunchKernelGGL(emit_kernel, dim3((unsigned)units.size()), dim3(256), 0, nullptr, static_cast<const UnitJob*>(d_jobs.p),
                     static_cast<Unit*>(d_units.p), static_cast<const uint32_t*>(off.p), static_cast<const uint16_t*>(sigma.p), (int)rows, k, kw,
                     static_cast<uint16_t*>(d_stream.p));
  PREP_TRY(hipGetLastError());
  PREP_TRY(hipEventRecord(ev[3], nullptr));
  PREP_TRY(hipMemcpy(units.data(), d_units.p, units.size() * sizeof(Unit), hipMemcpyDeviceToHost));  // (synchronises)
  float ms = 0;
  PREP_TRY(hipEventElapsedTime(&ms, ev[0], ev[1])); out->ms_values = ms;
  PREP_TRY(hipEventElapsedTime(&ms, ev[1], ev[2])); out->ms_sort = ms;
  PREP_TRY(hipEventElapsedTime(&ms, ev[2], ev[3])); out->ms_emit = ms;
  out->stored_rows = 0; out->segments = 0;
  for (const Unit& u : units) {
    out->stored_rows += u.nrows;
    if (u.npos) out->segments += u.nheads + 1;
  }
  out->nunits = (int64_t)units.size();
  out->max_units_per_block = max_units;
  out->flag_bytes = flag_bytes;
  out->parts = parts;
  out->stream_bytes = stream_bytes;
  out->unit_bytes = units.size() * sizeof(Unit);
  out->blk_bytes = blk_unit.size() * 4;
  out->d_stream = d_stream.release();
  out->d_units = d_units.release();
  out->d_blk_unit = d_blk.release();
  return 0;
}

}  // namespace rsr_internal
