// C ABI (include/rsr.h) and the gfx950 kernels of the RSR++ vector x binary/ternary-matrix product.
//
// Kernel structure (one launch per product):
//   * A workgroup stages one activation vector in LDS (plus a zero behind it for the null row
//     index) and owns a contiguous range of column blocks, i.e. a contiguous byte range of the
//     index streams.  Column blocks are independent (the paper's parallelisation I, Appendix C.1).
//   * Its wavefronts take work units (one window of 2^kw row values of one block and part, see
//     rsr_format.h) from an LDS counter.  For a unit a wavefront
//       1. reads the unit's stream with 16-byte buffer loads (the next unit's loads go out while
//          the current one is summed) and walks its positions: every lane owns a run of
//          consecutive sorted rows and gathers v[sigma(p)] from LDS into its running sum - the
//          segmented sums of Eq. SS2 - and where a row's flag says that a new value starts it
//          first drops the sum into the current slot of its private window of u in LDS and moves
//          to the next slot (plain stores: a slot is stored by the lane in which its segment
//          ends; the part of a segment that a lane is left with at the end of its run is added
//          to the slot afterwards);
//       2. reads the window back in value order;
//       3. takes the low kw levels of the RSR++ fold (Section 4.3, Algorithm 3): "sum the
//          odd-indexed entries, then add neighbours" - three levels inside a lane's 8 consecutive
//          values, the next six across the 64 lanes - and leaves kw sums plus the window total
//          in a per-unit record.
//   * The wavefront that completes the last unit of a block adds the records up: low bits sum
//     over windows, the k-kw high levels of the fold see only window totals; the two parts of a
//     ternary matrix are reduced separately and subtracted once (Proposition 2.1); k outputs are
//     stored.
// All float additions happen in a fixed order (no floating-point atomics), so results are
// reproducible from run to run.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "../../include/rsr.h"
#include "rsr_format.h"
#include "rsr_internal.h"
#include "rsr_pack.h"

namespace {

thread_local std::string g_error;

int fail(int code, const std::string& msg) {
  g_error = msg;
  return code;
}

}  // namespace

namespace rsr_internal {
// shared with the other translation units of the library (rsr_dense.hip)
int set_error(int code, const std::string& msg) { return fail(code, msg); }
}  // namespace rsr_internal

namespace {

#define RSR_HIP_TRY(expr)                                                                   \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      (void)hipGetLastError();                                                              \
      return fail(RSR_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));         \
    }                                                                                       \
  } while (0)

constexpr uint64_t kMagic = 0x5253522b2b763031ull;  // "RSR++v01"

}  // namespace

// One row tile of the index on the device (a matrix of up to rsr::kTileRows rows has one).
struct DeviceTile {
  int64_t rows = 0, row0 = 0;
  uint32_t max_units_per_block = 0;
  int64_t nunits = 0;
  size_t stream_bytes = 0, unit_bytes = 0, blk_bytes = 0;
  void* d_stream = nullptr;
  void* d_units = nullptr;
  void* d_blk_unit = nullptr;
};

struct rsr_handle {
  uint64_t magic = 0;
  int device = 0, num_cu = 0;
  size_t lds_max = 0;
  // shape
  int64_t rows = 0, cols = 0, nblocks = 0;
  int k = 0, kw = 0, parts = 0, last_width = 0;
  int64_t stored_rows = 0, segments = 0, nunits = 0;
  int64_t flag_bytes = 0, stream_bytes = 0, schedule_bytes = 0;
  std::vector<DeviceTile> tiles;
  int waves = 16;  // wavefronts per workgroup at most
  bool step2_plain = false;  // rsr_set_step2
  // host copy of the device tables, fetched on the first rsr_export_block
  std::unique_ptr<rsr::Index> downloaded;
};

struct rsr_host_index {
  uint64_t magic = 0;
  rsr::Index X;
};

namespace {

constexpr uint64_t kHostMagic = 0x525352686f737431ull;  // "RSRhost1"

bool valid(const rsr_host_index* x) { return x && x->magic == kHostMagic; }

void fill_info(const rsr::Index& X, rsr_info_t* info) {
  std::memset(info, 0, sizeof(*info));
  const rsr::Packed& P = X.tiles[0];
  info->rows = X.rows; info->cols = X.cols; info->k = P.k; info->parts = P.parts;
  info->nblocks = P.nblocks; info->last_block_width = P.last_width;
  info->lo_bits = P.kw; info->hi_bits = P.k - P.kw;
  for (const rsr::Packed& T : X.tiles) {
    info->stored_rows += T.stored_rows; info->segments += T.segments; info->work_units += (int64_t)T.units.size();
    info->segment_bytes += T.flag_bytes;
    info->index_bytes += (int64_t)(T.stream.size() * sizeof(uint16_t)) - T.flag_bytes;
    info->schedule_bytes += (int64_t)(T.units.size() * sizeof(rsr::Unit) + T.blk_unit.size() * sizeof(uint32_t));
  }
  info->table_bytes = info->index_bytes + info->segment_bytes + info->schedule_bytes;
  info->device = -1; info->compute_units = 0;
  info->row_tiles = (int32_t)X.tiles.size();
}

bool valid(const rsr_handle* h) { return h && h->magic == kMagic; }

// ---------------------------------------------------------------------------------------------
// device code
// ---------------------------------------------------------------------------------------------
struct KArgs {
  int rows, cols, k, kw, parts, nblocks, last_width, batch;
  int vstride;   // elements between the activation vectors of consecutive batch lanes (the matrix's row count)
  int row0;      // first row of this row tile
  int accumulate;  // add to `out` instead of overwriting it (second and later row tiles, rsr_matvec_acc)
  int scaled;      // multiply the product by `scale` first (rsr_matvec_acc)
  uint32_t scale;  // bits of a float (float activations) or of an int (int8 activations)
  int g1;        // workgroups per batch lane
  int waves;     // wavefronts that take units (the LDS layout has a window for each)
  int ucap;      // unit records per round
  int nslot;     // block completion counters per round
  int nunits;    // unit descriptors in the index
  uint32_t off_win, off_rec, off_done, off_ctr, off_bu;  // LDS byte offsets
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- wavefront sums with DPP (no LDS traffic).  The total ends up in lane 63. ----
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ float dpp_get(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, BANK_MASK, false));
}
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ int dpp_get(int x) {
  return __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, BANK_MASK, false);
}
// Inclusive prefix sum over the 64 lanes.  Lanes whose DPP source does not exist, or that the
// masks exclude, receive 0.
__device__ __forceinline__ int wave_inclusive_scan(int x) {
  int y = x + dpp_get<0x111, 0xf, 0xf>(x);   // row_shr:1
  y += dpp_get<0x112, 0xf, 0xf>(x);           // row_shr:2
  y += dpp_get<0x113, 0xf, 0xf>(x);           // row_shr:3   -> y[i] = x[i-3..i]
  y += dpp_get<0x114, 0xf, 0xe>(y);           // row_shr:4, lanes 4..15 of each row
  y += dpp_get<0x118, 0xf, 0xc>(y);           // row_shr:8, lanes 8..15 -> prefix sums inside each row of 16
  y += dpp_get<0x142, 0xa, 0xf>(y);           // row_bcast:15 into rows 1 and 3
  y += dpp_get<0x143, 0xc, 0xf>(y);           // row_bcast:31 into rows 2 and 3
  return y;
}

// Sum over the 64 lanes, returned to every lane (through a scalar register).
template <typename AT>
__device__ __forceinline__ AT wave_total(AT x) {
  AT y = x + dpp_get<0x111, 0xf, 0xf>(x);
  y += dpp_get<0x112, 0xf, 0xf>(x);
  y += dpp_get<0x113, 0xf, 0xf>(x);
  y += dpp_get<0x114, 0xf, 0xe>(y);
  y += dpp_get<0x118, 0xf, 0xc>(y);
  y += dpp_get<0x142, 0xa, 0xf>(y);
  y += dpp_get<0x143, 0xc, 0xf>(y);
  return __builtin_bit_cast(AT, __builtin_amdgcn_readlane(__builtin_bit_cast(int, y), 63));
}

// Sums of eight values over the 16 lanes of each DPP row, all at once: after every exchange a
// lane keeps half of its values and hands the other half to its partner, so the three halving
// exchanges (lane xor 1, 2, 4) cost 4 + 2 + 1 additions instead of 8 each; a last exchange
// (lane xor 8) completes the row.  On return every lane holds the row sum of v[lane & 7].
template <typename AT>
__device__ __forceinline__ AT row_sums_of_eight(const AT (&v)[8], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
  AT w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const AT keep = b0 ? v[2 * i + 1] : v[2 * i];
    const AT give = b0 ? v[2 * i] : v[2 * i + 1];
    w[i] = keep + dpp_get<0xB1, 0xf, 0xf>(give);  // quad_perm [1,0,3,2]: lane xor 1
  }
  AT x2[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const AT keep = b1 ? w[2 * i + 1] : w[2 * i];
    const AT give = b1 ? w[2 * i] : w[2 * i + 1];
    x2[i] = keep + dpp_get<0x4E, 0xf, 0xf>(give);  // quad_perm [2,3,0,1]: lane xor 2
  }
  const AT keep = b2 ? x2[1] : x2[0];
  const AT give = b2 ? x2[0] : x2[1];
  // lane xor 4: lanes 0-3 and 8-11 of a row read 4 lanes up, lanes 4-7 and 12-15 read 4 lanes down
  const AT y = keep + dpp_get<0x104, 0xf, 0x5>(give) + dpp_get<0x114, 0xf, 0xa>(give);
  return y + dpp_get<0x128, 0xf, 0xf>(y);  // row_ror:8 is lane xor 8 inside a row
}

// Lane swaps of a value with itself, in assembly: the compiler takes the two results of the swap
// builtins for equal when they are combined as floats.  (The s_nop covers the wait states a lane
// swap needs after a vector write of its operands.)
struct Swapped { uint32_t x, y; };
__device__ __forceinline__ Swapped swap32(uint32_t v) {  // .x: lanes 0-31 twice, .y: lanes 32-63 twice
  Swapped r{v, v};
  asm volatile("s_nop 1\n v_permlane32_swap_b32 %0, %1" : "+v"(r.x), "+v"(r.y));
  return r;
}
__device__ __forceinline__ Swapped swap16(uint32_t v) {  // .x: rows 0,0,2,2 of v, .y: rows 1,1,3,3
  Swapped r{v, v};
  asm volatile("s_nop 1\n v_permlane16_swap_b32 %0, %1" : "+v"(r.x), "+v"(r.y));
  return r;
}

// counter += 1 on behalf of the wavefront; returns the old value (wavefront-uniform).  One lane
// does it, with the execution mask set by hand: the compiler's own version of "lane 0 only" costs
// a dozen instructions.  LDS operations of a wavefront execute in order, so stores issued before
// this are in place before the counter moves.
__device__ __forceinline__ uint32_t lds_count_up(uint32_t lds_byte_addr) {
  uint32_t old;
  uint64_t saved;
  asm volatile(
      "s_mov_b64 %[sv], exec\n s_mov_b64 exec, 1\n ds_add_rtn_u32 %[o], %[ad], %[one]\n s_mov_b64 exec, %[sv]\n s_waitcnt lgkmcnt(0)\n"
      : [o] "=&v"(old), [sv] "=&s"(saved)
      : [ad] "v"(lds_byte_addr), [one] "v"(1u)
      : "memory");
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)old);
}

template <typename VT> struct Acc;
template <> struct Acc<float> { using type = float; };
template <> struct Acc<int8_t> { using type = int32_t; };

// ---- the stream positions of a unit, eight (one granule) or two (one dword) at a time ----
// Per position and lane the stream holds a row index x (uint16) and a flag, the top bit of `f`
// (f is shifted left by one per position).  A flagged entry starts a new value: the running sum
// `a` of the segment that ends here goes to the current window slot (LDS byte address `sa`), the
// lane moves to the next slot and the sum restarts; then, flagged or not, the activation with row
// index x is added.  All eight gathers are issued before the first sum so that their latencies
// overlap.  Written in assembly: a position costs one address extraction, one LDS read, one
// add-with-carry that shifts the flags and puts the flag of every lane into vcc, three
// instructions under that mask (store, next slot, restart) and one add; there are no branches.
// (The wait before the add of position q allows 7 - q LDS operations to be outstanding: the
// gathers behind it, whether or not the stores of masked-off lanes are counted.)
//   float activations:  LDS byte address of row x = 4 * x (the vector sits at LDS offset 0)
//   int8 activations:   LDS byte address of row x = x
#define RSR_X4_LO(d, w) "v_lshlrev_b32_sdwa " d ", 2, " w " dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n"
#define RSR_X4_HI(d, w) "v_lshlrev_b32_sdwa " d ", 2, " w " dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n"
#define RSR_X1_LO(d, w) "v_and_b32 " d ", 0xffff, " w "\n"
#define RSR_X1_HI(d, w) "v_lshrrev_b32 " d ", 16, " w "\n"
#define RSR_POS(q, cnt, ADD)                                                                             \
  "v_add_co_u32 %[f], vcc, %[f], %[f]\n s_mov_b64 exec, vcc\n ds_write_b32 %[sa], %[a]\n"              \
  "v_add_u32 %[sa], 4, %[sa]\n v_mov_b32 %[a], 0\n s_mov_b64 exec, -1\n s_waitcnt lgkmcnt(" #cnt ")\n " \
  ADD " %[a], %[a], %[t" #q "]\n"

// In a granule the eight flags are shifted out first, each carry into a scalar register pair: the execution
// masks are then ready when their positions come up, and no position waits for a vector result to reach
// the scalar unit (0.4 us per product at 16384 x 16384).  The wait count of a position in a granule is 8:
// behind the read it needs, the granule has issued 7 - q more reads and q + 1 stores, and LDS operations
// complete in order.
#define RSR_MASK(q) "v_add_co_u32_e64 %[f], %[m" #q "], %[f], %[f]\n"
#define RSR_POSM(q, ADD)                                                                              \
  "s_mov_b64 exec, %[m" #q "]\n ds_write_b32 %[sa], %[a]\n"                                          \
  "v_add_u32 %[sa], 4, %[sa]\n v_mov_b32 %[a], 0\n s_mov_b64 exec, -1\n s_waitcnt lgkmcnt(8)\n "     \
  ADD " %[a], %[a], %[t" #q "]\n"
#define RSR_MASK_REGS                                                                                              \
  [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3), [m4] "=&s"(m4), [m5] "=&s"(m5), [m6] "=&s"(m6), \
      [m7] "=&s"(m7)

__device__ __forceinline__ void granule_step(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, float& a, uint32_t& sa,
                                             uint32_t& f, const float*) {
  uint32_t s0, s1, s2, s3, s4, s5, s6, s7;
  float t0, t1, t2, t3, t4, t5, t6, t7;
  uint64_t m0, m1, m2, m3, m4, m5, m6, m7;
  asm volatile(
      RSR_X4_LO("%[s0]", "%[w0]") RSR_X4_HI("%[s1]", "%[w0]") RSR_X4_LO("%[s2]", "%[w1]") RSR_X4_HI("%[s3]", "%[w1]")
      RSR_X4_LO("%[s4]", "%[w2]") RSR_X4_HI("%[s5]", "%[w2]") RSR_X4_LO("%[s6]", "%[w3]") RSR_X4_HI("%[s7]", "%[w3]")
      "ds_read_b32 %[t0], %[s0]\n ds_read_b32 %[t1], %[s1]\n ds_read_b32 %[t2], %[s2]\n ds_read_b32 %[t3], %[s3]\n"
      "ds_read_b32 %[t4], %[s4]\n ds_read_b32 %[t5], %[s5]\n ds_read_b32 %[t6], %[s6]\n ds_read_b32 %[t7], %[s7]\n"
      RSR_MASK(0) RSR_MASK(1) RSR_MASK(2) RSR_MASK(3) RSR_MASK(4) RSR_MASK(5) RSR_MASK(6) RSR_MASK(7)
      RSR_POSM(0, "v_add_f32") RSR_POSM(1, "v_add_f32") RSR_POSM(2, "v_add_f32") RSR_POSM(3, "v_add_f32")
      RSR_POSM(4, "v_add_f32") RSR_POSM(5, "v_add_f32") RSR_POSM(6, "v_add_f32") RSR_POSM(7, "v_add_f32")
      : [a] "+v"(a), [sa] "+v"(sa), [f] "+v"(f), [s0] "=&v"(s0), [s1] "=&v"(s1), [s2] "=&v"(s2), [s3] "=&v"(s3),
        [s4] "=&v"(s4), [s5] "=&v"(s5), [s6] "=&v"(s6), [s7] "=&v"(s7), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2),
        [t3] "=&v"(t3), [t4] "=&v"(t4), [t5] "=&v"(t5), [t6] "=&v"(t6), [t7] "=&v"(t7), RSR_MASK_REGS
      : [w0] "v"(w0), [w1] "v"(w1), [w2] "v"(w2), [w3] "v"(w3)
      : "vcc", "memory");
}
__device__ __forceinline__ void pair_step(uint32_t w0, float& a, uint32_t& sa, uint32_t& f, const float*) {
  uint32_t s0, s1;
  float t0, t1;
  asm volatile(
      RSR_X4_LO("%[s0]", "%[w0]") RSR_X4_HI("%[s1]", "%[w0]")
      "ds_read_b32 %[t0], %[s0]\n ds_read_b32 %[t1], %[s1]\n"
      RSR_POS(0, 1, "v_add_f32") RSR_POS(1, 0, "v_add_f32")
      : [a] "+v"(a), [sa] "+v"(sa), [f] "+v"(f), [s0] "=&v"(s0), [s1] "=&v"(s1), [t0] "=&v"(t0), [t1] "=&v"(t1)
      : [w0] "v"(w0)
      : "vcc", "memory");
}
__device__ __forceinline__ void single_step(uint32_t w0, float& a, uint32_t& sa, uint32_t& f, const float*) {
  uint32_t s0;
  float t0;
  asm volatile(RSR_X4_LO("%[s0]", "%[w0]") "ds_read_b32 %[t0], %[s0]\n" RSR_POS(0, 0, "v_add_f32")
               : [a] "+v"(a), [sa] "+v"(sa), [f] "+v"(f), [s0] "=&v"(s0), [t0] "=&v"(t0)
               : [w0] "v"(w0)
               : "vcc", "memory");
}
__device__ __forceinline__ void granule_step(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, int32_t& a, uint32_t& sa,
                                             uint32_t& f, const int8_t*) {
  uint32_t s0, s1, s2, s3, s4, s5, s6, s7;
  int32_t t0, t1, t2, t3, t4, t5, t6, t7;
  uint64_t m0, m1, m2, m3, m4, m5, m6, m7;
  asm volatile(
      RSR_X1_LO("%[s0]", "%[w0]") RSR_X1_HI("%[s1]", "%[w0]") RSR_X1_LO("%[s2]", "%[w1]") RSR_X1_HI("%[s3]", "%[w1]")
      RSR_X1_LO("%[s4]", "%[w2]") RSR_X1_HI("%[s5]", "%[w2]") RSR_X1_LO("%[s6]", "%[w3]") RSR_X1_HI("%[s7]", "%[w3]")
      "ds_read_i8 %[t0], %[s0]\n ds_read_i8 %[t1], %[s1]\n ds_read_i8 %[t2], %[s2]\n ds_read_i8 %[t3], %[s3]\n"
      "ds_read_i8 %[t4], %[s4]\n ds_read_i8 %[t5], %[s5]\n ds_read_i8 %[t6], %[s6]\n ds_read_i8 %[t7], %[s7]\n"
      RSR_MASK(0) RSR_MASK(1) RSR_MASK(2) RSR_MASK(3) RSR_MASK(4) RSR_MASK(5) RSR_MASK(6) RSR_MASK(7)
      RSR_POSM(0, "v_add_u32") RSR_POSM(1, "v_add_u32") RSR_POSM(2, "v_add_u32") RSR_POSM(3, "v_add_u32")
      RSR_POSM(4, "v_add_u32") RSR_POSM(5, "v_add_u32") RSR_POSM(6, "v_add_u32") RSR_POSM(7, "v_add_u32")
      : [a] "+v"(a), [sa] "+v"(sa), [f] "+v"(f), [s0] "=&v"(s0), [s1] "=&v"(s1), [s2] "=&v"(s2), [s3] "=&v"(s3),
        [s4] "=&v"(s4), [s5] "=&v"(s5), [s6] "=&v"(s6), [s7] "=&v"(s7), [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2),
        [t3] "=&v"(t3), [t4] "=&v"(t4), [t5] "=&v"(t5), [t6] "=&v"(t6), [t7] "=&v"(t7), RSR_MASK_REGS
      : [w0] "v"(w0), [w1] "v"(w1), [w2] "v"(w2), [w3] "v"(w3)
      : "vcc", "memory");
}
__device__ __forceinline__ void pair_step(uint32_t w0, int32_t& a, uint32_t& sa, uint32_t& f, const int8_t*) {
  uint32_t s0, s1;
  int32_t t0, t1;
  asm volatile(
      RSR_X1_LO("%[s0]", "%[w0]") RSR_X1_HI("%[s1]", "%[w0]")
      "ds_read_i8 %[t0], %[s0]\n ds_read_i8 %[t1], %[s1]\n"
      RSR_POS(0, 1, "v_add_u32") RSR_POS(1, 0, "v_add_u32")
      : [a] "+v"(a), [sa] "+v"(sa), [f] "+v"(f), [s0] "=&v"(s0), [s1] "=&v"(s1), [t0] "=&v"(t0), [t1] "=&v"(t1)
      : [w0] "v"(w0)
      : "vcc", "memory");
}

// The scalar fields of a unit descriptor.  The unit number is wavefront-uniform, so the descriptor is
// read with scalar loads: these do not queue with the vector loads of the compute unit, which
// return in the order they were issued across all its wavefronts - a descriptor that has to come
// from memory would hold back everything requested after it (the other wavefronts' share of the
// activation vector at the start, stream data later).
__device__ __forceinline__ void single_step(uint32_t w0, int32_t& a, uint32_t& sa, uint32_t& f, const int8_t*) {
  uint32_t s0;
  int32_t t0;
  asm volatile(RSR_X1_LO("%[s0]", "%[w0]") "ds_read_i8 %[t0], %[s0]\n" RSR_POS(0, 0, "v_add_u32")
               : [a] "+v"(a), [sa] "+v"(sa), [f] "+v"(f), [s0] "=&v"(s0), [t0] "=&v"(t0)
               : [w0] "v"(w0)
               : "vcc", "memory");
}

struct Desc {
  uint32_t stream_off, block;
  int window, part, npos, units_in_block, index_in_block, slot0;
};
__device__ __forceinline__ Desc load_desc(const uint32_t* __restrict__ unit_words, uint32_t u) {
  const uint32_t* w = unit_words + (size_t)__builtin_amdgcn_readfirstlane((int)u) * 8;
  Desc d;
  d.stream_off = w[0];
  d.block = w[1];
  const uint32_t w2 = w[2], w3 = w[3], w4 = w[4];
  d.window = (int)(w2 & 0xffffu);
  d.part = (int)((w2 >> 16) & 0xffu);
  d.npos = (int)(w2 >> 24);
  d.units_in_block = (int)(w3 & 0xffffu);
  d.index_in_block = (int)(w3 >> 16);
  d.slot0 = (int)(w4 & 0xffffu);
  return d;
}

constexpr int NG = rsr::kMaxGranules;
#ifndef RSR_HEAD_GRANULES
#define RSR_HEAD_GRANULES 1
#endif

// The work of one workgroup: `wg` is its number among the workgroups of this product (a launch may
// carry several products, see rsr_multi_kernel).  The workgroup may have more wavefronts than the
// product's LDS layout has windows for (p.waves): the others help to stage the activation vector
// and take no units.
// PLAIN selects step 2 of Algorithm 2 as printed there (the product u . Bin_[k] term by term,
// O(k 2^k)) instead of the RSR++ fold of Algorithm 3: kept for the comparison of Appendix F.2.
template <typename VT, bool PLAIN>
__device__ __forceinline__ void rsr_body(const unsigned char* __restrict__ stream, const uint32_t* __restrict__ unit_words,
                                         const uint32_t* __restrict__ blk_unit, const VT* __restrict__ vin,
                                         typename Acc<VT>::type* __restrict__ out, const KArgs& p, const int wg) {
  using AT = typename Acc<VT>::type;
  extern __shared__ __align__(16) unsigned char lds[];
  VT* vl = reinterpret_cast<VT*>(lds);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwaves = p.waves;
  const bool worker = wave < nwaves;

  // workgroup -> (batch lane b, block range g): the `batch` siblings of a block range sit 8
  // workgroup ids apart so that round-robin dispatch puts them on the same XCD (shared L2).
  const int per = 8 * p.batch;
  const int grp = wg / per, rem = wg % per;
  const int b = rem >> 3;
  const int g = grp * 8 + (rem & 7);
  if (g >= p.g1) return;
  const int blk_begin = (int)((int64_t)g * p.nblocks / p.g1);
  const int blk_end = (int)((int64_t)(g + 1) * p.nblocks / p.g1);
  if (blk_begin >= blk_end) return;

  const uint32_t winbase = p.off_win + (uint32_t)(worker ? wave : 0) * (rsr::kWindow * 4);
  AT* win = reinterpret_cast<AT*>(lds + winbase);
  AT* rec = reinterpret_cast<AT*>(lds + p.off_rec);
  unsigned* done = reinterpret_cast<unsigned*>(lds + p.off_done);
  unsigned* ctr = reinterpret_cast<unsigned*>(lds + p.off_ctr);
  uint32_t* bu = reinterpret_cast<uint32_t*>(lds + p.off_bu);  // first unit of the round's blocks
  AT* outp = out + (int64_t)b * p.cols;
  const uint32_t lane16 = (uint32_t)lane * 16u, lane4 = (uint32_t)lane * 4u, lane2 = (uint32_t)lane * 2u;

  // Two register buffers: while one unit is summed from one, the next unit's stream arrives in the
  // other.  Every unit issues the same number of loads (the ones it does not need read the first
  // bytes of the stream, which stay cached), so that the wait counts between units are exact and a
  // wait for the current unit never waits for the next one.
  uint32_t eA[NG][4], eB[NG][4];
  uint32_t tA[4], tB[4];  // positions behind the last full granule: up to three rows of dwords and one of uint16
  uint32_t fA[2], fB[2];  // the lane's flags: positions 0..31 from bit 31 down, positions 32..47 from bit 15 down
  // A unit's stream is read through a buffer descriptor that covers exactly the unit: a load past
  // its end (a granule, a dword row or the second flag word the unit does not have, or a unit that
  // does not exist: npos = 0) returns zeros without touching memory, and an address costs no
  // vector arithmetic.
  auto unit_rsrc = [&](uint32_t stream_off, int npos) {
    unsigned char* us = const_cast<unsigned char*>(stream) + (size_t)stream_off * rsr::kStreamAlign;
    const int bytes = npos * rsr::kPositionBytes + (npos > 0 ? rsr::kFlagBytes0 : 0) + (npos > 32 ? rsr::kFlagBytes1 : 0);
    return __builtin_amdgcn_make_buffer_rsrc(us, 0, bytes, 0x00020000);
  };
  constexpr int kNonTemporal = 2;  // the stream is read once per product: keep it from displacing reused data
  // (the offsets go into the per-lane offset, which the range check covers; the scalar offset stays 0)
  const uint32_t lane16_hi = lane16 + 4096u;
  auto issue_granule = [&](__amdgpu_buffer_rsrc_t rs, int gq, uint32_t (&e)[NG][4]) {
    const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(gq < 4 ? lane16 : lane16_hi) + (gq & 3) * 1024, 0, kNonTemporal);
    e[gq][0] = x.x; e[gq][1] = x.y; e[gq][2] = x.z; e[gq][3] = x.w;
  };
  auto issue_pair = [&](__amdgpu_buffer_rsrc_t rs, uint32_t pair_base, int j, uint32_t (&et)[4]) {
    et[j] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)pair_base + j * 256, 0, kNonTemporal);
  };
  // the last position of an odd count: a row of uint16 behind the dword rows (for an even count this
  // reads flag bytes, which nobody uses)
  auto issue_single = [&](__amdgpu_buffer_rsrc_t rs, int npos, uint32_t (&et)[4]) {
    et[3] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rs, (int)((uint32_t)(npos & ~1) * rsr::kPositionBytes + lane2), 0, kNonTemporal);
  };
  auto issue_flags = [&](__amdgpu_buffer_rsrc_t rs, int npos, uint32_t (&f)[2]) {
    const uint32_t fbase = (uint32_t)npos * rsr::kPositionBytes;
    f[0] = __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(fbase + lane4), 0, kNonTemporal);
    f[1] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rs, (int)(fbase + rsr::kFlagBytes0 + lane2), 0, kNonTemporal);
  };
  // A wavefront's first unit is requested in two parts: the flags and the first kHeadGranules
  // granules before the workgroup's barrier, the rest behind it (see there).
  constexpr int kHeadGranules = RSR_HEAD_GRANULES;
  auto issue_head = [&](uint32_t stream_off, int npos, uint32_t (&e)[NG][4], uint32_t (&f)[2]) {
    const __amdgpu_buffer_rsrc_t rs = unit_rsrc(stream_off, npos);
    issue_flags(rs, npos, f);
#pragma unroll
    for (int gq = 0; gq < kHeadGranules; ++gq) issue_granule(rs, gq, e);
  };
  auto issue_rest = [&](uint32_t stream_off, int npos, uint32_t (&e)[NG][4], uint32_t (&et)[4]) {
    const __amdgpu_buffer_rsrc_t rs = unit_rsrc(stream_off, npos);
#pragma unroll
    for (int gq = kHeadGranules; gq < NG; ++gq) issue_granule(rs, gq, e);
#pragma unroll
    for (int j = 0; j < 3; ++j) issue_pair(rs, lane4 + (uint32_t)(npos >> 3) * 1024u, j, et);
    issue_single(rs, npos, et);
  };

  // The activation vector is staged first: its loads go out before anything else so that they do
  // not queue behind the (much larger) first stream loads of the other wavefronts.
  const VT* __restrict__ v = vin + (int64_t)b * p.vstride + p.row0;
  constexpr int per16 = 16 / (int)sizeof(VT);
  const int n16 = ((reinterpret_cast<uintptr_t>(v) & 15) == 0) ? p.rows / per16 : 0;
  const uint4* v16 = reinterpret_cast<const uint4*>(v);
  constexpr int kEarly = 4;  // 16-byte pieces per thread fetched before the descriptors
  uint4 sv[kEarly];
#pragma unroll
  for (int j = 0; j < kEarly; ++j) {
    const int i = tid + j * (int)blockDim.x;
    sv[j] = make_uint4(0, 0, 0, 0);
    if (i < n16) sv[j] = v16[i];
  }

  // where a lane puts its part of a unit record (see below), in bytes from the record's start
  const uint32_t rec_lane = 4u * (lane < 7 ? (uint32_t)lane : lane == 7 ? 9u : lane == 15 ? 7u : lane == 23 ? 8u : lane == 31 ? 10u : 12u);
  bool first_round = true;
  for (int rb0 = blk_begin; rb0 < blk_end;) {
    // ---- round set-up.  A round covers as many consecutive blocks as there are completion
    //      counters (nslot <= 64) and unit records (ucap). ----
    // Usually all blocks of the workgroup fit in one round; otherwise the block table of the next
    // nslot blocks is fetched to find out how many do.  (By the last threads of the workgroup:
    // vector loads return in the order of issue across the wavefronts of a compute unit.)
    const uint32_t u_begin = blk_unit[rb0];
    const uint32_t u_last = blk_unit[blk_end];
    const bool one_round = (blk_end - rb0 <= p.nslot) && (u_last - u_begin <= (uint32_t)p.ucap);
    if (!one_round) {
      for (int i = (int)blockDim.x - 1 - tid; i <= p.nslot; i += (int)blockDim.x) {
        const int blk = rb0 + i;
        bu[i] = blk_unit[blk < blk_end ? blk : blk_end];
      }
    }
    if (tid < p.nslot) done[tid] = 0;
    // the first unit of every wavefront is fixed (u_begin + wave), so that its descriptor can be
    // fetched before the barrier; later ones come from the counter
    if (tid == 0) *ctr = (unsigned)nwaves;
    // The first stream loads go out before anything waits for the activation vector: they are
    // behind it in the queue anyway.
    const uint32_t u_first = u_begin + (uint32_t)wave;
    Desc D = load_desc(unit_words, u_first < (uint32_t)p.nunits ? u_first : 0u);
    if (!worker) D.npos = 0;  // (its loads then fall outside the buffer descriptor and read nothing)
    issue_head(D.stream_off, D.npos, eA, fA);
    if (first_round) {
      // vl[rows] = 0 serves the null row index.
      uint4* l16 = reinterpret_cast<uint4*>(vl);
#pragma unroll
      for (int j = 0; j < kEarly; ++j) {
        const int i = tid + j * (int)blockDim.x;
        if (i < n16) l16[i] = sv[j];
      }
      for (int i = tid + kEarly * (int)blockDim.x; i < n16; i += blockDim.x) l16[i] = v16[i];
      for (int i = n16 * per16 + tid; i < p.rows; i += blockDim.x) vl[i] = v[i];
      if (tid == 0) vl[p.rows] = (VT)0;
      first_round = false;
    }
    __syncthreads();
    issue_rest(D.stream_off, D.npos, eA, tA);
    int nblk = blk_end - rb0;
    if (!one_round) {
      const bool ok = (lane < p.nslot) && (rb0 + lane < blk_end) && (bu[lane + 1] - u_begin <= (uint32_t)p.ucap);
      const uint64_t mask = __ballot(ok);
      nblk = (~mask == 0) ? 64 : __builtin_ctzll(~mask);
      if (nblk < 1) nblk = 1;  // a single block always fits: ucap >= the largest block
    }
    const int rb1 = rb0 + nblk;
    const uint32_t n_tot = (one_round ? u_last : bu[nblk]) - u_begin;  // units of this round, numbered 0 .. n_tot-1

    // A wavefront reserves its next unit only when it starts on the current one (not earlier): the
    // last units of the round then go to the wavefronts that get there first.
    auto take = [&]() { return lds_count_up(p.off_ctr); };
    auto fetch_desc = [&](uint32_t ixq) {  // past the end it reads unit 0 (unused)
      return load_desc(unit_words, ixq < n_tot ? u_begin + ixq : 0u);
    };
    uint32_t ix = worker ? (uint32_t)wave : n_tot;

    // One unit from buffer (e, et, f); the next unit's stream goes into (en, etn, fn) meanwhile.
    auto unit = [&](uint32_t (&e)[NG][4], uint32_t (&et)[4], uint32_t (&f)[2], uint32_t (&en)[NG][4], uint32_t (&etn)[4],
                    uint32_t (&fn)[2]) {
      const uint32_t ix1 = take();
      Desc D1 = fetch_desc(ix1);
      // (the next unit's descriptor arrives during the first granules; its loads go out one by one
      // between the later steps: a wavefront that issues a whole unit at once waits for room in
      // the memory pipeline while it could be summing)

      // ---- step 1: segmented sums (Eq. SS2) into the window (u of Algorithm 2, this window's slice) ----
      {
        uint4* w16 = reinterpret_cast<uint4*>(win);
        w16[lane] = make_uint4(0, 0, 0, 0);
        w16[lane + 64] = make_uint4(0, 0, 0, 0);
        static_assert(rsr::kWindow == 512, "zeroing above");
      }
      // The lane's first slot: the unit's first slot plus the flags of the lanes before it.
      const uint32_t f1 = f[1] << 16;
      const int nflag = __builtin_popcount(f[0]) + __builtin_popcount(f1);
      const int flags_before = wave_inclusive_scan(nflag) - nflag;
      uint32_t sa = winbase + (uint32_t)(D.slot0 + flags_before) * 4u;
      AT a = (AT)0;
      const int full = D.npos >> 3;
      uint32_t fl = f[0];
      auto step = [&](int gq) {
        if (gq == 4) fl = f1;
        if (gq < full) granule_step(e[gq][0], e[gq][1], e[gq][2], e[gq][3], a, sa, fl, vl);
      };
#pragma unroll
      for (int gq = 0; gq < NG / 2; ++gq) step(gq);
      if (ix1 >= n_tot) D1.npos = 0;
      const __amdgpu_buffer_rsrc_t rs1 = unit_rsrc(D1.stream_off, D1.npos);
      const uint32_t pair_base1 = lane4 + (uint32_t)(D1.npos >> 3) * 1024u;
      issue_flags(rs1, D1.npos, fn);
#pragma unroll
      for (int gq = NG / 2; gq < NG; ++gq) {
        step(gq);
        issue_granule(rs1, 2 * (gq - NG / 2), en);
        issue_granule(rs1, 2 * (gq - NG / 2) + 1, en);
      }
      {
        // the positions behind the last full granule; their flags follow those of the granules
        const int pairs = (D.npos & 7) >> 1;
        fl = (full < 4) ? (f[0] << (8 * full)) : (f1 << (8 * (full - 4)));
#pragma unroll
        for (int j = 0; j < 3; ++j) {
          if (j < pairs) pair_step(et[j], a, sa, fl, vl);
          issue_pair(rs1, pair_base1, j, etn);
        }
        if (D.npos & 1) single_step(et[3], a, sa, fl, vl);
        issue_single(rs1, D1.npos, etn);
      }
      // What a lane is left with belongs to a segment that goes on in the next lane (or ends with
      // the unit): it is added to its slot, which by now holds what the lane that saw the end of the
      // segment has stored there (or zero).  Consecutive lanes without any flag share a slot: their
      // sums are first added up along the lanes, and the last lane of such a run adds the total.
      {
        const bool owner = (nflag > 0) || (lane == 0);
        const bool has = (a != (AT)0);
        if (__builtin_amdgcn_ballot_w64(!owner && has) != 0) {
#pragma unroll
          for (int d = 1; d < 64; d *= 2) {
            const AT oa = __shfl_up(a, d);
            const uint32_t osa = (uint32_t)__shfl_up((int)sa, d);
            if (lane >= d && osa == sa) a += oa;
          }
          const uint32_t nsa = (uint32_t)__shfl_down((int)sa, 1);
          if (lane == 63 || nsa != sa) *reinterpret_cast<AT*>(lds + sa) += a;
        } else if (owner) {
          *reinterpret_cast<AT*>(lds + sa) += a;
        }
      }

      // ---- step 2: the low levels of the RSR++ fold on this window ----
      // lane l holds the values 8l .. 8l+7 of the window: three levels in registers ...
      AT u[8];
      {
        const uint4 x0 = reinterpret_cast<const uint4*>(win)[2 * lane];
        const uint4 x1 = reinterpret_cast<const uint4*>(win)[2 * lane + 1];
        const uint32_t raw[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] = __builtin_bit_cast(AT, raw[i]);
      }
      AT total, bit7, bit8;
      if constexpr (PLAIN) {
        // u . Bin_[kw] by its definition: for every column (value bit) the sum of bit * u[j] over all j.
        AT sb[rsr::kMaxWindowBits];
#pragma unroll
        for (int bit = 0; bit < rsr::kMaxWindowBits; ++bit) {
          AT acc = (AT)0;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc += (AT)(((8 * lane + i) >> bit) & 1) * u[i];
          sb[bit] = wave_total<AT>(acc);
        }
        AT all = (AT)0;
#pragma unroll
        for (int i = 0; i < 8; ++i) all += u[i];
        total = wave_total<AT>(all);  // the window's total, for the value bits above the window
#pragma unroll
        for (int bit = 0; bit < 7; ++bit) total = ((lane & 7) == bit) ? sb[bit] : total;  // lanes 0..6 carry the bit sums
        bit7 = sb[7];
        bit8 = sb[8];
      } else {
      // vals[0..2]: the three levels inside the lane; vals[3..6]: lane bits 0..3 (value bits 3..6);
      // vals[7]: the lane's total, from which the two row-index bits (value bits 7, 8) and the
      // window total follow.
      AT vals[8];
      const AT s01 = u[0] + u[1], s23 = u[2] + u[3], s45 = u[4] + u[5], s67 = u[6] + u[7];
      vals[0] = (u[1] + u[3]) + (u[5] + u[7]);  // odd-indexed entries
      vals[1] = s23 + s67;                      // odd-indexed pair sums
      vals[2] = s45 + s67;                      // odd-indexed sums of four
      const AT x = (s01 + s23) + (s45 + s67);
#pragma unroll
      for (int beta = 0; beta < 4; ++beta) vals[3 + beta] = ((lane >> beta) & 1) ? x : (AT)0;
      vals[7] = x;
      // Sums over the 16 lanes of each row, then across the four rows with lane swaps: total
      // (all rows), value bit 7 (rows 1 and 3) and value bit 8 (rows 2 and 3).
      const uint32_t rowsum = __builtin_bit_cast(uint32_t, row_sums_of_eight<AT>(vals, lane));
      const Swapped h32 = swap32(rowsum);                                              // .x: rows 0,1,0,1  .y: rows 2,3,2,3
      const AT s02_13 = __builtin_bit_cast(AT, h32.x) + __builtin_bit_cast(AT, h32.y);  // rows 0+2, 1+3, 0+2, 1+3
      const Swapped t16 = swap16(__builtin_bit_cast(uint32_t, s02_13));                // .x: 0+2 everywhere  .y: 1+3 everywhere
      const Swapped b16 = swap16(h32.y);                                               // .x: row 2 everywhere  .y: row 3
      total = __builtin_bit_cast(AT, t16.x) + __builtin_bit_cast(AT, t16.y);
      bit7 = __builtin_bit_cast(AT, t16.y);
      bit8 = __builtin_bit_cast(AT, b16.x) + __builtin_bit_cast(AT, b16.y);
      }
      // ---- record, and completion of the block: lanes 0..7 finish the sums ----
      // One store writes the record: lanes 0..6 hold the sums of value bits 0..6, lane 7 the
      // window's total, lane 15 (second row) bit 7, lane 23 bit 8; lane 31 adds part and window.
      const int slot = (int)D.block - rb0;
      {
        AT val = total;
        val = (lane == 15) ? bit7 : val;  // lane bit 4 = rows 1 and 3 = value bit 7
        val = (lane == 23) ? bit8 : val;  // lane bit 5 = rows 2 and 3 = value bit 8
        val = (lane == 31) ? __builtin_bit_cast(AT, (uint32_t)((D.part << 16) | D.window)) : val;
        *reinterpret_cast<AT*>(lds + p.off_rec + ix * (rsr::kRecordWords * 4) + rec_lane) = val;
      }
      const unsigned before = lds_count_up(p.off_done + (uint32_t)slot * 4u);
      if ((int)before + 1 == D.units_in_block) {
        // ---- last unit of the block: remaining fold levels, ternary combine, store ----
        // Lane (bit + 16 * part) adds up, over the block's units, "sum of u[j] over the values j
        // with bit `bit` set".  Bits below kw are in the unit records; a higher bit sees only
        // window totals (the remaining levels of the fold act on the windows' sums).
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");  // the records were written by this workgroup
        // (the two halves of the wavefront take every other record, two records per step, so that
        // four LDS reads are in flight instead of one dependent pair)
        const int bit = lane & 15, q = (lane >> 4) & 1, half = lane >> 5;
        const AT* base = rec + (size_t)((int)ix - D.index_in_block) * rsr::kRecordWords;  // the block's units are consecutive
        const int word = (bit < p.kw) ? bit : 9;
        auto term = [&](uint32_t meta, AT t) {
          const bool use = ((int)(meta >> 16) == q) && (bit < p.kw || (((meta & 0xffffu) >> (bit - p.kw)) & 1u));
          return use ? t : (AT)0;
        };
        AT sum_a = (AT)0, sum_b = (AT)0;
        int j = half;
        for (; j + 2 < D.units_in_block; j += 4) {
          const AT* ra = base + (size_t)j * rsr::kRecordWords;
          const AT* rb = ra + 2 * rsr::kRecordWords;
          const uint32_t ma = __builtin_bit_cast(uint32_t, ra[10]), mb = __builtin_bit_cast(uint32_t, rb[10]);
          const AT ta = ra[word], tb = rb[word];
          sum_a += term(ma, ta);
          sum_b += term(mb, tb);
        }
        if (j < D.units_in_block) {
          const AT* ra = base + (size_t)j * rsr::kRecordWords;
          sum_a += term(__builtin_bit_cast(uint32_t, ra[10]), ra[word]);
        }
        // the two halves of the wavefront, then part 1 (second 16-lane row) from part 0: lane swaps
        const Swapped hs = swap32(__builtin_bit_cast(uint32_t, sum_a + sum_b));
        const AT sum = __builtin_bit_cast(AT, hs.x) + __builtin_bit_cast(AT, hs.y);
        const Swapped ps = swap16(__builtin_bit_cast(uint32_t, sum));  // .x: row 0 (part 0), .y: row 1 (part 1)
        const AT res = __builtin_bit_cast(AT, ps.x) - __builtin_bit_cast(AT, ps.y);  // Proposition 2.1: v.B(1) - v.B(2)
        // value bit `bit` belongs to column k-1-bit of the block (first column most significant)
        const int width = ((int)D.block == p.nblocks - 1) ? p.last_width : p.k;
        const int col = p.k - 1 - bit;
        if (lane < 16 && bit < p.k && col < width) {
          AT* dst = outp + (int64_t)D.block * p.k + col;
          const AT term = p.scaled ? res * __builtin_bit_cast(AT, p.scale) : res;
          *dst = p.accumulate ? *dst + term : term;  // row tiles add up: the product is linear in the rows
        }
      }
      ix = ix1; D = D1;
    };

    while (ix < n_tot) {
      unit(eA, tA, fA, eB, tB, fB);
      if (ix >= n_tot) break;
      unit(eB, tB, fB, eA, tA, fA);
      if (ix >= n_tot) break;
    }
    rb0 = rb1;
    __syncthreads();
  }
}

template <typename VT, bool PLAIN>
__global__ void __launch_bounds__(1024)
rsr_matvec_kernel(const unsigned char* __restrict__ stream, const uint32_t* __restrict__ unit_words,
                  const uint32_t* __restrict__ blk_unit, const VT* __restrict__ vin,
                  typename Acc<VT>::type* __restrict__ out, const KArgs p) {
  rsr_body<VT, PLAIN>(stream, unit_words, blk_unit, vin, out, p, (int)blockIdx.x);
}

// Several products in one launch (rsr_matvec_multi): every product owns a range of workgroups and
// brings its own tables, activations, results and LDS layout.
constexpr int kMaxJobs = 8;
struct KJob {
  const unsigned char* stream;
  const uint32_t* unit_words;
  const uint32_t* blk_unit;
  const void* vin;
  void* out;
  int wg_begin;  // first workgroup of this product
  int pad;
  KArgs p;
};
struct MultiArgs {
  int njobs;
  int pad;
  KJob job[kMaxJobs];
};

template <typename VT>
__global__ void __launch_bounds__(1024) rsr_multi_kernel(const MultiArgs m) {
  int j = 0;
#pragma unroll
  for (int i = 1; i < kMaxJobs; ++i)
    if (i < m.njobs && (int)blockIdx.x >= m.job[i].wg_begin) j = i;
  // (selected with a wavefront-uniform index: the arguments stay in scalar registers)
  const KJob& J = m.job[j];
  rsr_body<VT, false>(J.stream, J.unit_words, J.blk_unit, static_cast<const VT*>(J.vin),
               static_cast<typename Acc<VT>::type*>(J.out), J.p, (int)blockIdx.x - J.wg_begin);
}

// ---------------------------------------------------------------------------------------------
// host code
// ---------------------------------------------------------------------------------------------
size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct LaunchPlan {
  KArgs p;
  int64_t grid = 0;
  int waves = 0;
  size_t lds = 0;
};

// Launch shape of one row tile for `batch` vectors on `num_cu` compute units.
// `max_wg_per_cu`: how many workgroups of this product may share a compute unit (a launch that carries
// several products gives every workgroup the largest LDS size any of them needs, so it plans with 1).
template <typename VT>
int plan_tile(const rsr_handle* h, const DeviceTile& T, bool accumulate, int batch, int num_cu, int max_wg_per_cu, LaunchPlan* plan) {
  KArgs& p = plan->p;
  std::memset(&p, 0, sizeof(p));
  p.rows = (int)T.rows; p.cols = (int)h->cols; p.k = h->k; p.kw = h->kw; p.parts = h->parts;
  p.nblocks = (int)h->nblocks; p.last_width = h->last_width; p.batch = batch;
  p.vstride = (int)h->rows; p.row0 = (int)T.row0; p.accumulate = accumulate ? 1 : 0;

  // LDS budget: activation vector + per-wavefront windows + unit records + counters
  const size_t vbytes = align_up(((size_t)T.rows + 1) * sizeof(VT), 16);
  const size_t win_bytes = (size_t)rsr::kWindow * 4;
  const size_t rec_bytes = (size_t)rsr::kRecordWords * 4;
  int nslot = 64;
  // Unit records of a round: room for wavefronts comes first, then as many records as fit (a round
  // ends with a barrier); a block's units always fit in a round.
  size_t ucap = 0;
  int waves = 0;
  auto total = [&](int w, size_t uc) { return vbytes + (size_t)w * win_bytes + uc * rec_bytes + (size_t)nslot * 4 + 16 + ((size_t)nslot + 1) * 4 + 12; };
  for (size_t cand : {(size_t)512, (size_t)256, (size_t)128, (size_t)64, (size_t)1}) {
    const size_t uc = std::max<size_t>(T.max_units_per_block, cand);
    int w = h->waves;
    while (w > 1 && total(w, uc) > h->lds_max) --w;
    if (total(w, uc) <= h->lds_max && w > waves) { waves = w; ucap = uc; }
  }
  if (waves == 0)
    return fail(RSR_ERR_UNSUPPORTED, "a row tile of " + std::to_string(T.rows) + " rows with " + std::to_string(T.max_units_per_block) +
                                         " work units in a column block does not fit in " + std::to_string(h->lds_max) + " bytes of LDS");
  // Grid and workgroup size.  Up to four workgroups per compute unit if they fit together (LDS, and 16
  // wavefronts per compute unit at this kernel's register count); never more workgroups than blocks; and
  // no more wavefronts than the largest share of a workgroup has units: idle wavefronts only lengthen
  // the start of the launch (1024 x 1024: 5.5 -> 4.0 us per product).
  const int waves_fit = waves;
  const size_t ucap_fit = ucap;
  int64_t g1 = 1;
  for (int wg = max_wg_per_cu; wg >= 1; --wg) {
    g1 = ((int64_t)num_cu * wg + batch - 1) / batch;
    g1 = (g1 + 7) / 8 * 8;
    if (g1 > h->nblocks) g1 = h->nblocks;
    if (g1 < 1) g1 = 1;
    const int64_t blocks_per_wg = (h->nblocks + g1 - 1) / g1;
    // Equal shares: no more workgroups than it takes to keep the largest share this small.  (1366 blocks
    // over 256 compute units would be 5 or 6 blocks each; 228 workgroups get 6 each, 28 compute units
    // stay idle, and the product is 0.5 us faster: the stream is shared by all compute units and the
    // workgroups with the larger share finish last either way, only later when more of them compete.)
    g1 = (h->nblocks + blocks_per_wg - 1) / blocks_per_wg;
    const int64_t units_per_wg = blocks_per_wg * (int64_t)std::max<uint32_t>(1, T.max_units_per_block);
    waves = (int)std::min<int64_t>(waves_fit, units_per_wg);
    ucap = std::min<size_t>(ucap_fit, (size_t)units_per_wg);  // records for the units a workgroup can have
    if (wg == 1 || (wg * waves <= 16 && (size_t)wg * total(waves, ucap) <= h->lds_max)) break;
  }
  p.g1 = (int)g1;
  const int64_t grid = (g1 + 7) / 8 * 8 * (int64_t)batch;
  if (grid > 0x7fffffff) return fail(RSR_ERR_INVALID_ARGUMENT, "batch too large");

  plan->lds = total(waves, ucap);
  plan->grid = grid;
  plan->waves = waves;
  p.waves = waves;
  p.ucap = (int)ucap; p.nslot = nslot;
  p.off_win = (uint32_t)vbytes;
  p.off_rec = (uint32_t)(vbytes + (size_t)waves * win_bytes);
  p.off_done = (uint32_t)(p.off_rec + ucap * rec_bytes);
  p.off_ctr = (uint32_t)(p.off_done + (size_t)nslot * 4);
  p.off_bu = p.off_ctr + 16;
  p.nunits = (int)T.nunits;
  return RSR_OK;
}

template <typename VT>
int launch_tile(rsr_handle* h, const DeviceTile& T, bool accumulate, const uint32_t* scale, const VT* v, void* out, int batch, void* stream) {
  LaunchPlan plan;
  const int rc = plan_tile<VT>(h, T, accumulate, batch, h->num_cu, 4, &plan);
  if (rc != RSR_OK) return rc;
  if (scale) { plan.p.scaled = 1; plan.p.scale = *scale; }
  auto kern = h->step2_plain ? rsr_matvec_kernel<VT, true> : rsr_matvec_kernel<VT, false>;
  hipLaunchKernelGGL(kern, dim3((unsigned)plan.grid), dim3((unsigned)(plan.waves * 64)), plan.lds, static_cast<hipStream_t>(stream),
                     static_cast<const unsigned char*>(T.d_stream), static_cast<const uint32_t*>(T.d_units), static_cast<const uint32_t*>(T.d_blk_unit), v,
                     static_cast<typename Acc<VT>::type*>(out), plan.p);
  RSR_HIP_TRY(hipGetLastError());
  return RSR_OK;
}

// Several products as one launch: the compute units are shared out in proportion to the bytes of the
// products' tables; every product is then planned as if it had its share of the device to itself.
template <typename VT>
int launch_multi(const rsr_job* jobs, int njobs, int batch, void* stream) {
  if (!jobs || njobs < 1) return fail(RSR_ERR_INVALID_ARGUMENT, "no jobs");
  if (njobs > kMaxJobs) return fail(RSR_ERR_INVALID_ARGUMENT, "at most " + std::to_string(kMaxJobs) + " products per launch");
  if (batch < 1 || batch > 65535) return fail(RSR_ERR_INVALID_ARGUMENT, "batch must be in 1..65535");
  double bytes_total = 0;
  for (int j = 0; j < njobs; ++j) {
    if (!valid(jobs[j].h)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid handle in job " + std::to_string(j));
    if (!jobs[j].v || !jobs[j].out) return fail(RSR_ERR_INVALID_ARGUMENT, "null pointer in job " + std::to_string(j));
    if (jobs[j].h->tiles.size() != 1) return fail(RSR_ERR_UNSUPPORTED, "a matrix with more than 32768 rows takes a launch per row tile: use rsr_matvec");
    if (jobs[j].h->device != jobs[0].h->device) return fail(RSR_ERR_INVALID_ARGUMENT, "the handles belong to different devices");
    bytes_total += (double)jobs[j].h->stream_bytes + 1.0;
  }
  MultiArgs m;
  std::memset(&m, 0, sizeof(m));
  m.njobs = njobs;
  int64_t grid = 0;
  int waves = 1;
  size_t lds = 0;
  const int num_cu = jobs[0].h->num_cu;
  // shares in multiples of 8 compute units (one per XCD), at least 8, together no more than the device has
  // (a workgroup that has to wait for a free compute unit would start when the others are nearly done)
  int share[kMaxJobs];
  int given = 0;
  for (int j = 0; j < njobs; ++j) {
    share[j] = std::max(8, (int)((double)num_cu * ((double)jobs[j].h->stream_bytes + 1.0) / bytes_total) / 8 * 8);
    given += share[j];
  }
  while (given > num_cu) {
    int big = 0;
    for (int j = 1; j < njobs; ++j) if (share[j] > share[big]) big = j;
    if (share[big] <= 8) break;
    share[big] -= 8; given -= 8;
  }
  while (given + 8 <= num_cu) {  // what is left over goes to the products with the most bytes per compute unit
    int best = 0;
    for (int j = 1; j < njobs; ++j)
      if ((double)jobs[j].h->stream_bytes / share[j] > (double)jobs[best].h->stream_bytes / share[best]) best = j;
    share[best] += 8; given += 8;
  }
  for (int j = 0; j < njobs; ++j) {
    rsr_handle* h = jobs[j].h;
    LaunchPlan plan;
    const int rc = plan_tile<VT>(h, h->tiles[0], false, batch, std::min(share[j], num_cu), 1, &plan);
    if (rc != RSR_OK) return rc;
    KJob& J = m.job[j];
    J.stream = static_cast<const unsigned char*>(h->tiles[0].d_stream);
    J.unit_words = static_cast<const uint32_t*>(h->tiles[0].d_units);
    J.blk_unit = static_cast<const uint32_t*>(h->tiles[0].d_blk_unit);
    J.vin = jobs[j].v; J.out = jobs[j].out;
    J.wg_begin = (int)grid;
    J.p = plan.p;
    grid += plan.grid;  // (a multiple of 8: every product starts on the first XCD of the round-robin)
    waves = std::max(waves, plan.waves);
    lds = std::max(lds, plan.lds);
    if (grid > 0x7fffffff) return fail(RSR_ERR_INVALID_ARGUMENT, "batch too large");
  }
  auto kern = rsr_multi_kernel<VT>;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3((unsigned)(waves * 64)), lds, static_cast<hipStream_t>(stream), m);
  RSR_HIP_TRY(hipGetLastError());
  return RSR_OK;
}

// One launch per row tile, in order, on the caller's stream: the first overwrites `out`, the others add.
template <typename VT>
// With `scale` (rsr_matvec_acc) every launch adds scale * (its tile's product) to `out`.
int launch(rsr_handle* h, const VT* v, void* out, int batch, void* stream, const uint32_t* scale = nullptr) {
  if (!valid(h)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid handle");
  if (!v || !out) return fail(RSR_ERR_INVALID_ARGUMENT, "null pointer");
  if (batch < 1) return fail(RSR_ERR_INVALID_ARGUMENT, "batch must be >= 1");
  if (batch > 65535) return fail(RSR_ERR_INVALID_ARGUMENT, "batch must be <= 65535");
  for (size_t t = 0; t < h->tiles.size(); ++t) {
    const int rc = launch_tile<VT>(h, h->tiles[t], t > 0 || scale != nullptr, scale, v, out, batch, stream);
    if (rc != RSR_OK) return rc;
  }
  return RSR_OK;
}

void free_tables(rsr_handle* h) {
  for (DeviceTile& T : h->tiles) {
    if (T.d_stream) (void)hipFree(T.d_stream);
    if (T.d_units) (void)hipFree(T.d_units);
    if (T.d_blk_unit) (void)hipFree(T.d_blk_unit);
    T.d_stream = T.d_units = T.d_blk_unit = nullptr;
  }
}

int upload(DeviceTile* T, const rsr::Packed& P) {
  T->stream_bytes = P.stream.size() * sizeof(uint16_t);
  T->unit_bytes = P.units.size() * sizeof(rsr::Unit);
  T->blk_bytes = P.blk_unit.size() * sizeof(uint32_t);
  RSR_HIP_TRY(hipMalloc(&T->d_stream, T->stream_bytes + 1024));
  RSR_HIP_TRY(hipMalloc(&T->d_units, T->unit_bytes + 32));
  RSR_HIP_TRY(hipMalloc(&T->d_blk_unit, T->blk_bytes + 16));
  RSR_HIP_TRY(hipMemset(static_cast<unsigned char*>(T->d_stream) + T->stream_bytes, 0, 1024));
  if (T->stream_bytes) RSR_HIP_TRY(hipMemcpy(T->d_stream, P.stream.data(), T->stream_bytes, hipMemcpyHostToDevice));
  if (T->unit_bytes) RSR_HIP_TRY(hipMemcpy(T->d_units, P.units.data(), T->unit_bytes, hipMemcpyHostToDevice));
  RSR_HIP_TRY(hipMemcpy(T->d_blk_unit, P.blk_unit.data(), T->blk_bytes, hipMemcpyHostToDevice));
  RSR_HIP_TRY(hipDeviceSynchronize());
  return RSR_OK;
}

}  // namespace

extern "C" {

rsr_handle* rsr_preprocess(const int8_t* A, int64_t rows, int64_t cols, int k) {
  g_error.clear();
  std::unique_ptr<rsr_handle> h(new (std::nothrow) rsr_handle());
  if (!h) { fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory"); return nullptr; }
  rsr::Index X;
  std::string err;
  int rc;
  try {
    rc = rsr::pack_tiles(A, rows, cols, k, 0, &X, &err);
  } catch (const std::bad_alloc&) {
    fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory while packing");
    return nullptr;
  }
  if (rc != 0) { fail(rc, "rsr_preprocess: " + err); return nullptr; }

  hipError_t e = hipGetDevice(&h->device);
  if (e != hipSuccess) { (void)hipGetLastError(); fail(RSR_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e)); return nullptr; }
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, h->device);
  if (e != hipSuccess) { (void)hipGetLastError(); fail(RSR_ERR_HIP, std::string("hipGetDeviceProperties: ") + hipGetErrorString(e)); return nullptr; }
  h->num_cu = prop.multiProcessorCount;
  h->lds_max = prop.sharedMemPerBlock;
  rsr_info_t info;
  fill_info(X, &info);
  h->rows = rows; h->cols = cols; h->nblocks = info.nblocks;
  h->k = info.k; h->kw = info.lo_bits; h->parts = info.parts; h->last_width = info.last_block_width;
  h->stored_rows = info.stored_rows; h->segments = info.segments; h->nunits = info.work_units;
  h->flag_bytes = info.segment_bytes; h->stream_bytes = info.index_bytes + info.segment_bytes; h->schedule_bytes = info.schedule_bytes;
  // both kernels may use the whole LDS of a compute unit as dynamic shared memory
  for (const void* kern : {reinterpret_cast<const void*>(rsr_matvec_kernel<float, false>),
                           reinterpret_cast<const void*>(rsr_matvec_kernel<int8_t, false>),
                           reinterpret_cast<const void*>(rsr_matvec_kernel<float, true>),
                           reinterpret_cast<const void*>(rsr_matvec_kernel<int8_t, true>),
                           reinterpret_cast<const void*>(rsr_multi_kernel<float>),
                           reinterpret_cast<const void*>(rsr_multi_kernel<int8_t>)}) {
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)h->lds_max);
    if (e != hipSuccess) { (void)hipGetLastError(); fail(RSR_ERR_HIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e)); return nullptr; }
  }
  h->tiles.resize(X.tiles.size());
  for (size_t t = 0; t < X.tiles.size(); ++t) {
    DeviceTile& T = h->tiles[t];
    T.rows = X.tiles[t].rows; T.row0 = X.row0[t];
    T.max_units_per_block = X.tiles[t].max_units_per_block;
    T.nunits = (int64_t)X.tiles[t].units.size();
    if (upload(&T, X.tiles[t]) != RSR_OK) { free_tables(h.get()); return nullptr; }
  }
  h->magic = kMagic;
  return h.release();
}

rsr_handle* rsr_preprocess_device(const int8_t* A, int64_t rows, int64_t cols, int k) {
  g_error.clear();
  if (!A) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_preprocess_device: null pointer"); return nullptr; }
  if (rows < 1 || rows > rsr::kMaxRows) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_preprocess_device: rows must be in 1..65534"); return nullptr; }
  if (cols < 1) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_preprocess_device: cols must be >= 1"); return nullptr; }
  if (k < 1 || k > rsr::kMaxK) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_preprocess_device: k must be in 1..16"); return nullptr; }
  std::unique_ptr<rsr_handle> h(new (std::nothrow) rsr_handle());
  if (!h) { fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory"); return nullptr; }
  hipError_t e = hipGetDevice(&h->device);
  hipDeviceProp_t prop;
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, h->device);
  if (e != hipSuccess) { (void)hipGetLastError(); fail(RSR_ERR_HIP, std::string("rsr_preprocess_device: ") + hipGetErrorString(e)); return nullptr; }
  h->num_cu = prop.multiProcessorCount;
  h->lds_max = prop.sharedMemPerBlock;
  std::string err;
  int kind = 0;
  int rc = rsr_internal::device_matrix_kind(A, rows * cols, &kind, &err);
  if (rc != 0) { fail(rc, "rsr_preprocess_device: " + err); return nullptr; }
  if (kind == 0) { fail(RSR_ERR_INVALID_ARGUMENT, "rsr_preprocess_device: an entry lies outside {-1,0,1}"); return nullptr; }
  h->rows = rows; h->cols = cols; h->k = k; h->kw = std::min(k, rsr::kMaxWindowBits); h->parts = kind;
  h->nblocks = (cols + k - 1) / k;
  h->last_width = (int)(cols - (h->nblocks - 1) * k);
  for (const void* kern : {reinterpret_cast<const void*>(rsr_matvec_kernel<float, false>),
                           reinterpret_cast<const void*>(rsr_matvec_kernel<int8_t, false>),
                           reinterpret_cast<const void*>(rsr_matvec_kernel<float, true>),
                           reinterpret_cast<const void*>(rsr_matvec_kernel<int8_t, true>),
                           reinterpret_cast<const void*>(rsr_multi_kernel<float>),
                           reinterpret_cast<const void*>(rsr_multi_kernel<int8_t>)}) {
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)h->lds_max);
    if (e != hipSuccess) { (void)hipGetLastError(); fail(RSR_ERR_HIP, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e)); return nullptr; }
  }
  const int64_t ntiles = (rows + rsr::kTileRows - 1) / rsr::kTileRows;
  const int64_t height = ((rows + ntiles - 1) / ntiles + 15) / 16 * 16;
  for (int64_t t = 0; t < ntiles; ++t) {
    const int64_t r0 = t * height, r1 = std::min(rows, r0 + height);
    rsr_internal::BuiltTile B;
    rc = rsr_internal::device_build_tile(A + r0 * cols, r1 - r0, cols, cols, k, kind, &B, &err);
    if (rc != 0) { free_tables(h.get()); fail(rc, "rsr_preprocess_device: " + err); return nullptr; }
    DeviceTile T;
    T.rows = r1 - r0; T.row0 = r0;
    T.max_units_per_block = B.max_units_per_block; T.nunits = B.nunits;
    T.stream_bytes = B.stream_bytes; T.unit_bytes = B.unit_bytes; T.blk_bytes = B.blk_bytes;
    T.d_stream = B.d_stream; T.d_units = B.d_units; T.d_blk_unit = B.d_blk_unit;
    h->tiles.push_back(T);
    h->stored_rows += B.stored_rows; h->segments += B.segments; h->nunits += B.nunits;
    h->flag_bytes += B.flag_bytes; h->stream_bytes += (int64_t)B.stream_bytes;
    h->schedule_bytes += (int64_t)(B.unit_bytes + B.blk_bytes);
  }
  h->magic = kMagic;
  return h.release();
}

int rsr_matvec(rsr_handle* h, const float* v, float* out, int batch, void* stream) {
  return launch<float>(h, v, out, batch, stream);
}

int rsr_matvec_i8(rsr_handle* h, const int8_t* v, int32_t* out, int batch, void* stream) {
  return launch<int8_t>(h, v, out, batch, stream);
}

int rsr_matvec_acc(rsr_handle* h, const float* v, float* out, float scale, int batch, void* stream) {
  if (!(scale == scale) || scale - scale != 0.0f) return fail(RSR_ERR_INVALID_ARGUMENT, "rsr_matvec_acc: scale must be finite");
  const uint32_t bits = __builtin_bit_cast(uint32_t, scale);
  return launch<float>(h, v, out, batch, stream, &bits);
}

int rsr_matvec_acc_i8(rsr_handle* h, const int8_t* v, int32_t* out, int32_t scale, int batch, void* stream) {
  const uint32_t bits = (uint32_t)scale;
  return launch<int8_t>(h, v, out, batch, stream, &bits);
}

int rsr_matvec_multi(const rsr_job* jobs, int njobs, int batch, void* stream) {
  return launch_multi<float>(jobs, njobs, batch, stream);
}

int rsr_matvec_multi_i8(const rsr_job* jobs, int njobs, int batch, void* stream) {
  return launch_multi<int8_t>(jobs, njobs, batch, stream);
}

int rsr_set_step2(rsr_handle* h, int step2) {
  if (!valid(h)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid handle");
  if (step2 != RSR_STEP2_FOLD && step2 != RSR_STEP2_PLAIN) return fail(RSR_ERR_INVALID_ARGUMENT, "unknown step 2 variant");
  h->step2_plain = (step2 == RSR_STEP2_PLAIN);
  return RSR_OK;
}

int rsr_model_k(int64_t rows, int k_min, int k_max) {
  if (rows < 1 || k_min < 1 || k_max > rsr::kMaxK || k_min > k_max) return fail(RSR_ERR_INVALID_ARGUMENT, "rsr_model_k: bad range");
  int best = k_min;
  double best_cost = 0;
  for (int k = k_min; k <= k_max; ++k) {
    const double cost = ((double)rows + (double)(1u << k)) / (double)k;  // per column: (n + 2^k) / k
    if (k == k_min || cost < best_cost) { best = k; best_cost = cost; }
  }
  return best;
}

int rsr_autotune_k(const int8_t* A, int64_t rows, int64_t cols, int batch, int k_min, int k_max, int reps, int cold,
                   int* best_k, double* us_per_k) {
  g_error.clear();
  if (!A || !best_k) return fail(RSR_ERR_INVALID_ARGUMENT, "null pointer");
  if (k_min < 1 || k_max > rsr::kMaxK || k_min > k_max) return fail(RSR_ERR_INVALID_ARGUMENT, "k range must lie in 1..16");
  if (batch < 1 || batch > 65535 || reps < 1) return fail(RSR_ERR_INVALID_ARGUMENT, "batch and reps must be >= 1");
  float* v = nullptr;
  float* out = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  std::vector<rsr_handle*> hs;
  auto cleanup = [&]() {
    (void)hipDeviceSynchronize();
    for (rsr_handle* h : hs) rsr_destroy(h);
    hs.clear();
  };
  auto release = [&]() {
    cleanup();
    if (v) (void)hipFree(v);
    if (out) (void)hipFree(out);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  };
  auto bail = [&](int code, const std::string& msg) { release(); return fail(code, msg); };
  if (hipMalloc(&v, (size_t)batch * rows * sizeof(float)) != hipSuccess || hipMalloc(&out, (size_t)batch * cols * sizeof(float)) != hipSuccess)
    return bail(RSR_ERR_HIP, "rsr_autotune_k: device allocation failed");
  if (hipMemset(v, 0, (size_t)batch * rows * sizeof(float)) != hipSuccess) return bail(RSR_ERR_HIP, "rsr_autotune_k: hipMemset failed");
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return bail(RSR_ERR_HIP, "rsr_autotune_k: hipEventCreate failed");
  double best_us = 0;
  for (int k = k_min; k <= k_max; ++k) {
    rsr_handle* h = rsr_preprocess(A, rows, cols, k);
    if (!h) { const std::string msg = g_error; return bail(RSR_ERR_INVALID_ARGUMENT, msg); }
    hs.push_back(h);
    if (cold) {  // enough copies that the tables of consecutive calls do not come from the last-level cache
      rsr_info_t info;
      rsr_info(h, &info);
      const int64_t want = ((int64_t)512 << 20) / std::max<int64_t>(1, info.table_bytes) + 1;
      const int copies = (int)std::min<int64_t>(16, std::max<int64_t>(1, want));
      for (int c = 1; c < copies; ++c) {
        rsr_handle* hc = rsr_preprocess(A, rows, cols, k);
        if (!hc) { const std::string msg = g_error; return bail(RSR_ERR_HIP, msg); }
        hs.push_back(hc);
      }
    }
    const int n = (int)hs.size();
    int rc = RSR_OK;
    for (int i = 0; i < std::max(3, n) && rc == RSR_OK; ++i) rc = rsr_matvec(hs[(size_t)(i % n)], v, out, batch, nullptr);
    if (rc == RSR_OK && hipEventRecord(e0, nullptr) != hipSuccess) rc = RSR_ERR_HIP;
    for (int i = 0; i < reps && rc == RSR_OK; ++i) rc = rsr_matvec(hs[(size_t)(i % n)], v, out, batch, nullptr);
    if (rc == RSR_OK && (hipEventRecord(e1, nullptr) != hipSuccess || hipEventSynchronize(e1) != hipSuccess)) rc = RSR_ERR_HIP;
    float ms = 0;
    if (rc == RSR_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = RSR_ERR_HIP;
    if (rc != RSR_OK) { const std::string msg = g_error.empty() ? "rsr_autotune_k: timing failed" : g_error; return bail(rc, msg); }
    const double us = (double)ms * 1e3 / reps;
    if (us_per_k) us_per_k[k - k_min] = us;
    if (k == k_min || us < best_us) { best_us = us; *best_k = k; }
    cleanup();
  }
  release();
  return RSR_OK;
}

void rsr_destroy(rsr_handle* h) {
  if (!valid(h)) return;
  free_tables(h);
  h->magic = 0;
  delete h;
}

const char* rsr_last_error(void) { return g_error.c_str(); }

int rsr_info(const rsr_handle* h, rsr_info_t* info) {
  if (!valid(h) || !info) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid handle or null info");
  std::memset(info, 0, sizeof(*info));
  info->rows = h->rows; info->cols = h->cols; info->k = h->k; info->parts = h->parts;
  info->nblocks = h->nblocks; info->last_block_width = h->last_width;
  info->lo_bits = h->kw; info->hi_bits = h->k - h->kw;
  info->stored_rows = h->stored_rows; info->segments = h->segments; info->work_units = h->nunits;
  info->segment_bytes = h->flag_bytes;
  info->index_bytes = h->stream_bytes - h->flag_bytes;
  info->schedule_bytes = h->schedule_bytes;
  info->table_bytes = info->index_bytes + info->segment_bytes + info->schedule_bytes;
  info->device = h->device; info->compute_units = h->num_cu;
  info->row_tiles = (int32_t)h->tiles.size();
  return RSR_OK;
}

int rsr_export_block(rsr_handle* h, int part, int64_t block, int32_t* sigma, int32_t* L) {
  if (!valid(h)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid handle");
  if (!h->downloaded) {
    std::unique_ptr<rsr::Index> X(new (std::nothrow) rsr::Index());
    if (!X) return fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory");
    int dev = 0;
    RSR_HIP_TRY(hipGetDevice(&dev));
    RSR_HIP_TRY(hipSetDevice(h->device));
    X->rows = h->rows; X->cols = h->cols;
    try {
      X->tiles.resize(h->tiles.size());
      for (size_t t = 0; t < h->tiles.size(); ++t) {
        const DeviceTile& T = h->tiles[t];
        rsr::Packed& P = X->tiles[t];
        X->row0.push_back(T.row0);
        P.stream.resize(T.stream_bytes / sizeof(uint16_t));
        P.units.resize(T.unit_bytes / sizeof(rsr::Unit));
        P.blk_unit.resize(T.blk_bytes / sizeof(uint32_t));
        P.rows = T.rows; P.cols = h->cols; P.k = h->k; P.kw = h->kw; P.parts = h->parts;
        P.nblocks = h->nblocks; P.last_width = h->last_width;
        if (T.stream_bytes) RSR_HIP_TRY(hipMemcpy(P.stream.data(), T.d_stream, T.stream_bytes, hipMemcpyDeviceToHost));
        if (T.unit_bytes) RSR_HIP_TRY(hipMemcpy(P.units.data(), T.d_units, T.unit_bytes, hipMemcpyDeviceToHost));
        RSR_HIP_TRY(hipMemcpy(P.blk_unit.data(), T.d_blk_unit, T.blk_bytes, hipMemcpyDeviceToHost));
      }
    } catch (const std::bad_alloc&) {
      (void)hipSetDevice(dev);
      return fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory");
    }
    RSR_HIP_TRY(hipSetDevice(dev));
    h->downloaded = std::move(X);
  }
  std::string err;
  const int rc = rsr::decode_block(*h->downloaded, part, block, sigma, L, &err);
  if (rc != 0) return fail(rc, "rsr_export_block: " + err);
  return RSR_OK;
}

rsr_host_index* rsr_host_pack(const int8_t* A, int64_t rows, int64_t cols, int k) {
  g_error.clear();
  std::unique_ptr<rsr_host_index> x(new (std::nothrow) rsr_host_index());
  if (!x) { fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory"); return nullptr; }
  std::string err;
  int rc;
  try {
    rc = rsr::pack_tiles(A, rows, cols, k, 0, &x->X, &err);
  } catch (const std::bad_alloc&) {
    fail(RSR_ERR_OUT_OF_MEMORY, "out of host memory while packing");
    return nullptr;
  }
  if (rc != 0) { fail(rc, "rsr_host_pack: " + err); return nullptr; }
  x->magic = kHostMagic;
  return x.release();
}

void rsr_host_free(rsr_host_index* x) {
  if (!valid(x)) return;
  x->magic = 0;
  delete x;
}

int rsr_host_info(const rsr_host_index* x, rsr_info_t* info) {
  if (!valid(x) || !info) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid host index or null info");
  fill_info(x->X, info);
  return RSR_OK;
}

int rsr_host_export_block(const rsr_host_index* x, int part, int64_t block, int32_t* sigma, int32_t* L) {
  if (!valid(x)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid host index");
  std::string err;
  const int rc = rsr::decode_block(x->X, part, block, sigma, L, &err);
  if (rc != 0) return fail(rc, "rsr_host_export_block: " + err);
  return RSR_OK;
}

int rsr_host_streams(const rsr_host_index* x, int tile, const uint16_t** stream, int64_t* n_stream, const void** units,
                     int64_t* n_units, const uint32_t** blk_unit, int64_t* tile_row0, int64_t* tile_rows) {
  if (!valid(x)) return fail(RSR_ERR_INVALID_ARGUMENT, "invalid host index");
  if (tile < 0 || tile >= (int)x->X.tiles.size()) return fail(RSR_ERR_INVALID_ARGUMENT, "row tile out of range");
  const rsr::Packed& P = x->X.tiles[(size_t)tile];
  if (stream) *stream = P.stream.data();
  if (n_stream) *n_stream = (int64_t)P.stream.size();
  if (units) *units = P.units.data();
  if (n_units) *n_units = (int64_t)P.units.size();
  if (blk_unit) *blk_unit = P.blk_unit.data();
  if (tile_row0) *tile_row0 = x->X.row0[(size_t)tile];
  if (tile_rows) *tile_rows = P.rows;
  return RSR_OK;
}

}  // extern "C"
