// Host side of rsr_preprocess: Algorithm 1 (Section 3.4) and the device packing.
#include "rsr_pack.h"

#include <algorithm>
#include <atomic>
#include <cstring>
#include <thread>

namespace rsr {
namespace {

struct BlockOut {
  std::vector<uint16_t> stream;
  std::vector<Unit> units;
  int64_t stored_rows = 0, heads = 0, flag_bytes = 0;
};

struct Scratch {
  std::vector<uint16_t> val[2];     // value of every row, per part
  std::vector<uint32_t> off;        // 2^k + 1 exclusive prefix counts (the full segmentation)
  std::vector<uint32_t> pos;
  std::vector<uint16_t> sigma;      // sorted rows (Definition 3.2, equal rows in ascending order)
  std::vector<uint16_t> entry;      // a window's entries: rows in sorted order, nulls for absent values
  std::vector<uint8_t> flag;        // 1 = the entry's value is the previous entry's plus one
  std::vector<uint16_t> slot;       // the entry's window slot (kept for cutting units)
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- LDS banks ----
// A gather instruction reads one activation per lane.  The LDS has 32 banks of 4 bytes and serves
// the two halves of a wavefront (lanes 0..31, 32..63) one after the other; a half costs as many
// cycles as its fullest bank has distinct addresses (measured on gfx950 with a stride sweep: 64 lanes
// at stride 1, 2, 4, 8 words take 2.4, 4.1, 8.1, 16.1 cycles; two lanes of the same half on one bank
// cost one cycle more, two lanes of different halves do not).  The bank of a float activation is
// its row number modulo 32.  The order of the rows inside a segment is free (a segment is a sum), so
// within every run of a lane that belongs to one segment the rows are dealt out position by position
// in such a way that the lanes of a half meet in few banks: at each position the lanes with the
// fewest rows left to choose from pick first, and each picks, among the rows its run still holds,
// the one whose bank has been picked least at that position.
constexpr int kBanks = 32;
constexpr int kHalf = 32;
constexpr int kImprovePasses = 4;

void spread_over_banks(uint16_t (*ent)[kMaxPositions], const uint8_t (*flg)[kMaxPositions], int npos, uint16_t null_index) {
  for (int h = 0; h < kLanes / kHalf; ++h) {
    int run_end[kHalf];  // end (exclusive) of the run that covers the current position, per lane
    for (int l = 0; l < kHalf; ++l) run_end[l] = 0;
    for (int p = 0; p < npos; ++p) {
      int order[kHalf], left[kHalf];
      for (int l = 0; l < kHalf; ++l) {
        const int L = h * kHalf + l;
        if (run_end[l] <= p) {  // a new run starts here: up to the next flag
          int q = p + 1;
          while (q < npos && !flg[L][q]) ++q;
          run_end[l] = q;
        }
        left[l] = run_end[l] - p;
        order[l] = l;
      }
      std::stable_sort(order, order + kHalf, [&](int x, int y) { return left[x] < left[y]; });
      int load[kBanks] = {0};
      for (int o = 0; o < kHalf; ++o) {
        const int l = order[o], L = h * kHalf + l;
        int best = p;
        for (int q = p; q < run_end[l]; ++q) {
          if (ent[L][q] == null_index) continue;  // a null entry reads one shared word: it is placed last
          if (ent[L][best] == null_index || load[ent[L][q] % kBanks] < load[ent[L][best] % kBanks]) best = q;
        }
        std::swap(ent[L][p], ent[L][best]);
        if (ent[L][p] != null_index) ++load[ent[L][p] % kBanks];
      }
    }
    // Then a few passes of local improvement: two rows of one run trade places when that lowers the sum of
    // the squared bank loads of their two positions (a cheap stand-in for the depth of the fullest bank).
    static thread_local uint8_t bank_load[kMaxPositions][kBanks];
    for (int p = 0; p < npos; ++p) {
      for (int b = 0; b < kBanks; ++b) bank_load[p][b] = 0;
      for (int l = 0; l < kHalf; ++l)
        if (ent[h * kHalf + l][p] != null_index) ++bank_load[p][ent[h * kHalf + l][p] % kBanks];
    }
    for (int pass = 0; pass < kImprovePasses; ++pass) {
      bool changed = false;
      for (int l = 0; l < kHalf; ++l) {
        const int L = h * kHalf + l;
        int p0 = 0;
        while (p0 < npos) {
          int p1 = p0 + 1;
          while (p1 < npos && !flg[L][p1]) ++p1;  // the run [p0, p1)
          for (int p = p0; p < p1; ++p)
            for (int q = p + 1; q < p1; ++q) {
              const uint16_t rp = ent[L][p], rq = ent[L][q];
              if (rp == null_index || rq == null_index) continue;
              const int bp = rp % kBanks, bq = rq % kBanks;
              if (bp == bq) continue;
              const int delta = ((int)bank_load[p][bq] - (int)bank_load[p][bp] + 1) + ((int)bank_load[q][bp] - (int)bank_load[q][bq] + 1);
              if (delta < 0) {
                --bank_load[p][bp]; ++bank_load[p][bq]; --bank_load[q][bq]; ++bank_load[q][bp];
                std::swap(ent[L][p], ent[L][q]);
                changed = true;
              }
            }
          p0 = p1;
        }
      }
      if (!changed) break;
    }
  }
}

// One unit: entries e[0 .. n) with their flags, the first one in window slot `slot0`.
void emit_unit(const uint16_t* e, const uint8_t* f, int n, int slot0, uint32_t block, uint32_t window, int part,
               uint16_t null_index, BlockOut* out) {
  const int npos = ceil_div(n, kLanes);
  Unit u;
  std::memset(&u, 0, sizeof(u));
  u.stream_off = (uint32_t)(out->stream.size() * sizeof(uint16_t) / kStreamAlign);
  u.block = block;
  u.window = (uint16_t)window;
  u.part = (uint8_t)part;
  u.npos = (uint8_t)npos;
  u.slot0 = (uint16_t)slot0;
  u.nentries = (uint32_t)n;
  if (npos > 0) {
    // entry of lane l at position p (the first entry's flag is dropped: its slot is slot0)
    uint16_t ent[kLanes][kMaxPositions];
    uint8_t flg[kLanes][kMaxPositions];
    for (int l = 0; l < kLanes; ++l)
      for (int p = 0; p < npos; ++p) {
        const int i = l * npos + p;
        ent[l][p] = i < n ? e[i] : null_index;
        flg[l][p] = (i > 0 && i < n) ? f[i] : 0;
      }
    spread_over_banks(ent, flg, npos, null_index);
    auto at = [&](int l, int p) { return ent[l][p]; };
    auto flag_at = [&](int l, int p) { return (int)flg[l][p]; };
    const int full = npos / kGranulePositions;
    for (int g = 0; g < full; ++g)
      for (int l = 0; l < kLanes; ++l)
        for (int q = 0; q < kGranulePositions; ++q) out->stream.push_back(at(l, g * kGranulePositions + q));
    for (int p = full * kGranulePositions; p + 1 < npos; p += 2)
      for (int l = 0; l < kLanes; ++l) {
        out->stream.push_back(at(l, p));
        out->stream.push_back(at(l, p + 1));
      }
    if (npos & 1)
      for (int l = 0; l < kLanes; ++l) out->stream.push_back(at(l, npos - 1));
    for (int l = 0; l < kLanes; ++l) {
      uint32_t w = 0;
      for (int p = 0; p < npos && p < 32; ++p) w |= (uint32_t)flag_at(l, p) << (31 - p);
      out->stream.push_back((uint16_t)(w & 0xffffu));
      out->stream.push_back((uint16_t)(w >> 16));
    }
    out->flag_bytes += kFlagBytes0;
    if (npos > 32) {
      for (int l = 0; l < kLanes; ++l) {
        uint32_t w = 0;
        for (int p = 32; p < npos; ++p) w |= (uint32_t)flag_at(l, p) << (47 - p);
        out->stream.push_back((uint16_t)w);
      }
      out->flag_bytes += kFlagBytes1;
    }
    while (out->stream.size() * sizeof(uint16_t) % kStreamAlign) out->stream.push_back(0);
    for (int i = 0; i < n; ++i) {
      u.nrows += (e[i] != null_index);
      u.nheads += (i > 0 && f[i]);
    }
    out->heads += u.nheads + 1;
  }
  out->stored_rows += u.nrows;
  out->units.push_back(u);
}

// All windows of one (block, part): sort the rows by value, list each window's rows in sorted
// order (one null entry for every absent value between two present ones), cut the list into
// units of at most kMaxUnitEntries entries.
void pack_part(int64_t rows, int k, int kw, uint32_t block, int part, Scratch* S, BlockOut* out) {
  const uint32_t nvals = 1u << k;
  const uint32_t W = 1u << kw;
  const uint16_t null_index = (uint16_t)rows;
  const std::vector<uint16_t>& val = S->val[part];
  // counting sort of the rows by value (Definition 3.2; "bucket sort" in the proof of Theorem 3.6)
  S->off.assign((size_t)nvals + 1, 0);
  for (int64_t r = 0; r < rows; ++r) ++S->off[(size_t)val[r] + 1];
  for (uint32_t j = 0; j < nvals; ++j) S->off[j + 1] += S->off[j];
  S->pos.assign(S->off.begin(), S->off.end() - 1);
  S->sigma.resize((size_t)rows);
  for (int64_t r = 0; r < rows; ++r) S->sigma[S->pos[val[r]]++] = (uint16_t)r;

  const uint32_t nwin = nvals >> kw;
  for (uint32_t w = 0; w < nwin; ++w) {
    const uint32_t j0 = w * W;
    const uint32_t jfirst = (w == 0 ? 1 : 0);  // value 0 contributes nothing
    if (S->off[j0 + W] == S->off[j0 + jfirst]) continue;
    S->entry.clear(); S->flag.clear(); S->slot.clear();
    for (uint32_t jl = jfirst; jl < W; ++jl) {
      const uint32_t b = S->off[j0 + jl], e = S->off[j0 + jl + 1];
      if (b == e) {
        if (S->entry.empty()) continue;  // nothing before it: the unit starts at the first present value
        S->entry.push_back(null_index); S->flag.push_back(1); S->slot.push_back((uint16_t)jl);
        continue;
      }
      for (uint32_t p = b; p < e; ++p) {
        S->entry.push_back(S->sigma[p]);
        S->flag.push_back(p == b);
        S->slot.push_back((uint16_t)jl);
      }
    }
    // the nulls behind the last present value are of no use
    while (!S->entry.empty() && S->entry.back() == null_index) { S->entry.pop_back(); S->flag.pop_back(); S->slot.pop_back(); }
    // units of equal size; a unit neither starts nor ends with a null entry
    const int total = (int)S->entry.size();
    const int nunits = ceil_div(total, kMaxUnitEntries);
    for (int ui = 0; ui < nunits; ++ui) {
      int b = (int)((int64_t)total * ui / nunits), e = (int)((int64_t)total * (ui + 1) / nunits);
      while (b < e && S->entry[(size_t)b] == null_index) ++b;
      while (e > b && S->entry[(size_t)e - 1] == null_index) --e;
      if (b == e) continue;
      emit_unit(&S->entry[(size_t)b], &S->flag[(size_t)b], e - b, S->slot[(size_t)b], block, w, part, null_index, out);
    }
  }
}

constexpr int kGroup = 8;  // column blocks whose row values are extracted in one pass over A

// Definition 3.2 for kGroup consecutive blocks at once: the row's bits, first column most
// significant.  One pass over the rows reads each cache line of A once for the whole group.
void extract_values(const int8_t* A, int64_t rows, int64_t cols, int k, int parts, int64_t block0, int nb,
                    std::vector<uint16_t> (*val)[2]) {
  int width[kGroup], shift[kGroup];
  for (int g = 0; g < nb; ++g) {
    width[g] = (int)std::min<int64_t>(k, cols - (block0 + g) * k);
    shift[g] = k - width[g];
    for (int p = 0; p < parts; ++p) val[g][p].resize((size_t)rows);
  }
  const int64_t c0 = block0 * k;
  for (int64_t r = 0; r < rows; ++r) {
    const int8_t* a = A + r * cols + c0;
    for (int g = 0; g < nb; ++g) {
      uint32_t plus = 0, minus = 0;
      for (int c = 0; c < width[g]; ++c) {
        const int x = a[c];
        plus = (plus << 1) | (uint32_t)(x == 1);
        minus = (minus << 1) | (uint32_t)(x == -1);
      }
      a += width[g];
      val[g][0][(size_t)r] = (uint16_t)(plus << shift[g]);
      if (parts == 2) val[g][1][(size_t)r] = (uint16_t)(minus << shift[g]);
    }
  }
}

void pack_block(int64_t rows, int k, int kw, int parts, int64_t block, Scratch* S, BlockOut* out) {
  for (int p = 0; p < parts; ++p) pack_part(rows, k, kw, (uint32_t)block, p, S, out);
  if (out->units.empty())  // an all-zero block still has to write its outputs: a unit without positions
    emit_unit(nullptr, nullptr, 0, 0, (uint32_t)block, 0, 0, (uint16_t)rows, out);
}

}  // namespace

int pack_matrix(const int8_t* A, int64_t rows, int64_t cols, int k, int threads, int force_parts, Packed* out, std::string* err) {
  if (!A || !out) { *err = "null pointer"; return -1; }
  if (rows < 1 || rows > kMaxRows) { *err = "rows must be in 1..65534"; return -1; }
  if (cols < 1) { *err = "cols must be >= 1"; return -1; }
  if (k < 1 || k > kMaxK) { *err = "k must be in 1..16"; return -1; }
  const int64_t nblocks = (cols + k - 1) / k;
  if (nblocks > (int64_t)0x7fffffff) { *err = "too many column blocks"; return -1; }
  if (threads <= 0) {
    threads = (int)std::thread::hardware_concurrency();
    if (threads < 1) threads = 1;
    if (threads > 16) threads = 16;
  }
  if ((int64_t)threads > (nblocks + kGroup - 1) / kGroup) threads = (int)((nblocks + kGroup - 1) / kGroup);

  // entries must be in {-1,0,1}; any -1 makes the matrix ternary (Proposition 2.1)
  std::atomic<int64_t> bad(-1);
  std::atomic<int> any_minus(0);
  {
    const int64_t total = rows * cols;
    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t) {
      pool.emplace_back([&, t]() {
        const int64_t b = total * t / threads, e = total * (t + 1) / threads;
        int minus = 0;
        for (int64_t i = b; i < e; ++i) {
          const int x = A[i];
          if (x < -1 || x > 1) {
            int64_t expect = -1;
            bad.compare_exchange_strong(expect, i);
            return;
          }
          minus |= (x < 0);
        }
        if (minus) any_minus.store(1);
      });
    }
    for (auto& th : pool) th.join();
  }
  if (bad.load() >= 0) {
    const int64_t i = bad.load();
    *err = "entry outside {-1,0,1} at row " + std::to_string(i / cols) + ", column " + std::to_string(i % cols);
    return -1;
  }
  const int parts = force_parts ? force_parts : (any_minus.load() ? 2 : 1);
  const int kw = std::min(k, kMaxWindowBits);

  std::vector<BlockOut> blocks((size_t)nblocks);
  std::atomic<int> failed(0);
  {
    std::atomic<int64_t> next(0);
    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t) {
      pool.emplace_back([&]() {
        try {
          Scratch S;
          std::vector<uint16_t> val[kGroup][2];
          for (;;) {
            const int64_t b0 = next.fetch_add(kGroup);
            if (b0 >= nblocks || failed.load()) break;
            const int nb = (int)std::min<int64_t>(kGroup, nblocks - b0);
            extract_values(A, rows, cols, k, parts, b0, nb, val);
            for (int g = 0; g < nb; ++g) {
              for (int p = 0; p < parts; ++p) S.val[p].swap(val[g][p]);
              pack_block(rows, k, kw, parts, b0 + g, &S, &blocks[(size_t)(b0 + g)]);
              for (int p = 0; p < parts; ++p) S.val[p].swap(val[g][p]);
            }
          }
        } catch (...) {
          failed.store(1);
        }
      });
    }
    for (auto& th : pool) th.join();
  }
  if (failed.load()) { *err = "out of host memory while packing"; return -4; }

  Packed& P = *out;
  P = Packed();
  P.rows = rows; P.cols = cols; P.k = k; P.kw = kw; P.parts = parts; P.nblocks = nblocks;
  P.last_width = (int)(cols - (nblocks - 1) * k);
  size_t ne = 0, nu = 0;
  for (const BlockOut& b : blocks) { ne += b.stream.size(); nu += b.units.size(); }
  if (ne * sizeof(uint16_t) / kStreamAlign > 0xffffffffull || nu > 0xffffffffull) { *err = "index too large"; return -2; }
  try {
    P.stream.resize(ne); P.units.resize(nu); P.blk_unit.resize((size_t)nblocks + 1);
  } catch (...) { *err = "out of host memory while packing"; return -4; }
  size_t pe = 0, pu = 0;
  for (int64_t b = 0; b < nblocks; ++b) {
    BlockOut& B = blocks[(size_t)b];
    P.blk_unit[(size_t)b] = (uint32_t)pu;
    if (!B.stream.empty()) std::memcpy(&P.stream[pe], B.stream.data(), B.stream.size() * sizeof(uint16_t));
    if (B.units.size() > 0xffffu) { *err = "too many work units in one column block"; return -2; }
    for (size_t i = 0; i < B.units.size(); ++i) {
      Unit u = B.units[i];
      u.stream_off += (uint32_t)(pe * sizeof(uint16_t) / kStreamAlign);
      u.units_in_block = (uint16_t)B.units.size();
      u.index_in_block = (uint16_t)i;
      P.units[pu + i] = u;
    }
    P.max_units_per_block = std::max<uint32_t>(P.max_units_per_block, (uint32_t)B.units.size());
    P.stored_rows += B.stored_rows;
    P.segments += B.heads;
    P.flag_bytes += B.flag_bytes;
    pe += B.stream.size(); pu += B.units.size();
    std::vector<uint16_t>().swap(B.stream);
  }
  P.blk_unit[(size_t)nblocks] = (uint32_t)pu;
  return 0;
}

// Position p, lane l of a unit's stream.
static inline uint16_t stream_at(const uint16_t* us, int npos, int p, int l) {
  const int full = npos / kGranulePositions;
  if (p < full * kGranulePositions)
    return us[((size_t)(p / kGranulePositions) * kLanes + l) * kGranulePositions + p % kGranulePositions];
  const int q = p - full * kGranulePositions;
  const uint16_t* rest = us + (size_t)full * kGranulePositions * kLanes;
  if ((npos & 1) && p == npos - 1) return rest[(size_t)(q / 2) * 2 * kLanes + l];  // the last, single row
  return rest[((size_t)(q / 2) * kLanes + l) * 2 + (q & 1)];
}

static inline int flag_at(const uint16_t* us, int npos, int p, int l) {
  const uint16_t* f0 = us + (size_t)npos * kLanes;
  if (p < 32) {
    const uint32_t w = (uint32_t)f0[2 * l] | ((uint32_t)f0[2 * l + 1] << 16);
    return (int)((w >> (31 - p)) & 1u);
  }
  const uint16_t* f1 = f0 + 2 * kLanes;
  return (int)((f1[l] >> (47 - p)) & 1u);
}

int pack_tiles(const int8_t* A, int64_t rows, int64_t cols, int k, int threads, Index* out, std::string* err) {
  if (!A || !out) { *err = "null pointer"; return -1; }
  if (rows < 1 || rows > kMaxRows) { *err = "rows must be in 1..65534"; return -1; }
  if (cols < 1) { *err = "cols must be >= 1"; return -1; }
  out->rows = rows; out->cols = cols;
  out->tiles.clear(); out->row0.clear();
  const int64_t ntiles = (rows + kTileRows - 1) / kTileRows;
  // equal heights, multiples of 16 rows (a tile's share of an activation vector stays 16-byte aligned)
  const int64_t height = ((rows + ntiles - 1) / ntiles + 15) / 16 * 16;
  int parts = 0;
  if (ntiles > 1) {  // the kind is a property of the whole matrix
    parts = 1;
    for (int64_t i = 0; i < rows * cols; ++i)
      if (A[i] < 0) { parts = 2; break; }
  }
  for (int64_t t = 0; t < ntiles; ++t) {
    const int64_t r0 = t * height, r1 = std::min(rows, r0 + height);
    out->tiles.emplace_back();
    out->row0.push_back(r0);
    const int rc = pack_matrix(A + r0 * cols, r1 - r0, cols, k, threads, parts, &out->tiles.back(), err);
    if (rc != 0) {
      // (positions in the message count from the tile's first row)
      if (ntiles > 1) *err += " (rows counted from row " + std::to_string(r0) + ")";
      return rc;
    }
  }
  return 0;
}

int decode_block(const Index& X, int part, int64_t block, int32_t* sigma, int32_t* L, std::string* err) {
  const Packed& P0 = X.tiles[0];
  if (part < 0 || part >= P0.parts) { *err = "part out of range"; return -1; }
  if (block < 0 || block >= P0.nblocks) { *err = "block out of range"; return -1; }
  const int width = (block == P0.nblocks - 1) ? P0.last_width : P0.k;
  const int shift = P0.k - width;
  const uint32_t nvals = 1u << width;
  std::vector<std::vector<int32_t>> by_value(nvals);
  std::vector<uint8_t> listed((size_t)X.rows, 0);
  for (size_t t = 0; t < X.tiles.size(); ++t) {
    const Packed& P = X.tiles[t];
    const int64_t r0 = X.row0[t];
    const uint16_t null_index = (uint16_t)P.rows;
    for (uint32_t ui = P.blk_unit[(size_t)block]; ui < P.blk_unit[(size_t)block + 1]; ++ui) {
      const Unit& u = P.units[ui];
      if (u.part != part) continue;
      if (u.npos > kMaxPositions) { *err = "corrupt unit: position count"; return -1; }
      const uint16_t* us = &P.stream[(size_t)u.stream_off * (kStreamAlign / sizeof(uint16_t))];
      uint32_t sl = u.slot0;
      for (int l = 0; l < kLanes; ++l)
        for (int p = 0; p < u.npos; ++p) {
          sl += (uint32_t)flag_at(us, u.npos, p, l);
          const uint16_t row = stream_at(us, u.npos, p, l);
          if (row == null_index) continue;
          if (row > null_index) { *err = "corrupt unit: row index out of range"; return -1; }
          if (sl >= (1u << P.kw)) { *err = "corrupt unit: slot outside the window"; return -1; }
          const uint32_t value = (((uint32_t)u.window << P.kw) + sl) >> shift;
          if (value >= nvals || value == 0 || listed[(size_t)(r0 + row)]) { *err = "corrupt unit: bad value or repeated row"; return -1; }
          listed[(size_t)(r0 + row)] = 1;
          by_value[value].push_back((int32_t)(r0 + row));
        }
    }
  }
  for (int64_t r = 0; r < X.rows; ++r)
    if (!listed[(size_t)r]) by_value[0].push_back((int32_t)r);  // the rows that were left out have value 0
  int64_t p = 0;
  for (uint32_t j = 0; j < nvals; ++j) {
    if (L) L[j] = (int32_t)p;
    std::sort(by_value[j].begin(), by_value[j].end());
    for (int32_t r : by_value[j]) {
      if (sigma) sigma[p] = r;
      ++p;
    }
  }
  if (L) L[nvals] = (int32_t)p;
  return 0;
}

}  // namespace rsr
