// Host side of rsr_preprocess: Algorithm 1 (Section 3.4) and the device packing.
#include "rsr_pack.h"

#include <algorithm>
#include <atomic>
#include <cstring>
#include <thread>

namespace rsr {
namespace {

struct Piece {
  uint32_t start;   // first sorted position of the piece inside the block's permutation
  uint16_t len;     // rows in the piece, 1 .. kMaxDiag
  uint16_t slot;    // value of the segment inside its window (0 .. 2^kw - 1)
};

struct BlockOut {
  std::vector<uint16_t> entries, slots;
  std::vector<Unit> units;
  int64_t stored_rows = 0, segments = 0;
};

struct Scratch {
  std::vector<uint16_t> val[2];     // value of every row, per part
  std::vector<uint32_t> off;        // 2^k + 1 exclusive prefix counts (the full segmentation)
  std::vector<uint32_t> pos;
  std::vector<uint16_t> sigma;      // sorted rows (Definition 3.2, equal rows in ascending order)
  std::vector<Piece> pieces, sorted, leftover, unit_pieces;
  std::vector<uint16_t> unit_slot, parents;
  std::vector<uint8_t> seen;
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// One unit: up to 512 pieces (already sorted by descending length) of one window.
void emit_unit(const std::vector<Piece>& pcs, const std::vector<uint16_t>& slot_ids,
               const std::vector<uint16_t>& parents, const std::vector<uint16_t>& sigma, uint32_t block,
               uint32_t window, int part, uint16_t null_index, BlockOut* out) {
  Unit u;
  std::memset(&u, 0, sizeof(u));
  const int np = (int)pcs.size();
  const int nt = np ? pcs[0].len : 0;
  u.entry_off = (uint32_t)(out->entries.size() / kPerLane);
  u.slot_off = (uint32_t)(out->slots.size() / kPerLane);
  u.block = block;
  u.window = (uint16_t)window;
  u.npieces = (uint16_t)np;
  u.nt = (uint8_t)nt;
  u.part = (uint8_t)part;
  u.nov = (uint8_t)parents.size();
  int cnt = np;
  int nt_main = nt;
  int granules = 0;
  for (int t = 0; t < nt; ++t) {
    while (cnt > 0 && pcs[cnt - 1].len <= t) --cnt;
    if (nt_main == nt && cnt <= kTailRanks) nt_main = t;  // from here on one entry per lane suffices
    if (t < nt_main) {
      const int c8 = ceil_div(cnt, kPerLane);
      u.cnt8[t] = (uint8_t)c8;
      granules += c8;
      for (int q = 0; q < c8 * kPerLane; ++q)
        out->entries.push_back(q < cnt ? sigma[pcs[q].start + t] : null_index);
    } else {
      u.cnt8[t] = (uint8_t)cnt;
      for (int q = 0; q < cnt; ++q) out->entries.push_back(sigma[pcs[q].start + t]);
    }
    out->stored_rows += cnt;
  }
  while (out->entries.size() % kPerLane) out->entries.push_back(null_index);
  u.nt_main = (uint8_t)nt_main;
  u.main_granules = (uint16_t)granules;
  const int ns = ceil_div(np, kPerLane) * kPerLane;
  for (int q = 0; q < ns; ++q) out->slots.push_back(q < np ? slot_ids[q] : (uint16_t)kWindow);
  const int nov = (int)parents.size();
  const int npar = ceil_div(nov, kPerLane) * kPerLane;
  for (int o = 0; o < npar; ++o) out->slots.push_back(o < nov ? parents[o] : (uint16_t)0);
  out->segments += np;
  out->units.push_back(u);
}

// All windows of one (block, part): cut segments into pieces, rank by length, emit units.
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
    if (S->off[j0 + W] == S->off[j0 + (w == 0 ? 1 : 0)]) continue;  // nothing but value 0 here
    S->pieces.clear();
    for (uint32_t jl = (w == 0 ? 1 : 0); jl < W; ++jl) {  // value 0 contributes nothing
      const uint32_t j = j0 + jl;
      const uint32_t c = S->off[j + 1] - S->off[j];
      if (c == 0) continue;
      if (c <= (uint32_t)kMaxDiag) {
        S->pieces.push_back(Piece{S->off[j], (uint16_t)c, (uint16_t)jl});
      } else {
        const uint32_t m = (c + kMaxDiag - 1) / kMaxDiag, base = c / m, rem = c % m;
        uint32_t s = S->off[j];
        for (uint32_t i = 0; i < m; ++i) {
          const uint32_t len = base + (i < rem ? 1 : 0);
          S->pieces.push_back(Piece{s, (uint16_t)len, (uint16_t)jl});
          s += len;
        }
      }
    }
    // stable counting sort by descending length
    uint32_t bucket[kMaxDiag + 2] = {0};
    for (const Piece& p : S->pieces) ++bucket[kMaxDiag - p.len + 1];
    for (int i = 0; i <= kMaxDiag; ++i) bucket[i + 1] += bucket[i];
    S->sorted.resize(S->pieces.size());
    for (const Piece& p : S->pieces) S->sorted[bucket[kMaxDiag - p.len]++] = p;

    // fill units; a second piece of a value inside one unit takes an overflow slot
    std::vector<Piece>* cur = &S->sorted;
    while (!cur->empty()) {
      S->unit_pieces.clear();
      S->unit_slot.clear();
      S->parents.clear();
      S->leftover.clear();
      S->seen.assign(W, 0);
      for (const Piece& p : *cur) {
        if ((int)S->unit_pieces.size() >= kTileRanks) { S->leftover.push_back(p); continue; }
        if (!S->seen[p.slot]) {
          S->seen[p.slot] = 1;
          S->unit_pieces.push_back(p);
          S->unit_slot.push_back(p.slot);
        } else if ((int)S->parents.size() < kMaxOverflow) {
          S->unit_pieces.push_back(p);
          S->unit_slot.push_back((uint16_t)(kOverflowBase + S->parents.size()));
          S->parents.push_back(p.slot);
        } else {
          S->leftover.push_back(p);
        }
      }
      emit_unit(S->unit_pieces, S->unit_slot, S->parents, S->sigma, block, w, part, null_index, out);
      S->sorted.swap(S->leftover);  // leftover keeps the descending order
      cur = &S->sorted;
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
  if (out->units.empty()) {  // an all-zero block still has to write its outputs
    const std::vector<Piece> none;
    const std::vector<uint16_t> no_ids;
    emit_unit(none, no_ids, no_ids, S->sigma, (uint32_t)block, 0, 0, (uint16_t)rows, out);
  }
}

}  // namespace

int pack_matrix(const int8_t* A, int64_t rows, int64_t cols, int k, int threads, Packed* out, std::string* err) {
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
  const int parts = any_minus.load() ? 2 : 1;
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
  size_t ne = 0, ns = 0, nu = 0;
  for (const BlockOut& b : blocks) { ne += b.entries.size(); ns += b.slots.size(); nu += b.units.size(); }
  if (ne / kPerLane > 0xffffffffull || nu > 0xffffffffull) { *err = "index too large"; return -2; }
  try {
    P.entries.resize(ne); P.slots.resize(ns); P.units.resize(nu); P.blk_unit.resize((size_t)nblocks + 1);
  } catch (...) { *err = "out of host memory while packing"; return -4; }
  size_t pe = 0, ps = 0, pu = 0;
  for (int64_t b = 0; b < nblocks; ++b) {
    BlockOut& B = blocks[(size_t)b];
    P.blk_unit[(size_t)b] = (uint32_t)pu;
    if (!B.entries.empty()) std::memcpy(&P.entries[pe], B.entries.data(), B.entries.size() * sizeof(uint16_t));
    if (!B.slots.empty()) std::memcpy(&P.slots[ps], B.slots.data(), B.slots.size() * sizeof(uint16_t));
    for (size_t i = 0; i < B.units.size(); ++i) {
      Unit u = B.units[i];
      u.entry_off += (uint32_t)(pe / kPerLane);
      u.slot_off += (uint32_t)(ps / kPerLane);
      u.units_in_block = (uint16_t)B.units.size();
      P.units[pu + i] = u;
    }
    if (B.units.size() > 0xffffu) { *err = "too many work units in one column block"; return -2; }
    P.max_units_per_block = std::max<uint32_t>(P.max_units_per_block, (uint32_t)B.units.size());
    P.stored_rows += B.stored_rows;
    P.segments += B.segments;
    pe += B.entries.size(); ps += B.slots.size(); pu += B.units.size();
    BlockOut().entries.swap(B.entries);
    BlockOut().slots.swap(B.slots);
  }
  P.blk_unit[(size_t)nblocks] = (uint32_t)pu;
  return 0;
}

int decode_block(const Packed& P, int part, int64_t block, int32_t* sigma, int32_t* L, std::string* err) {
  if (part < 0 || part >= P.parts) { *err = "part out of range"; return -1; }
  if (block < 0 || block >= P.nblocks) { *err = "block out of range"; return -1; }
  const int width = (block == P.nblocks - 1) ? P.last_width : P.k;
  const int shift = P.k - width;
  const uint32_t nvals = 1u << width;
  const uint16_t null_index = (uint16_t)P.rows;
  std::vector<std::vector<int32_t>> by_value(nvals);
  std::vector<uint8_t> listed((size_t)P.rows, 0);
  for (uint32_t ui = P.blk_unit[(size_t)block]; ui < P.blk_unit[(size_t)block + 1]; ++ui) {
    const Unit& u = P.units[ui];
    if (u.part != part) continue;
    const uint16_t* e = &P.entries[(size_t)u.entry_off * kPerLane];
    const uint16_t* s = &P.slots[(size_t)u.slot_off * kPerLane];
    const int ns = ceil_div(u.npieces, kPerLane) * kPerLane;
    for (int t = 0; t < u.nt; ++t) {
      const int n = (t < u.nt_main) ? u.cnt8[t] * kPerLane : u.cnt8[t];
      for (int q = 0; q < n; ++q) {
        const uint16_t row = e[q];
        if (row == null_index) continue;
        if (q >= u.npieces || row > null_index) { *err = "corrupt unit: entry beyond its pieces"; return -1; }
        uint32_t slot = s[q];
        if (slot >= (uint32_t)kOverflowBase) {
          const uint32_t o = slot - kOverflowBase;
          if (o >= u.nov) { *err = "corrupt unit: overflow slot out of range"; return -1; }
          slot = s[ns + o];
        }
        if (slot >= (uint32_t)kWindow) { *err = "corrupt unit: row in a dummy slot"; return -1; }
        const uint32_t value = (((uint32_t)u.window << P.kw) + slot) >> shift;
        if (value >= nvals || value == 0 || listed[row]) { *err = "corrupt unit: bad value or repeated row"; return -1; }
        listed[row] = 1;
        by_value[value].push_back((int32_t)row);
      }
      e += n;
    }
  }
  for (int64_t r = 0; r < P.rows; ++r)
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
