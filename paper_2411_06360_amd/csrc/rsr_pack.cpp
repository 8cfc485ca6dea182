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
  uint16_t len;     // rows, 1 .. kMaxPieceRows
  uint16_t slot;    // value of the segment inside its window (0 .. 2^kw - 1)
};

struct BlockOut {
  std::vector<uint16_t> stream;
  std::vector<Unit> units;
  int64_t stored_rows = 0, segments = 0, header_positions = 0;
};

// Cost of a work unit beyond its positions (descriptor, window clearing, fold), in positions.
constexpr int kUnitCost = 3;

struct Scratch {
  std::vector<uint16_t> val[2];     // value of every row, per part
  std::vector<uint32_t> off;        // 2^k + 1 exclusive prefix counts (the full segmentation)
  std::vector<uint32_t> pos;
  std::vector<uint16_t> sigma;      // sorted rows (Definition 3.2, equal rows in ascending order)
  std::vector<Piece> pieces, sorted;
  std::vector<uint16_t> unit_slot, parents, positions;
  std::vector<uint8_t> seen;
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Longest piece: its group (header + rows) and all parent positions have to fit into one unit.
constexpr int kMaxPieceRows = kMaxPositions - 1 - kMaxOverflow / kLanes;

// ---- LDS banks ----
// A gather instruction reads one activation per lane; the LDS serves the 32 lanes of a half
// wavefront together and takes one pass per distinct address in the fullest bank (bank of a
// float activation = row mod 32).  Two things are free in the layout and are used to bring every
// position as close to one pass as possible:
//   * which pieces share a half wavefront: pieces of equal length may trade places anywhere in
//     the unit, any two pieces may trade places inside their group.  A randomised search moves
//     pieces until no bank has more rows in a half group than the group has positions (or the
//     iteration budget is spent);
//   * at which of the group's positions a lane reads which of its rows (a piece is a sum).  This is
//     an edge colouring of the bipartite multigraph lanes x banks (an edge per row, a colour per
//     position): with at most n rows per lane and per bank, n colours suffice (Koenig), i.e. every
//     position is conflict-free.  Rows of a bank beyond n are placed afterwards where they cost
//     the fewest extra passes.
constexpr int kBanks = 32;
constexpr int kHalf = 32;

struct HalfGroup {
  int n = 0;                 // positions of the group
  uint16_t deg[kBanks];      // rows per bank
};

inline int half_cost(const HalfGroup& h) {
  int mx = h.n, sq = 0;
  for (int b = 0; b < kBanks; ++b) {
    const int d = h.deg[b];
    if (d > mx) mx = d;
    const int e = d - h.n;
    if (e > 0) sq += 8 * e * e;
    if (e + 1 > 0) sq += (e + 1) * (e + 1);
  }
  return 1024 * mx + sq;
}

// Edge colouring of one half group.  row_of[l][0 .. len[l]) are the rows of lane l; on return
// place[l][t] is the row lane l reads at position t (or `null_index`).
//
// A bank with more than n rows cannot be conflict-free.  Its rows beyond the n-th go to a second
// (third, fourth) copy of the bank; the graph lanes x bank copies still has at most n edges per
// node, so it has a proper colouring, in which a position sees every copy at most once: a
// position costs as many passes as it uses copies of its fullest bank.  The rows of the extra
// copies are coloured first and take the lowest colour that is free, which gathers them in few
// positions.  (Rows beyond the fourth copy are placed afterwards wherever their lane is free.)
constexpr int kBankCopies = 4;

void colour_half(int n, const uint16_t (*row_of)[kMaxPieceRows], const int* len, uint16_t null_index,
                 uint16_t (*place)[kMaxPieceRows]) {
  constexpr int kNodes = kBanks * kBankCopies;
  int16_t at_lane[kHalf][kMaxPieceRows], at_bank[kNodes][kMaxPieceRows];  // edge at (node, colour) or -1
  for (int l = 0; l < kHalf; ++l)
    for (int c = 0; c < n; ++c) { at_lane[l][c] = -1; place[l][c] = null_index; }
  for (int v = 0; v < kNodes; ++v)
    for (int c = 0; c < n; ++c) at_bank[v][c] = -1;
  struct Edge { uint8_t lane, node; int8_t colour; uint16_t row; };
  Edge edges[kHalf * kMaxPieceRows];
  int ne = 0;
  int bank_count[kBanks] = {0};
  int16_t todo[kHalf * kMaxPieceRows];  // edges in the order they are coloured
  int n_extra = 0, n_todo = 0;
  int16_t late[kHalf * kMaxPieceRows];
  int n_late = 0;
  // Lanes with the most rows first: the rows that find their bank full, and go to its extra copies,
  // then belong to the lanes with the most room.
  int order[kHalf];
  for (int l = 0; l < kHalf; ++l) order[l] = l;
  std::stable_sort(order, order + kHalf, [&](int x, int y) { return len[x] > len[y]; });
  for (int o = 0; o < kHalf; ++o) {
    const int l = order[o];
    for (int t = 0; t < len[l]; ++t) {
      Edge& e = edges[ne];
      e.lane = (uint8_t)l; e.row = row_of[l][t]; e.colour = -1;
      const int bank = e.row & (kBanks - 1);
      const int copy = bank_count[bank]++ / n;
      e.node = (uint8_t)(bank + kBanks * (copy < kBankCopies ? copy : 0));
      if (copy >= kBankCopies) {
        late[n_late++] = (int16_t)ne;
      } else if (copy > 0) {  // coloured before the others
        for (int j = n_todo; j > n_extra; --j) todo[j] = todo[j - 1];
        todo[n_extra++] = (int16_t)ne;
        ++n_todo;
      } else {
        todo[n_todo++] = (int16_t)ne;
      }
      ++ne;
    }
  }
  for (int q = 0; q < n_todo; ++q) {
    const int i = todo[q];
    Edge& e = edges[i];
    const int u = e.lane, v = e.node;
    int a = 0, b = 0;
    if (q < n_extra) {
      while (at_lane[u][a] >= 0 || at_bank[v][a] >= 0) { if (++a == n) break; }  // lowest colour free at both ends
      if (a < n) { e.colour = (int8_t)a; at_lane[u][a] = (int16_t)i; at_bank[v][a] = (int16_t)i; continue; }
      a = 0;
    }
    // (the other rows take the highest free colours, so that the swaps below rarely touch the low
    // colours where the extra copies sit)
    a = n - 1; b = n - 1;
    while (at_lane[u][a] >= 0) --a;  // a colour the lane has not used (it has at most n rows)
    while (at_bank[v][b] >= 0) --b;  // a colour the bank copy has not used (it has at most n rows)
    if (at_bank[v][a] >= 0) {
      // make `a` free at the bank copy: swap a and b along the path that starts there with colour a
      int16_t path[2 * kHalf + kNodes + 2];
      int np = 0, node = v, col = a;
      bool at_bank_side = true;
      for (;;) {
        const int ei = at_bank_side ? at_bank[node][col] : at_lane[node][col];
        if (ei < 0) break;
        path[np++] = (int16_t)ei;
        node = at_bank_side ? edges[ei].lane : edges[ei].node;
        at_bank_side = !at_bank_side;
        col = (col == a) ? b : a;
      }
      for (int j = 0; j < np; ++j) {
        Edge& f = edges[path[j]];
        at_lane[f.lane][f.colour] = -1; at_bank[f.node][f.colour] = -1;
      }
      for (int j = 0; j < np; ++j) {
        Edge& f = edges[path[j]];
        f.colour = (int8_t)(f.colour == a ? b : a);
        at_lane[f.lane][f.colour] = path[j]; at_bank[f.node][f.colour] = path[j];
      }
    }
    e.colour = (int8_t)a;
    at_lane[u][a] = (int16_t)i; at_bank[v][a] = (int16_t)i;
  }
  // rows beyond the last copy: a free position of the lane where the bank is used least
  if (n_late > 0) {
    uint8_t mult[kMaxPieceRows][kBanks];
    std::memset(mult, 0, sizeof(mult));
    for (int i = 0; i < ne; ++i) if (edges[i].colour >= 0) ++mult[edges[i].colour][edges[i].node & (kBanks - 1)];
    for (int j = 0; j < n_late; ++j) {
      Edge& e = edges[late[j]];
      const int bank = e.node & (kBanks - 1);
      int best = -1;
      for (int c = 0; c < n; ++c)
        if (at_lane[e.lane][c] < 0 && (best < 0 || mult[c][bank] < mult[best][bank])) best = c;
      e.colour = (int8_t)best;  // the lane has at most n rows, so a position is free
      at_lane[e.lane][best] = late[j];
      ++mult[best][bank];
    }
  }
  for (int i = 0; i < ne; ++i) place[edges[i].lane][edges[i].colour] = edges[i].row;
}

// One unit: pcs[0 .. count) (sorted by descending length), their slots, and the parents of the
// overflow slots among them.
void emit_unit(const Piece* pcs, const uint16_t* slot_ids, int count, const std::vector<uint16_t>& parents,
               const std::vector<uint16_t>& sigma, uint32_t block, uint32_t window, int part, uint16_t null_index,
               std::vector<uint16_t>& positions, BlockOut* out) {
  positions.clear();
  int npos = 0;
  auto add_position = [&](uint16_t fill) {
    positions.resize((size_t)(npos + 1) * kLanes, fill);
    return &positions[(size_t)npos++ * kLanes];
  };
  const int nov = (int)parents.size();
  for (int c = 0; c * kLanes < nov; ++c) {
    uint16_t* q = add_position(null_index);
    for (int l = 0; l < kLanes && c * kLanes + l < nov; ++l) q[l] = parents[(size_t)c * kLanes + l];
  }

  // ---- which piece sits where: place i = (group i / 64, lane i % 64) holds piece at_place[i] ----
  const int G = ceil_div(count, kLanes);
  std::vector<int> at_place((size_t)G * kLanes);
  for (int i = 0; i < G * kLanes; ++i) at_place[i] = i < count ? i : -1;
  std::vector<HalfGroup> hg((size_t)G * 2);
  auto bank_of = [&](int piece, int t) { return (int)(sigma[pcs[piece].start + t] & (kBanks - 1)); };
  auto plen = [&](int piece) { return piece < 0 ? 0 : (int)pcs[piece].len; };
  for (int g = 0; g < G; ++g)
    for (int h = 0; h < 2; ++h) {
      HalfGroup& x = hg[(size_t)g * 2 + h];
      x.n = pcs[(size_t)g * kLanes].len;
      std::memset(x.deg, 0, sizeof(x.deg));
      for (int l = 0; l < kHalf; ++l) {
        const int pc = at_place[(size_t)g * kLanes + h * kHalf + l];
        for (int t = 0; t < plen(pc); ++t) ++x.deg[bank_of(pc, t)];
      }
    }
  {
    uint64_t rng = 0x9E3779B97F4A7C15ull ^ ((uint64_t)block << 24) ^ ((uint64_t)window << 8) ^ (uint64_t)part ^ ((uint64_t)count << 44);
    auto next = [&]() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return (uint32_t)(rng >> 32); };
    const int nplaces = G * kLanes;
    auto overfull = [&](const HalfGroup& x) {
      for (int b = 0; b < kBanks; ++b) if (x.deg[b] > x.n) return true;
      return false;
    };
    int bad = 0;
    for (const HalfGroup& x : hg) bad += overfull(x);
    const int budget = 3000;
    for (int it = 0; it < budget && bad > 0 && nplaces > kHalf; ++it) {
      // a place in an overfull half group whose piece has a row in that half group's fullest bank
      int i = (int)(next() % (uint32_t)nplaces);
      {
        int tries = 0;
        while (tries < 8 && !overfull(hg[(size_t)(i / kLanes) * 2 + (i % kLanes) / kHalf])) { i = (int)(next() % (uint32_t)nplaces); ++tries; }
      }
      const int gi = i / kLanes, hi = (i % kLanes) / kHalf;
      HalfGroup& X = hg[(size_t)gi * 2 + hi];
      int worst = 0;
      for (int b = 1; b < kBanks; ++b) if (X.deg[b] > X.deg[worst]) worst = b;
      {
        const int base = gi * kLanes + hi * kHalf, l0 = (int)(next() % kHalf);
        for (int d = 0; d < kHalf; ++d) {
          const int cand = base + (l0 + d) % kHalf, pc = at_place[cand];
          bool has = false;
          for (int t = 0; t < plen(pc); ++t) if (bank_of(pc, t) == worst) { has = true; break; }
          if (has) { i = cand; break; }
        }
      }
      const int j = (int)(next() % (uint32_t)nplaces);
      const int gj = j / kLanes, hj = (j % kLanes) / kHalf;
      if (gi == gj && hi == hj) continue;
      const int pi = at_place[i], pj = at_place[j];
      if (gi != gj && plen(pi) != plen(pj)) continue;  // every group keeps its lengths
      HalfGroup& Y = hg[(size_t)gj * 2 + hj];
      const int before = half_cost(X) + half_cost(Y);
      const bool bad_x = overfull(X), bad_y = overfull(Y);
      for (int t = 0; t < plen(pi); ++t) { const int b = bank_of(pi, t); --X.deg[b]; ++Y.deg[b]; }
      for (int t = 0; t < plen(pj); ++t) { const int b = bank_of(pj, t); --Y.deg[b]; ++X.deg[b]; }
      const int after = half_cost(X) + half_cost(Y);
      if (after < before || (after == before && (next() & 3) == 0)) {
        at_place[i] = pj; at_place[j] = pi;
        bad += (int)overfull(X) + (int)overfull(Y) - (int)bad_x - (int)bad_y;
      } else {
        for (int t = 0; t < plen(pi); ++t) { const int b = bank_of(pi, t); ++X.deg[b]; --Y.deg[b]; }
        for (int t = 0; t < plen(pj); ++t) { const int b = bank_of(pj, t); ++Y.deg[b]; --X.deg[b]; }
      }
    }
  }

  uint64_t hdr = 0;
  int ngroups = 0;
  uint32_t nidx = 0;
  for (int g = 0; g < G; ++g) {
    const int n = pcs[(size_t)g * kLanes].len;  // the group's longest piece
    hdr |= 1ull << npos;
    uint16_t* h = add_position(0);
    for (int l = 0; l < kLanes; ++l) {
      const int pc = at_place[(size_t)g * kLanes + l];
      h[l] = pc >= 0 ? slot_ids[pc] : (uint16_t)(kWindow + (l & (kDummySlots - 1)));
    }
    const int first = npos;
    for (int t = 0; t < n; ++t) add_position(null_index);
    for (int half = 0; half < 2; ++half) {
      uint16_t row_of[kHalf][kMaxPieceRows], place[kHalf][kMaxPieceRows];
      int len[kHalf];
      for (int l = 0; l < kHalf; ++l) {
        const int pc = at_place[(size_t)g * kLanes + half * kHalf + l];
        len[l] = plen(pc);
        for (int t = 0; t < len[l]; ++t) row_of[l][t] = sigma[pcs[pc].start + t];
        nidx += (uint32_t)len[l];
      }
      colour_half(n, row_of, len, null_index, place);
      for (int t = 0; t < n; ++t)
        for (int l = 0; l < kHalf; ++l) positions[(size_t)(first + t) * kLanes + half * kHalf + l] = place[l][t];
    }
    ++ngroups;
  }
  if (npos & 1) add_position(null_index);  // dword rows hold two positions
  Unit u;
  std::memset(&u, 0, sizeof(u));
  u.stream_off = (uint32_t)(out->stream.size() * sizeof(uint16_t) / kStreamAlign);
  u.block = block;
  u.window = (uint16_t)window;
  u.part = (uint8_t)part;
  u.npar = (uint8_t)ceil_div(nov, kLanes);
  u.npos = (uint8_t)npos;
  u.ngroups = (uint8_t)ngroups;
  u.hdr_lo = (uint32_t)hdr;
  u.hdr_hi = (uint16_t)(hdr >> 32);
  u.nidx = nidx;
  u.npieces = (uint32_t)count;
  const int full = npos / kGranulePositions;
  for (int g = 0; g < full; ++g)
    for (int l = 0; l < kLanes; ++l)
      for (int q = 0; q < kGranulePositions; ++q)
        out->stream.push_back(positions[(size_t)(g * kGranulePositions + q) * kLanes + l]);
  for (int p = full * kGranulePositions; p < npos; p += 2)
    for (int l = 0; l < kLanes; ++l) {
      out->stream.push_back(positions[(size_t)p * kLanes + l]);
      out->stream.push_back(positions[(size_t)(p + 1) * kLanes + l]);
    }
  out->stored_rows += nidx;
  out->segments += count;
  out->header_positions += ngroups;
  out->units.push_back(u);
}

// All windows of one (block, part): sort the rows, cut each window's segments into pieces of at
// most T rows, rank the pieces by length, fill units group by group.
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
    // ---- the cut length T: the one with the fewest positions (plus a charge per unit) ----
    uint32_t longest = 0;
    for (uint32_t jl = jfirst; jl < W; ++jl) longest = std::max(longest, S->off[j0 + jl + 1] - S->off[j0 + jl]);
    int best_T = 1, best_cost = 0x7fffffff;
    for (int T = std::min<uint32_t>(longest, kMaxPieceRows); T >= 1; --T) {
      uint32_t hist[kMaxPieceRows + 1] = {0};
      uint32_t nov = 0, nov_cls[4] = {0, 0, 0, 0};  // further pieces, also per row class (value bits 7, 8)
      for (uint32_t jl = jfirst; jl < W; ++jl) {
        const uint32_t c = S->off[j0 + jl + 1] - S->off[j0 + jl];
        if (!c) continue;
        hist[T] += c / (uint32_t)T;
        if (c % (uint32_t)T) ++hist[c % (uint32_t)T];
        const uint32_t more = (c + (uint32_t)T - 1) / (uint32_t)T - 1;
        nov += more;
        nov_cls[(jl >> 7) & 3] += more;
      }
      // groups of 64 in descending length: a group costs its header and its longest piece
      int cost = 0;
      uint32_t in_group = 0;
      for (int len = T; len >= 1; --len) {
        uint32_t n = hist[len];
        while (n) {
          if (in_group == 0) cost += 1 + len;
          const uint32_t take = std::min<uint32_t>(n, kLanes - in_group);
          in_group = (in_group + take) % kLanes;
          n -= take;
        }
      }
      // parent positions: a row class has 16 overflow slots per position
      const uint32_t cls_max = std::max(std::max(nov_cls[0], nov_cls[1]), std::max(nov_cls[2], nov_cls[3]));
      cost += ceil_div((int)cls_max, kLanes / 4);
      const int units = std::max(ceil_div(cost, kMaxPositions - 2), ceil_div((int)cls_max, kMaxOverflow / 4));
      cost += units * kUnitCost;
      if (cost < best_cost) { best_cost = cost; best_T = T; }
      if (nov > (uint32_t)8 * kMaxOverflow && cost > 2 * best_cost) break;  // shorter pieces only get worse
    }
    // ---- pieces, ranked by descending length (stable counting sort) ----
    const uint32_t T = (uint32_t)best_T;
    S->pieces.clear();
    for (uint32_t jl = jfirst; jl < W; ++jl) {
      const uint32_t j = j0 + jl;
      const uint32_t c = S->off[j + 1] - S->off[j];
      for (uint32_t done = 0; done < c; done += T)
        S->pieces.push_back(Piece{S->off[j] + done, (uint16_t)std::min(T, c - done), (uint16_t)jl});
    }
    uint32_t bucket[kMaxPieceRows + 2] = {0};
    for (const Piece& p : S->pieces) ++bucket[kMaxPieceRows - p.len + 1];
    for (int i = 0; i <= kMaxPieceRows; ++i) bucket[i + 1] += bucket[i];
    S->sorted.resize(S->pieces.size());
    for (const Piece& p : S->pieces) S->sorted[bucket[kMaxPieceRows - p.len]++] = p;

    // ---- units: consecutive groups while positions and overflow slots last ----
    // Overflow slot x sits in lane x % 64 of the fold; the kernel adds its sum to that lane's total,
    // so the lane's 16-lane row (which stands for value bits 7 and 8) has to match the parent's:
    // class c = parent >> 7 owns the overflow slots 64i + 16c .. 64i + 16c + 15, i = 0 .. 3.
    const int np = (int)S->sorted.size();
    S->unit_slot.resize((size_t)np);
    int first = 0;        // first piece of the unit being filled
    int posn = 0;         // its positions without the parent positions
    int cls_used[4] = {0, 0, 0, 0};
    S->parents.clear();   // parent of every overflow slot up to the highest one in use (null = unused)
    S->seen.assign(W, 0);
    auto ovf_index = [](int cls, int n) { return (n / 16) * kLanes + 16 * cls + n % 16; };
    auto flush_unit = [&](int end) {
      emit_unit(&S->sorted[(size_t)first], &S->unit_slot[(size_t)first], end - first, S->parents, S->sigma, block, w, part,
                null_index, S->positions, out);
      first = end;
      posn = 0;
      for (int& c : cls_used) c = 0;
      S->parents.clear();
      S->seen.assign(W, 0);
    };
    for (int r0 = 0; r0 < np; r0 += kLanes) {
      const int cnt = std::min(kLanes, np - r0);
      const int need = 1 + (int)S->sorted[(size_t)r0].len;
      for (int attempt = 0;; ++attempt) {
        // pieces of this group whose segment already has a piece in the unit (or earlier in this group)
        int extra[4] = {0, 0, 0, 0};
        for (int l = 0; l < cnt; ++l) {
          const uint16_t sl = S->sorted[(size_t)(r0 + l)].slot;
          if (S->seen[sl]) ++extra[(sl >> 7) & 3]; else S->seen[sl] = 2;  // 2: tentatively, by this group
        }
        bool fits = true;
        int top = (int)S->parents.size();
        for (int c = 0; c < 4; ++c) {
          const int n = cls_used[c] + extra[c];
          if (n > kMaxOverflow / 4) fits = false;
          else if (extra[c]) top = std::max(top, ovf_index(c, n - 1) + 1);
        }
        if (posn + need + ceil_div(top, kLanes) > kMaxPositions) fits = false;
        if (fits || attempt == 1) {
          for (int l = 0; l < cnt; ++l) {
            Piece& pc = S->sorted[(size_t)(r0 + l)];
            if (S->seen[pc.slot] == 2) {
              S->seen[pc.slot] = 1;
              S->unit_slot[(size_t)(r0 + l)] = pc.slot;
            } else {
              const int c = (pc.slot >> 7) & 3;
              const int x = ovf_index(c, cls_used[c]++);
              if ((int)S->parents.size() <= x) S->parents.resize((size_t)x + 1, null_index);
              S->parents[(size_t)x] = pc.slot;
              S->unit_slot[(size_t)(r0 + l)] = (uint16_t)(kOverflowBase + x);
            }
          }
          posn += need;
          break;
        }
        for (int l = 0; l < cnt; ++l) {  // undo the tentative marks, close the unit, try again in an empty one
          uint8_t& m = S->seen[S->sorted[(size_t)(r0 + l)].slot];
          if (m == 2) m = 0;
        }
        flush_unit(r0);
      }
    }
    if (first < np) flush_unit(np);
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
  if (out->units.empty()) {  // an all-zero block still has to write its outputs: a unit without positions
    S->parents.clear();
    emit_unit(nullptr, nullptr, 0, S->parents, S->sigma, (uint32_t)block, 0, 0, (uint16_t)rows, S->positions, out);
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
    P.segments += B.segments;
    P.header_positions += B.header_positions;
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
  return us[(size_t)full * kGranulePositions * kLanes + ((size_t)(q / 2) * kLanes + l) * 2 + (q & 1)];
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
    if (u.npos > kMaxPositions || (u.npos & 1)) { *err = "corrupt unit: position count"; return -1; }
    const uint16_t* us = &P.stream[(size_t)u.stream_off * (kStreamAlign / sizeof(uint16_t))];
    const uint64_t hdr = ((uint64_t)u.hdr_hi << 32) | u.hdr_lo;
    const int npar = u.npar;
    if (npar > kMaxOverflow / kLanes || npar > u.npos) { *err = "corrupt unit: overflow slots"; return -1; }
    uint16_t slot[kLanes];
    for (int l = 0; l < kLanes; ++l) slot[l] = (uint16_t)kWindow;
    for (int p = npar; p < u.npos; ++p) {
      if ((hdr >> p) & 1) {
        for (int l = 0; l < kLanes; ++l) slot[l] = stream_at(us, u.npos, p, l);
        continue;
      }
      for (int l = 0; l < kLanes; ++l) {
        const uint16_t row = stream_at(us, u.npos, p, l);
        if (row == null_index) continue;
        if (row > null_index) { *err = "corrupt unit: row index out of range"; return -1; }
        uint32_t sl = slot[l];
        if (sl >= (uint32_t)kOverflowBase) {  // a further piece of a segment: filed under its parent
          const uint32_t o = sl - kOverflowBase;
          if (o >= (uint32_t)npar * kLanes) { *err = "corrupt unit: overflow slot out of range"; return -1; }
          sl = stream_at(us, u.npos, (int)(o / kLanes), (int)(o % kLanes));
          if (sl < (uint32_t)kWindow && ((sl >> 7) & 3) != ((o % kLanes) >> 4)) { *err = "corrupt unit: overflow slot in the wrong row"; return -1; }
        }
        if (sl >= (uint32_t)kWindow) { *err = "corrupt unit: row in a dummy slot"; return -1; }
        const uint32_t value = (((uint32_t)u.window << P.kw) + sl) >> shift;
        if (value >= nvals || value == 0 || listed[row]) { *err = "corrupt unit: bad value or repeated row"; return -1; }
        listed[row] = 1;
        by_value[value].push_back((int32_t)row);
      }
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
