// Host-side builder of the per-suit decomposition table (the "pre-computed
// statistics for all possible suit combinations" of paper section 3.1, item 2),
// in the form the kernels use.
//
// A suit pattern is nine counts 0..4.  It is valid when it splits into runs
// and triplets ("sets only") or into sets plus one pair: 21,743 patterns with
// 23,533 decompositions (at most four each).
//
// The key is split into prefix5 (base-5 number of ranks 1..5, 3125 values) and
// suffix5 (ranks 6..9, 625 values).  Prefixes that accept the same set of
// suffixes share one row; there are only 97 different rows.
//
//  probe tables, staged into LDS (about 11 KB):
//   rowid[prefix5]            u8   row of this prefix, 0 = the empty row
//   bitmap[row][20]           u32  bit suffix5 set <=> (prefix5, suffix5) is valid
//  record tables, read from global memory when a winning hand is scored:
//   base[prefix5]             u16  number of valid keys with a smaller prefix
//   rowrank[row][20]          u16  set bits of the row before each bitmap word
//   recs[key][4]              u32  the key's decompositions (at most four), unused entries 0; bits 28..29 of the
//                                  first one hold their number - 1, so one 4-byte load per suit serves the usual
//                                  case of a single decomposition.  A record: bits 0..3 pair rank + 1 (0 = none); four set slots
//                                  of 5 bits from bit 4: type << 4 | rank (1 = triplet, 0 = run start), 0x1F = empty
//                                  (so a record is never 0)
#pragma once
#include <algorithm>
#include <cstdint>
#include <map>
#include <vector>

namespace mjt {

constexpr int kPrefixes = 3125;   // 5^5
constexpr int kSuffixes = 625;    // 5^4

constexpr int kRowWords = 20;      // 625 bits

struct SuitTables {
  std::vector<uint8_t> rowid;      // kPrefixes, padded to a multiple of 16 bytes
  std::vector<uint32_t> bitmap;    // n_rows * kRowWords
  std::vector<uint16_t> base;      // kPrefixes (+ pad)
  std::vector<uint16_t> rowrank;   // n_rows * kRowWords
  std::vector<uint32_t> recs;      // n_keys * 4
  int n_rows = 0, n_keys = 0, n_recs = 0;
};

inline void emit(std::map<uint32_t, std::vector<uint32_t>> &out, const int trip[9], const int run[7], int pair)
{
  int c[9] = {0};
  for (int r = 0; r < 9; r++) c[r] += 3 * trip[r];
  for (int r = 0; r < 7; r++) { c[r] += run[r]; c[r + 1] += run[r]; c[r + 2] += run[r]; }
  if (pair >= 0) c[pair] += 2;
  for (int r = 0; r < 9; r++) if (c[r] > 4) return;
  uint32_t key = 0, p5 = 1;
  for (int r = 0; r < 9; r++) { key += (uint32_t)c[r] * p5; p5 *= 5; }
  uint32_t rec = (uint32_t)(pair + 1);
  int slot = 0;
  for (int r = 0; r < 9; r++) {
    if (trip[r]) rec |= (uint32_t)(0x10 | r) << (4 + 5 * slot++);
    if (r < 7) for (int j = 0; j < run[r]; j++) rec |= (uint32_t)r << (4 + 5 * slot++);
  }
  for (; slot < 4; slot++) rec |= 0x1Fu << (4 + 5 * slot);
  out[key].push_back(rec);
}

// every multiset of at most four sets, with and without a pair
inline void enumerate(std::map<uint32_t, std::vector<uint32_t>> &out)
{
  int trip[9] = {0}, run[7] = {0};
  // choose the sets in non-decreasing order of an id: 0..8 triplets, 9..15 runs
  struct Rec {
    static void go(std::map<uint32_t, std::vector<uint32_t>> &out, int trip[9], int run[7], int first, int left)
    {
      for (int pair = -1; pair < 9; pair++) emit(out, trip, run, pair);
      if (left == 0) return;
      for (int id = first; id < 16; id++) {
        if (id < 9) { if (trip[id]) continue; trip[id] = 1; go(out, trip, run, id, left - 1); trip[id] = 0; }
        else { if (run[id - 9] == 4) continue; run[id - 9]++; go(out, trip, run, id, left - 1); run[id - 9]--; }
      }
    }
  };
  Rec::go(out, trip, run, 0, 4);
  for (auto &kv : out) {                 // the same multiset is reached once only, but keep the lists tidy
    std::sort(kv.second.begin(), kv.second.end());
    kv.second.erase(std::unique(kv.second.begin(), kv.second.end()), kv.second.end());
  }
}

inline SuitTables build()
{
  std::map<uint32_t, std::vector<uint32_t>> keys;     // key5 = prefix5 + 3125 * suffix5
  enumerate(keys);
  // suffix sets per prefix, and the records in (prefix, suffix) order
  std::vector<std::vector<int>> cols(kPrefixes);
  std::map<std::pair<int, int>, const std::vector<uint32_t> *> ordered;
  for (auto &kv : keys) {
    int p = (int)(kv.first % kPrefixes), sfx = (int)(kv.first / kPrefixes);
    cols[p].push_back(sfx);
    ordered[{p, sfx}] = &kv.second;
  }
  SuitTables t;
  t.rowid.assign((kPrefixes + 15) & ~15, 0);
  t.base.assign((kPrefixes + 7) & ~7, 0);
  std::map<std::vector<int>, int> row_of;
  row_of[std::vector<int>()] = 0;                     // row 0 accepts nothing
  t.bitmap.assign(kRowWords, 0);
  t.rowrank.assign(kRowWords, 0);
  int running = 0;
  for (int p = 0; p < kPrefixes; p++) {
    std::sort(cols[p].begin(), cols[p].end());
    auto it = row_of.find(cols[p]);
    if (it == row_of.end()) {
      int id = (int)row_of.size();
      it = row_of.emplace(cols[p], id).first;
      std::vector<uint32_t> bits(kRowWords, 0);
      for (int c : cols[p]) bits[c >> 5] |= 1u << (c & 31);
      int before = 0;
      for (int w = 0; w < kRowWords; w++) {
        t.bitmap.push_back(bits[w]);
        t.rowrank.push_back((uint16_t)before);
        before += __builtin_popcount(bits[w]);
      }
    }
    t.rowid[p] = (uint8_t)it->second;
    t.base[p] = (uint16_t)running;
    running += (int)cols[p].size();
  }
  t.n_rows = (int)row_of.size();
  for (auto &kv : ordered) {
    for (int j = 0; j < 4; j++) t.recs.push_back(j < (int)kv.second->size() ? (*kv.second)[j] : 0u);
    t.recs[t.recs.size() - 4] |= (uint32_t)(kv.second->size() - 1) << 28;      // how many there are, with the first one
    t.n_keys++;
    t.n_recs += (int)kv.second->size();
  }
  return t;
}

// ---------------------------------------------------------------- shanten
// Block statistics of one suit for the shanten number (paper section 3.2 lists the shanten number among the
// observation's scalars; section 3.1, item 2 is the idea of a per-suit table).  For a pattern of counts and a number
// m = 0..4 of complete sets (triplets, runs) taken from it, the entry gives the largest number of partial sets
// (pair, two adjacent, two with a gap; capped at 4) that the remaining tiles still hold, once without and once
// with one pair set aside as the head: ten 3-bit fields, 7 = "m sets are not possible" (bits 0..14 without head,
// 15..29 with).  The key is the base-5 number of the counts, prefix5 + 3125 * suffix5 for a numbered suit
// (1,953,125 entries), seven digits for the honors (78,125 entries, no runs).  Filled by dynamic programming over
// the lowest occupied rank: every block that starts there, or the tile belongs to nothing.
struct Frontier { int8_t n[5], h[5]; };
inline uint32_t pack_frontier(const Frontier &f)
{
  uint32_t v = 0;
  for (int m = 0; m < 5; m++) {
    const int without = f.n[m], with = f.h[m];
    v |= (uint32_t)(without < 0 ? 7 : without) << (3 * m);
    v |= (uint32_t)(with < 0 ? 7 : with) << (15 + 3 * m);
  }
  return v;
}
inline std::vector<uint32_t> build_shanten_table(int n_ranks, bool runs)
{
  int pw[10];
  pw[0] = 1;
  for (int r = 1; r <= n_ranks; r++) pw[r] = pw[r - 1] * 5;
  const int N = pw[n_ranks];
  std::vector<Frontier> F((size_t)N);
  Frontier empty;
  for (int m = 0; m < 5; m++) { empty.n[m] = m == 0 ? 0 : -1; empty.h[m] = -1; }
  F[0] = empty;
  std::vector<uint32_t> out((size_t)N);
  out[0] = pack_frontier(F[0]);
  for (int key = 1; key < N; key++) {
    int c[11] = {0};
    for (int r = 0, k = key; r < n_ranks; r++, k /= 5) c[r] = k % 5;
    int i = 0;
    while (c[i] == 0) i++;
    Frontier f;
    for (int m = 0; m < 5; m++) f.n[m] = f.h[m] = -1;
    auto relax = [&f](const Frontier &g, int dm, int dt) {
      for (int m = 0; m + dm < 5; m++) {
        if (g.n[m] >= 0) f.n[m + dm] = std::max<int8_t>(f.n[m + dm], (int8_t)std::min(g.n[m] + dt, 4));
        if (g.h[m] >= 0) f.h[m + dm] = std::max<int8_t>(f.h[m + dm], (int8_t)std::min(g.h[m] + dt, 4));
      }
    };
    if (c[i] >= 3) relax(F[key - 3 * pw[i]], 1, 0);
    if (runs && i + 2 < n_ranks && c[i + 1] && c[i + 2]) relax(F[key - pw[i] - pw[i + 1] - pw[i + 2]], 1, 0);
    if (c[i] >= 2) relax(F[key - 2 * pw[i]], 0, 1);
    if (runs && i + 1 < n_ranks && c[i + 1]) relax(F[key - pw[i] - pw[i + 1]], 0, 1);
    if (runs && i + 2 < n_ranks && c[i + 2]) relax(F[key - pw[i] - pw[i + 2]], 0, 1);
    relax(F[key - pw[i]], 0, 0);
    if (c[i] >= 2) {                                            // the pair at rank i is the head
      const Frontier &g = F[key - 2 * pw[i]];
      for (int m = 0; m < 5; m++) if (g.n[m] >= 0) f.h[m] = std::max(f.h[m], g.n[m]);
    }
    F[key] = f;
    out[key] = pack_frontier(f);
  }
  return out;
}

// ---------------------------------------------------------------- neighbours
// For every pattern of nine counts 0..4 of one suit (key = base-5 number of the counts = prefix5 + 3125 * suffix5,
// 1,953,125 entries of 32 bits): what the search for tenpai-keeping discards asks about a suit, answered by one read
// instead of some thirty probes of the pattern table:
//   bit 0        the pattern itself is valid (sets, or sets and a pair)
//   bits 1..9    rank r holds fewer than four and the pattern with one more tile of rank r is valid
//   bits 10..18  rank r is held and the pattern with one tile of rank r less is valid
//   bits 19..27  rank r is held and the pattern with one tile of rank r less can be made valid by adding some tile
inline std::vector<uint32_t> build_neighbour_table()
{
  std::map<uint32_t, std::vector<uint32_t>> keys;
  enumerate(keys);
  const int N = 1953125;
  std::vector<uint8_t> valid((size_t)N, 0);
  for (auto &kv : keys) valid[kv.first] = 1;
  int pw[9];
  pw[0] = 1;
  for (int r = 1; r < 9; r++) pw[r] = pw[r - 1] * 5;
  // first pass: valid + "can take a tile of rank r"
  std::vector<uint32_t> out((size_t)N, 0);
  int c[9] = {0};
  for (int key = 0; key < N; key++) {
    uint32_t v = valid[key];
    for (int r = 0; r < 9; r++) if (c[r] < 4 && valid[key + pw[r]]) v |= 1u << (1 + r);
    out[key] = v;
    for (int r = 0; r < 9; r++) { if (++c[r] < 5) break; c[r] = 0; }      // next count vector
  }
  // second pass: what removing a tile of rank r leaves
  for (int r = 0; r < 9; r++) c[r] = 0;
  for (int key = 0; key < N; key++) {
    uint32_t v = out[key];
    for (int r = 0; r < 9; r++) if (c[r] > 0) {
      const uint32_t less = out[key - pw[r]];
      if (less & 1u) v |= 1u << (10 + r);
      if (less & 0x3FEu) v |= 1u << (19 + r);
    }
    out[key] = v;
    for (int r = 0; r < 9; r++) { if (++c[r] < 5) break; c[r] = 0; }
  }
  return out;
}

}  // namespace mjt
