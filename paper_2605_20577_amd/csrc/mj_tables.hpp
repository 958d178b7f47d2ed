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
//   keyinfo[key]              u32  first record | number of records << 16
//   recs[]                    u32  bits 0..3 pair rank + 1 (0 = none); four set slots of 5 bits
//                                  from bit 4: type << 4 | rank (1 = triplet, 0 = run start), 0x1F = empty
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
  std::vector<uint32_t> keyinfo;   // n_keys
  std::vector<uint32_t> recs;      // n_recs
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
    t.keyinfo.push_back((uint32_t)t.recs.size() | (uint32_t)kv.second->size() << 16);
    for (uint32_t r : *kv.second) t.recs.push_back(r);
  }
  t.n_keys = (int)t.keyinfo.size();
  t.n_recs = (int)t.recs.size();
  return t;
}

}  // namespace mjt
