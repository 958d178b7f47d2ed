// Per-environment logic of the batched Riichi Mahjong step, written for one
// GPU lane per environment (gfx950).  Every function is MJ_HD so that the same
// source also compiles for the host, where the test-only host build runs it
// under a debugger or sanitizer; the product only ever runs it inside the HIP
// kernels of mj_lib.hip.
//
// What is computed follows the paper's environment (section 3.1: State, init,
// step; section 3.2: rules, modes, action ids, legal_action_mask, illegal
// action => termination; section 4.1: random policy).  How it is computed is
// this library's own design:
//   - hands are four words per seat of 3-bit packed counts (three suits, honors);
//   - win detection looks each suit word up in a two-level table of all valid
//     suit patterns (prefix -> shared row -> suffix bitmap, in LDS), honors by
//     bit arithmetic;
//   - scoring turns decomposition records into bit masks (triplet kinds, packed
//     run multiplicities) so every yaku and the fu are mask / popcount tests;
//   - waits of every seat are cached as 34-bit masks and refreshed only when
//     that seat's concealed hand changes.
#pragma once
#include <stdint.h>

#ifndef MJ_HD
#define MJ_HD __host__ __device__ __forceinline__
#endif
// Branch weights.  The step kernels are one very large function at the limit of the register file; the register
// allocator and the block placement follow these hints.  Which hints help was found by measuring builds that differ in
// one hint each: see the places that use them.
#define MJ_RARE(x) __builtin_expect(!!(x), 0)
#define MJ_USUAL(x) __builtin_expect(!!(x), 1)
#ifndef MJ_STAT
#define MJ_STAT(x) ((void)0)
#endif
// -DMJ_PROFILE (never in the shipped library): wave-level region timers of the step kernels.  MJ_RB notes which
// lanes need a region and the time; MJ_RE adds, once per wavefront, the cycles spent in it, one entry and the
// number of lanes that needed it to three counters per region in LDS, which k_rollout prints for one block.
#if defined(MJ_PROFILE) && defined(__HIPCC__)
enum { PR_LOOP, PR_REFILL, PR_SAMPLE, PR_STEP, PR_RESET, PR_DEAL, PR_DEAL_NEXT, PR_DEAL_WAVE, PR_FINISH,
       PR_S0, PR_S1_TURN, PR_DISCARD, PR_KAN, PR_DECL, PR_S1_RESP, PR_CALL, PR_S2, PR_W_SHORT, PR_W_FACTS, PR_W_REFRESH,
       PR_WF_CAND, PR_WF_SPECIAL, PR_S3, PR_S3_RON, PR_WIN, PR_ABORT, PR_EXH, PR_DRAW, PR_KANDRAW,
       PR_TM_FACTS, PR_TM_EXACT, PR_TP_STD, PR_TP_OWN, PR_TP_SPECIAL, PR_TM_TSUMO, PR_TM_RIICHI, PR_TM_BITS, PR_EVAL, PR_N };
__shared__ unsigned long long mj_prof[3 * PR_N];
#endif
#if defined(MJ_PROFILE) && defined(__HIP_DEVICE_COMPILE__)
#define MJ_RB(name, cond) const unsigned long long rbm_##name = __ballot((cond) ? 1 : 0); const long long rbt_##name = clock64()
#define MJ_RE(name, idx)                                                                                   \
  do {                                                                                                     \
    if (rbm_##name) {                                                                                      \
      const unsigned long long act_ = __ballot(1);                                                         \
      if ((int)(threadIdx.x & 63) == __ffsll((long long)act_) - 1) {                                       \
        atomicAdd(&mj_prof[3 * (idx)], (unsigned long long)(clock64() - rbt_##name));                      \
        atomicAdd(&mj_prof[3 * (idx) + 1], 1ull);                                                          \
        atomicAdd(&mj_prof[3 * (idx) + 2], (unsigned long long)__popcll(rbm_##name));                      \
      }                                                                                                    \
    }                                                                                                      \
  } while (0)
#elif defined(MJ_MARKS) && defined(__HIP_DEVICE_COMPILE__)
// -DMJ_MARKS (never in the shipped library): the same region boundaries as comments in the generated assembly
#define MJ_RB(name, cond) asm volatile("; MJMARK B " #name)
#define MJ_RE(name, idx) asm volatile("; MJMARK E " #name)
#else
#define MJ_RB(name, cond) ((void)0)
#define MJ_RE(name, idx) ((void)0)
#endif
// Everything is force-inlined: the kernels contain no function calls.  Out-of-line device functions (tried for
// the hand evaluator and the waits search) gave wrong results on the GPU on rare paths while the same source was
// right on the host, and each call site cost a few hundred instructions of register save and restore.  The big
// functions therefore have few call sites each (loops over seats are kept rolled around them).

namespace mj {

// ---------------------------------------------------------------- constants
enum { F_RED = 1, F_ABORT = 2, F_KUITAN = 4, F_ENDGAME = 16, F_KANDORA_LATE = 32, F_NAGASHI = 64, F_ANKAN_ROB = 128, F_PAO = 256 };
enum { PH_TURN = 0, PH_RESPOND = 1, PH_RESPOND_KAKAN = 2, PH_TERMINAL = 3 };
enum { A_DISCARD = 0, A_DISCARD_RED = 34, A_KAN = 37, A_RIICHI = 71, A_TSUMO = 72, A_KYUUSHU = 73, A_RON = 74,
       A_PON = 75, A_PON_RED = 76, A_MINKAN = 77, A_CHI_L = 78, A_CHI_L_RED = 81, A_PASS = 84, N_ACTIONS = 85 };
enum { MT_CHI = 1, MT_PON = 2, MT_MINKAN = 3, MT_ANKAN = 4, MT_KAKAN = 5 };

constexpr uint64_t K_TERMINALS = 0x4060301ull;                       // kinds 0,8,9,17,18,26
constexpr uint64_t K_HONORS = 0x7Full << 27;
constexpr uint64_t K_YAOCHU = K_TERMINALS | K_HONORS;
// "Facts" of a hand, kept next to the caches that depend on it so that a hand which changed in one suit costs one
// table probe instead of four: tile count mod 3 of suit s in bits 2s..2s+1, "suit s is a valid pattern" in bit 8+s.
// They ride in bits 40..51 of a waits word (W_FACTS_VALID set) and of the tenpai-discards word (TD_FACTS set).
constexpr int FACTS_SHIFT = 40;
constexpr uint64_t W_FACTS_VALID = 1ull << 52, TD_FACTS = 1ull << 52;
constexpr uint64_t TD_UNKNOWN = 1ull << 62;     // tenpai_discards_of without the search: "some discard may keep tenpai"
constexpr uint64_t TD_VALID = 1ull << 63;       // Env::tdisc holds the tenpai-keeping discards of the hand as it is now
constexpr uint64_t K_WINDS = 0xFull << 27;
constexpr uint64_t K_DRAGONS = 0x7ull << 31;
constexpr uint64_t K_ALL = (1ull << 34) - 1;
constexpr uint32_t O111 = 0111111111u;                               // bit 0 of each of nine 3-bit fields

struct Rules {
  uint32_t flags, env_id_base;
  int32_t start_score;
  float illegal_penalty;
  uint32_t mode;
  uint32_t seed;
};

// the per-suit pattern table: probe part (LDS) and record part (global memory).  The kernels hold this struct by
// value (in registers): after inlining, the probes then compile to LDS reads instead of generic-address loads.
struct Lut {
  const uint8_t *rowid;      // [3125] row of a prefix
  const uint32_t *bitmap;    // [rows][20] valid suffixes of a row
  const uint16_t *base;      // [3125] keys before this prefix
  const uint16_t *rowrank;   // [rows][20] set bits before each word
  const uint32_t *recs;      // [keys][4] the decompositions of a key, unused entries 0; the first one carries their number
  const uint32_t *nb;        // [5^9] neighbours of every count pattern (global memory): valid | can take r | can lose r | ...
};

// One environment's view of the structure-of-arrays state.  "Hot" fields (touched by every step) live at
// ptr[i * hs]; the step kernels keep them in LDS (hs = block size, ptr = LDS base + thread) and every other
// user reads them in HBM (hs = n).  "Cold" fields always live in HBM at ptr[i * n] (n = B, ptr = base + b).
struct Env {
  int64_t n, hs;
  uint64_t *dk, *waits, *mask, *meld;                 // hot  [4] [4] [8] [4]
  uint64_t *tdisc;                                    // hot  [1]: discards of the seat to move that keep its hand tenpai (TD_VALID set), a cache
  int32_t *score, *delta;                             // hot  [4] [4]
  uint32_t *episode, *serial, *hand, *seatw;          // hot  [1] [1] [16] [4]
  uint64_t *yaku, *resw;                              // cold [4] [4]
  int32_t *gain;                                      // cold [4]
  uint32_t *glob;                                     // cold [7] (held in registers during a step)
  uint32_t *wallw;                                    // cold [2][34]: two wall buffers of 136 bytes, four per word;
                                                      // Glob::wall_sel names the current one, the other holds
  uint32_t *nserial;                                  // cold [1]: ... the wall of this kyoku_serial, made ahead of time
  uint32_t *nexth, *nextred;                          // cold [16] [1]: its four dealt hands by seat wind, red fives
  uint64_t *nextwaits;                                // cold [4]: their waits
  uint8_t *river;                                     // cold [128]
  uint16_t *hist;                                     // this environment's row of 128 entries: the kyoku's public actions
                                                      // in order, action | seat << 8
  uint8_t *hstage, *hbase;                            // null, or a staging column for the history in LDS (bytes at
                                                      // stride hs) and the history index of its first slot (hist_push)

};

// control bytes kept in registers during a step (7 words in HBM)
struct Glob {
  uint8_t kyoku, honba, kyotaku, terminated;
  uint8_t draw_ptr, n_kan, live_left, n_dora;
  uint8_t drawn, phase, cur, actor_mask;
  uint8_t riichi_pending, kanflags, last_discard, last_discarder;   // kanflags: bit 0 the drawn tile is a replacement
                                                                    // tile, bit 1 a kan indicator waits to be turned (F_KANDORA_LATE)
  uint8_t kakan_tile, kuikae0, kuikae1, first_wind;
  uint8_t same_wind_cnt, illegal_seat, end_type, winners;
  uint8_t loser, tenpai_mask;
  uint8_t wall_sel;     // which of the two wall buffers holds the current wall (not part of the logical state)
  uint8_t hist_len;     // entries of Env::hist in use
};
union GlobU { Glob g; uint32_t w[7]; };

// per-seat control word
//  0-2 hand_red | 3-5 n_meld | 6-11 n_river | 12-19 riichi_idx | 20-21 riichi | 22 ippatsu | 23 first_turn
//  24 furiten_temp | 25 furiten_riichi | 26-28 kan_by | 29-30 final_rank
enum { SW_RED = 0, SW_NMELD = 3, SW_NRIVER = 6, SW_RIDX = 12, SW_RIICHI = 20, SW_IPPATSU = 22, SW_FIRST = 23,
       SW_FTEMP = 24, SW_FRIICHI = 25, SW_KANBY = 26, SW_RANK = 29 };
MJ_HD uint32_t sw_get(uint32_t w, int pos, int bits) { return (w >> pos) & ((1u << bits) - 1); }
MJ_HD uint32_t sw_set(uint32_t w, int pos, int bits, uint32_t v) { return (w & ~(((1u << bits) - 1) << pos)) | (v << pos); }

// ------------------------------------------------------------------ helpers
MJ_HD int popc32(uint32_t x) { return __builtin_popcount(x); }
MJ_HD int popc64(uint64_t x) { return __builtin_popcountll(x); }
MJ_HD int ctz64(uint64_t x) { return __builtin_ctzll(x); }
MJ_HD uint32_t mulhi(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * b) >> 32); }
MJ_HD int suit_of(int k) { return k >= 27 ? 3 : k >= 18 ? 2 : k >= 9 ? 1 : 0; }
MJ_HD int rank_of(int k, int su) { return k - 9 * su; }
MJ_HD bool is_five(int k) { return k == 4 || k == 13 || k == 22; }
MJ_HD int cnt3(uint32_t w, int r) { return (int)((w >> (3 * r)) & 7u); }
MJ_HD uint64_t kbit(int k) { return 1ull << k; }
MJ_HD int code_kind(int c) { return c & 63; }
MJ_HD int code_red(int c) { return (c >> 6) & 1; }

// a 32-bit word of a byte row (rows of river bytes and history entries start at multiples of four bytes)
MJ_HD uint32_t row_word(const void *row, int i)
{
  uint32_t w;
  __builtin_memcpy(&w, __builtin_assume_aligned((const uint8_t *)row + 4 * i, 4), 4);      // one 4-byte load
  return w;
}

MJ_HD int m_type(uint32_t m) { return (int)(m & 7); }
MJ_HD int m_kind(uint32_t m) { return (int)((m >> 3) & 63); }
MJ_HD uint32_t m_make(int type, int kind, int from_rel, int pos, int has_red, int called_red)
{
  return (uint32_t)(type | kind << 3 | from_rel << 9 | pos << 11 | has_red << 13 | called_red << 14);
}
MJ_HD uint32_t meld_at(uint64_t mw, int j) { return (uint32_t)(mw >> (16 * j)) & 0xFFFFu; }

// Philox4x32-10 (Salmon et al., SC'11)
MJ_HD void philox(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, uint32_t out[4])
{
#pragma unroll
  for (int i = 0; i < 10; i++) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ------------------------------------------------------------ suit patterns
MJ_HD uint32_t prefix5(uint32_t w) { return cnt3(w, 0) + 5 * cnt3(w, 1) + 25 * cnt3(w, 2) + 125 * cnt3(w, 3) + 625 * cnt3(w, 4); }
MJ_HD uint32_t suffix5(uint32_t w) { return cnt3(w, 5) + 5 * cnt3(w, 6) + 25 * cnt3(w, 7) + 125 * cnt3(w, 8); }
// is the suit word (counts 0..4) a valid pattern?  Two dependent LDS reads.
MJ_HD bool lut_valid(const Lut &L, uint32_t w)
{
  MJ_STAT(n_lut);
  uint32_t s = suffix5(w);
  uint32_t row = L.rowid[prefix5(w)];
  return (L.bitmap[row * 20 + (s >> 5)] >> (s & 31)) & 1u;
}
// The decomposition records of the three numbered suits of a hand, every table read of one kind issued together:
// the probe (two LDS reads per suit), the key's number (two small global reads per suit), the first record (one
// global read per suit; it also says how many records the key has).  n[s] = number of records (0 = the suit is not
// a valid pattern), rec0[s] = the first one, key[s] = where the others are (recs[4 key + i]): they are read only when
// they are used, so that the usual hand with one decomposition per suit keeps few values alive.
MJ_HD void lut_records3(const Lut &L, const uint32_t h[4], int n[3], uint32_t rec0[3], uint32_t key[3])
{
  uint32_t p[3], sfx[3], row[3], word[3];
#pragma unroll
  for (int s = 0; s < 3; s++) { p[s] = prefix5(h[s]); sfx[s] = suffix5(h[s]); row[s] = L.rowid[p[s]]; }
#pragma unroll
  for (int s = 0; s < 3; s++) word[s] = L.bitmap[row[s] * 20 + (sfx[s] >> 5)];
#pragma unroll
  for (int s = 0; s < 3; s++) {
    const bool valid = (word[s] >> (sfx[s] & 31)) & 1u;
    const uint32_t k = (uint32_t)L.base[p[s]] + L.rowrank[row[s] * 20 + (sfx[s] >> 5)] + (uint32_t)popc32(word[s] & ((1u << (sfx[s] & 31)) - 1u));
    key[s] = valid ? k : 0u;
    n[s] = valid ? 1 : 0;
  }
#pragma unroll
  for (int s = 0; s < 3; s++) {
    rec0[s] = L.recs[4 * (size_t)key[s]];
    n[s] = n[s] ? 1 + (int)(rec0[s] >> 28 & 3u) : 0;
  }
}

MJ_HD int tiles_in(uint32_t w)      // sum of the nine 3-bit fields
{
  uint32_t a = (w & 0007007007u) + ((w >> 3) & 0007007007u) + ((w >> 6) & 0007007007u);   // three 9-bit sums
  return (int)((a & 0x1FF) + ((a >> 9) & 0x1FF) + ((a >> 18) & 0x1FF));
}
// honors: valid when every count is 0 or 3, or exactly one is 2
MJ_HD bool honors_valid(uint32_t w)
{
  uint32_t b0 = w & O111, b1 = (w >> 1) & O111, b2 = (w >> 2) & O111;
  uint32_t one = b0 & ~b1 & ~b2, two = b1 & ~b0 & ~b2, four = b2;
  return one == 0 && four == 0 && popc32(two) <= 1;
}
MJ_HD uint32_t fields_eq(uint32_t w, int v)   // bit 3r set where field r == v
{
  uint32_t b0 = w & O111, b1 = (w >> 1) & O111, b2 = (w >> 2) & O111;
  uint32_t m0 = (v & 1) ? b0 : ~b0, m1 = (v & 2) ? b1 : ~b1, m2 = (v & 4) ? b2 : ~b2;
  return m0 & m1 & m2 & O111;
}
MJ_HD uint32_t fields_nonzero(uint32_t w) { return (w | (w >> 1) | (w >> 2)) & O111; }
// compress the bits at positions 0,3,6,...,24 of nine fields into 9 consecutive bits (four fold-and-mask steps)
MJ_HD uint32_t squeeze9(uint32_t m)
{
  uint32_t x = m & O111;
  x = (x | (x >> 2)) & 0x10C30C3u;      // pairs   at 0,6,12,18 and bit 24
  x = (x | (x >> 4)) & 0x100F00Fu;      // nibbles at 0,12      and bit 24
  x = (x | (x >> 8)) & 0x10000FFu;      // byte    at 0         and bit 24
  return (x | (x >> 16)) & 0x1FFu;
}

// kinds (34-bit mask) of which the seat owns four, concealed and melds together
MJ_HD int meld_count(uint32_t m, int k)
{
  int t = m_type(m), b = m_kind(m);
  if (t == MT_CHI) return (k >= b && k <= b + 2) ? 1 : 0;
  if (t == MT_PON) return k == b ? 3 : 0;
  if (t >= MT_MINKAN) return k == b ? 4 : 0;
  return 0;
}
// element su of four values without an indexed array (arrays indexed at run time live in scratch memory)
MJ_HD uint32_t pick4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, int su)
{
  uint32_t lo = (su & 1) ? a1 : a0, hi = (su & 1) ? a3 : a2;
  return (su & 2) ? hi : lo;
}
MJ_HD uint64_t pick4q(uint64_t a0, uint64_t a1, uint64_t a2, uint64_t a3, int su)
{
  uint64_t lo = (su & 1) ? a1 : a0, hi = (su & 1) ? a3 : a2;
  return (su & 2) ? hi : lo;
}
MJ_HD int hand_count(const uint32_t h[4], int k) { int su = suit_of(k); return cnt3(pick4(h[0], h[1], h[2], h[3], su), rank_of(k, su)); }

MJ_HD bool suit_valid(const Lut &L, int su, uint32_t w) { return su == 3 ? honors_valid(w) : lut_valid(L, w); }
// ranks r (bit r) with count < 4 whose addition makes the suit word valid
MJ_HD uint32_t suit_addmask(const Lut *Lp, int su, uint32_t w)
{
  const Lut &L = *Lp;
  uint32_t m = 0;
  if (su < 3) {
    // nine probes whose keys differ from the key of w by one power of five: adding to ranks 1..5 changes the
    // prefix (five row reads), adding to ranks 6..9 keeps the row of w and moves along it.  All row reads are
    // issued before the first bitmap read, so the LDS latency is paid twice, not eighteen times.
    const uint32_t p = prefix5(w), sfx = suffix5(w);
    const uint32_t full = (w >> 2) & O111;                 // fields that already hold four
    uint32_t row[6];
    row[5] = L.rowid[p];
    uint32_t pw = 1;
#pragma unroll
    for (int r = 0; r < 5; r++) { row[r] = L.rowid[p + ((full >> (3 * r) & 1u) ? 0u : pw)]; pw *= 5; }   // full field: no probe
    pw = 1;
#pragma unroll
    for (int r = 0; r < 9; r++) {
      const uint32_t sr = (r < 5 || (full >> (3 * r) & 1u)) ? sfx : sfx + pw;
      if (r >= 5) pw *= 5;
      const uint32_t bit = (L.bitmap[row[r < 5 ? r : 5] * 20 + (sr >> 5)] >> (sr & 31)) & 1u;
      m |= bit << r;
    }
    m &= ~squeeze9(full);
  } else {
    // honors: a single becomes the pair, a pair becomes a triplet; the other counts must already fit
    uint32_t one = fields_eq(w, 1), two = fields_eq(w, 2), four = (w >> 2) & O111;
    if (four) return 0;
    int n1 = popc32(one), n2 = popc32(two);
    uint32_t cand = 0;
    if (n1 == 1 && n2 == 0) cand = one;                 // 1 -> 2: the pair
    else if (n1 == 0 && n2 == 1) cand = two;            // 2 -> 3, no pair left here
    else if (n1 == 0 && n2 == 2) cand = two;            // one of two pairs becomes a triplet
    else if (n1 == 1 && n2 == 1) cand = 0;              // a single and a pair can not both be fixed
    m = squeeze9(cand) & 0x7Fu;
  }
  return m;
}
// honors: ranks whose removal leaves the counts valid (closed form, like honors_valid)
MJ_HD uint32_t honors_submask(uint32_t w)
{
  uint32_t one = fields_eq(w, 1), two = fields_eq(w, 2), three = fields_eq(w, 3), four = (w >> 2) & O111;
  int n1 = popc32(one), n2 = popc32(two), n4 = popc32(four);
  uint32_t cand = 0;
  if (n1 == 1 && n4 == 0 && n2 <= 1) cand |= one;       // the lone single goes
  if (n1 == 0 && n4 == 0 && n2 == 0) cand |= three;     // a triplet becomes the pair
  if (n1 == 0 && n4 == 1 && n2 <= 1) cand |= four;      // the four become a triplet
  return squeeze9(cand) & 0x7Fu;
}
// what the search for tenpai-keeping discards asks about one numbered suit: is it valid, which ranks can take a tile
// (count < 4) so that it becomes valid, which held ranks can lose a tile so that it is valid
struct SuitFacts { uint32_t valid, addm, subm; };
// kinds of which the seat owns four once its melds are counted: the melds' tiles are added to the concealed
// counts field by field (a kind never exceeds four copies, so no field overflows)
MJ_HD uint64_t own4_mask(const uint32_t h[4], uint64_t meldw, int n_meld)
{
  uint32_t o0 = h[0], o1 = h[1], o2 = h[2], o3 = h[3];
  for (int j = 0; j < n_meld; j++) {
    const uint32_t m = meld_at(meldw, j);
    const int t = m_type(m), b = m_kind(m), su = suit_of(b);
    const uint32_t add = (t == MT_CHI ? 0111u : t == MT_PON ? 3u : 4u) << (3 * rank_of(b, su));
    o0 += su == 0 ? add : 0u; o1 += su == 1 ? add : 0u; o2 += su == 2 ? add : 0u; o3 += su == 3 ? add : 0u;
  }
  return (uint64_t)squeeze9((o0 >> 2) & O111) | (uint64_t)squeeze9((o1 >> 2) & O111) << 9 |
         (uint64_t)squeeze9((o2 >> 2) & O111) << 18 | (uint64_t)squeeze9((o3 >> 2) & O111) << 27;
}
// cheap necessary condition for seven pairs: kinds held at least twice
MJ_HD int kinds_held_twice(const uint32_t h[4])
{
  int n = 0;
#pragma unroll
  for (int su = 0; su < 4; su++) n += popc32(((h[su] >> 1) | (h[su] >> 2)) & O111);
  return n;
}
struct SpecialCounts { int c1, c2, c3, c4, yao_tiles, total; };
MJ_HD SpecialCounts special_counts(const uint32_t h[4])
{
  SpecialCounts c = {0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int su = 0; su < 4; su++) {
    c.c1 += popc32(fields_eq(h[su], 1)); c.c2 += popc32(fields_eq(h[su], 2));
    c.c3 += popc32(fields_eq(h[su], 3)); c.c4 += popc32(fields_eq(h[su], 4));
    c.yao_tiles += su == 3 ? tiles_in(h[3]) : cnt3(h[su], 0) + cnt3(h[su], 8);
  }
  c.total = c.c1 + 2 * c.c2 + 3 * c.c3 + 4 * c.c4;
  return c;
}
MJ_HD uint64_t kinds_where(const uint32_t h[4], int v)     // 34-bit mask of kinds whose count equals v
{
  uint64_t m = 0;
#pragma unroll
  for (int su = 0; su < 4; su++) m |= (uint64_t)squeeze9(fields_eq(h[su], v)) << (9 * su);
  return m;
}

// at most `limit` (0 or 1) tiles that are neither terminals nor honors (no counting: masks only)
MJ_HD bool few_simples(const uint32_t h[4], int limit)
{
  const uint32_t inner = ~(7u | 7u << 24);
  const uint32_t a = h[0] & inner, b = h[1] & inner, c = h[2] & inner;
  if (limit == 0) return (a | b | c) == 0;
  const int kinds = popc32(fields_nonzero(a)) + popc32(fields_nonzero(b)) + popc32(fields_nonzero(c));
  return kinds <= 1 && ((a | b | c) & (O111 * 6u)) == 0;          // one kind at most, held once
}
MJ_HD uint32_t hand_facts(const Lut &L, const uint32_t h[4])     // four probes
{
  uint32_t f = 0;
#pragma unroll
  for (int s = 0; s < 4; s++) {
    f |= (uint32_t)(tiles_in(h[s]) % 3) << (2 * s);
    if (suit_valid(L, s, h[s])) f |= 1u << (8 + s);
  }
  return f;
}
MJ_HD uint32_t facts_update(const Lut &L, uint32_t f, int su, uint32_t hw)      // suit su changed to hw: one probe
{
  const uint32_t rem = (uint32_t)(tiles_in(hw) % 3);
  const bool v = su == 3 ? honors_valid(hw) : lut_valid(L, hw);
  return (f & ~(3u << (2 * su)) & ~(1u << (8 + su))) | rem << (2 * su) | (v ? 1u << (8 + su) : 0u);
}

// Waits of a (13 - 3*n_meld)-tile hand: kinds whose addition completes it and of which the seat owns fewer than
// four, in bits 0..33; the hand's facts ride along in bits 40..52 (see above).  waits_from_facts takes the facts as
// given, waits_of looks them up.
MJ_HD uint64_t waits_from_facts(const Lut *Lp, uint32_t h0, uint32_t h1, uint32_t h2, uint32_t h3, uint64_t meldw, int n_meld,
                                uint32_t facts)
{
  MJ_STAT(n_waits);
  const uint32_t h[4] = {h0, h1, h2, h3};
  uint64_t w = 0;
  int r1 = 0, r2 = 0;
  uint32_t bad = 0, nonzero = 0;
#pragma unroll
  for (int s = 0; s < 4; s++) {
    const int rem = (int)(facts >> (2 * s) & 3u);
    r1 += rem == 1; r2 += rem == 2;
    if (rem != 0) nonzero |= 1u << s;
    if (rem == 1 || !(facts >> (8 + s) & 1u)) bad |= 1u << s;
  }
  // standard form: the suit that takes the tile has remainder 1 (it then holds the pair) or is one of two
  // suits with remainder 2; every other suit must already be valid.  With remainder pattern (1,0,0,0) the
  // remainder-1 suit is the only "bad" one allowed; with (2,2,0,0) either no suit is bad (both are candidates)
  // or one of the two is (then it must take the tile).
  MJ_RB(wfc, ((r1 == 1 && r2 == 0) || (r1 == 0 && r2 == 2)) && (bad & (bad - 1)) == 0);
  if (((r1 == 1 && r2 == 0) || (r1 == 0 && r2 == 2)) && (bad & (bad - 1)) == 0) {
    uint32_t cands = bad ? (bad & nonzero) : nonzero;
    while (cands) {
      MJ_STAT(n_waits_cand);
      const int s = __builtin_ctz(cands);
      cands &= cands - 1;
      w |= (uint64_t)suit_addmask(Lp, s, pick4(h0, h1, h2, h3, s)) << (9 * s);
    }
  }
  MJ_RE(wfc, PR_WF_CAND);
  MJ_RB(wfs, n_meld == 0 && (kinds_held_twice(h) == 6 || few_simples(h, 0)));
  if (n_meld == 0 && (kinds_held_twice(h) == 6 || few_simples(h, 0))) {
    SpecialCounts c = special_counts(h);
    if (c.c2 == 6 && c.c1 == 1 && c.c3 == 0 && c.c4 == 0) w |= kinds_where(h, 1);      // seven pairs
    if (c.yao_tiles == c.total && c.c3 == 0 && c.c4 == 0) {                            // thirteen orphans
      if (c.c1 == 13) w |= K_YAOCHU;
      else if (c.c1 == 11 && c.c2 == 1) w |= K_YAOCHU & ~(kinds_where(h, 1) | kinds_where(h, 2));
    }
  }
  MJ_RE(wfs, PR_WF_SPECIAL);
  if (w) w &= ~own4_mask(h, meldw, n_meld);
  return w | (uint64_t)facts << FACTS_SHIFT | W_FACTS_VALID;
}
MJ_HD uint64_t waits_of(const Lut *Lp, uint32_t h0, uint32_t h1, uint32_t h2, uint32_t h3, uint64_t meldw, int n_meld)
{
  const uint32_t h[4] = {h0, h1, h2, h3};
  return waits_from_facts(Lp, h0, h1, h2, h3, meldw, n_meld, hand_facts(*Lp, h));
}

// Kinds whose discard leaves the 14 - 3*n_meld tiles of a hand tenpai (non-empty waits_of).  Per suit, three
// facts are looked up once for the hand as it is: valid, ranks that may leave (the rest stays valid), ranks that
// may come (the suit becomes valid and the kind is not exhausted).  A discard from suit s1 whose wait lies in
// another suit s2 is then pure mask logic; only a discard whose wait lies in its own suit needs a lookup per
// candidate, and that case needs the three other suits to be valid already.
// With exact == false only the cheap necessary conditions are tested: the result is 0 (no discard keeps tenpai)
// or TD_UNKNOWN.
MJ_HD uint64_t tenpai_discards_from_facts(const Lut *Lp, uint32_t h0, uint32_t h1, uint32_t h2, uint32_t h3, uint64_t meldw,
                                          int n_meld, bool exact, uint32_t facts)
{
  const Lut &L = *Lp;
  MJ_STAT(n_tenpai);
  const uint32_t h[4] = {h0, h1, h2, h3};
  const uint32_t remp = facts & 0xFFu;
  uint32_t valid = 0;
  int t1 = 0, t2 = 0;
#pragma unroll
  for (int s = 0; s < 4; s++) {
    const int r = (int)(remp >> (2 * s) & 3u);
    t1 += r == 1; t2 += r == 2;
    if (r != 1 && (facts >> (8 + s) & 1u)) valid |= 1u << s;
  }
  uint64_t out = 0;
  const bool special = n_meld == 0 && (kinds_held_twice(h) >= 6 || few_simples(h, 1));
  const bool standard = popc32(~valid & 15u) <= 2;      // a discard and a draw touch at most two suits
  if (!exact) return (standard || special) ? TD_UNKNOWN : 0;
  if (standard) MJ_STAT(n_tp_standard);
  MJ_RB(tps, standard);
  if (standard) {                       // rare: the search proper
    // the three numbered suits' neighbours: one read each from the table of all patterns, issued together
    const uint32_t e0 = L.nb[prefix5(h0) + 3125u * suffix5(h0)], e1 = L.nb[prefix5(h1) + 3125u * suffix5(h1)];
    const uint32_t e2 = L.nb[prefix5(h2) + 3125u * suffix5(h2)];
    SuitFacts f0, f1, f2;
    f0.valid = e0 & 1u; f0.addm = e0 >> 1 & 0x1FFu; f0.subm = e0 >> 10 & 0x1FFu;
    f1.valid = e1 & 1u; f1.addm = e1 >> 1 & 0x1FFu; f1.subm = e1 >> 10 & 0x1FFu;
    f2.valid = e2 & 1u; f2.addm = e2 >> 1 & 0x1FFu; f2.subm = e2 >> 10 & 0x1FFu;
    // numbered ranks whose tile may leave with the wait in the same suit (tiles the seat owns four of not yet excluded)
    const uint64_t xchg = (uint64_t)(e0 >> 19 & 0x1FFu) | (uint64_t)(e1 >> 19 & 0x1FFu) << 9 | (uint64_t)(e2 >> 19 & 0x1FFu) << 18 | K_HONORS;
    const uint64_t full = own4_mask(h, meldw, n_meld);
    const uint64_t subp = (uint64_t)f0.subm | (uint64_t)f1.subm << 9 | (uint64_t)f2.subm << 18 | (uint64_t)honors_submask(h3) << 27;
    const uint64_t addp = ((uint64_t)f0.addm | (uint64_t)f1.addm << 9 | (uint64_t)f2.addm << 18 |
                           (uint64_t)suit_addmask(Lp, 3, h3) << 27) & ~full;
    uint32_t can_take = 0;
#pragma unroll
    for (int s = 0; s < 4; s++) if ((addp >> (9 * s)) & 0x1FF) can_take |= 1u << s;
    uint64_t own_suit = 0;              // held kinds whose discard has to be tried with the wait in the same suit
#pragma unroll
    for (int s1 = 0; s1 < 4; s1++) {
      if (h[s1] == 0) continue;
      const int rem1 = (int)(remp >> (2 * s1) & 3);
      // which suits may take the new tile when a tile leaves s1: the final remainders must be one 2 and three 0.
      // A suit that loses a tile goes 0 -> 2, 1 -> 0, 2 -> 1; one that gains a tile goes 0 -> 1, 1 -> 2, 2 -> 0.
      uint32_t feas = 0;
      if (t1 == 0 && t2 == 1) feas |= 1u << s1;                                  // the tile comes back into s1
#pragma unroll
      for (int s2 = 0; s2 < 4; s2++) {
        if (s2 == s1) continue;
        const int rem2 = (int)(remp >> (2 * s2) & 3);
        bool f = (rem1 == 0 && rem2 == 2 && t2 == 1 && t1 == 0) || (rem1 == 1 && rem2 == 1 && t1 == 2 && t2 == 0) ||
                 (rem1 == 1 && rem2 == 2 && t1 == 1 && t2 == 2);
        if (f) feas |= 1u << s2;
      }
      // the untouched suits must be valid as they are (at most one of them may be the one that takes the tile)
      const uint32_t bad_others = ~valid & 15u & ~(1u << s1);
      if (popc32(bad_others) > 1) continue;
      const uint64_t field = 0x1FFull << (9 * s1);
      // the wait lies in another suit s2: what stays in s1 must be valid, and s2 is the only suit that may be invalid
      uint32_t cand = feas & ~(1u << s1);
      if (bad_others) cand &= bad_others;
      if (cand & can_take) out |= subp & field;
      // the wait lies in s1 itself
      if ((feas >> s1 & 1) && bad_others == 0)
        own_suit |= (uint64_t)squeeze9(fields_nonzero(h[s1])) << (9 * s1);
    }
    own_suit &= ~out & xchg;
    MJ_RB(tpo, own_suit != 0);
    while (own_suit) {
      MJ_STAT(n_tp_own);
      const int k = ctz64(own_suit);
      own_suit &= own_suit - 1;
      const int su = suit_of(k), r = rank_of(k, su);
      const uint32_t g = pick4(h0, h1, h2, h3, su) - (1u << (3 * r));
      const uint32_t blocked = (uint32_t)(full >> (9 * su) & 0x1FF) & ~(1u << r);     // the discarded kind is owned one less
      if (suit_addmask(Lp, su, g) & ~blocked) out |= kbit(k);
    }
    MJ_RE(tpo, PR_TP_OWN);
  }
  MJ_RE(tps, PR_TP_STD);
  MJ_RB(tpx, special);
  if (special) {
    // seven pairs and thirteen orphans in closed form: the counts of singles, pairs, triplets after the discard
    const SpecialCounts c = special_counts(h);
    if (c.c4 == 0) {
      const uint64_t one = kinds_where(h, 1), two = kinds_where(h, 2), three = kinds_where(h, 3);
      if (c.c3 == 0 && c.c2 == 6 && c.c1 == 2) out |= one;
      if (c.c3 == 0 && c.c2 == 7 && c.c1 == 0) out |= two;
      if (c.c3 == 1 && c.c2 == 5 && c.c1 == 1) out |= three;
      const int nonyao = c.total - c.yao_tiles;
      if (nonyao == 0) {
        if (c.c3 == 0 && c.c1 == 12 && c.c2 == 1) out |= one | two;
        if (c.c3 == 0 && c.c1 == 10 && c.c2 == 2) out |= two;
        if (c.c3 == 1 && c.c1 == 11 && c.c2 == 0) out |= three;
      } else if (nonyao == 1 && c.c3 == 0) {
        if ((c.c1 == 14 && c.c2 == 0) || (c.c1 == 12 && c.c2 == 1)) out |= one & ~K_YAOCHU;
      }
    }
  }
  MJ_RE(tpx, PR_TP_SPECIAL);
  return out;
}

MJ_HD uint64_t tenpai_discards_of(const Lut *Lp, uint32_t h0, uint32_t h1, uint32_t h2, uint32_t h3, uint64_t meldw, int n_meld,
                                  bool exact)
{
  const uint32_t h[4] = {h0, h1, h2, h3};
  return tenpai_discards_from_facts(Lp, h0, h1, h2, h3, meldw, n_meld, exact, hand_facts(*Lp, h));
}

// ------------------------------------------------------------------ shanten
// Shanten number of a concealed hand with n_meld melds (paper section 3.2, observation scalars): -1 complete,
// 0 tenpai, ...  Standard form: 2 * need - max(2 m + min(t, need - m)) - head with need = 4 - n_meld, m sets and
// t partial sets summed over the four suits; each suit contributes, for every m, its largest t from the block
// tables of mj_tables.hpp (sh_suit for the numbered suits, sh_honor for the honors), with the head in at most one
// suit.  Seven pairs and thirteen orphans compete when there is no meld.
struct ShFront { int v[5]; };
MJ_HD ShFront sh_front(uint32_t e, int head)
{
  ShFront f;
#pragma unroll
  for (int m = 0; m < 5; m++) { int x = (int)(e >> (15 * head + 3 * m)) & 7; f.v[m] = x == 7 ? -64 : x; }
  return f;
}
MJ_HD ShFront sh_join(const ShFront &a, const ShFront &b)     // sets and partial sets of two disjoint groups of tiles
{
  ShFront c;
#pragma unroll
  for (int m = 0; m < 5; m++) {
    int best = -64;
#pragma unroll
    for (int i = 0; i <= m; i++) { int x = a.v[i] + b.v[m - i]; best = x > best ? x : best; }
    c.v[m] = best;
  }
  return c;
}
MJ_HD ShFront sh_max(const ShFront &a, const ShFront &b)
{
  ShFront c;
#pragma unroll
  for (int m = 0; m < 5; m++) c.v[m] = a.v[m] > b.v[m] ? a.v[m] : b.v[m];
  return c;
}
MJ_HD int sh_value(const ShFront &f, int need)                // max of 2 m + min(t, need - m) over m <= need
{
  int best = -64;
#pragma unroll
  for (int m = 0; m < 5; m++) {
    if (m > need || f.v[m] < 0) continue;
    int t = f.v[m] < need - m ? f.v[m] : need - m;
    best = 2 * m + t > best ? 2 * m + t : best;
  }
  return best;
}
MJ_HD int shanten_of(const uint32_t *sh_suit, const uint32_t *sh_honor, uint32_t h0, uint32_t h1, uint32_t h2, uint32_t h3,
                     int n_meld)
{
  const uint32_t hkey = (uint32_t)cnt3(h3, 0) + 5u * cnt3(h3, 1) + 25u * cnt3(h3, 2) + 125u * cnt3(h3, 3) + 625u * cnt3(h3, 4) +
                        3125u * cnt3(h3, 5) + 15625u * cnt3(h3, 6);
  const uint32_t e0 = sh_suit[prefix5(h0) + 3125u * suffix5(h0)], e1 = sh_suit[prefix5(h1) + 3125u * suffix5(h1)];
  const uint32_t e2 = sh_suit[prefix5(h2) + 3125u * suffix5(h2)], e3 = sh_honor[hkey];
  const int need = 4 - n_meld;
  const ShFront n0 = sh_front(e0, 0), n1 = sh_front(e1, 0), n2 = sh_front(e2, 0), n3 = sh_front(e3, 0);
  const ShFront g0 = sh_front(e0, 1), g1 = sh_front(e1, 1), g2 = sh_front(e2, 1), g3 = sh_front(e3, 1);
  const ShFront n01 = sh_join(n0, n1), n23 = sh_join(n2, n3);
  const ShFront g01 = sh_max(sh_join(g0, n1), sh_join(n0, g1)), g23 = sh_max(sh_join(g2, n3), sh_join(n2, g3));
  int sh = 2 * need - sh_value(sh_join(n01, n23), need);
  const int with_head = sh_value(sh_max(sh_join(g01, n23), sh_join(n01, g23)), need);
  if (with_head >= 0 && 2 * need - with_head - 1 < sh) sh = 2 * need - with_head - 1;
  if (n_meld == 0) {
    const uint32_t h[4] = {h0, h1, h2, h3};
    int pairs = kinds_held_twice(h), kinds = 0, yao = 0, yao_pair = 0;
#pragma unroll
    for (int su = 0; su < 4; su++) {
      const uint32_t nz = fields_nonzero(h[su]), two = ((h[su] >> 1) | (h[su] >> 2)) & O111;
      const uint32_t ym = su == 3 ? O111 : (1u | 1u << 24);     // the yaochu ranks of this suit
      kinds += popc32(nz);
      yao += popc32(nz & ym);
      if (two & ym) yao_pair = 1;
    }
    const int chiitoi = 6 - pairs + (kinds < 7 ? 7 - kinds : 0), kokushi = 13 - yao - yao_pair;
    sh = chiitoi < sh ? chiitoi : sh;
    sh = kokushi < sh ? kokushi : sh;
  }
  return sh;
}

// --------------------------------------------------------------- evaluation
struct HandIn {
  uint32_t h[4];        // concealed, winning tile included
  uint64_t meldw;
  int n_meld, win, flags, riichi, seat_wind, round_wind, n_ind, n_aka, kuitan;
  uint8_t ind[5], ura[5];
};
struct HandOut {
  uint64_t yaku;
  int32_t points;
  int han, fu, units, shape_ok, yaku_ok, n_dora, n_ura, n_aka;
};

MJ_HD int32_t up100(int32_t x) { return (x + 99) / 100 * 100; }
MJ_HD int32_t base_points(int han, int fu, int units)
{
  if (units > 0) return 8000 * units;
  if (han >= 13) return 8000;
  if (han >= 11) return 6000;
  if (han >= 8) return 4000;
  if (han >= 6) return 3000;
  if (han >= 5) return 2000;
  int32_t b = (int32_t)fu << (han + 2);
  return b > 2000 ? 2000 : b;
}
MJ_HD int32_t total_points(int32_t base, bool dealer, bool tsumo)
{
  if (!tsumo) return up100(base * (dealer ? 6 : 4));
  if (dealer) return 3 * up100(base * 2);
  return up100(base * 2) + 2 * up100(base);
}
MJ_HD int dora_of(int k)
{
  if (k < 27) { int su = k / 9, r = k - 9 * su; return 9 * su + (r == 8 ? 0 : r + 1); }
  if (k < 31) return k == 30 ? 27 : k + 1;
  return k == 33 ? 31 : k + 1;
}

// yaku bit numbers
enum { Y_RIICHI = 0, Y_DRIICHI, Y_IPPATSU, Y_TSUMO, Y_PINFU, Y_TANYAO, Y_IIPEIKOU, Y_HAKU, Y_HATSU, Y_CHUN, Y_SEATW,
       Y_ROUNDW, Y_RINSHAN, Y_CHANKAN, Y_HAITEI, Y_HOUTEI, Y_CHIITOI, Y_SANSHOKU, Y_ITTSU, Y_CHANTA, Y_TOITOI,
       Y_SANANKOU, Y_DOUKOU, Y_SANKANTSU, Y_HONROUTOU, Y_SHOUSANGEN, Y_HONITSU, Y_JUNCHAN, Y_RYANPEIKOU, Y_CHINITSU,
       Y_KOKUSHI = 32, Y_SUUANKOU, Y_DAISANGEN, Y_SHOUSUUSHII, Y_DAISUUSHII, Y_TSUUIISOU, Y_CHINROUTOU, Y_RYUUIISOU,
       Y_CHUUREN, Y_SUUKANTSU, Y_TENHOU, Y_CHIIHOU };
#define YB(x) (1ull << (x))
// han value classes, closed / open
constexpr uint64_t HC1 = YB(Y_RIICHI) | YB(Y_IPPATSU) | YB(Y_TSUMO) | YB(Y_PINFU) | YB(Y_TANYAO) | YB(Y_IIPEIKOU) |
                         YB(Y_HAKU) | YB(Y_HATSU) | YB(Y_CHUN) | YB(Y_SEATW) | YB(Y_ROUNDW) | YB(Y_RINSHAN) |
                         YB(Y_CHANKAN) | YB(Y_HAITEI) | YB(Y_HOUTEI);
constexpr uint64_t HC2 = YB(Y_DRIICHI) | YB(Y_CHIITOI) | YB(Y_SANSHOKU) | YB(Y_ITTSU) | YB(Y_CHANTA) | YB(Y_TOITOI) |
                         YB(Y_SANANKOU) | YB(Y_DOUKOU) | YB(Y_SANKANTSU) | YB(Y_HONROUTOU) | YB(Y_SHOUSANGEN);
constexpr uint64_t HC3 = YB(Y_HONITSU) | YB(Y_JUNCHAN) | YB(Y_RYANPEIKOU);
constexpr uint64_t HC6 = YB(Y_CHINITSU);
constexpr uint64_t HO1 = YB(Y_TANYAO) | YB(Y_HAKU) | YB(Y_HATSU) | YB(Y_CHUN) | YB(Y_SEATW) | YB(Y_ROUNDW) |
                         YB(Y_RINSHAN) | YB(Y_CHANKAN) | YB(Y_HAITEI) | YB(Y_HOUTEI) | YB(Y_SANSHOKU) | YB(Y_ITTSU) |
                         YB(Y_CHANTA);
constexpr uint64_t HO2 = YB(Y_TOITOI) | YB(Y_SANANKOU) | YB(Y_DOUKOU) | YB(Y_SANKANTSU) | YB(Y_HONROUTOU) |
                         YB(Y_SHOUSANGEN) | YB(Y_HONITSU) | YB(Y_JUNCHAN);
constexpr uint64_t HO5 = YB(Y_CHINITSU);

struct EvalCtx {
  bool menzen, tsumo, dealer;
  int riichi, flags, n_meld, n_dora, n_ura, n_aka, seat_k, round_k, win;
  uint64_t situ, first_ym, colour_y, colour_ym;
  bool found;
  HandOut best;
};

MJ_HD void offer(EvalCtx &c, uint64_t y, uint64_t ym, int fu)
{
  HandOut r;
  ym |= c.first_ym;
  if (ym) {
    r.units = popc64(ym >> 32); r.yaku = ym; r.han = 13 * r.units; r.fu = 0;
    r.points = total_points(8000 * r.units, c.dealer, c.tsumo);
  } else {
    y |= c.situ;
    int han = c.menzen ? popc64(y & HC1) + 2 * popc64(y & HC2) + 3 * popc64(y & HC3) + 6 * popc64(y & HC6)
                       : popc64(y & HO1) + 2 * popc64(y & HO2) + 5 * popc64(y & HO5);
    if (han == 0) return;
    han += c.n_dora + c.n_ura + c.n_aka;
    r.units = 0; r.yaku = y; r.han = han; r.fu = fu;
    r.points = total_points(base_points(han, fu, 0), c.dealer, c.tsumo);
  }
  bool better;
  if (!c.found) better = true;
  else if (r.points != c.best.points) better = r.points > c.best.points;
  else if (r.han != c.best.han) better = r.han > c.best.han;
  else if (r.fu != c.best.fu) better = r.fu > c.best.fu;
  else better = r.yaku > c.best.yaku;
  if (better) {
    c.best.yaku = r.yaku; c.best.points = r.points; c.best.han = r.han; c.best.fu = r.fu; c.best.units = r.units;
    c.found = true;
  }
}

// one decomposition as masks
struct Decomp {
  uint64_t trip_c, trip_o, kan_c, kan_o;   // kinds
  uint32_t crun[3], orun[3];               // packed multiplicities of run starts, concealed / called
  int pair;
};

MJ_HD void add_record(Decomp &d, uint32_t rec, int su)
{
  int p = (int)(rec & 15);
  if (p) d.pair = 9 * su + p - 1;
#pragma unroll
  for (int j = 0; j < 4; j++) {
    uint32_t s = (rec >> (4 + 5 * j)) & 31u;
    if (s == 31u) continue;
    int r = (int)(s & 15);
    if (s & 16) d.trip_c |= kbit(9 * su + r);
    else d.crun[su] += 1u << (3 * r);
  }
}

// value of one decomposition under one way of waiting
MJ_HD void eval_placed(EvalCtx &c, const Decomp &d, uint64_t trip_c, uint64_t trip_o, int wait_fu, bool two_sided)
{
  MJ_STAT(n_placed);
  uint64_t y = c.colour_y, ym = c.colour_ym;
  uint32_t run[3] = {d.crun[0] + d.orun[0], d.crun[1] + d.orun[1], d.crun[2] + d.orun[2]};
  int n_run = tiles_in(run[0]) + tiles_in(run[1]) + tiles_in(run[2]);
  uint64_t trips = trip_c | trip_o | d.kan_c | d.kan_o;
  uint64_t concealed = trip_c | d.kan_c, kans = d.kan_c | d.kan_o;
  uint64_t pairb = kbit(d.pair);
  int n_conc = popc64(concealed), n_kan = popc64(kans);

  y |= (trips >> 31 & 7) << Y_HAKU;
  if (trips & kbit(c.seat_k)) y |= YB(Y_SEATW);
  if (trips & kbit(c.round_k)) y |= YB(Y_ROUNDW);
  int pair_fu = 0;
  if (pairb & K_DRAGONS) pair_fu += 2;
  if (d.pair == c.seat_k) pair_fu += 2;
  if (d.pair == c.round_k) pair_fu += 2;
  bool pinfu = c.menzen && n_run == 4 && pair_fu == 0 && two_sided;
  if (pinfu) y |= YB(Y_PINFU);
  if (c.menzen) {
    int doubles = 0;
#pragma unroll
    for (int s = 0; s < 3; s++) {
      uint32_t x = (d.crun[s] >> 1) & 0333333333u;
      doubles += popc32(x & O111) + 2 * popc32(x & (O111 << 1));
    }
    if (doubles >= 2) y |= YB(Y_RYANPEIKOU);
    else if (doubles == 1) y |= YB(Y_IIPEIKOU);
  }
  uint32_t rm0 = fields_nonzero(run[0]), rm1 = fields_nonzero(run[1]), rm2 = fields_nonzero(run[2]);
  if (rm0 & rm1 & rm2) y |= YB(Y_SANSHOKU);
  const uint32_t ITTSU = 1u | 1u << 9 | 1u << 18;
  if ((rm0 & ITTSU) == ITTSU || (rm1 & ITTSU) == ITTSU || (rm2 & ITTSU) == ITTSU) y |= YB(Y_ITTSU);
  const uint32_t ENDS = 1u | 1u << 18;          // runs 123 and 789
  bool every_yao = ((rm0 | rm1 | rm2) & ~ENDS) == 0 && (trips & ~K_YAOCHU) == 0 && (pairb & K_YAOCHU) != 0;
  if (every_yao && n_run >= 1) y |= ((trips | pairb) & K_HONORS) ? YB(Y_CHANTA) : YB(Y_JUNCHAN);
  if (n_run == 0) y |= YB(Y_TOITOI);
  if (n_conc == 3) y |= YB(Y_SANANKOU);
  uint32_t t0 = (uint32_t)(trips & 0x1FF), t1 = (uint32_t)(trips >> 9 & 0x1FF), t2 = (uint32_t)(trips >> 18 & 0x1FF);
  if (t0 & t1 & t2) y |= YB(Y_DOUKOU);
  if (n_kan == 3) y |= YB(Y_SANKANTSU);
  int n_dragon = popc64(trips & K_DRAGONS), n_wind = popc64(trips & K_WINDS);
  if (n_dragon == 2 && (pairb & K_DRAGONS)) y |= YB(Y_SHOUSANGEN);

  if (n_conc == 4) ym |= YB(Y_SUUANKOU);
  if (n_dragon == 3) ym |= YB(Y_DAISANGEN);
  if (n_wind == 3 && (pairb & K_WINDS)) ym |= YB(Y_SHOUSUUSHII);
  if (n_wind == 4) ym |= YB(Y_DAISUUSHII);
  if (n_kan == 4) ym |= YB(Y_SUUKANTSU);

  int fu;
  if (pinfu) fu = c.tsumo ? 20 : 30;
  else {
    fu = 20 + ((c.menzen && !c.tsumo) ? 10 : 0) + (c.tsumo ? 2 : 0) + pair_fu + wait_fu;
    fu += 2 * popc64(trip_o & ~K_YAOCHU) + 4 * popc64(trip_o & K_YAOCHU) + 4 * popc64(trip_c & ~K_YAOCHU) +
          8 * popc64(trip_c & K_YAOCHU) + 8 * popc64(d.kan_o & ~K_YAOCHU) + 16 * popc64(d.kan_o & K_YAOCHU) +
          16 * popc64(d.kan_c & ~K_YAOCHU) + 32 * popc64(d.kan_c & K_YAOCHU);
    if (!c.menzen && fu == 20) fu = 30;
    fu = (fu + 9) / 10 * 10;
  }
  offer(c, y, ym, fu);
}

// all ways the winning tile can sit in this decomposition
MJ_HD void eval_decomp(EvalCtx &c, const Decomp &d)
{
  int w = c.win;
  if (d.pair == w) eval_placed(c, d, d.trip_c, d.trip_o, 2, false);
  if (d.trip_c & kbit(w)) {
    if (c.tsumo) eval_placed(c, d, d.trip_c, d.trip_o, 0, false);
    else eval_placed(c, d, d.trip_c & ~kbit(w), d.trip_o | kbit(w), 0, false);
  }
  if (w < 27) {
    int su = suit_of(w), r = rank_of(w, su);
    uint32_t cr = pick4(d.crun[0], d.crun[1], d.crun[2], 0u, su);
    bool mid = r >= 1 && r <= 7 && cnt3(cr, r - 1) > 0;                 // run r-1, r, r+1
    bool low = r <= 6 && cnt3(cr, r) > 0;                               // run r, r+1, r+2
    bool high = r >= 2 && cnt3(cr, r - 2) > 0;                          // run r-2, r-1, r
    bool edge = (low && r == 6) || (high && r == 2);
    bool two = (low && r != 6) || (high && r != 2);
    if (mid || edge) eval_placed(c, d, d.trip_c, d.trip_o, 2, false);
    if (two) eval_placed(c, d, d.trip_c, d.trip_o, 0, true);
  }
}

MJ_HD void eval_hand(const Lut *Lp, const HandIn &q, HandOut &out)
{
  const Lut &L = *Lp;
  MJ_STAT(n_eval);
  out.yaku = 0; out.points = 0; out.han = out.fu = out.units = out.shape_ok = out.yaku_ok = 0;
  out.n_dora = out.n_ura = out.n_aka = 0;
  int n_meld = q.n_meld, w = q.win;
  if (n_meld > 4 || w >= 34 || hand_count(q.h, w) == 0) return;
  int total = tiles_in(q.h[0]) + tiles_in(q.h[1]) + tiles_in(q.h[2]) + tiles_in(q.h[3]);
  if (total != 14 - 3 * n_meld) return;
  // counts above four make no valid pattern
  uint32_t over = 0;
#pragma unroll
  for (int s = 0; s < 4; s++) over |= ((q.h[s] >> 2) & O111) & ((q.h[s] | (q.h[s] >> 1)) & O111);
  if (over) return;

  // per-suit probes
  int nd[3]; uint32_t rec0[3], key[3];
  int n_pair_suits = 0; bool std_ok = true;
  lut_records3(L, q.h, nd, rec0, key);
#pragma unroll
  for (int s = 0; s < 3; s++) {
    if (nd[s] == 0) std_ok = false;
    if (tiles_in(q.h[s]) % 3 == 2) n_pair_suits++;
  }
  if (!honors_valid(q.h[3])) std_ok = false;
  uint32_t hon_pair = fields_eq(q.h[3], 2), hon_trip = fields_eq(q.h[3], 3);
  if (hon_pair) n_pair_suits++;
  if (n_pair_suits != 1) std_ok = false;

  // special forms
  uint32_t pairs = 0, other = 0; uint64_t present = 0;
#pragma unroll
  for (int s = 0; s < 4; s++) {
    uint32_t e2 = fields_eq(q.h[s], 2), nz = fields_nonzero(q.h[s]);
    pairs += popc32(e2); other += popc32(nz & ~e2 & ~fields_eq(q.h[s], 1));
    present |= (uint64_t)squeeze9(nz) << (9 * s);
  }
  bool chiitoi = n_meld == 0 && pairs == 7 && popc64(present) == 7;
  bool kokushi = n_meld == 0 && (present & ~K_YAOCHU) == 0 && popc64(present) == 13 && pairs == 1 && other == 0;
  if (!std_ok && !chiitoi && !kokushi) return;
  out.shape_ok = 1;
  MJ_STAT(n_eval_shape);

  // context shared by every interpretation
  EvalCtx c;
  c.found = false;
  c.best.yaku = 0; c.best.points = 0; c.best.han = c.best.fu = c.best.units = 0;
  c.n_meld = n_meld; c.win = w; c.flags = q.flags;
  c.tsumo = q.flags & 1; c.dealer = q.seat_wind == 0;
  c.seat_k = 27 + q.seat_wind; c.round_k = 27 + q.round_wind;
  Decomp base;
  base.trip_c = base.trip_o = base.kan_c = base.kan_o = 0;
  base.crun[0] = base.crun[1] = base.crun[2] = 0;
  base.orun[0] = base.orun[1] = base.orun[2] = 0;
  base.pair = 63;
  uint32_t all[4] = {q.h[0], q.h[1], q.h[2], q.h[3]};
  c.menzen = true;
  for (int j = 0; j < n_meld; j++) {
    uint32_t m = meld_at(q.meldw, j);
    int t = m_type(m), k = m_kind(m), su = suit_of(k), r = rank_of(k, su);
    if (t != MT_ANKAN) c.menzen = false;
    uint32_t add_all, add_run = 0;
    if (t == MT_CHI) { add_run = 1u << (3 * r); add_all = 0111u << (3 * r); }
    else if (t == MT_PON) { base.trip_o |= kbit(k); add_all = 3u << (3 * r); }
    else if (t == MT_ANKAN) { base.kan_c |= kbit(k); add_all = 4u << (3 * r); }
    else { base.kan_o |= kbit(k); add_all = 4u << (3 * r); }
#pragma unroll
    for (int i = 0; i < 4; i++) all[i] += su == i ? add_all : 0u;
#pragma unroll
    for (int i = 0; i < 3; i++) base.orun[i] += su == i ? add_run : 0u;
  }
  c.riichi = c.menzen ? q.riichi : 0;
  c.n_dora = c.n_ura = 0;
  for (int i = 0; i < q.n_ind && i < 5; i++) {
    c.n_dora += hand_count(all, dora_of(q.ind[i]));
    if (c.riichi) c.n_ura += hand_count(all, dora_of(q.ura[i]));
  }
  c.n_aka = q.n_aka;
  int f = q.flags;
  uint64_t situ = 0;
  if (c.riichi == 1) situ |= YB(Y_RIICHI);
  if (c.riichi == 2) situ |= YB(Y_DRIICHI);
  if (c.riichi && (f & 2)) situ |= YB(Y_IPPATSU);
  if (c.tsumo && c.menzen) situ |= YB(Y_TSUMO);
  if (c.tsumo && (f & 4)) situ |= YB(Y_RINSHAN);
  if (!c.tsumo && (f & 8)) situ |= YB(Y_CHANKAN);
  if (c.tsumo && (f & 16) && !(f & 4)) situ |= YB(Y_HAITEI);
  if (!c.tsumo && (f & 32) && !(f & 8)) situ |= YB(Y_HOUTEI);
  c.situ = situ;
  c.first_ym = ((f & 64) && c.tsumo && n_meld == 0 && !(f & 4)) ? YB(c.dealer ? Y_TENHOU : Y_CHIIHOU) : 0;

  // yaku of the tile multiset alone
  {
    const uint32_t TERM = 7u | 7u << 24;
    bool s0 = all[0] != 0, s1 = all[1] != 0, s2 = all[2] != 0, hon = all[3] != 0;
    int n_suits = (int)s0 + (int)s1 + (int)s2;
    uint32_t suited = all[0] | all[1] | all[2];
    bool no_term = (suited & TERM) == 0, only_term = (suited & ~TERM) == 0;
    uint64_t y = 0, ym = 0;
    if (no_term && !hon && (c.menzen || q.kuitan)) y |= YB(Y_TANYAO);
    if (n_suits == 1 && hon) y |= YB(Y_HONITSU);
    if (n_suits == 1 && !hon) y |= YB(Y_CHINITSU);
    if (only_term && hon && n_suits >= 1) y |= YB(Y_HONROUTOU);
    if (n_suits == 0) ym |= YB(Y_TSUUIISOU);
    if (only_term && !hon) ym |= YB(Y_CHINROUTOU);
    const uint32_t GREEN_S = 7u << 3 | 7u << 6 | 7u << 9 | 7u << 15 | 7u << 21;   // 2 3 4 6 8 of souzu
    if (all[0] == 0 && all[1] == 0 && (all[2] & ~GREEN_S) == 0 && (all[3] & ~(7u << 15)) == 0) ym |= YB(Y_RYUUIISOU);
    c.colour_y = y; c.colour_ym = ym;
  }

  if (std_ok) {
    // nine gates: closed, one suit, at least 3 1 1 1 1 1 1 1 3
    uint64_t gates = 0;
    if (n_meld == 0 && (c.colour_y & YB(Y_CHINITSU))) {
      uint32_t x = all[0] | all[1] | all[2];        // only one of them is non-zero
      bool each = fields_nonzero(x) == O111;
      if (each && cnt3(x, 0) >= 3 && cnt3(x, 8) >= 3) gates = YB(Y_CHUUREN);
    }
    c.colour_ym |= gates;
    if (hon_pair) base.pair = 27 + (ctz64(hon_pair) / 3);
    uint32_t ht = hon_trip;
    while (ht) { int b = ctz64(ht); ht &= ht - 1; base.trip_c |= kbit(27 + b / 3); }
    for (int i0 = 0; i0 < nd[0]; i0++)
      for (int i1 = 0; i1 < nd[1]; i1++)
        for (int i2 = 0; i2 < nd[2]; i2++) {
          MJ_STAT(n_decomp);
          Decomp d = base;
          add_record(d, i0 == 0 ? rec0[0] : L.recs[4 * (size_t)key[0] + i0], 0);
          add_record(d, i1 == 0 ? rec0[1] : L.recs[4 * (size_t)key[1] + i1], 1);
          add_record(d, i2 == 0 ? rec0[2] : L.recs[4 * (size_t)key[2] + i2], 2);
          eval_decomp(c, d);
        }
    c.colour_ym &= ~gates;
  }
  if (chiitoi) offer(c, c.colour_y | YB(Y_CHIITOI), c.colour_ym, 25);
  if (kokushi) offer(c, 0, YB(Y_KOKUSHI), 0);

  if (c.found) {
    out.yaku = c.best.yaku; out.points = c.best.points; out.han = c.best.han; out.fu = c.best.fu;
    out.units = c.best.units; out.yaku_ok = 1;
    out.n_dora = c.n_dora; out.n_ura = c.n_ura; out.n_aka = c.n_aka;
  }
}

}  // namespace mj
