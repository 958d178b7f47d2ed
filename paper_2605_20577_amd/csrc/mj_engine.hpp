// The phase machine of one environment (deal, draw, discard, calls, kans,
// wins, draws, kyoku and game transitions, legal masks) on the packed state of
// mj_core.hpp.  One GPU lane runs one environment; see mj_core.hpp for the
// host-compilation note.  Rules: paper section 3.2 (standard four-player
// East-South Riichi, red / no-red variants, single / east / half modes,
// illegal action => termination); the concrete readings (action numbering,
// simultaneous responses, wall geography, tie-breaks) are this library's and
// are listed in the design document.
#pragma once
#include <cassert>
#include "mj_core.hpp"

namespace mj {

// checked in the host build of this code (tests, sanitizers), nothing on the device
#ifdef __HIP_DEVICE_COMPILE__
#define MJ_HOST_ASSERT(x) ((void)0)
#else
#define MJ_HOST_ASSERT(x) assert(x)
#endif

// pins a per-lane value in a vector register at this point (otherwise the compiler turns bit tests of it back into
// booleans that each occupy a scalar register pair for as long as they live)
#ifdef __HIP_DEVICE_COMPILE__
#define MJ_KEEP_IN_VGPR(x) asm volatile("" : "+v"(x))
#else
#define MJ_KEEP_IN_VGPR(x) ((void)0)
#endif

struct Ctx {
  Env e;
  Lut L;               // table pointers, by value (see BlockMem)
  Rules R;
  Glob g;
  uint32_t env_id;
  bool need_deal;      // set when a step ends in "deal the next kyoku": the caller shuffles and deals
  bool need_turn;      // the seat to move still needs its legal mask (step_finish)
  uint32_t live_word;  // the wall word that holds the next live tile, loaded at the start of the step ...
  int live_ptr;        // ... for this draw pointer (-1: nothing loaded)
};

// ------------------------------------------------------------- field access
MJ_HD uint32_t &HW(Ctx &c, int s, int su) { return c.e.hand[(int64_t)(s * 4 + su) * c.e.hs]; }
MJ_HD uint32_t &SW(Ctx &c, int s) { return c.e.seatw[(int64_t)s * c.e.hs]; }
MJ_HD uint64_t &MELDW(Ctx &c, int s) { return c.e.meld[(int64_t)s * c.e.hs]; }
MJ_HD uint64_t &WAITS(Ctx &c, int s) { return c.e.waits[(int64_t)s * c.e.hs]; }
MJ_HD uint64_t &DK(Ctx &c, int s) { return c.e.dk[(int64_t)s * c.e.hs]; }
MJ_HD uint64_t &TD(Ctx &c) { return c.e.tdisc[0]; }
MJ_HD uint64_t &MASK(Ctx &c, int s, int w) { return c.e.mask[(int64_t)(s * 2 + w) * c.e.hs]; }
MJ_HD int32_t &SCORE(Ctx &c, int s) { return c.e.score[(int64_t)s * c.e.hs]; }
MJ_HD int32_t &DELTA(Ctx &c, int s) { return c.e.delta[(int64_t)s * c.e.hs]; }
// tile i of wall buffer `sel`
MJ_HD int wall_at(const Env &e, int sel, int i) { return (int)(e.wallw[(int64_t)(sel * 34 + (i >> 2)) * e.n] >> (8 * (i & 3)) & 255u); }
MJ_HD void wall_set(const Env &e, int sel, int i, int v)
{
  uint32_t &w = e.wallw[(int64_t)(sel * 34 + (i >> 2)) * e.n];
  w = (w & ~(255u << (8 * (i & 3)))) | (uint32_t)v << (8 * (i & 3));
}
MJ_HD int WALL(Ctx &c, int i) { return wall_at(c.e, c.g.wall_sel, i); }
MJ_HD uint8_t &RIVER(Ctx &c, int s, int i) { return c.e.river[(int64_t)(s * 32 + i) * c.e.n]; }

MJ_HD int swf(Ctx &c, int s, int pos, int bits) { return (int)sw_get(SW(c, s), pos, bits); }
MJ_HD void swf_set(Ctx &c, int s, int pos, int bits, int v) { SW(c, s) = sw_set(SW(c, s), pos, bits, (uint32_t)v); }

MJ_HD int count_of(Ctx &c, int s, int k) { int su = suit_of(k); return cnt3(HW(c, s, su), rank_of(k, su)); }
MJ_HD void hand_add(Ctx &c, int s, int k, int d)
{
  int su = suit_of(k);
  HW(c, s, su) += (uint32_t)d << (3 * rank_of(k, su));     // d may be negative: two's complement on the field
}
MJ_HD bool has_red(Ctx &c, int s, int k) { return is_five(k) && ((SW(c, s) >> (k / 9)) & 1u); }
MJ_HD int nonred_of(Ctx &c, int s, int k) { return count_of(c, s, k) - (has_red(c, s, k) ? 1 : 0); }
MJ_HD int concealed_total(Ctx &c, int s)
{
  return tiles_in(HW(c, s, 0)) + tiles_in(HW(c, s, 1)) + tiles_in(HW(c, s, 2)) + tiles_in(HW(c, s, 3));
}
MJ_HD int dealer_of(const Ctx &c) { return c.g.kyoku & 3; }
MJ_HD bool is_red_id(const Ctx &c, int id) { return (c.R.flags & F_RED) && (id == 16 || id == 52 || id == 88); }

MJ_HD void refresh_waits(Ctx &c, int s)
{
  WAITS(c, s) = waits_of(&c.L, HW(c, s, 0), HW(c, s, 1), HW(c, s, 2), HW(c, s, 3), MELDW(c, s), swf(c, s, SW_NMELD, 3));
}
MJ_HD int take_tile(Ctx &c, int s, int id)
{
  int k = id >> 2, red = is_red_id(c, id) ? 1 : 0;
  hand_add(c, s, k, 1);
  if (red) SW(c, s) |= 1u << (k / 9);
  return k | red << 6;
}
MJ_HD bool menzen_of(Ctx &c, int s)
{
  uint64_t mw = MELDW(c, s);
  int n = swf(c, s, SW_NMELD, 3);
  for (int j = 0; j < n; j++) if (m_type(meld_at(mw, j)) != MT_ANKAN) return false;
  return true;
}
MJ_HD void clear_masks(Ctx &c)
{
#pragma unroll
  for (int i = 0; i < 8; i++) c.e.mask[(int64_t)i * c.e.hs] = 0;
  c.g.actor_mask = 0;
}
MJ_HD void clear_first_and_ippatsu(Ctx &c)
{
#pragma unroll
  for (int s = 0; s < 4; s++) SW(c, s) &= ~((1u << SW_IPPATSU) | (1u << SW_FIRST));
}

// value of seat s winning on kind w now
MJ_HD void eval_seat(Ctx &c, int s, int w, bool tsumo, bool chankan, HandOut &out)
{
  HandIn q;
#pragma unroll
  for (int su = 0; su < 4; su++) q.h[su] = HW(c, s, su);
  if (!tsumo) { int su = suit_of(w); q.h[su] += 1u << (3 * rank_of(w, su)); }
  uint32_t sw = SW(c, s);
  q.meldw = MELDW(c, s);
  q.n_meld = (int)sw_get(sw, SW_NMELD, 3);
  q.win = w;
  int f = 0;
  if (tsumo) f |= 1;
  if (sw >> SW_IPPATSU & 1) f |= 2;
  if (tsumo && (c.g.kanflags & 1)) f |= 4;
  if (chankan) f |= 8;
  if (tsumo && c.g.live_left == 0 && !(c.g.kanflags & 1)) f |= 16;
  if (!tsumo && !chankan && c.g.live_left == 0) f |= 32;
  if (tsumo && (sw >> SW_FIRST & 1)) f |= 64;
  q.flags = f;
  q.riichi = (int)sw_get(sw, SW_RIICHI, 2);
  q.seat_wind = (s - dealer_of(c)) & 3;
  q.round_wind = c.g.kyoku >> 2;
  q.n_ind = c.g.n_dora;
#pragma unroll
  for (int i = 0; i < 5; i++) { q.ind[i] = WALL(c, 126 + i) >> 2; q.ura[i] = WALL(c, 131 + i) >> 2; }
  int aka = popc32(sw & 7u);
  for (int j = 0; j < q.n_meld; j++) aka += (int)(meld_at(q.meldw, j) >> 13 & 1u);
  if (!tsumo && !chankan && code_red(c.g.last_discard) && code_kind(c.g.last_discard) == w) aka++;
  if (chankan && code_red(c.g.kakan_tile)) aka++;
  q.n_aka = aka;
  q.kuitan = (c.R.flags & F_KUITAN) ? 1 : 0;
  MJ_RB(ev, true);
  eval_hand(&c.L, q, out);
  MJ_RE(ev, PR_EVAL);
}

// A complete hand certainly has a yaku when the situation alone gives one: riichi, a self-drawn closed hand, a win on
// a replacement tile or on the tile of a kan, or on the last tile.  (These are exactly the situational yaku that the
// evaluator adds to every interpretation, so "some interpretation has a yaku" holds without looking at the tiles.)
// Used where only the yes / no is needed, i.e. when a win is OFFERED; the value is computed when the win is taken.
MJ_HD bool sure_yaku(Ctx &c, int s, bool tsumo, bool chankan)
{
  const uint32_t sw = SW(c, s);
  const bool menzen = menzen_of(c, s);
  const bool rinshan = (c.g.kanflags & 1) != 0;
  if (menzen && (tsumo || sw_get(sw, SW_RIICHI, 2))) return true;
  if (tsumo ? (rinshan || c.g.live_left == 0) : (chankan || c.g.live_left == 0)) return true;
  return false;
}

MJ_HD bool furiten(Ctx &c, int s)
{
  uint32_t sw = SW(c, s);
  return (sw >> SW_FTEMP & 1) || (sw >> SW_FRIICHI & 1) || (WAITS(c, s) & DK(c, s)) != 0;
}
MJ_HD void mark_furiten(Ctx &c, int s)
{
  SW(c, s) |= sw_get(SW(c, s), SW_RIICHI, 2) ? (1u << SW_FRIICHI) : (1u << SW_FTEMP);
}

// a legal-action mask in two registers (no indexed array, so it never lands in scratch memory)
struct Mask2 { uint64_t w0, w1; };
MJ_HD void set_action(Mask2 &m, int a)
{
  uint64_t bit = 1ull << (a & 63);
  if (a < 64) m.w0 |= bit; else m.w1 |= bit;
}

// discards available from a hand (four suit words, red bits in sw), restricted to the kinds in `allowed`: the
// non-red discard of kind k is action k, so the set of held kinds IS the low part of the mask; red fives are
// patched in
MJ_HD void discard_bits(const uint32_t h[4], uint32_t sw, uint64_t allowed, Mask2 &m)
{
  uint64_t held = 0;
#pragma unroll
  for (int su = 0; su < 4; su++) {
    held |= (uint64_t)squeeze9(fields_nonzero(h[su])) << (9 * su);
    if (su < 3 && (sw >> su & 1u)) {                       // the red five of this suit is in the hand
      uint64_t five = kbit(9 * su + 4);
      if (allowed & five) m.w0 |= 1ull << (A_DISCARD_RED + su);
      if (cnt3(h[su], 4) == 1) held &= ~five;              // ... and it is the only five
    }
  }
  m.w0 |= held & allowed;
}

// legal actions of the seat to move; the seat's words are read once and handed to the helpers
MJ_HD void turn_mask(Ctx &c)
{
  MJ_STAT(n_turn);
  const int s = c.g.cur;
  Mask2 m = {0, 0};
  clear_masks(c);
  c.g.phase = PH_TURN;
  c.g.actor_mask = (uint8_t)(1 << s);
  const int drawn_k = c.g.drawn == 255 ? -1 : code_kind(c.g.drawn);
  const uint32_t sw = SW(c, s);
  const uint32_t h[4] = {HW(c, s, 0), HW(c, s, 1), HW(c, s, 2), HW(c, s, 3)};
  const uint64_t mw = MELDW(c, s), wfull = WAITS(c, s), waits = wfull & K_ALL;
  const int riichi = (int)sw_get(sw, SW_RIICHI, 2), n_meld = (int)sw_get(sw, SW_NMELD, 3);

  // Discards that keep the hand tenpai: needed for the riichi declaration and the discard that follows it, and
  // kept for the next step, where the discard then tells whether the seat's waits are empty without a search.
  // A seat in riichi can only discard the drawn tile, which gives back the hand it had: nothing to find out.
  bool menzen = true;
  for (int j = 0; j < n_meld; j++) if (m_type(meld_at(mw, j)) != MT_ANKAN) menzen = false;
  const bool may_riichi = !c.g.riichi_pending && !riichi && drawn_k >= 0 && menzen && SCORE(c, s) >= 1000 && c.g.live_left >= 4;
  // The hand differs from the 13 - 3m tiles whose facts sit in the waits word by the tile drawn, or by the tiles a
  // call took (all of the called tile's suit): one probe brings the facts up to date.
  const int changed = drawn_k >= 0 ? drawn_k : (c.g.kuikae0 != 255 ? (int)c.g.kuikae0 : -1);
  uint32_t facts;
  MJ_RB(tmf, true);
  if ((wfull & W_FACTS_VALID) && changed >= 0) {
    const int cs = suit_of(changed);
    facts = facts_update(c.L, (uint32_t)(wfull >> FACTS_SHIFT) & 0xFFFu, cs, pick4(h[0], h[1], h[2], h[3], cs));
  } else facts = hand_facts(c.L, h);
  const bool exact = !riichi && (may_riichi || c.g.riichi_pending);        // the set itself is only searched for when
  uint64_t td = 0;                                                         // the mask needs it
  MJ_RE(tmf, PR_TM_FACTS);
  MJ_RB(tme, exact);
  if (exact) MJ_STAT(n_exact);
  if (exact) td = tenpai_discards_from_facts(&c.L, h[0], h[1], h[2], h[3], mw, n_meld, true, facts);
  TD(c) = (exact || riichi ? td | TD_VALID : 0) | (uint64_t)facts << FACTS_SHIFT | TD_FACTS;
  MJ_RE(tme, PR_TM_EXACT);
  MJ_RB(tmt, !c.g.riichi_pending && drawn_k >= 0 && (waits >> drawn_k & 1));
  if (MJ_RARE(!c.g.riichi_pending && drawn_k >= 0 && (waits >> drawn_k & 1))) {
    if (sure_yaku(c, s, true, false)) set_action(m, A_TSUMO);
    else {
      MJ_STAT(n_tsumo_eval);
      HandOut r;
      eval_seat(c, s, drawn_k, true, false, r);
      if (r.yaku_ok) set_action(m, A_TSUMO);
    }
  }
  MJ_RE(tmt, PR_TM_TSUMO);
  const bool kan_ok = !c.g.riichi_pending && drawn_k >= 0 && c.g.live_left > 0 && c.g.n_kan < 4;
  MJ_RB(tmr, riichi != 0);
  MJ_RB(tmb, riichi == 0);
  if (riichi) {
    if (code_red(c.g.drawn)) set_action(m, A_DISCARD_RED + drawn_k / 9);
    else set_action(m, A_DISCARD + drawn_k);
    if (kan_ok && hand_count(h, drawn_k) == 4) {
      // a concealed kan is allowed in riichi only when it leaves the waits as they were
      const int su = suit_of(drawn_k);
      const uint32_t four = 4u << (3 * rank_of(drawn_k, su));
      const uint64_t mw2 = mw | (uint64_t)m_make(MT_ANKAN, drawn_k, 0, 0, 0, 0) << (16 * n_meld);
      if ((waits_of(&c.L, h[0] - (su == 0 ? four : 0u), h[1] - (su == 1 ? four : 0u), h[2] - (su == 2 ? four : 0u),
                   h[3] - (su == 3 ? four : 0u), mw2, n_meld + 1) & K_ALL) == waits)
        set_action(m, A_KAN + drawn_k);
    }
  } else {
    uint64_t allowed = td;                                  // after the declaration: tenpai-keeping discards only
    if (!c.g.riichi_pending) {
      allowed = K_ALL;
      if (c.g.kuikae0 != 255) allowed &= ~kbit(c.g.kuikae0);
      if (c.g.kuikae1 != 255) allowed &= ~kbit(c.g.kuikae1);
    }
    discard_bits(h, sw, allowed, m);
    if (!c.g.riichi_pending) {
      uint64_t kans = 0;                                    // kinds that may be declared as a kan
#pragma unroll
      for (int su = 0; su < 4; su++) kans |= (uint64_t)squeeze9(fields_eq(h[su], 4)) << (9 * su);
      for (int j = 0; j < n_meld; j++) {
        const uint32_t ml = meld_at(mw, j);
        if (m_type(ml) == MT_PON && hand_count(h, m_kind(ml)) >= 1) kans |= kbit(m_kind(ml));
      }
      if (kan_ok) {                                         // KAN k is action 37 + k: bits 37..70
        m.w0 |= kans << A_KAN;
        m.w1 |= kans >> (64 - A_KAN);
      }
      if (td && may_riichi) set_action(m, A_RIICHI);
      if ((c.R.flags & F_ABORT) && (sw >> SW_FIRST & 1) && drawn_k >= 0) {
        uint64_t present = 0;
#pragma unroll
        for (int su = 0; su < 4; su++) present |= (uint64_t)squeeze9(fields_nonzero(h[su])) << (9 * su);
        if (popc64(present & K_YAOCHU) >= 9) set_action(m, A_KYUUSHU);
      }
    }
  }
  MJ_RE(tmr, PR_TM_RIICHI);
  MJ_RE(tmb, PR_TM_BITS);
  MASK(c, s, 0) = m.w0;
  MASK(c, s, 1) = m.w1;
}

MJ_HD void draw_live(Ctx &c, int s)
{
  c.g.cur = (uint8_t)s;
  int id = c.live_ptr == (int)c.g.draw_ptr ? (int)(c.live_word >> (8 * (c.g.draw_ptr & 3)) & 255u) : WALL(c, c.g.draw_ptr);
  c.live_ptr = -1;
  c.g.draw_ptr++;
  c.g.live_left--;
  c.g.kanflags &= (uint8_t)~1u;
  c.g.drawn = (uint8_t)take_tile(c, s, id);
}

// Fisher-Yates over the 136 tile ids: key (seed, env_id), counter (kyoku_serial, j, 0, 0); position i swaps
// with i + mulhi(r[i], 136 - i).  Plain per-environment form (the kernels do the same steps wave-cooperatively).
MJ_HD void shuffle_wall(Ctx &c)
{
  uint32_t serial = c.e.serial[0];
  for (int i = 0; i < 136; i++) wall_set(c.e, c.g.wall_sel, i, i);
  for (int j = 0; j < 34; j++) {
    uint32_t r[4];
    philox(serial, (uint32_t)j, 0, 0, c.R.seed, c.env_id, r);
#pragma unroll
    for (int t = 0; t < 4; t++) {
      int i = 4 * j + t;
      if (i >= 135) break;
      int k = i + (int)mulhi(r[t], (uint32_t)(136 - i));
      int a = WALL(c, i), b = WALL(c, k);
      wall_set(c.e, c.g.wall_sel, i, b); wall_set(c.e, c.g.wall_sel, k, a);
    }
  }
}

// a deal, part 1: every per-kyoku field back to its start (the final rank of the game is kept)
MJ_HD void deal_reset(Ctx &c)
{
  MJ_STAT(n_deal);
#pragma unroll
  for (int i = 0; i < 16; i++) c.e.hand[(int64_t)i * c.e.hs] = 0;
  for (int s = 0; s < 4; s++) {
    uint32_t keep = SW(c, s) & (3u << SW_RANK);
    SW(c, s) = keep | (255u << SW_RIDX) | (1u << SW_FIRST);
    MELDW(c, s) = 0;
    DK(c, s) = 0;
  }
  c.g.n_kan = 0; c.g.n_dora = 1; c.g.hist_len = 0;
  c.g.riichi_pending = 0; c.g.kanflags = 0;
  c.g.last_discard = 255; c.g.last_discarder = 255; c.g.kakan_tile = 255;
  c.g.kuikae0 = c.g.kuikae1 = 255;
  c.g.first_wind = 255; c.g.same_wind_cnt = 0;
  c.g.cur = (uint8_t)dealer_of(c);
  c.g.draw_ptr = 52; c.g.live_left = 70; c.g.drawn = 255;
}
// part 2: 4 x 13 tiles from the wall; the seat with seat wind j takes wall[13j .. 13j+12]
MJ_HD void deal_hands(Ctx &c)
{
  int dealer = dealer_of(c);
  for (int j = 0; j < 4; j++) {
    int s = (dealer + j) & 3;
    for (int t = 0; t < 13; t++) take_tile(c, s, WALL(c, 13 * j + t));
  }
}
// part 3: the waits of the four 13-tile hands;  part 4: the dealer draws (the mask follows in step_finish)
MJ_HD void deal_waits(Ctx &c)
{
  for (int s = 0; s < 4; s++) refresh_waits(c, s);
}
MJ_HD void deal_first_draw(Ctx &c)
{
  draw_live(c, dealer_of(c));
  c.need_deal = false;
  c.need_turn = true;
}
MJ_HD void step_finish(Ctx &c)
{
  if (c.need_turn) turn_mask(c);
  c.need_turn = false;
}
// whole deal from the environment's own wall in HBM
MJ_HD void deal(Ctx &c, bool reshuffle)
{
  if (reshuffle) shuffle_wall(c);
  deal_reset(c);
  deal_hands(c);
  deal_waits(c);
  deal_first_draw(c);
  step_finish(c);
}

MJ_HD void new_game(Ctx &c)
{
  for (int s = 0; s < 4; s++) {
    SCORE(c, s) = c.R.start_score;
    SW(c, s) = 0;                                        // final rank 0
  }
  c.g.kyoku = 0; c.g.honba = 0; c.g.kyotaku = 0; c.g.terminated = 0;
  c.need_deal = true;
}

MJ_HD void clear_result(Ctx &c)
{
  c.g.end_type = 0; c.g.winners = 0; c.g.loser = 255; c.g.tenpai_mask = 0;
#pragma unroll
  for (int s = 0; s < 4; s++) {
    c.e.resw[(int64_t)s * c.e.n] = 0;
    c.e.yaku[(int64_t)s * c.e.n] = 0;
    c.e.gain[(int64_t)s * c.e.n] = 0;
  }
}
MJ_HD void credit(Ctx &c, int s, int32_t x) { SCORE(c, s) += x; DELTA(c, s) += x; }

MJ_HD void finish_kyoku(Ctx &c, bool renchan, bool honba_up)
{
  int last = c.R.mode == 0 ? 0 : c.R.mode == 1 ? 3 : 7;
  bool over = c.R.mode == 0;
  const int32_t sc0[4] = {SCORE(c, 0), SCORE(c, 1), SCORE(c, 2), SCORE(c, 3)};
  for (int s = 0; s < 4; s++) if (sc0[s] < 0) over = true;
  if ((c.R.flags & F_ENDGAME) && c.R.mode != 0) {
    // end of game by points: see MJ_F_ENDGAME
    const int dealer = dealer_of(c), limit = last + 4;
    const int32_t sd = pick4((uint32_t)sc0[0], (uint32_t)sc0[1], (uint32_t)sc0[2], (uint32_t)sc0[3], dealer);
    int32_t top = sc0[0];
    bool lead = true;
    for (int s = 0; s < 4; s++) {
      top = sc0[s] > top ? sc0[s] : top;
      if (s != dealer && sc0[s] >= sd) lead = false;
    }
    if (c.g.kyoku >= last) {
      if (!renchan) { if (top >= 30000 || c.g.kyoku == limit) over = true; }
      else if ((lead && sd >= 30000) || (c.g.kyoku > last && top >= 30000)) over = true;
    }
  } else if (!renchan && c.g.kyoku == last) over = true;
  if (honba_up) { if (c.g.honba < 255) c.g.honba++; } else c.g.honba = 0;
  if (!renchan && !over) c.g.kyoku++;
  if (over) {
    int32_t sc[4] = {SCORE(c, 0), SCORE(c, 1), SCORE(c, 2), SCORE(c, 3)};
    int top = 0;
    for (int s = 1; s < 4; s++) if (sc[s] > sc[top]) top = s;
    int32_t sticks = 1000 * (int32_t)c.g.kyotaku;
    credit(c, top, sticks);
    sc[top] += sticks;
    c.g.kyotaku = 0;
    for (int s = 0; s < 4; s++) {
      int r = 0;
      for (int o = 0; o < 4; o++) r += (sc[o] > sc[s] || (sc[o] == sc[s] && o < s)) ? 1 : 0;
      swf_set(c, s, SW_RANK, 2, r);
    }
    c.g.terminated = 1; c.g.phase = PH_TERMINAL;
    clear_masks(c);
    return;
  }
  c.e.serial[0]++;
  c.need_deal = true;
}

// MJ_F_PAO: who fed the last exposed set of winner s's three dragons / four winds (-1: nobody is liable).  The meld
// word keeps the melds in the order they were made, each with the seat it was claimed from.
MJ_HD int pao_seat(Ctx &c, int s, uint64_t yaku)
{
  const int big3 = (int)(yaku >> Y_DAISANGEN & 1), big4 = (int)(yaku >> Y_DAISUUSHII & 1);
  if (!(big3 | big4)) return -1;
  const int lo = big3 ? 31 : 27, need = big3 ? 3 : 4;
  const uint64_t mw = MELDW(c, s);
  const int nm = swf(c, s, SW_NMELD, 3);
  int cnt = 0;
  uint32_t last = 0;
  for (int j = 0; j < nm; j++) {
    const uint32_t m = meld_at(mw, j);
    const int k = m_kind(m);
    if (k >= lo && k < lo + need) { cnt++; last = m; }         // honors are never part of a run
  }
  if (cnt != need || m_type(last) == MT_ANKAN) return -1;
  return (s + (int)(last >> 9 & 3)) & 3;
}

MJ_HD void win(Ctx &c, int winners, bool tsumo, int loser, int w, bool chankan)
{
  int dealer = dealer_of(c);
  clear_result(c);
  c.g.end_type = tsumo ? 1 : 2;
  c.g.winners = (uint8_t)winners;
  c.g.loser = tsumo ? 255 : (uint8_t)loser;
  // the sticks go to the only winner, or to the first winner after the loser
  int stick_seat = 0;
  if (tsumo) stick_seat = ctz64((uint64_t)winners);
  else for (int d = 3; d >= 1; d--) if (winners >> ((loser + d) & 3) & 1) stick_seat = (loser + d) & 3;
  int32_t honba = c.g.honba;
  for (int s = 0; s < 4; s++) {
    if (!(winners >> s & 1)) continue;
    HandOut r;
    eval_seat(c, s, w, tsumo, chankan, r);
    c.e.yaku[(int64_t)s * c.e.n] = r.yaku;
    c.e.resw[(int64_t)s * c.e.n] = (uint64_t)(uint8_t)r.han | (uint64_t)(uint8_t)r.fu << 8 | (uint64_t)r.units << 16 |
                                   (uint64_t)r.n_dora << 24 | (uint64_t)r.n_ura << 32 | (uint64_t)r.n_aka << 40;
    int32_t base = base_points(r.han, r.fu, r.units), got = 0;
    int liable = -1;
    if ((c.R.flags & F_PAO) && r.units) liable = pao_seat(c, s, r.yaku);
    if (liable >= 0 && (tsumo || liable != loser)) {
      // one unit of the hand is the liable seat's: all of it (and the counter bonus) on a self-draw, half of it on
      // a ron off somebody else, who pays the other half, the bonus and whatever else the hand is worth
      const int32_t mult = s == dealer ? 6 : 4, part = 8000 * mult, other = base - 8000;
      if (tsumo) {
        got = part + 300 * honba;
        credit(c, liable, -got);
        if (other > 0)
          for (int o = 0; o < 4; o++) {
            if (o == s) continue;
            const int32_t x = (s == dealer || o == dealer) ? other * 2 : other;
            credit(c, o, -x);
            got += x;
          }
      } else {
        const int32_t from_loser = part / 2 + other * mult + 300 * honba;
        credit(c, liable, -(part / 2));
        credit(c, loser, -from_loser);
        got = part / 2 + from_loser;
      }
    } else if (tsumo) {
      for (int o = 0; o < 4; o++) {
        if (o == s) continue;
        int32_t x = ((s == dealer || o == dealer) ? up100(base * 2) : up100(base)) + 100 * honba;
        credit(c, o, -x);
        got += x;
      }
    } else {
      got = up100(base * (s == dealer ? 6 : 4)) + 300 * honba;
      credit(c, loser, -got);
    }
    if (s == stick_seat) { got += 1000 * (int32_t)c.g.kyotaku; c.g.kyotaku = 0; }
    credit(c, s, got);
    c.e.gain[(int64_t)s * c.e.n] = got;
  }
  bool renchan = winners >> dealer & 1;
  finish_kyoku(c, renchan, renchan);
}

MJ_HD void exhaustive_draw(Ctx &c)
{
  clear_result(c);
  c.g.end_type = 3;
  int T = 0;
  for (int s = 0; s < 4; s++) if ((WAITS(c, s) & K_ALL) != 0 || swf(c, s, SW_RIICHI, 2)) T |= 1 << s;
  c.g.tenpai_mask = (uint8_t)T;
  int n = popc32((uint32_t)T);
  // MJ_F_NAGASHI: seats that discarded terminals and honors only (the set of discarded kinds says so) and whose
  // discards nobody took (every open meld names the seat it took from)
  int N = 0;
  if (c.R.flags & F_NAGASHI) {
    for (int s = 0; s < 4; s++) if (!(DK(c, s) & ~K_YAOCHU)) N |= 1 << s;
    if (N)
      for (int o = 0; o < 4; o++) {
        const uint64_t mw = MELDW(c, o);
        const int nm = swf(c, o, SW_NMELD, 3);
        for (int j = 0; j < nm; j++) {
          const uint32_t m = meld_at(mw, j);
          if (m_type(m) != MT_ANKAN) N &= ~(1 << ((o + (int)(m >> 9 & 3)) & 3));
        }
      }
  }
  if (N) {
    const int dealer = dealer_of(c);
    c.g.end_type = 10;
    c.g.winners = (uint8_t)N;
    for (int w = 0; w < 4; w++) if (N >> w & 1) {
      int32_t got = 0;
      for (int o = 0; o < 4; o++) if (o != w) {
        const int32_t pay = (w == dealer || o == dealer) ? 4000 : 2000;
        credit(c, o, -pay); got += pay;
      }
      credit(c, w, got);
      c.e.gain[(int64_t)w * c.e.n] = got;
    }
  } else if (n >= 1 && n <= 3) {
    int32_t get = 3000 / n, give = 3000 / (4 - n);
    for (int s = 0; s < 4; s++) credit(c, s, (T >> s & 1) ? get : -give);
  }
  finish_kyoku(c, T >> dealer_of(c) & 1, true);
}
MJ_HD void abortive_draw(Ctx &c, int type)
{
  clear_result(c);
  c.g.end_type = (uint8_t)type;
  finish_kyoku(c, true, true);
}

// indicators of earlier open / added kans that wait to be turned are turned now (see MJ_F_KANDORA_LATE)
MJ_HD void turn_pending_indicators(Ctx &c)
{
  c.g.n_dora = (uint8_t)(c.g.n_dora + (c.g.kanflags >> 1 & 1));
  c.g.kanflags &= (uint8_t)~2u;
}

// the replacement draw that completes any kan (the mask follows in step_finish); `open` = a kan from a discard or
// a tile added to a pon, whose indicator waits for the seat's discard when the rules say so
MJ_HD void kan_draw(Ctx &c, bool open)
{
  int s = c.g.cur;
  swf_set(c, s, SW_KANBY, 3, swf(c, s, SW_KANBY, 3) + 1);
  if ((c.R.flags & F_KANDORA_LATE) && open) c.g.kanflags |= 2;
  else c.g.n_dora++;
  int id = WALL(c, 122 + c.g.n_kan);
  c.g.n_kan++;
  c.g.live_left--;
  clear_first_and_ippatsu(c);
  c.g.drawn = (uint8_t)take_tile(c, s, id);
  c.g.kanflags |= 1;
  c.g.kakan_tile = 255;
}

// The discard was not won on: a pending riichi is established and paid for.  Returns the type of the abortive
// draw that is now due (0 = none).
MJ_HD int settle_discard(Ctx &c)
{
  int d = c.g.last_discarder;
  const bool riichi_now = c.g.riichi_pending != 0;
  if (c.g.riichi_pending) {
    credit(c, d, -1000);
    c.g.kyotaku++;
    uint32_t sw = SW(c, d);
    sw = sw_set(sw, SW_RIICHI, 2, c.g.riichi_pending);
    sw |= 1u << SW_IPPATSU;
    sw = sw_set(sw, SW_RIDX, 8, sw_get(sw, SW_NRIVER, 6) - 1);
    SW(c, d) = sw;
    c.g.riichi_pending = 0;
  }
  if (c.R.flags & F_ABORT) {
    if (c.g.same_wind_cnt == 4) return 5;
    // four riichi can only become true with the riichi that this discard establishes, four kans only with four kans
    // on the table: the seats' words are looked at in those two cases only
    if (MJ_RARE(riichi_now || c.g.n_kan == 4)) {
      bool all_riichi = true, one_seat = false;
      for (int s = 0; s < 4; s++) {
        uint32_t sw = SW(c, s);
        if (!sw_get(sw, SW_RIICHI, 2)) all_riichi = false;
        if (sw_get(sw, SW_KANBY, 3) == 4) one_seat = true;
      }
      if (all_riichi) return 6;
      if (c.g.n_kan == 4 && !one_seat) return 7;
    }
  }
  return 0;
}

// can seat o win on kind k discarded (or added to a kan) by someone else?  A fitting tile that can not be
// won on leaves the seat furiten.
MJ_HD bool ron_option(Ctx &c, int o, int k, bool chankan)
{
  if (!(WAITS(c, o) >> k & 1)) return false;
  bool ok = false;
  if (!furiten(c, o)) {
    if (MJ_USUAL(sure_yaku(c, o, false, chankan))) ok = true;
    else {
      MJ_STAT(n_ron_eval);
      HandOut r;
      eval_seat(c, o, k, false, chankan, r);
      ok = r.yaku_ok;
    }
  }
  if (!ok) mark_furiten(c, o);
  return ok;
}

// Responses live in word 1 of a mask (actions 74..84 are its bits 10..20), so a seat's options are one 32-bit value.
constexpr uint32_t R_BIT(int a) { return 1u << (a - 64); }
// pon / open kan of kind (su, r) by a seat with control word sw and counts hw in that suit
MJ_HD uint32_t pon_kan_options(const Ctx &c, int su, int r, uint32_t sw, uint32_t hw)
{
  uint32_t m = 0;
  if (!sw_get(sw, SW_RIICHI, 2) && c.g.live_left > 0) {
    const int have = cnt3(hw, r);
    const int total = 13 - 3 * (int)sw_get(sw, SW_NMELD, 3);      // a seat that is not on turn holds exactly this many
    const bool red_held = su < 3 && r == 4 && (sw >> su & 1u);
    const int nonred = have - (red_held ? 1 : 0);
    if (total - have > 0) {
      if (nonred >= 2) m |= R_BIT(A_PON);
      if (red_held && nonred >= 1) m |= R_BIT(A_PON_RED);
    }
    if (have >= 3 && c.g.n_kan < 4) m |= R_BIT(A_MINKAN);
  }
  return m;
}
// chi of rank r of a numbered suit by the next seat
MJ_HD uint32_t chi_options(const Ctx &c, int su, int r, uint32_t sw, uint32_t hw)
{
  uint32_t m = 0;
  if (!sw_get(sw, SW_RIICHI, 2) && c.g.live_left > 0 && su < 3) {
    const int have = cnt3(hw, r);
    const int total = 13 - 3 * (int)sw_get(sw, SW_NMELD, 3);
    const bool red_in_suit = sw >> su & 1u;
#pragma unroll
    for (int pos = 0; pos < 3; pos++) {
      int lo = r - pos;
      if (lo < 0 || lo > 6) continue;
      int ra = pos == 0 ? lo + 1 : lo, rb = pos == 2 ? lo + 1 : lo + 2;       // the two ranks taken from the hand
      int ca = cnt3(hw, ra), cb = cnt3(hw, rb);
      if (ca == 0 || cb == 0) continue;
      int extra = 0;
      if (pos == 0 && r + 3 <= 8) extra = cnt3(hw, r + 3);
      if (pos == 2 && r - 3 >= 0) extra = cnt3(hw, r - 3);
      if (total - 2 - have - extra <= 0) continue;
      bool five_used = ra == 4 || rb == 4;
      int na = ca - ((ra == 4 && red_in_suit) ? 1 : 0), nb = cb - ((rb == 4 && red_in_suit) ? 1 : 0);
      if (na >= 1 && nb >= 1) m |= R_BIT(A_CHI_L) << pos;
      if (five_used && red_in_suit) m |= R_BIT(A_CHI_L_RED) << pos;
    }
  }
  return m;
}

// seat s puts the tile (kind k, red flag) into its river; everything that follows from it comes later.
// The three words it changes are read together, changed in registers and written once; returns the suit word of the
// hand after the discard and, in was_riichi, whether the seat is in riichi.
MJ_HD uint32_t apply_discard(Ctx &c, int s, int k, int red, bool &was_riichi)
{
  turn_pending_indicators(c);
  const int su = suit_of(k);
  uint32_t sw = SW(c, s);
  uint32_t hw = HW(c, s, su);
  const uint64_t dk = DK(c, s);
  hw -= 1u << (3 * rank_of(k, su));
  was_riichi = sw_get(sw, SW_RIICHI, 2) != 0;
  if (red) sw &= ~(1u << (k / 9));
  int nr = (int)sw_get(sw, SW_NRIVER, 6);
  // at most 30 discards per seat and kyoku (4 (n - 1) <= 70 live draws + 3 seats x 16 claims), so 32 entries suffice
  MJ_HOST_ASSERT(nr < 32);
  RIVER(c, s, nr) = (uint8_t)(k | red << 6);
  sw = sw_set(sw, SW_NRIVER, 6, nr + 1);
  sw &= ~(1u << SW_FTEMP);
  if (sw_get(sw, SW_RIICHI, 2)) sw &= ~(1u << SW_IPPATSU);
  if ((sw >> SW_FIRST & 1) && c.g.same_wind_cnt != 255) {
    if (k >= 27 && k <= 30 && (c.g.same_wind_cnt == 0 || k == c.g.first_wind)) { c.g.first_wind = (uint8_t)k; c.g.same_wind_cnt++; }
    else c.g.same_wind_cnt = 255;
  }
  sw &= ~(1u << SW_FIRST);
  HW(c, s, su) = hw;
  DK(c, s) = dk | kbit(k);
  SW(c, s) = sw;
  c.g.kuikae0 = c.g.kuikae1 = 255;
  c.g.last_discard = (uint8_t)(k | red << 6);
  c.g.last_discarder = (uint8_t)s;
  c.g.drawn = 255;
  return hw;
}

MJ_HD void remove_tiles(Ctx &c, int s, int k, int n_nonred, int take_red)
{
  hand_add(c, s, k, -(n_nonred + take_red));
  if (take_red) SW(c, s) &= ~(1u << (k / 9));
}
MJ_HD void push_meld(Ctx &c, int s, uint32_t m)
{
  int j = swf(c, s, SW_NMELD, 3);
  MELDW(c, s) |= (uint64_t)m << (16 * j);
  swf_set(c, s, SW_NMELD, 3, j + 1);
}

// seat s takes the last discard with action a; returns true for an open kan (replacement draw due).
// The words it touches are read once, changed in registers and written once.
MJ_HD bool apply_call(Ctx &c, int s, int a)
{
  const int d = c.g.last_discarder, k = code_kind(c.g.last_discard), cred = code_red(c.g.last_discard);
  const int from_rel = (d - s) & 3, su = suit_of(k), r = rank_of(k, su);
  uint32_t sws[4];
#pragma unroll
  for (int t = 0; t < 4; t++) sws[t] = SW(c, t);
  const uint32_t sw_d = pick4(sws[0], sws[1], sws[2], sws[3], d);
  uint32_t sw = pick4(sws[0], sws[1], sws[2], sws[3], s);
  uint32_t hw = HW(c, s, su);
  uint64_t mw = MELDW(c, s);
  RIVER(c, d, (int)sw_get(sw_d, SW_NRIVER, 6) - 1) = (uint8_t)(c.g.last_discard | 0x80);      // the called tile, marked
  c.g.cur = (uint8_t)s;
  c.g.drawn = 255;
  c.g.kanflags &= (uint8_t)~1u;
  const bool red_held = su < 3 && r == 4 && (sw >> su & 1u);
  int tr = 0;                        // the red five leaves the hand
  uint32_t gone, meld;               // tiles taken from the hand (3-bit fields), the meld record
  bool kan = false;
  if (a == A_PON || a == A_PON_RED) {
    tr = a == A_PON_RED;
    gone = 2u << (3 * r);
    meld = m_make(MT_PON, k, from_rel, 0, tr | cred, cred);
    c.g.kuikae0 = (uint8_t)k; c.g.kuikae1 = 255;
  } else if (a == A_MINKAN) {
    tr = red_held ? 1 : 0;
    gone = 3u << (3 * r);
    meld = m_make(MT_MINKAN, k, from_rel, 0, tr | cred, cred);
    kan = true;
  } else {
    const int v = a - A_CHI_L, pos = v % 3, lo = r - pos;
    tr = v >= 3 ? 1 : 0;
    gone = (0111u << (3 * lo)) & ~(1u << (3 * r));          // one each of the run's ranks except the called one
    meld = m_make(MT_CHI, k - pos, from_rel, pos, tr | cred, cred);
    c.g.kuikae0 = (uint8_t)k;
    c.g.kuikae1 = 255;
    if (pos == 0 && r + 3 <= 8) c.g.kuikae1 = (uint8_t)(k + 3);
    if (pos == 2 && r - 3 >= 0) c.g.kuikae1 = (uint8_t)(k - 3);
  }
  HW(c, s, su) = hw - gone;
  if (tr) sw &= ~(1u << su);
  const int j = (int)sw_get(sw, SW_NMELD, 3);
  MELDW(c, s) = mw | (uint64_t)meld << (16 * j);
  sw = sw_set(sw, SW_NMELD, 3, (uint32_t)(j + 1));
  // any call ends everybody's first turn and ippatsu
#pragma unroll
  for (int t = 0; t < 4; t++) SW(c, t) = (t == s ? sw : sws[t]) & ~((1u << SW_IPPATSU) | (1u << SW_FIRST));
  return kan;
}

// KAN on the own turn; returns true for a concealed kan, false for a tile added to a pon (which can be robbed)
MJ_HD bool apply_own_kan(Ctx &c, int k)
{
  int s = c.g.cur;
  int tr = has_red(c, s, k) ? 1 : 0;
  c.g.drawn = 255;
  turn_pending_indicators(c);
  if (count_of(c, s, k) == 4) {
    remove_tiles(c, s, k, tr ? 3 : 4, tr);
    push_meld(c, s, m_make(MT_ANKAN, k, 0, 0, tr, 0));
    return true;
  }
  remove_tiles(c, s, k, tr ? 0 : 1, tr);
  uint64_t mw = MELDW(c, s);
  int n_meld = swf(c, s, SW_NMELD, 3);
  for (int j = 0; j < n_meld; j++) {
    uint32_t ml = meld_at(mw, j);
    if (m_type(ml) == MT_PON && m_kind(ml) == k) {
      uint32_t nm = (ml & ~7u) | MT_KAKAN | (tr ? 1u << 13 : 0u);
      mw = (mw & ~(0xFFFFull << (16 * j))) | (uint64_t)nm << (16 * j);
    }
  }
  MELDW(c, s) = mw;
  c.g.kakan_tile = (uint8_t)(k | tr << 6);
  return false;
}

MJ_HD int act_of(uint32_t acts, int s) { return (int)(int8_t)(acts >> (8 * s)); }

// seats (bit set in ron_offered) that were offered a win and let it go are furiten
MJ_HD void mark_passed_ron(Ctx &c, int ron_offered)
{
#pragma unroll
  for (int s = 0; s < 4; s++)
    if (ron_offered >> s & 1) mark_furiten(c, s);
}

// the action history (section 3.2, "Observation Space"): one entry per public action, action | seat << 8
// A 2-byte store of its own leaves the cache as a partial line of 32 to 64 bytes, so a kernel that runs many steps per
// launch gives the environment a staging ring in LDS (e.hstage: kHistRing entries, two bytes each at stride hs; entry
// i of the history sits in slot i mod kHistRing; *e.hbase = the number of entries of this kyoku that the row already
// holds): entries
// collect there and go to the row in one run of stores, hist_flush.  The kernel must flush at least every
// kHistFlushEvery steps: a step adds one entry, or up to three that end the kyoku (wins on one tile), and a deal
// starts the history afresh, so at most kHistFlushEvery + 2 entries wait in the ring.  71 B of HBM writes per env step
// became 28.
constexpr int kHistRing = 64, kHistFlushEvery = 32;
static_assert(kHistFlushEvery + 2 <= kHistRing && (kHistRing & (kHistRing - 1)) == 0, "the ring holds a flush interval");
// writes the staged entries to the row.  (After a deal *hbase may still hold the old kyoku's count until the first
// entry of the new one resets it; the history is empty then and there is nothing to write.)
MJ_HD void hist_flush(const Env &e, int hist_len)
{
  int j = *e.hbase;
  MJ_HOST_ASSERT(hist_len - j <= kHistRing);
#pragma unroll 1
  for (; j < hist_len; j++) {
    const int k = 2 * (j & (kHistRing - 1));
    e.hist[j] = (uint16_t)(e.hstage[(int64_t)k * e.hs] | e.hstage[(int64_t)(k + 1) * e.hs] << 8);
  }
  *e.hbase = (uint8_t)hist_len;
}
// STAGED: 1 the staging ring is there (known at compile time), 0 look at the pointer
template <int STAGED>
MJ_HD void hist_push(Ctx &c, int s, int a)
{
  const int i = c.g.hist_len;
  if (i >= 128) return;
  if (STAGED || c.e.hstage) {
    const int k = 2 * (i & (kHistRing - 1));
    if (i == 0) *c.e.hbase = 0;                          // the first entry after a deal: the row holds nothing of this kyoku
    c.e.hstage[(int64_t)k * c.e.hs] = (uint8_t)a;
    c.e.hstage[(int64_t)(k + 1) * c.e.hs] = (uint8_t)s;
  } else c.e.hist[i] = (uint16_t)(a | s << 8);
  c.g.hist_len = (uint8_t)(i + 1);
}

// One step of one environment, as a fixed sequence of stages that every lane walks through in the same order
// (each lane skips the stages it does not need), so that a wavefront executes each piece of code once per step:
//   0 check the actions   1 apply them (discard, call, kan, declarations)   2 refresh the actor's waits
//   3 offer responses (ron / pon / kan / chi, or robbing an added kan)      4 wins and draws: pay, rotate
//   5 draw (live wall or replacement tile)
// then, outside: deal when need_deal is set, and step_finish() for the mask of the seat to move.
// `acts` packs the four seats' actions as signed bytes (seat s in byte s).
// `sampled_ron` >= 0 says that the actions were drawn from the masks by the library's own sampler (they are legal by
// construction, so stage 0 is skipped) and carries the seats whose mask offered a win.
template <int STAGED = 0>
MJ_HD void step_env(Ctx &c, uint32_t acts, int sampled_ron = -1)
{
  c.need_deal = false;
  c.need_turn = false;
#pragma unroll
  for (int s = 0; s < 4; s++) DELTA(c, s) = 0;
  c.g.illegal_seat = 255;
  c.live_ptr = -1;
  if (c.g.terminated) return;
  MJ_RB(s0, true);
  // the next live tile is needed at the end of most steps: start its load now
  if (c.g.draw_ptr <= 121) {
    c.live_word = c.e.wallw[(int64_t)(c.g.wall_sel * 34 + (c.g.draw_ptr >> 2)) * c.e.n];
    c.live_ptr = c.g.draw_ptr;
  }
  // stage 0: an action outside the mask ends the game at once.  The eight mask words are read once, together.
  const int actors = c.g.actor_mask;
  int illegal = 0, ron_offered = sampled_ron;
  if (sampled_ron < 0) {
    uint64_t mk0[4], mk1[4];
#pragma unroll
    for (int s = 0; s < 4; s++) { mk0[s] = MASK(c, s, 0); mk1[s] = MASK(c, s, 1); }
    ron_offered = 0;
#pragma unroll
    for (int s = 0; s < 4; s++) {
      const int x = act_of(acts, s);
      const uint64_t w = x < 64 ? mk0[s] : mk1[s];
      const bool ok = x >= 0 && x < N_ACTIONS && (w >> (x & 63) & 1);
      if ((actors >> s & 1) && !ok) illegal |= 1 << s;
      if ((actors >> s & 1) && (mk1[s] >> (A_RON - 64) & 1)) ron_offered |= 1 << s;
    }
  }
  if (illegal) {
    c.g.illegal_seat = (uint8_t)__builtin_ctz((unsigned)illegal);
    clear_result(c);
    c.g.end_type = 9;
    c.g.terminated = 1;
    c.g.phase = PH_TERMINAL;
    clear_masks(c);
    return;
  }
  // stage 1: apply
  int waits_seat = -1, waits_k = -1, win_mask = 0, win_loser = -1, win_tile = 0, end_abort = 0;
  // what the later stages have to do, as bits of one per-lane word (six separate booleans would each live in a
  // scalar register pair across the stages)
  enum : uint32_t { DO_RESPOND = 1, DO_ROB = 2, DO_ADVANCE = 4, DO_KANFIN = 8, WIN_TSUMO = 16, WIN_ROB = 32, KAN_CONCEALED = 64 };
  uint32_t todo = 0;
  uint32_t discard_hw = 0;           // the discarder's hand word of the discarded tile's suit, after the discard
  MJ_RE(s0, PR_S0);
  MJ_RB(s1t, c.g.phase == PH_TURN);
  MJ_RB(s1r, c.g.phase != PH_TURN);
  if (c.g.phase == PH_TURN) {
    int s = c.g.cur, act = act_of(acts, s);
    hist_push<STAGED>(c, s, act);
    MJ_RB(dis, act < A_KAN);
    MJ_RB(kan, act >= A_KAN && act < A_RIICHI);
    MJ_RB(dcl, act >= A_RIICHI);
    if (act < A_KAN) {
      const int k = act < A_DISCARD_RED ? act : 4 + 9 * (act - A_DISCARD_RED);
      // a seat in riichi gives back the drawn tile: its waits stay; any other seat's waits follow from the discard
      bool was_riichi;
      discard_hw = apply_discard(c, s, k, act < A_DISCARD_RED ? 0 : 1, was_riichi);
      if (!was_riichi) { waits_seat = s; waits_k = k; }
      todo |= DO_RESPOND;
    } else if (act < A_RIICHI) {
      const int kk = act - A_KAN;
      if (!apply_own_kan(c, kk)) todo |= DO_ROB;
      else if ((c.R.flags & F_ANKAN_ROB) && (K_YAOCHU >> kk & 1)) {
        // MJ_F_ANKAN_ROB: the thirteen orphans may win on this tile; the tile code carries bit 7 while that is open
        c.g.kakan_tile = (uint8_t)(kk | 0x80);
        todo |= DO_ROB | KAN_CONCEALED;
      } else todo |= DO_KANFIN | KAN_CONCEALED;
      waits_seat = s;
    } else if (act == A_RIICHI) {
      c.g.riichi_pending = (SW(c, s) >> SW_FIRST & 1) ? 2 : 1;
      c.need_turn = true;
    } else if (act == A_TSUMO) {
      win_mask = 1 << s; todo |= WIN_TSUMO; win_tile = code_kind(c.g.drawn);
    } else end_abort = 4;
    MJ_RE(dis, PR_DISCARD);
    MJ_RE(kan, PR_KAN);
    MJ_RE(dcl, PR_DECL);
  } else {
    int ronners = 0;
    for (int s = 0; s < 4; s++) if ((actors >> s & 1) && act_of(acts, s) == A_RON) ronners |= 1 << s;
    if (ronners) {
      // wins on a discard or on the tile of a kan, in turn order from the seat that gave the tile
      const int from = c.g.phase == PH_RESPOND ? c.g.last_discarder : c.g.cur;
#pragma unroll 1
      for (int j = 1; j < 4; j++) {
        const int o = (from + j) & 3;
        if (ronners >> o & 1) hist_push<STAGED>(c, o, A_RON);
      }
    }
    if (c.g.phase == PH_RESPOND) {
      int d = c.g.last_discarder;
      if (popc32((uint32_t)ronners) == 3 && (c.R.flags & F_ABORT)) end_abort = 8;
      else if (ronners) { win_mask = ronners; win_loser = d; win_tile = code_kind(c.g.last_discard); }
      else {
        mark_passed_ron(c, ron_offered);
        int caller = -1, call = 0;
        for (int s = 0; s < 4; s++) if ((actors >> s & 1) && act_of(acts, s) >= A_PON && act_of(acts, s) <= A_MINKAN) { caller = s; call = act_of(acts, s); }
        int nx = (d + 1) & 3;
        if (caller < 0 && (actors >> nx & 1) && act_of(acts, nx) >= A_CHI_L && act_of(acts, nx) < A_PASS) { caller = nx; call = act_of(acts, nx); }
        end_abort = settle_discard(c);
        if (!end_abort) {
          if (caller >= 0) hist_push<STAGED>(c, caller, call);
          MJ_RB(cal, caller >= 0);
          if (caller < 0) todo |= DO_ADVANCE;
          else if (apply_call(c, caller, call)) { waits_seat = caller; todo |= DO_KANFIN; }
          else c.need_turn = true;
          MJ_RE(cal, PR_CALL);
        }
      }
    } else {
      if (ronners) { win_mask = ronners; win_loser = c.g.cur; win_tile = code_kind(c.g.kakan_tile); todo |= WIN_ROB; }
      else { mark_passed_ron(c, ron_offered); todo |= (c.g.kakan_tile & 0x80) ? (DO_KANFIN | KAN_CONCEALED) : DO_KANFIN; }
    }
  }
  MJ_RE(s1t, PR_S1_TURN);
  MJ_RE(s1r, PR_S1_RESP);
  clear_masks(c);
  MJ_RB(s2, waits_seat >= 0);
  // stage 2: the seat whose concealed hand is back to 13 - 3 * melds tiles gets its waits refreshed
  if (waits_seat >= 0) {
    MJ_STAT(n_waits_stage);
    const uint64_t td = TD(c);
    if (waits_k >= 0 && (td & TD_FACTS)) {
      // a discard: the facts of the 14-tile hand came with the turn's mask, the discard changed one suit; the set of
      // tenpai-keeping discards, when it was searched for, says at once whether any wait is left
      const int cs = suit_of(waits_k);
      const uint32_t facts = facts_update(c.L, (uint32_t)(td >> FACTS_SHIFT) & 0xFFFu, cs, discard_hw);
      MJ_RB(wsh, (td & TD_VALID) && !(td >> waits_k & 1));
      MJ_RB(wfa, !((td & TD_VALID) && !(td >> waits_k & 1)));
      if ((td & TD_VALID) && !(td >> waits_k & 1)) WAITS(c, waits_seat) = (uint64_t)facts << FACTS_SHIFT | W_FACTS_VALID;
      else
        WAITS(c, waits_seat) = waits_from_facts(&c.L, HW(c, waits_seat, 0), HW(c, waits_seat, 1), HW(c, waits_seat, 2),
                                                HW(c, waits_seat, 3), MELDW(c, waits_seat), swf(c, waits_seat, SW_NMELD, 3), facts);
      MJ_RE(wsh, PR_W_SHORT);
      MJ_RE(wfa, PR_W_FACTS);
    } else {
      MJ_RB(wre, true);
      refresh_waits(c, waits_seat);
      MJ_RE(wre, PR_W_REFRESH);
    }
  }
  MJ_RE(s2, PR_S2);
  // stage 3: responses of the other seats
  MJ_KEEP_IN_VGPR(todo);
  MJ_RB(s3, (todo & (DO_RESPOND | DO_ROB)) != 0);
  if (todo & (DO_RESPOND | DO_ROB)) {
    MJ_STAT(n_respond_stage);
    const bool respond = todo & DO_RESPOND, rob = todo & DO_ROB;
    const int from = respond ? c.g.last_discarder : c.g.cur;
    const int code = respond ? c.g.last_discard : c.g.kakan_tile;
    const int k = code_kind(code), su = suit_of(k);
    // what the three seats' options depend on, read together
    uint32_t sws[4], hws[4];
    uint64_t wts[4];
#pragma unroll
    for (int t = 0; t < 4; t++) { sws[t] = SW(c, t); hws[t] = HW(c, t, su); wts[t] = WAITS(c, t); }
    const int r = rank_of(k, su);
    // pon / kan and "the tile is one of my waits" for each seat in place (no selection by seat number), ...
    uint32_t opt[4], hit = 0;
#pragma unroll
    for (int t = 0; t < 4; t++) {
      const bool other = t != from;
      opt[t] = (respond && other) ? pon_kan_options(c, su, r, sws[t], hws[t]) : 0u;
      if (other && (wts[t] >> k & 1)) hit |= 1u << t;
    }
    // the tile of a concealed kan: only a hand without melds and without simples can wait for it as thirteen orphans
    // (the declarer holds all four copies, so no ordinary wait of such a hand contains it)
    if (rob && (todo & KAN_CONCEALED)) {
#pragma unroll
      for (int t = 0; t < 4; t++)
        if (sw_get(sws[t], SW_NMELD, 3) || ((HW(c, t, 0) | HW(c, t, 1) | HW(c, t, 2)) & 0x00FFFFF8u)) hit &= ~(1u << t);
    }
    // ... chi once, for the next seat, ...
    if (respond) {
      const int nx = (from + 1) & 3;
      const uint32_t copt = chi_options(c, su, r, pick4(sws[0], sws[1], sws[2], sws[3], nx), pick4(hws[0], hws[1], hws[2], hws[3], nx));
#pragma unroll
      for (int t = 0; t < 4; t++) if (t == nx) opt[t] |= copt;
    }
    // ... and the wins: one evaluation site in a loop over the (rare) seats that wait on the tile, in turn order
    uint32_t ron = 0;
    MJ_RB(s3r, hit != 0);
    for (int j = 1; j < 4 && hit; j++) {
      MJ_STAT(n_ron_loop);
      const int o = (from + j) & 3;
      if ((hit >> o & 1) && ron_option(c, o, k, rob)) ron |= 1u << o;
    }
    MJ_RE(s3r, PR_S3_RON);
    int any = 0;
#pragma unroll
    for (int t = 0; t < 4; t++) {
      if (ron >> t & 1) opt[t] |= R_BIT(A_RON);
      if (opt[t]) { any |= 1 << t; MASK(c, t, 1) = opt[t] | R_BIT(A_PASS); }      // word 0 is clear already
    }
    if (any) {
      c.g.phase = respond ? PH_RESPOND : PH_RESPOND_KAKAN;
      c.g.actor_mask = (uint8_t)any;
    } else if (respond) {
      end_abort = settle_discard(c);
      if (!end_abort) todo |= DO_ADVANCE;
    } else todo |= DO_KANFIN;
  }
  MJ_RE(s3, PR_S3);
  bool exhaust = false;
  MJ_KEEP_IN_VGPR(todo);
  if ((todo & DO_ADVANCE) && c.g.live_left == 0) { exhaust = true; todo &= ~DO_ADVANCE; }
  // stage 4: the kyoku ends
  if (win_mask) MJ_STAT(n_win);
  if (exhaust) MJ_STAT(n_exhaust);
  MJ_RB(win, win_mask != 0);
  MJ_RB(abo, !win_mask && end_abort);
  MJ_RB(exh, !win_mask && !end_abort && exhaust);
  if (MJ_RARE(win_mask != 0)) win(c, win_mask, (todo & WIN_TSUMO) != 0, win_loser, win_tile, (todo & WIN_ROB) != 0);
  else if (end_abort) abortive_draw(c, end_abort);
  else if (exhaust) exhaustive_draw(c);
  MJ_RE(win, PR_WIN);
  MJ_RE(abo, PR_ABORT);
  MJ_RE(exh, PR_EXH);
  // stage 5: draws
  MJ_KEEP_IN_VGPR(todo);
  MJ_RB(drw, (todo & DO_ADVANCE) != 0);
  if (todo & DO_ADVANCE) { draw_live(c, (c.g.last_discarder + 1) & 3); c.need_turn = true; }
  MJ_RE(drw, PR_DRAW);
  MJ_RB(kdr, (todo & DO_KANFIN) != 0);
  if (todo & DO_KANFIN) { kan_draw(c, !(todo & KAN_CONCEALED)); c.need_turn = true; }
  MJ_RE(kdr, PR_KANDRAW);
}

// the mulhi(r, n)-th set bit of a mask of n legal actions (-1 for an empty mask)
MJ_HD int pick_action(uint64_t m0, uint64_t m1, uint32_t r)
{
  int n = popc64(m0) + popc64(m1);
  if (n == 0) return -1;
  int pick = (int)mulhi(r, (uint32_t)n);
  int n0 = popc64(m0);
  uint64_t m = m0; int base = 0;
  if (pick >= n0) { pick -= n0; m = m1; base = 64; }
  // position of the pick-th set bit of m by halving (no loop whose length depends on the lane)
  uint32_t w = (uint32_t)m;
  int c = popc32(w);
  if (pick >= c) { pick -= c; w = (uint32_t)(m >> 32); base += 32; }
#pragma unroll
  for (int half = 16; half >= 1; half >>= 1) {
    c = popc32(w & ((1u << half) - 1u));
    if (pick >= c) { pick -= c; w >>= half; base += half; }
  }
  return base;
}
// uniform choice among the set bits of a mask: key (seed, env_id), counter (step_lo, step_hi, seat, 1)
MJ_HD int sample_action(uint64_t m0, uint64_t m1, uint32_t seed, uint32_t env_id, uint64_t step, int seat)
{
  if ((m0 | m1) == 0) return -1;
  uint32_t r[4];
  philox((uint32_t)step, (uint32_t)(step >> 32), (uint32_t)seat, 1, seed, env_id, r);
  return pick_action(m0, m1, r[0]);
}

}  // namespace mj
