// Conversion between the packed structure-of-arrays state and the canonical
// per-environment record of include/mj.h, and the observation bit planes.
#pragma once
#include "../../include/mj.h"
#include "mj_engine.hpp"
#include "mj_layout.hpp"

namespace mj {

MJ_HD void export_env(const Env &e, MjEnvCanon &o)
{
  Glob g;
  load_glob(e, g);
  const int64_t n = e.n;
  for (int s = 0; s < 4; s++) {
    uint32_t sw = e.seatw[s * n];
    o.discarded_kinds[s] = e.dk[s * n];
    o.waits[s] = e.waits[s * n] & K_ALL;                    // without the facts that ride in the upper bits
    o.mask[s][0] = e.mask[(2 * s) * n]; o.mask[s][1] = e.mask[(2 * s + 1) * n];
    o.yaku[s] = e.yaku[s * n];
    o.score[s] = e.score[s * n]; o.delta[s] = e.delta[s * n]; o.gain[s] = e.gain[s * n];
    uint64_t mw = e.meld[s * n], rw = e.resw[s * n];
    for (int j = 0; j < 4; j++) o.meld[s][j] = (uint16_t)(mw >> (16 * j));
    for (int su = 0; su < 4; su++) {
      uint32_t hw = e.hand[(s * 4 + su) * n];
      int nr = su == 3 ? 7 : 9;
      for (int r = 0; r < nr; r++) o.hand[s][(su == 3 ? 27 : 9 * su) + r] = (uint8_t)cnt3(hw, r);
    }
    int nriv = (int)sw_get(sw, SW_NRIVER, 6);
    for (int i = 0; i < 32; i++) o.river[s][i] = i < nriv ? e.river[(s * 32 + i) * n] : 0;
    o.hand_red[s] = (uint8_t)sw_get(sw, SW_RED, 3);
    o.n_meld[s] = (uint8_t)sw_get(sw, SW_NMELD, 3);
    o.n_river[s] = (uint8_t)nriv;
    o.riichi_idx[s] = (uint8_t)sw_get(sw, SW_RIDX, 8);
    o.riichi[s] = (uint8_t)sw_get(sw, SW_RIICHI, 2);
    o.ippatsu[s] = (uint8_t)sw_get(sw, SW_IPPATSU, 1);
    o.first_turn[s] = (uint8_t)sw_get(sw, SW_FIRST, 1);
    o.furiten_temp[s] = (uint8_t)sw_get(sw, SW_FTEMP, 1);
    o.furiten_riichi[s] = (uint8_t)sw_get(sw, SW_FRIICHI, 1);
    o.kan_by[s] = (uint8_t)sw_get(sw, SW_KANBY, 3);
    o.final_rank[s] = (uint8_t)sw_get(sw, SW_RANK, 2);
    o.han[s] = (uint8_t)rw; o.fu[s] = (uint8_t)(rw >> 8); o.yakuman_units[s] = (uint8_t)(rw >> 16);
    o.r_dora[s] = (uint8_t)(rw >> 24); o.r_ura[s] = (uint8_t)(rw >> 32); o.r_aka[s] = (uint8_t)(rw >> 40);
  }
  o.episode = e.episode[0]; o.kyoku_serial = e.serial[0];
  for (int i = 0; i < 136; i++) o.wall[i] = (uint8_t)wall_at(e, g.wall_sel, i);
  o.kyoku = g.kyoku; o.honba = g.honba; o.kyotaku = g.kyotaku; o.terminated = g.terminated;
  o.draw_ptr = g.draw_ptr; o.n_kan = g.n_kan; o.live_left = g.live_left; o.n_dora = g.n_dora;
  o.drawn = g.drawn; o.phase = g.phase; o.cur = g.cur; o.actor_mask = g.actor_mask;
  o.riichi_pending = g.riichi_pending; o.rinshan = g.kanflags & 1; o.last_discard = g.last_discard;
  o.last_discarder = g.last_discarder; o.kakan_tile = g.kakan_tile; o.kuikae[0] = g.kuikae0; o.kuikae[1] = g.kuikae1;
  o.first_wind = g.first_wind; o.same_wind_cnt = g.same_wind_cnt; o.illegal_seat = g.illegal_seat;
  o.end_type = g.end_type; o.winners = g.winners; o.loser = g.loser; o.tenpai_mask = g.tenpai_mask;
  o.dora_pending = g.kanflags >> 1 & 1; o.n_hist = g.hist_len;
  for (int i = 0; i < 128; i++)
    o.hist[i] = i < g.hist_len ? e.hist[i] : (uint16_t)0;
}

MJ_HD void import_env(const Env &e, const MjEnvCanon &o)
{
  Glob g;
  const int64_t n = e.n;
  for (int s = 0; s < 4; s++) {
    e.dk[s * n] = o.discarded_kinds[s];
    e.waits[s * n] = o.waits[s];
    e.mask[(2 * s) * n] = o.mask[s][0]; e.mask[(2 * s + 1) * n] = o.mask[s][1];
    e.yaku[s * n] = o.yaku[s];
    e.score[s * n] = o.score[s]; e.delta[s * n] = o.delta[s]; e.gain[s * n] = o.gain[s];
    uint64_t mw = 0;
    for (int j = 0; j < 4; j++) mw |= (uint64_t)o.meld[s][j] << (16 * j);
    e.meld[s * n] = mw;
    e.resw[s * n] = (uint64_t)o.han[s] | (uint64_t)o.fu[s] << 8 | (uint64_t)o.yakuman_units[s] << 16 |
                    (uint64_t)o.r_dora[s] << 24 | (uint64_t)o.r_ura[s] << 32 | (uint64_t)o.r_aka[s] << 40;
    for (int su = 0; su < 4; su++) {
      uint32_t hw = 0;
      int nr = su == 3 ? 7 : 9;
      for (int r = 0; r < nr; r++) hw |= (uint32_t)(o.hand[s][(su == 3 ? 27 : 9 * su) + r] & 7) << (3 * r);
      e.hand[(s * 4 + su) * n] = hw;
    }
    for (int i = 0; i < 32; i++) e.river[(s * 32 + i) * n] = o.river[s][i];
    uint32_t sw = 0;
    sw = sw_set(sw, SW_RED, 3, o.hand_red[s] & 7); sw = sw_set(sw, SW_NMELD, 3, o.n_meld[s] & 7);
    sw = sw_set(sw, SW_NRIVER, 6, o.n_river[s] & 63); sw = sw_set(sw, SW_RIDX, 8, o.riichi_idx[s]);
    sw = sw_set(sw, SW_RIICHI, 2, o.riichi[s] & 3); sw = sw_set(sw, SW_IPPATSU, 1, o.ippatsu[s] & 1);
    sw = sw_set(sw, SW_FIRST, 1, o.first_turn[s] & 1); sw = sw_set(sw, SW_FTEMP, 1, o.furiten_temp[s] & 1);
    sw = sw_set(sw, SW_FRIICHI, 1, o.furiten_riichi[s] & 1); sw = sw_set(sw, SW_KANBY, 3, o.kan_by[s] & 7);
    sw = sw_set(sw, SW_RANK, 2, o.final_rank[s] & 3);
    e.seatw[s * n] = sw;
  }
  e.episode[0] = o.episode; e.serial[0] = o.kyoku_serial;
  e.nserial[0] = 0xFFFFFFFFu;                      // whatever was made ahead of time is gone
  e.tdisc[0] = 0;                                  // ... and so is the cache of tenpai-keeping discards
  for (int i = 0; i < 34; i++)
    e.wallw[i * n] = (uint32_t)o.wall[4 * i] | (uint32_t)o.wall[4 * i + 1] << 8 | (uint32_t)o.wall[4 * i + 2] << 16 |
                     (uint32_t)o.wall[4 * i + 3] << 24;
  g.kyoku = o.kyoku; g.honba = o.honba; g.kyotaku = o.kyotaku; g.terminated = o.terminated;
  g.draw_ptr = o.draw_ptr; g.n_kan = o.n_kan; g.live_left = o.live_left; g.n_dora = o.n_dora;
  g.drawn = o.drawn; g.phase = o.phase; g.cur = o.cur; g.actor_mask = o.actor_mask;
  g.riichi_pending = o.riichi_pending; g.kanflags = (uint8_t)((o.rinshan & 1) | (o.dora_pending & 1) << 1); g.last_discard = o.last_discard;
  g.last_discarder = o.last_discarder; g.kakan_tile = o.kakan_tile; g.kuikae0 = o.kuikae[0]; g.kuikae1 = o.kuikae[1];
  g.first_wind = o.first_wind; g.same_wind_cnt = o.same_wind_cnt; g.illegal_seat = o.illegal_seat;
  g.end_type = o.end_type; g.winners = o.winners; g.loser = o.loser; g.tenpai_mask = o.tenpai_mask;
  g.wall_sel = 0;                      // the imported wall goes to buffer 0
  g.hist_len = o.n_hist > 128 ? 128 : o.n_hist;
  for (int i = 0; i < 128; i++) e.hist[i] = o.hist[i];
  store_glob(e, g);
}

// ---------------------------------------------------------------- observation
// 56 planes of 34 bits per viewer.  Per absolute seat: 14 masks (hand >= 1..4, river >= 1..4, meld >= 1..4,
// score thermometer, riichi plane); per environment: 9 masks (indicator >= 1..4, red visible, round wind,
// scalars, responded tile, dealer seat as a number).
enum { OB_HAND = 0, OB_RIVER = 4, OB_MELD = 8, OB_SCORE = 12, OB_RIICHI = 13, OB_SEAT_WORDS = 14 };
enum { OG_IND = 0, OG_REDVIS = 4, OG_ROUND = 5, OG_SCALARS = 6, OG_RESP = 7, OG_MISC = 8, OG_WORDS = 9 };

MJ_HD uint64_t ge_mask(const uint32_t w[4], int c)      // kinds whose packed count is >= c
{
  uint64_t m = 0;
#pragma unroll
  for (int su = 0; su < 4; su++) {
    uint32_t b0 = w[su] & O111, b1 = (w[su] >> 1) & O111, b2 = (w[su] >> 2) & O111, f;
    if (c == 1) f = b0 | b1 | b2;
    else if (c == 2) f = b1 | b2;
    else if (c == 3) f = (b0 & b1) | b2;
    else f = b2;
    m |= (uint64_t)squeeze9(f) << (9 * su);
  }
  return m & K_ALL;
}
MJ_HD void bump(uint32_t w[4], int k, int d) { int su = suit_of(k); w[su] += (uint32_t)d << (3 * rank_of(k, su)); }

// masks of absolute seat s; returns the red-five kinds this seat shows in river and melds
MJ_HD uint64_t obs_seat_masks(const Env &e, int s, uint64_t out[OB_SEAT_WORDS])
{
  const int64_t n = e.n;
  uint32_t sw = e.seatw[s * n];
  uint32_t h[4] = {e.hand[(s * 4) * n], e.hand[(s * 4 + 1) * n], e.hand[(s * 4 + 2) * n], e.hand[(s * 4 + 3) * n]};
  uint32_t rv[4] = {0, 0, 0, 0}, ml[4] = {0, 0, 0, 0};
  uint64_t redvis = 0;
  int nriv = (int)sw_get(sw, SW_NRIVER, 6);
  // the river bytes are one load each from rows B apart: issue them in groups of eight before using them
  for (int i0 = 0; i0 < nriv; i0 += 8) {
    int t[8];
#pragma unroll
    for (int j = 0; j < 8; j++) t[j] = (i0 + j < nriv) ? e.river[(s * 32 + i0 + j) * n] : 255;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      if (t[j] == 255) continue;
      bump(rv, t[j] & 63, 1);
      if (t[j] & 64) redvis |= kbit(t[j] & 63);
    }
  }
  uint64_t mw = e.meld[s * n];
  int nm = (int)sw_get(sw, SW_NMELD, 3);
  for (int j = 0; j < nm; j++) {
    uint32_t m = meld_at(mw, j);
    int t = m_type(m), k = m_kind(m);
    if (t == MT_CHI) { bump(ml, k, 1); bump(ml, k + 1, 1); bump(ml, k + 2, 1); }
    else bump(ml, k, t == MT_PON ? 3 : 4);
    if (m >> 13 & 1) redvis |= kbit((k / 9) * 9 + 4);
  }
#pragma unroll
  for (int c = 1; c <= 4; c++) {
    out[OB_HAND + c - 1] = ge_mask(h, c);
    out[OB_RIVER + c - 1] = ge_mask(rv, c);
    out[OB_MELD + c - 1] = ge_mask(ml, c);
  }
  int32_t sc = e.score[s * n];
  int steps = sc < 2000 ? 0 : sc / 2000;
  out[OB_SCORE] = steps >= 34 ? K_ALL : (1ull << steps) - 1;
  out[OB_RIICHI] = sw_get(sw, SW_RIICHI, 2) ? K_ALL : 0;
  return redvis;
}

// the two words of the current wall that hold the dora indicators (wall positions 124..131; the indicators are 126..130)
MJ_HD void dora_words(const Env &e, int wall_sel, uint32_t dw[2])
{
  dw[0] = e.wallw[(int64_t)(wall_sel * 34 + 31) * e.n];
  dw[1] = e.wallw[(int64_t)(wall_sel * 34 + 32) * e.n];
}
MJ_HD void obs_env_masks(const Glob &g, uint32_t rule_flags, uint64_t seat_red, const uint32_t dw[2], uint64_t out[OG_WORDS])
{
  uint32_t ind[4] = {0, 0, 0, 0};
  uint64_t redvis = seat_red;
  for (int i = 0; i < g.n_dora; i++) {
    int id = (int)(dw[(i + 2) >> 2] >> (8 * ((i + 2) & 3)) & 255u);
    bump(ind, id >> 2, 1);
    if ((rule_flags & F_RED) && (id == 16 || id == 52 || id == 88)) redvis |= kbit(id >> 2);
  }
#pragma unroll
  for (int c = 1; c <= 4; c++) out[OG_IND + c - 1] = ge_mask(ind, c);
  out[OG_REDVIS] = redvis;
  out[OG_ROUND] = kbit(27 + (g.kyoku >> 2));
  int a = g.live_left / 4, hb = g.honba > 8 ? 8 : g.honba, ky = g.kyotaku > 8 ? 8 : g.kyotaku;
  out[OG_SCALARS] = ((1ull << a) - 1) | (((1ull << hb) - 1) << 18) | (((1ull << ky) - 1) << 26);
  uint64_t resp = 0;
  if (g.phase == PH_RESPOND) resp = kbit(code_kind(g.last_discard));
  if (g.phase == PH_RESPOND_KAKAN) resp = kbit(code_kind(g.kakan_tile));
  out[OG_RESP] = resp;
  uint64_t drawn = (g.phase == PH_TURN && g.drawn != 255) ? kbit(code_kind(g.drawn)) : 0;
  out[OG_MISC] = (uint64_t)(g.kyoku & 3) | (uint64_t)g.cur << 2 | drawn << 8;     // dealer, cur, drawn-kind bit
}

// plane p (0..55) as seen by `me`, from the per-seat masks S[4][OB_SEAT_WORDS], own red bits and the env masks
MJ_HD uint64_t obs_plane(int p, int me, const uint64_t *S, uint32_t own_red, const uint64_t *G)
{
  if (p < 4) return S[me * OB_SEAT_WORDS + OB_HAND + p];
  if (p == 4) return (own_red & 1 ? kbit(4) : 0) | (own_red & 2 ? kbit(13) : 0) | (own_red & 4 ? kbit(22) : 0);
  if (p < 21) { int q = p - 5; return S[((me + (q >> 2)) & 3) * OB_SEAT_WORDS + OB_RIVER + (q & 3)]; }
  if (p < 37) { int q = p - 21; return S[((me + (q >> 2)) & 3) * OB_SEAT_WORDS + OB_MELD + (q & 3)]; }
  if (p < 41) return G[OG_IND + p - 37];
  if (p == 41) return G[OG_REDVIS];
  if (p < 46) return S[((me + p - 42) & 3) * OB_SEAT_WORDS + OB_RIICHI];
  if (p == 46) return G[OG_ROUND];
  int dealer = (int)(G[OG_MISC] & 3), cur = (int)(G[OG_MISC] >> 2 & 3);
  if (p == 47) return kbit(27 + ((me - dealer) & 3));
  if (p == 48) return kbit((dealer - me) & 3);
  if (p < 53) return S[((me + p - 49) & 3) * OB_SEAT_WORDS + OB_SCORE];
  if (p == 53) return G[OG_SCALARS];
  if (p == 54) return G[OG_RESP];
  return cur == me ? (G[OG_MISC] >> 8) : 0;
}

// ------------------------------------------------------- token observation
// The record of a viewer (see MjTokenObs) is put together from four pieces, so that the kernel can compute what the
// four viewers of a game share only once: the viewer's own hand, the game's scalars, the seats' public words
// rotated to the viewer, and the rivers (token bytes by absolute seat, picked by relative seat on the way out).
MJ_HD uint8_t tile_token(int kind, int red) { return (uint8_t)(red ? 34 + (kind >= 9) + (kind >= 18) : kind); }
MJ_HD uint8_t river_token(int t) { return (uint8_t)(tile_token(t & 63, t >> 6 & 1) | (t & 0x80)); }
// own hand: tokens in ascending order (the red five first among the fives) and the shanten number
MJ_HD void tok_own(const Env &e, int me, const uint32_t *sh_suit, const uint32_t *sh_honor, MjTokenObs &o)
{
  const int64_t n = e.n;
  const uint32_t swm = e.seatw[me * n];
  uint32_t h[4];
  for (int su = 0; su < 4; su++) h[su] = e.hand[(me * 4 + su) * n];
  int cnt = 0;
  for (int su = 0; su < 4; su++) {
    const int nr = su == 3 ? 7 : 9;
    for (int r = 0; r < nr; r++) {
      int c = cnt3(h[su], r);
      const int k = (su == 3 ? 27 : 9 * su) + r;
      if (su < 3 && r == 4 && (swm >> su & 1u) && c > 0) { if (cnt < 14) o.hand[cnt] = tile_token(k, 1); cnt++; c--; }
      for (int i = 0; i < c; i++) { if (cnt < 14) o.hand[cnt] = tile_token(k, 0); cnt++; }
    }
  }
  for (int i = cnt; i < 14; i++) o.hand[i] = 255;
  o.n_hand = (uint8_t)cnt;
  o.shanten = (int8_t)shanten_of(sh_suit, sh_honor, h[0], h[1], h[2], h[3], (int)sw_get(swm, SW_NMELD, 3));
}
// the game's scalars as the viewer sees them
MJ_HD void tok_env(const Env &e, const Glob &g, int me, uint32_t rule_flags, MjTokenObs &o)
{
  o.drawn = (g.phase == PH_TURN && g.cur == me && g.drawn != 255) ? tile_token(code_kind(g.drawn), code_red(g.drawn)) : 255;
  o.phase = g.phase;
  o.cur = g.phase == PH_TURN ? (uint8_t)((g.cur - me) & 3) : 255;
  o.last_discarder = g.last_discarder == 255 ? 255 : (uint8_t)((g.last_discarder - me) & 3);
  o.last_discard = g.last_discard == 255 ? 255 : tile_token(code_kind(g.last_discard), code_red(g.last_discard));
  o.kyoku = g.kyoku; o.honba = g.honba; o.kyotaku = g.kyotaku;
  o.dealer = (uint8_t)(((g.kyoku & 3) - me) & 3);
  o.live_left = g.live_left; o.n_dora = g.n_dora;
  for (int i = 0; i < 5; i++) {
    const int id = wall_at(e, g.wall_sel, 126 + i);
    const bool red = (rule_flags & F_RED) && (id == 16 || id == 52 || id == 88);
    o.dora[i] = i < g.n_dora ? tile_token(id >> 2, red) : 255;
  }
}
// the four seats' public words (control word, points, melds; by absolute seat) rotated to the viewer
MJ_HD void tok_seats(const uint32_t sw[4], const int32_t score[4], const uint64_t meld[4], int me, MjTokenObs &o)
{
  for (int rel = 0; rel < 4; rel++) {
    const int s = (me + rel) & 3;
    const int nm = (int)sw_get(sw[s], SW_NMELD, 3);
    o.n_meld[rel] = (uint8_t)nm; o.n_river[rel] = (uint8_t)sw_get(sw[s], SW_NRIVER, 6);
    o.riichi[rel] = (uint8_t)sw_get(sw[s], SW_RIICHI, 2); o.riichi_idx[rel] = (uint8_t)sw_get(sw[s], SW_RIDX, 8);
    o.score[rel] = score[s];
    for (int j = 0; j < 4; j++) o.meld[rel][j] = j < nm ? (uint16_t)(meld[s] >> (16 * j)) : (uint16_t)0;
  }
}
// one seat's river as 32 token bytes
MJ_HD void tok_river(const Env &e, int s, uint8_t out[32])
{
  const int nriv = (int)sw_get(e.seatw[s * e.n], SW_NRIVER, 6);
  uint8_t t[32];
#pragma unroll
  for (int i = 0; i < 32; i++) t[i] = e.river[(int64_t)(s * 32 + i) * e.n];      // all 32 loads in flight together
#pragma unroll
  for (int i = 0; i < 32; i++) out[i] = i < nriv ? river_token(t[i]) : (uint8_t)255;
}
// one entry of the action history as viewer `me` sees it
MJ_HD uint16_t hist_token(uint32_t ev, int me) { return (uint16_t)((ev & 0xFFu) | (((ev >> 8) - (uint32_t)me) & 3u) << 8); }
// the whole record of viewer `me` (the plain composition; every field of the record is written)
MJ_HD void token_obs(const Env &e, const Glob &g, int me, uint32_t rule_flags, const uint32_t *sh_suit, const uint32_t *sh_honor,
                     MjTokenObs &o)
{
  uint32_t sw[4];
  int32_t score[4];
  uint64_t meld[4];
  for (int s = 0; s < 4; s++) { sw[s] = e.seatw[s * e.n]; score[s] = e.score[s * e.n]; meld[s] = e.meld[s * e.n]; }
  tok_own(e, me, sh_suit, sh_honor, o);
  tok_env(e, g, me, rule_flags, o);
  tok_seats(sw, score, meld, me, o);
  for (int rel = 0; rel < 4; rel++) tok_river(e, (me + rel) & 3, o.river[rel]);
  o.n_hist = g.hist_len;
  for (int i = 0; i < 15; i++) o.zero_[i] = 0;
  for (int i = 0; i < 128; i++)
    o.hist[i] = i < g.hist_len ? hist_token(e.hist[i], me) : (uint16_t)0xFFFF;
}

}  // namespace mj
