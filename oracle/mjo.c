/*
 * mjo.c -- CPU ORACLE (test infrastructure, see mjo.h).
 *
 * Plain single-threaded C.  Every function follows the plain definition of
 * the rule it implements; win detection and scoring recurse over the hand and
 * enumerate every decomposition, with no table and no caching beyond the
 * `waits` field that is part of the state itself.
 *
 * Passages followed: paper section 3.2 (standard four-player East-South
 * Riichi rules; red / no-red variants; single / east / half modes; discrete
 * action ids with a legal_action_mask; an illegal action terminates the game
 * with a penalty), section 3.1 (what the State holds), section 4.1 (batched
 * steps under a random policy).  The paper is silent on the concrete rule
 * text, tie-breaks, numbering and randomness; the reading taken is written
 * at each function.
 */
#include "mjo.h"
#include <stdlib.h>
#include <assert.h>
#include <string.h>

typedef MjoEnv E;
struct MjoHandle {
  int64_t  B;
  uint32_t seed;
  MjoRules rules;
  uint64_t step;
  E       *env;
};

/* ------------------------------------------------------------------ tiles */

static int is_suited(int k) { return k < 27; }
static int is_honor(int k) { return k >= 27; }
static int is_terminal(int k) { return k < 27 && (k % 9 == 0 || k % 9 == 8); }
static int is_yaochu(int k) { return is_honor(k) || is_terminal(k); }
static int is_five(int k) { return k < 27 && k % 9 == 4; }
static int is_wind(int k) { return k >= 27 && k <= 30; }
static int is_dragon(int k) { return k >= 31; }

/* meld word: type(3) kind(6) from_rel(2) called_pos(2) has_red(1) called_is_red(1) */
enum { M_CHI = 1, M_PON = 2, M_MINKAN = 3, M_ANKAN = 4, M_KAKAN = 5 };
static int m_type(uint16_t m) { return m & 7; }
static int m_kind(uint16_t m) { return (m >> 3) & 63; }
static int m_has_red(uint16_t m) { return (m >> 13) & 1; }
static uint16_t m_make(int type, int kind, int from_rel, int pos, int has_red, int called_red)
{
  return (uint16_t)(type | kind << 3 | from_rel << 9 | pos << 11 | has_red << 13 | called_red << 14);
}
/* number of tiles of kind k inside one meld */
static int m_count(uint16_t m, int k)
{
  int t = m_type(m), b = m_kind(m);
  if (t == M_CHI) return (k >= b && k <= b + 2) ? 1 : 0;
  if (t == M_PON) return k == b ? 3 : 0;
  if (t == M_MINKAN || t == M_ANKAN || t == M_KAKAN) return k == b ? 4 : 0;
  return 0;
}

/* tile code used by drawn / last_discard / kakan_tile: kind | red << 6 */
static int t_kind(int code) { return code & 63; }
static int t_red(int code) { return (code >> 6) & 1; }

/* ----------------------------------------------------------------- Philox */

/* Philox4x32-10 as published by Salmon, Moraes, Dror and Shaw (SC'11). */
void mjo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; round++) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static uint32_t mulhi32(uint32_t a, uint32_t b) { return (uint32_t)(((uint64_t)a * b) >> 32); }

/* Fisher-Yates over the 136 tile ids.  Key (seed, env_id); counter
 * (kyoku_serial, j, 0, 0) for j = 0..33 yields words r[4j..4j+3]; position i
 * swaps with i + mulhi(r[i], 136 - i).  (Reading: bounded draw by
 * multiply-shift, fixed trip count.) */
void mjo_shuffle_wall(uint32_t seed, uint32_t env_id, uint32_t kyoku_serial, uint8_t wall[136])
{
  uint32_t r[136], key[2] = { seed, env_id };
  for (uint32_t j = 0; j < 34; j++) {
    uint32_t ctr[4] = { kyoku_serial, j, 0, 0 };
    mjo_philox4x32_10(ctr, key, &r[4 * j]);
  }
  for (int i = 0; i < 136; i++) wall[i] = (uint8_t)i;
  for (int i = 0; i < 135; i++) {
    int k = i + (int)mulhi32(r[i], (uint32_t)(136 - i));
    uint8_t t = wall[i]; wall[i] = wall[k]; wall[k] = t;
  }
}

/* ------------------------------------------------------------ completeness */

/* can the counts c[from..33] be split into runs and triplets only? */
static int sets_only(int *c, int from)
{
  int i = from;
  while (i < 34 && c[i] == 0) i++;
  if (i == 34) return 1;
  int ok = 0;
  if (c[i] >= 3) { c[i] -= 3; ok = sets_only(c, i); c[i] += 3; if (ok) return 1; }
  if (is_suited(i) && i % 9 <= 6 && c[i + 1] > 0 && c[i + 2] > 0) {
    c[i]--; c[i + 1]--; c[i + 2]--;
    ok = sets_only(c, i);
    c[i]++; c[i + 1]++; c[i + 2]++;
  }
  return ok;
}

static int std_complete(const uint8_t hand[34])
{
  int c[34];
  for (int i = 0; i < 34; i++) c[i] = hand[i];
  for (int p = 0; p < 34; p++) if (c[p] >= 2) {
    c[p] -= 2;
    int ok = sets_only(c, 0);
    c[p] += 2;
    if (ok) return 1;
  }
  return 0;
}
static int seven_pairs(const uint8_t hand[34])
{
  int n = 0;
  for (int i = 0; i < 34; i++) { if (hand[i] == 2) n++; else if (hand[i] != 0) return 0; }
  return n == 7;
}
static int thirteen_orphans(const uint8_t hand[34])
{
  int dup = 0;
  for (int i = 0; i < 34; i++) {
    if (is_yaochu(i)) { if (hand[i] == 0 || hand[i] > 2) return 0; if (hand[i] == 2) dup++; }
    else if (hand[i] != 0) return 0;
  }
  return dup == 1;
}

/* A hand is complete when the concealed tiles (14 - 3*n_meld of them, the
 * winning tile included) form (4 - n_meld) sets and a pair, or, with no meld,
 * seven distinct pairs or the thirteen orphans. */
int mjo_is_complete(const uint8_t hand[34], int n_meld)
{
  int total = 0;
  for (int i = 0; i < 34; i++) { if (hand[i] > 4) return 0; total += hand[i]; }
  if (total != 14 - 3 * n_meld) return 0;
  if (std_complete(hand)) return 1;
  if (n_meld == 0 && (seven_pairs(hand) || thirteen_orphans(hand))) return 1;
  return 0;
}

/* Waits of a (13 - 3*n_meld)-tile hand: kinds k of which the player owns
 * fewer than four (concealed + own melds) and whose addition completes the
 * hand; yaku not required.  (Reading: a wait on a tile the player already
 * holds four of does not count towards tenpai.) */
uint64_t mjo_waits_of(const uint8_t hand[34], const uint16_t meld[4], int n_meld)
{
  uint8_t h[34];
  uint64_t w = 0;
  memcpy(h, hand, 34);
  for (int k = 0; k < 34; k++) {
    int own = h[k];
    for (int j = 0; j < n_meld; j++) own += m_count(meld[j], k);
    if (own >= 4) continue;
    h[k]++;
    if (mjo_is_complete(h, n_meld)) w |= 1ull << k;
    h[k]--;
  }
  return w;
}

/* ------------------------------------------------------------ shanten */

/* Shanten number (paper section 3.2 lists it among the scalar properties of
 * the observation): how many tile exchanges a hand is away from tenpai, -1 for
 * a complete hand.  The usual formula on blocks, written as an exhaustive
 * search: with `need` = 4 - n_meld sets still to be found among the concealed
 * tiles, m complete sets (triplet or run), t partial sets (pair, two adjacent,
 * two with a gap) taken from disjoint tiles with m + t <= need, and p = 1 when
 * a pair is set aside as the head, the standard form is
 *     2 * need - (2 m + t) - p,
 * minimised over every way of choosing head, sets and partial sets; seven
 * pairs (6 - pairs + missing kinds) and thirteen orphans (13 - kinds - pair)
 * compete when there is no meld.  Tile availability is not considered (a
 * partial set that waits on a tile the hand already holds four times still
 * counts), as in the customary definition. */
static void sh_search(uint8_t *c, int i, int m, int t, int need, int *best)
{
  while (i < 34 && c[i] == 0) i++;
  if (i == 34) {
    int tt = t < need - m ? t : need - m;
    if (2 * m + tt > *best) *best = 2 * m + tt;
    return;
  }
  int suited = i < 27, r = i % 9;
  if (m < need) {
    if (c[i] >= 3) { c[i] -= 3; sh_search(c, i, m + 1, t, need, best); c[i] += 3; }
    if (suited && r <= 6 && c[i + 1] && c[i + 2]) {
      c[i]--; c[i + 1]--; c[i + 2]--; sh_search(c, i, m + 1, t, need, best); c[i]++; c[i + 1]++; c[i + 2]++;
    }
  }
  if (c[i] >= 2) { c[i] -= 2; sh_search(c, i, m, t + 1, need, best); c[i] += 2; }
  if (suited && r <= 7 && c[i + 1]) { c[i]--; c[i + 1]--; sh_search(c, i, m, t + 1, need, best); c[i]++; c[i + 1]++; }
  if (suited && r <= 6 && c[i + 2]) { c[i]--; c[i + 2]--; sh_search(c, i, m, t + 1, need, best); c[i]++; c[i + 2]++; }
  c[i]--; sh_search(c, i, m, t, need, best); c[i]++;          /* this tile belongs to nothing */
}

int mjo_shanten(const uint8_t hand[34], int n_meld)
{
  uint8_t c[34];
  memcpy(c, hand, 34);
  int need = 4 - n_meld, best = 0;
  sh_search(c, 0, 0, 0, need, &best);
  int sh = 2 * need - best;                                    /* no head set aside */
  for (int k = 0; k < 34; k++) {
    if (c[k] < 2) continue;
    c[k] -= 2;
    best = 0;
    sh_search(c, 0, 0, 0, need, &best);
    c[k] += 2;
    if (2 * need - best - 1 < sh) sh = 2 * need - best - 1;
  }
  if (n_meld == 0) {
    int pairs = 0, kinds = 0, yao = 0, yao_pair = 0;
    for (int k = 0; k < 34; k++) {
      if (c[k] >= 1) kinds++;
      if (c[k] >= 2) pairs++;
      if (is_yaochu(k)) { if (c[k] >= 1) yao++; if (c[k] >= 2) yao_pair = 1; }
    }
    int chiitoi = 6 - pairs + (kinds < 7 ? 7 - kinds : 0);
    int kokushi = 13 - yao - yao_pair;
    if (chiitoi < sh) sh = chiitoi;
    if (kokushi < sh) sh = kokushi;
  }
  return sh;
}

/* ------------------------------------------------------------ evaluation */

enum { S_RUN = 0, S_TRIPLET = 1, S_KAN = 2 };
typedef struct { uint8_t type, kind, open; } Set;

enum {
  Y_RIICHI = 0, Y_DOUBLE_RIICHI, Y_IPPATSU, Y_TSUMO, Y_PINFU, Y_TANYAO, Y_IIPEIKOU,
  Y_HAKU, Y_HATSU, Y_CHUN, Y_SEAT_WIND, Y_ROUND_WIND, Y_RINSHAN, Y_CHANKAN, Y_HAITEI,
  Y_HOUTEI, Y_CHIITOI, Y_SANSHOKU, Y_ITTSU, Y_CHANTA, Y_TOITOI, Y_SANANKOU, Y_DOUKOU,
  Y_SANKANTSU, Y_HONROUTOU, Y_SHOUSANGEN, Y_HONITSU, Y_JUNCHAN, Y_RYANPEIKOU, Y_CHINITSU,
  Y_KOKUSHI = 32, Y_SUUANKOU, Y_DAISANGEN, Y_SHOUSUUSHII, Y_DAISUUSHII, Y_TSUUIISOU,
  Y_CHINROUTOU, Y_RYUUIISOU, Y_CHUUREN, Y_SUUKANTSU, Y_TENHOU, Y_CHIIHOU
};
/* han per yaku: closed hand / open hand (0 = not available) */
static const uint8_t HAN_CLOSED[30] = { 1,2,1,1,1,1,1, 1,1,1,1,1,1,1,1, 1,2,2,2,2,2,2,2, 2,2,2,3,3,3,6 };
static const uint8_t HAN_OPEN[30]   = { 0,0,0,0,0,1,0, 1,1,1,1,1,1,1,1, 1,0,1,1,1,2,2,2, 2,2,2,2,2,0,5 };

typedef struct {
  const MjoHandQuery *q;
  int all[34];            /* every tile of the hand, melds included */
  int menzen;             /* no open meld */
  int tsumo, dealer, riichi;
  int n_dora, n_ura, n_aka;
  int found;              /* some valid interpretation seen */
  MjoHandResult best;
} Eval;

static int32_t up100(int32_t x) { return (x + 99) / 100 * 100; }

/* base = fu * 2^(han+2) capped at 2000, then the limit table; yakuman 8000 per unit */
static int32_t base_points(int han, int fu, int units)
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
/* total received by the winner, without honba and sticks */
static int32_t total_points(int32_t base, int dealer, int tsumo)
{
  if (!tsumo) return up100(base * (dealer ? 6 : 4));
  if (dealer) return 3 * up100(base * 2);
  return up100(base * 2) + 2 * up100(base);
}

/* yaku that depend on the situation only; same for every form */
static uint64_t situational(const Eval *c)
{
  const MjoHandQuery *q = c->q;
  uint64_t y = 0;
  int f = q->flags;
  if (c->riichi == 1) y |= 1ull << Y_RIICHI;
  if (c->riichi == 2) y |= 1ull << Y_DOUBLE_RIICHI;
  if (c->riichi && (f & 2)) y |= 1ull << Y_IPPATSU;
  if (c->tsumo && c->menzen) y |= 1ull << Y_TSUMO;
  if (c->tsumo && (f & 4)) y |= 1ull << Y_RINSHAN;
  if (!c->tsumo && (f & 8)) y |= 1ull << Y_CHANKAN;
  if (c->tsumo && (f & 16) && !(f & 4)) y |= 1ull << Y_HAITEI;
  if (!c->tsumo && (f & 32) && !(f & 8)) y |= 1ull << Y_HOUTEI;
  return y;
}
static uint64_t first_turn_yakuman(const Eval *c)
{
  const MjoHandQuery *q = c->q;
  if ((q->flags & 64) && c->tsumo && q->n_meld == 0 && !(q->flags & 4))
    return 1ull << (c->dealer ? Y_TENHOU : Y_CHIIHOU);
  return 0;
}

/* Offer one interpretation: regular yaku y (situational bits not yet added),
 * yakuman bits ym, fu.  Keeps the maximum under (points, han, fu, yaku). */
static void offer(Eval *c, uint64_t y, uint64_t ym, int fu)
{
  MjoHandResult r;
  memset(&r, 0, sizeof r);
  ym |= first_turn_yakuman(c);
  if (ym) {
    int units = 0;
    for (int b = 32; b < 64; b++) if (ym >> b & 1) units++;
    r.yaku = ym; r.yakuman_units = (uint8_t)units; r.han = (uint8_t)(13 * units); r.fu = 0;
    r.points = total_points(base_points(0, 0, units), c->dealer, c->tsumo);
  } else {
    y |= situational(c);
    int han = 0;
    for (int b = 0; b < 30; b++) if (y >> b & 1) han += c->menzen ? HAN_CLOSED[b] : HAN_OPEN[b];
    if (han == 0) return;            /* dora alone never make a win */
    han += c->n_dora + c->n_ura + c->n_aka;
    r.yaku = y; r.han = (uint8_t)han; r.fu = (uint8_t)fu;
    r.points = total_points(base_points(han, fu, 0), c->dealer, c->tsumo);
  }
  r.shape_ok = 1; r.yaku_ok = 1;
  r.n_dora = (uint8_t)c->n_dora; r.n_ura = (uint8_t)c->n_ura; r.n_aka = (uint8_t)c->n_aka;
  int better;
  if (!c->found) better = 1;
  else if (r.points != c->best.points) better = r.points > c->best.points;
  else if (r.han != c->best.han) better = r.han > c->best.han;
  else if (r.fu != c->best.fu) better = r.fu > c->best.fu;
  else better = r.yaku > c->best.yaku;
  if (better) { c->best = r; c->found = 1; }
}

/* yaku that depend on the tile multiset only (any form) */
static void colour_yaku(const Eval *c, uint64_t *y, uint64_t *ym)
{
  int suits = 0, honors = 0, all_simple = 1, all_yaochu = 1, all_honor = 1, all_term = 1, all_green = 1;
  for (int k = 0; k < 34; k++) if (c->all[k]) {
    if (is_honor(k)) honors = 1; else suits |= 1 << (k / 9);
    if (is_yaochu(k)) all_simple = 0; else all_yaochu = 0;
    if (!is_honor(k)) all_honor = 0;
    if (!is_terminal(k)) all_term = 0;
    if (!(k == 19 || k == 20 || k == 21 || k == 23 || k == 25 || k == 32)) all_green = 0;
  }
  int one_suit = suits == 1 || suits == 2 || suits == 4;
  if (all_simple && (c->menzen || c->q->kuitan)) *y |= 1ull << Y_TANYAO;
  if (one_suit && honors) *y |= 1ull << Y_HONITSU;
  if (one_suit && !honors) *y |= 1ull << Y_CHINITSU;
  if (all_yaochu && !all_honor && !all_term) *y |= 1ull << Y_HONROUTOU;
  if (all_honor) *ym |= 1ull << Y_TSUUIISOU;
  if (all_term) *ym |= 1ull << Y_CHINROUTOU;
  if (all_green) *ym |= 1ull << Y_RYUUIISOU;
}

/* One standard interpretation: four sets (melds first), the pair, and how the
 * winning tile was waited for (wait_fu 0/2, two_sided for pinfu). */
static void eval_standard(Eval *c, const Set *sets, int pair, int wait_fu, int two_sided)
{
  const MjoHandQuery *q = c->q;
  uint64_t y = 0, ym = 0;
  int seat_k = 27 + q->seat_wind, round_k = 27 + q->round_wind;
  int n_run = 0, n_kan = 0, n_concealed = 0, n_dragon = 0, n_windset = 0;
  int run_cnt[27] = {0}, trip_rank[3] = {0, 0, 0}, run_rank[3] = {0, 0, 0};
  int every_yaochu = 1, any_honor = 0;
  for (int j = 0; j < 4; j++) {
    int k = sets[j].kind;
    if (sets[j].type == S_RUN) {
      n_run++; run_cnt[k]++; run_rank[k / 9] |= 1 << (k % 9);
      if (!(k % 9 == 0 || k % 9 == 6)) every_yaochu = 0;
    } else {
      if (sets[j].type == S_KAN) n_kan++;
      if (!sets[j].open) n_concealed++;
      if (is_dragon(k)) { n_dragon++; y |= 1ull << (Y_HAKU + (k - 31)); }
      if (is_wind(k)) n_windset++;
      if (k == seat_k) y |= 1ull << Y_SEAT_WIND;
      if (k == round_k) y |= 1ull << Y_ROUND_WIND;
      if (is_suited(k)) trip_rank[k / 9] |= 1 << (k % 9);
      if (!is_yaochu(k)) every_yaochu = 0;
      if (is_honor(k)) any_honor = 1;
    }
  }
  if (!is_yaochu(pair)) every_yaochu = 0;
  if (is_honor(pair)) any_honor = 1;

  int pair_fu = 0;
  if (is_dragon(pair)) pair_fu += 2;
  if (pair == seat_k) pair_fu += 2;
  if (pair == round_k) pair_fu += 2;

  int pinfu = c->menzen && n_run == 4 && pair_fu == 0 && two_sided;
  if (pinfu) y |= 1ull << Y_PINFU;
  if (c->menzen) {
    int doubles = 0;
    for (int k = 0; k < 27; k++) doubles += run_cnt[k] / 2;
    if (doubles >= 2) y |= 1ull << Y_RYANPEIKOU;
    else if (doubles == 1) y |= 1ull << Y_IIPEIKOU;
  }
  if (run_rank[0] & run_rank[1] & run_rank[2]) y |= 1ull << Y_SANSHOKU;
  for (int s = 0; s < 3; s++) if ((run_rank[s] & 0x49) == 0x49) y |= 1ull << Y_ITTSU;
  if (every_yaochu && n_run >= 1) y |= 1ull << (any_honor ? Y_CHANTA : Y_JUNCHAN);
  if (n_run == 0) y |= 1ull << Y_TOITOI;
  if (n_concealed == 3) y |= 1ull << Y_SANANKOU;
  if (trip_rank[0] & trip_rank[1] & trip_rank[2]) y |= 1ull << Y_DOUKOU;
  if (n_kan == 3) y |= 1ull << Y_SANKANTSU;
  if (n_dragon == 2 && is_dragon(pair)) y |= 1ull << Y_SHOUSANGEN;
  colour_yaku(c, &y, &ym);

  if (n_concealed == 4) ym |= 1ull << Y_SUUANKOU;
  if (n_dragon == 3) ym |= 1ull << Y_DAISANGEN;
  if (n_windset == 3 && is_wind(pair)) ym |= 1ull << Y_SHOUSUUSHII;
  if (n_windset == 4) ym |= 1ull << Y_DAISUUSHII;
  if (n_kan == 4) ym |= 1ull << Y_SUUKANTSU;
  if (q->n_meld == 0 && (y >> Y_CHINITSU & 1)) {       /* nine gates: 1112345678999 + any */
    int s = 0, ok = 1;
    while (s < 3 && c->all[9 * s] == 0) s++;
    for (int r = 0; r < 9; r++) {
      int need = (r == 0 || r == 8) ? 3 : 1;
      if (c->all[9 * s + r] < need) ok = 0;
    }
    if (ok) ym |= 1ull << Y_CHUUREN;
  }

  /* fu */
  int fu;
  if (pinfu) fu = c->tsumo ? 20 : 30;
  else {
    fu = 20;
    if (c->menzen && !c->tsumo) fu += 10;
    if (c->tsumo) fu += 2;
    for (int j = 0; j < 4; j++) if (sets[j].type != S_RUN) {
      int f = 2;
      if (!sets[j].open) f *= 2;
      if (is_yaochu(sets[j].kind)) f *= 2;
      if (sets[j].type == S_KAN) f *= 4;
      fu += f;
    }
    fu += pair_fu + wait_fu;
    if (!c->menzen && fu == 20) fu = 30;
    fu = (fu + 9) / 10 * 10;
  }
  offer(c, y, ym, fu);
}

/* every way the winning tile can have completed this decomposition */
static void placements(Eval *c, const Set *sets, int pair)
{
  int w = c->q->win_kind, m = c->q->n_meld;
  if (pair == w) eval_standard(c, sets, pair, 2, 0);
  for (int j = m; j < 4; j++) {
    int k = sets[j].kind;
    if (sets[j].type == S_TRIPLET && k == w) {
      Set t[4];
      memcpy(t, sets, sizeof t);
      if (!c->tsumo) t[j].open = 1;      /* a triplet finished by ron counts as open */
      eval_standard(c, t, pair, 0, 0);
    } else if (sets[j].type == S_RUN && w >= k && w <= k + 2) {
      int closed = w == k + 1;
      int edge = (w == k + 2 && k % 9 == 0) || (w == k && k % 9 == 6);
      if (closed || edge) eval_standard(c, sets, pair, 2, 0);
      else eval_standard(c, sets, pair, 0, 1);
    }
  }
}

static void enum_sets(Eval *c, int *h, int from, Set *sets, int ns, int pair)
{
  int i = from;
  while (i < 34 && h[i] == 0) i++;
  if (i == 34) { if (ns == 4) placements(c, sets, pair); return; }
  if (ns == 4) return;
  if (h[i] >= 3) {
    h[i] -= 3;
    sets[ns].type = S_TRIPLET; sets[ns].kind = (uint8_t)i; sets[ns].open = 0;
    enum_sets(c, h, i, sets, ns + 1, pair);
    h[i] += 3;
  }
  if (is_suited(i) && i % 9 <= 6 && h[i + 1] > 0 && h[i + 2] > 0) {
    h[i]--; h[i + 1]--; h[i + 2]--;
    sets[ns].type = S_RUN; sets[ns].kind = (uint8_t)i; sets[ns].open = 0;
    enum_sets(c, h, i, sets, ns + 1, pair);
    h[i]++; h[i + 1]++; h[i + 2]++;
  }
}

static int dora_next(int k)
{
  if (k < 27) return (k / 9) * 9 + (k % 9 + 1) % 9;
  if (k < 31) return 27 + (k - 27 + 1) % 4;
  return 31 + (k - 31 + 1) % 3;
}

/* Best value of a hand: maximum over every form, decomposition and placement
 * of the winning tile under the order (points, han, fu, yaku mask). */
void mjo_eval_hand(const MjoHandQuery *q, MjoHandResult *out)
{
  Eval c;
  memset(&c, 0, sizeof c);
  memset(out, 0, sizeof *out);
  c.q = q;
  int n_meld = q->n_meld;
  if (n_meld > 4 || q->win_kind >= 34 || q->hand[q->win_kind] == 0) return;
  if (!mjo_is_complete(q->hand, n_meld)) return;
  out->shape_ok = 1;

  c.menzen = 1;
  for (int k = 0; k < 34; k++) c.all[k] = q->hand[k];
  for (int j = 0; j < n_meld; j++) {
    if (m_type(q->meld[j]) != M_ANKAN) c.menzen = 0;
    for (int k = 0; k < 34; k++) c.all[k] += m_count(q->meld[j], k);
  }
  c.tsumo = q->flags & 1;
  c.dealer = q->seat_wind == 0;
  c.riichi = c.menzen ? q->riichi : 0;
  for (int i = 0; i < q->n_ind && i < 5; i++) {
    c.n_dora += c.all[dora_next(q->ind[i])];
    if (c.riichi) c.n_ura += c.all[dora_next(q->ura[i])];
  }
  c.n_aka = q->n_aka;

  /* standard form */
  Set sets[4];
  for (int j = 0; j < n_meld; j++) {
    int t = m_type(q->meld[j]);
    sets[j].kind = (uint8_t)m_kind(q->meld[j]);
    sets[j].type = t == M_CHI ? S_RUN : t == M_PON ? S_TRIPLET : S_KAN;
    sets[j].open = t != M_ANKAN;
  }
  int h[34];
  for (int k = 0; k < 34; k++) h[k] = q->hand[k];
  for (int p = 0; p < 34; p++) if (h[p] >= 2) {
    h[p] -= 2;
    enum_sets(&c, h, 0, sets, n_meld, p);
    h[p] += 2;
  }
  /* seven pairs: 25 fu */
  if (n_meld == 0 && seven_pairs(q->hand)) {
    uint64_t y = 1ull << Y_CHIITOI, ym = 0;
    colour_yaku(&c, &y, &ym);
    offer(&c, y, ym, 25);
  }
  /* thirteen orphans */
  if (n_meld == 0 && thirteen_orphans(q->hand)) offer(&c, 0, 1ull << Y_KOKUSHI, 0);

  if (c.found) *out = c.best;
}

/* ---------------------------------------------------------------- engine */

static void set_bit(uint64_t m[2], int a) { m[a >> 6] |= 1ull << (a & 63); }
static int get_bit(const uint64_t m[2], int a) { return (int)(m[a >> 6] >> (a & 63) & 1); }
static int nonred(const E *e, int s, int k)
{
  return e->hand[s][k] - ((is_five(k) && (e->hand_red[s] >> (k / 9) & 1)) ? 1 : 0);
}
static int concealed_total(const E *e, int s)
{
  int n = 0;
  for (int k = 0; k < 34; k++) n += e->hand[s][k];
  return n;
}
static int is_menzen(const E *e, int s)
{
  for (int j = 0; j < e->n_meld[s]; j++) if (m_type(e->meld[s][j]) != M_ANKAN) return 0;
  return 1;
}
static int dealer_of(const E *e) { return e->kyoku & 3; }

static void refresh_waits(E *e, int s) { e->waits[s] = mjo_waits_of(e->hand[s], e->meld[s], e->n_meld[s]); }

static int is_red_id(const MjoHandle *h, int id)
{
  return (h->rules.flags & MJO_F_RED) && (id == 16 || id == 52 || id == 88);
}
static int take_tile(const MjoHandle *h, E *e, int s, int id)   /* wall tile -> hand; returns tile code */
{
  int k = id >> 2, red = is_red_id(h, id);
  e->hand[s][k]++;
  if (red) e->hand_red[s] |= (uint8_t)(1 << (k / 9));
  return k | red << 6;
}

/* value of seat s winning on tile kind w now (tsumo: w already in hand) */
static void eval_seat(const MjoHandle *h, const E *e, int s, int w, int tsumo, int chankan, MjoHandResult *r)
{
  MjoHandQuery q;
  memset(&q, 0, sizeof q);
  memcpy(q.hand, e->hand[s], 34);
  if (!tsumo) q.hand[w]++;
  q.n_meld = e->n_meld[s];
  for (int j = 0; j < 4; j++) q.meld[j] = e->meld[s][j];
  q.win_kind = (uint8_t)w;
  int f = 0;
  if (tsumo) f |= 1;
  if (e->ippatsu[s]) f |= 2;
  if (tsumo && e->rinshan) f |= 4;
  if (chankan) f |= 8;
  if (tsumo && e->live_left == 0 && !e->rinshan) f |= 16;
  if (!tsumo && !chankan && e->live_left == 0) f |= 32;
  if (tsumo && e->first_turn[s]) f |= 64;
  q.flags = (uint8_t)f;
  q.riichi = e->riichi[s];
  q.seat_wind = (uint8_t)((s - dealer_of(e)) & 3);
  q.round_wind = (uint8_t)(e->kyoku >> 2);
  q.n_ind = e->n_dora;
  for (int i = 0; i < 5; i++) { q.ind[i] = e->wall[126 + i] >> 2; q.ura[i] = e->wall[131 + i] >> 2; }
  int aka = 0;
  for (int b = 0; b < 3; b++) aka += e->hand_red[s] >> b & 1;
  for (int j = 0; j < e->n_meld[s]; j++) aka += m_has_red(e->meld[s][j]);
  /* a red five won by ron is not in the hand yet */
  if (!tsumo && !chankan && t_red(e->last_discard) && t_kind(e->last_discard) == w) aka++;
  if (chankan && t_red(e->kakan_tile)) aka++;
  q.n_aka = (uint8_t)aka;
  q.kuitan = (h->rules.flags & MJO_F_KUITAN) ? 1 : 0;
  mjo_eval_hand(&q, r);
}

static int furiten(const E *e, int s)
{
  return e->furiten_temp[s] || e->furiten_riichi[s] || (e->waits[s] & e->discarded_kinds[s]) != 0;
}

static void clear_masks(E *e) { memset(e->mask, 0, sizeof e->mask); e->actor_mask = 0; }

static void clear_first_turn_and_ippatsu(E *e)
{
  for (int s = 0; s < 4; s++) { e->ippatsu[s] = 0; e->first_turn[s] = 0; }
}

/* legal actions of the seat to move (phase TURN) */
static void turn_mask(const MjoHandle *h, E *e)
{
  int s = e->cur;
  uint64_t m[2] = {0, 0};
  clear_masks(e);
  e->phase = MJO_TURN;
  e->actor_mask = (uint8_t)(1 << s);
  int drawn_k = e->drawn == 255 ? -1 : t_kind(e->drawn);

  int can_tsumo = 0;
  if (drawn_k >= 0 && mjo_is_complete(e->hand[s], e->n_meld[s])) {
    MjoHandResult r;
    eval_seat(h, e, s, drawn_k, 1, 0, &r);
    can_tsumo = r.yaku_ok;
  }

  if (e->riichi_pending) {
    /* only discards that keep the hand tenpai */
    for (int k = 0; k < 34; k++) if (e->hand[s][k]) {
      e->hand[s][k]--;
      uint64_t w = mjo_waits_of(e->hand[s], e->meld[s], e->n_meld[s]);
      e->hand[s][k]++;
      if (!w) continue;
      if (nonred(e, s, k) > 0) set_bit(m, MJO_A_DISCARD + k);
      if (is_five(k) && (e->hand_red[s] >> (k / 9) & 1)) set_bit(m, MJO_A_DISCARD_RED + k / 9);
    }
  } else if (e->riichi[s]) {
    /* in riichi: cut the drawn tile, or win, or a concealed kan that keeps the waits */
    if (t_red(e->drawn)) set_bit(m, MJO_A_DISCARD_RED + drawn_k / 9);
    else set_bit(m, MJO_A_DISCARD + drawn_k);
    if (can_tsumo) set_bit(m, MJO_A_TSUMO);
    if (e->live_left > 0 && e->n_kan < 4 && e->hand[s][drawn_k] == 4) {
      uint8_t hh[34];
      uint16_t mm[4];
      memcpy(hh, e->hand[s], 34);
      memcpy(mm, e->meld[s], sizeof mm);
      hh[drawn_k] = 0;
      mm[e->n_meld[s]] = m_make(M_ANKAN, drawn_k, 0, 0, 0, 0);
      if (mjo_waits_of(hh, mm, e->n_meld[s] + 1) == e->waits[s]) set_bit(m, MJO_A_KAN + drawn_k);
    }
  } else {
    for (int k = 0; k < 34; k++) if (e->hand[s][k] && k != e->kuikae[0] && k != e->kuikae[1]) {
      if (nonred(e, s, k) > 0) set_bit(m, MJO_A_DISCARD + k);
      if (is_five(k) && (e->hand_red[s] >> (k / 9) & 1)) set_bit(m, MJO_A_DISCARD_RED + k / 9);
    }
    if (can_tsumo) set_bit(m, MJO_A_TSUMO);
    if (drawn_k >= 0 && e->live_left > 0 && e->n_kan < 4) {
      for (int k = 0; k < 34; k++) {
        if (e->hand[s][k] == 4) set_bit(m, MJO_A_KAN + k);
        else if (e->hand[s][k] >= 1)
          for (int j = 0; j < e->n_meld[s]; j++)
            if (m_type(e->meld[s][j]) == M_PON && m_kind(e->meld[s][j]) == k) set_bit(m, MJO_A_KAN + k);
      }
    }
    if (drawn_k >= 0 && is_menzen(e, s) && e->score[s] >= 1000 && e->live_left >= 4) {
      int ok = 0;
      for (int k = 0; k < 34 && !ok; k++) if (e->hand[s][k]) {
        e->hand[s][k]--;
        if (mjo_waits_of(e->hand[s], e->meld[s], e->n_meld[s])) ok = 1;
        e->hand[s][k]++;
      }
      if (ok) set_bit(m, MJO_A_RIICHI);
    }
    if ((h->rules.flags & MJO_F_ABORT) && e->first_turn[s] && drawn_k >= 0) {
      int n = 0;
      for (int k = 0; k < 34; k++) if (is_yaochu(k) && e->hand[s][k]) n++;
      if (n >= 9) set_bit(m, MJO_A_KYUUSHU);
    }
  }
  e->mask[s][0] = m[0]; e->mask[s][1] = m[1];
}

static void draw_live(const MjoHandle *h, E *e, int s)
{
  e->cur = (uint8_t)s;
  int id = e->wall[e->draw_ptr++];
  e->live_left--;
  e->rinshan = 0;
  e->drawn = (uint8_t)take_tile(h, e, s, id);
}

static void deal(MjoHandle *h, int64_t b, int reshuffle)
{
  E *e = &h->env[b];
  if (reshuffle) mjo_shuffle_wall(h->seed, h->rules.env_id_base + (uint32_t)b, e->kyoku_serial, e->wall);
  memset(e->hand, 0, sizeof e->hand);
  memset(e->hand_red, 0, 4);
  memset(e->meld, 0, sizeof e->meld);
  memset(e->n_meld, 0, 4);
  memset(e->river, 0, sizeof e->river);
  memset(e->n_river, 0, 4);
  memset(e->riichi_idx, 255, 4);
  memset(e->riichi, 0, 4);
  memset(e->ippatsu, 0, 4);
  memset(e->first_turn, 1, 4);
  memset(e->furiten_temp, 0, 4);
  memset(e->furiten_riichi, 0, 4);
  memset(e->kan_by, 0, 4);
  memset(e->discarded_kinds, 0, sizeof e->discarded_kinds);
  e->draw_ptr = 52; e->n_kan = 0; e->live_left = 70; e->n_dora = 1; e->dora_pending = 0;
  e->n_hist = 0; memset(e->hist, 0, sizeof e->hist);
  e->drawn = 255; e->riichi_pending = 0; e->rinshan = 0;
  e->last_discard = 255; e->last_discarder = 255; e->kakan_tile = 255;
  e->kuikae[0] = e->kuikae[1] = 255;
  e->first_wind = 255; e->same_wind_cnt = 0;
  int dealer = dealer_of(e);
  for (int j = 0; j < 4; j++) {
    int s = (dealer + j) & 3;
    for (int t = 0; t < 13; t++) take_tile(h, e, s, e->wall[13 * j + t]);
  }
  for (int s = 0; s < 4; s++) refresh_waits(e, s);
  draw_live(h, e, dealer);
  turn_mask(h, e);
}

static void new_game(MjoHandle *h, int64_t b)
{
  E *e = &h->env[b];
  for (int s = 0; s < 4; s++) { e->score[s] = h->rules.start_score; e->final_rank[s] = 0; }
  e->kyoku = 0; e->honba = 0; e->kyotaku = 0; e->terminated = 0;
  deal(h, b, 1);
}

static void clear_result(E *e)
{
  e->end_type = 0; e->winners = 0; e->loser = 255; e->tenpai_mask = 0;
  for (int s = 0; s < 4; s++) {
    e->han[s] = e->fu[s] = e->yakuman_units[s] = 0;
    e->r_dora[s] = e->r_ura[s] = e->r_aka[s] = 0;
    e->yaku[s] = 0; e->gain[s] = 0;
  }
}

static void pay(E *e, int from, int to, int32_t amount)
{
  e->score[from] -= amount; e->delta[from] -= amount;
  e->score[to] += amount; e->delta[to] += amount;
}

/* After the payments of a finished kyoku: rotate or repeat the dealer, end
 * the game by mode / bust / last round, or deal the next kyoku in this step. */
static void finish_kyoku(MjoHandle *h, int64_t b, int renchan, int honba_up)
{
  E *e = &h->env[b];
  int last = h->rules.mode == 0 ? 0 : h->rules.mode == 1 ? 3 : 7;
  int over = h->rules.mode == 0;
  for (int s = 0; s < 4; s++) if (e->score[s] < 0) over = 1;
  if ((h->rules.flags & MJO_F_ENDGAME) && h->rules.mode != 0) {
    /* End of game by points (the paper's rule set follows Tenhou, section 3.2; this is this library's reading of
     * that site's ending rules): the last regular kyoku ends the game only if somebody has 30,000; otherwise play
     * goes on for at most one more round, ending after any kyoku that leaves somebody at 30,000; a dealer who
     * repeats in the last regular kyoku or later ends the game when alone in the lead with 30,000. */
    int dealer = dealer_of(e), limit = last + 4, lead = 1;
    int32_t top = e->score[0];
    for (int s = 1; s < 4; s++) if (e->score[s] > top) top = e->score[s];
    for (int s = 0; s < 4; s++) if (s != dealer && e->score[s] >= e->score[dealer]) lead = 0;
    if (e->kyoku >= last) {
      if (!renchan) { if (top >= 30000 || e->kyoku == limit) over = 1; }
      else if ((lead && e->score[dealer] >= 30000) || (e->kyoku > last && top >= 30000)) over = 1;
    }
  } else if (!renchan && e->kyoku == last) over = 1;
  if (honba_up) { if (e->honba < 255) e->honba++; } else e->honba = 0;
  if (!renchan && !over) e->kyoku++;
  if (over) {
    int top = 0;
    for (int s = 1; s < 4; s++) if (e->score[s] > e->score[top]) top = s;
    int32_t sticks = 1000 * (int32_t)e->kyotaku;
    e->score[top] += sticks; e->delta[top] += sticks; e->kyotaku = 0;
    for (int s = 0; s < 4; s++) {
      int r = 0;
      for (int o = 0; o < 4; o++)
        if (e->score[o] > e->score[s] || (e->score[o] == e->score[s] && o < s)) r++;
      e->final_rank[s] = (uint8_t)r;
    }
    e->terminated = 1; e->phase = MJO_TERMINAL;
    clear_masks(e);
    return;
  }
  e->kyoku_serial++;
  deal(h, b, 1);
}

/* win by the seats in `winners` (bit mask).  tsumo: one winner, everybody
 * pays.  ron: `loser` pays every winner in full, honba included; the sticks
 * go to the winner closest after the loser in turn order. */
/* MJO_F_PAO: the seat liable for winner s's big three dragons or big four winds, or -1.  Reading (section 3.2
 * names the rule set, not this detail): all three dragon sets (all four wind sets) are exposed, and the one exposed
 * last was claimed from a discard; the discarder of that tile is liable.  Melds are stored in the order they were
 * made, and a pon that later took its fourth tile keeps its place and its source. */
static int pao_seat(const E *e, int s, uint64_t yaku)
{
  int lo, need;
  if (yaku >> Y_DAISANGEN & 1) { lo = 31; need = 3; }
  else if (yaku >> Y_DAISUUSHII & 1) { lo = 27; need = 4; }
  else return -1;
  int cnt = 0, last = -1;
  for (int j = 0; j < e->n_meld[s]; j++) {
    int k = m_kind(e->meld[s][j]);
    if (m_type(e->meld[s][j]) != M_CHI && k >= lo && k < lo + need) { cnt++; last = j; }
  }
  if (cnt != need || m_type(e->meld[s][last]) == M_ANKAN) return -1;
  return (s + (e->meld[s][last] >> 9 & 3)) & 3;
}

static void win(MjoHandle *h, int64_t b, int winners, int tsumo, int loser, int w, int chankan)
{
  E *e = &h->env[b];
  int dealer = dealer_of(e);
  clear_result(e);
  e->end_type = tsumo ? 1 : 2;
  e->winners = (uint8_t)winners;
  e->loser = tsumo ? 255 : (uint8_t)loser;
  int stick_seat = -1;
  if (tsumo) { for (int s = 0; s < 4; s++) if (winners >> s & 1) stick_seat = s; }
  else for (int d = 3; d >= 1; d--) if (winners >> ((loser + d) & 3) & 1) stick_seat = (loser + d) & 3;
  for (int s = 0; s < 4; s++) if (winners >> s & 1) {
    MjoHandResult r;
    eval_seat(h, e, s, w, tsumo, chankan, &r);
    e->han[s] = r.han; e->fu[s] = r.fu; e->yakuman_units[s] = r.yakuman_units; e->yaku[s] = r.yaku;
    e->r_dora[s] = r.n_dora; e->r_ura[s] = r.n_ura; e->r_aka[s] = r.n_aka;
    int32_t base = base_points(r.han, r.fu, r.yakuman_units);
    int32_t before = e->score[s];
    int liable = (h->rules.flags & MJO_F_PAO) ? pao_seat(e, s, r.yaku) : -1;
    if (liable >= 0 && (tsumo || liable != loser)) {
      /* The liable yakuman is one unit, worth `part` to this winner by ron or by self-draw alike.  Self-draw: the
       * liable seat pays all of it and the counter bonus; any further yakuman of the hand is paid by all three as
       * usual.  Ron off somebody else: the two share the liable part evenly, the discarder pays the rest and the
       * counter bonus.  (Ron off the liable seat itself is an ordinary ron.) */
      int32_t part = 8000 * (s == dealer ? 6 : 4), rest = 8000 * (r.yakuman_units - 1), bonus = 300 * (int32_t)e->honba;
      if (tsumo) {
        pay(e, liable, s, part + bonus);
        if (rest > 0)
          for (int o = 0; o < 4; o++) if (o != s) pay(e, o, s, (s == dealer || o == dealer) ? rest * 2 : rest);
      } else {
        pay(e, liable, s, part / 2);
        pay(e, loser, s, part / 2 + rest * (s == dealer ? 6 : 4) + bonus);
      }
    } else if (tsumo) {
      for (int o = 0; o < 4; o++) if (o != s) {
        int32_t x = (s == dealer || o == dealer) ? up100(base * 2) : up100(base);
        pay(e, o, s, x + 100 * (int32_t)e->honba);
      }
    } else {
      pay(e, loser, s, up100(base * (s == dealer ? 6 : 4)) + 300 * (int32_t)e->honba);
    }
    if (s == stick_seat) {
      int32_t sticks = 1000 * (int32_t)e->kyotaku;
      e->score[s] += sticks; e->delta[s] += sticks; e->kyotaku = 0;
    }
    e->gain[s] = e->score[s] - before;
  }
  int renchan = winners >> dealer & 1;
  finish_kyoku(h, b, renchan, renchan);
}

static void exhaustive_draw(MjoHandle *h, int64_t b)
{
  E *e = &h->env[b];
  clear_result(e);
  e->end_type = 3;
  int T = 0, n = 0;
  for (int s = 0; s < 4; s++) if (e->waits[s] || e->riichi[s]) { T |= 1 << s; n++; }
  e->tenpai_mask = (uint8_t)T;
  /* Reading (the paper names the rule set, section 3.2, not this detail), with MJO_F_NAGASHI: a seat whose river
   * holds terminals and honors only, none of them claimed by another seat, is paid as for a self-drawn mangan
   * (4000 from or to the dealer, 2000 between the others), without counter bonus; deposits stay on the table.
   * Several seats can qualify; the payments for tenpai are not made then.  The dealer still repeats when tenpai
   * and the counter goes up, as after any exhaustive draw.  end_type 10, winners = the seats paid. */
  int N = 0;
  if (h->rules.flags & MJO_F_NAGASHI)
    for (int s = 0; s < 4; s++) {
      int ok = e->n_river[s] > 0;
      for (int i = 0; i < e->n_river[s]; i++)
        if (!is_yaochu(e->river[s][i] & 63) || (e->river[s][i] & 0x80)) ok = 0;
      if (ok) N |= 1 << s;
    }
  if (N) {
    int dealer = dealer_of(e);
    e->end_type = 10;
    e->winners = (uint8_t)N;
    for (int w = 0; w < 4; w++) if (N >> w & 1)
      for (int o = 0; o < 4; o++) if (o != w) {
        int32_t pay = (w == dealer || o == dealer) ? 4000 : 2000;
        e->score[o] -= pay; e->delta[o] -= pay;
        e->score[w] += pay; e->delta[w] += pay; e->gain[w] += pay;
      }
  } else if (n >= 1 && n <= 3) {
    int32_t give = 3000 / (4 - n), get = 3000 / n;
    for (int s = 0; s < 4; s++) {
      int32_t x = (T >> s & 1) ? get : -give;
      e->score[s] += x; e->delta[s] += x;
    }
  }
  finish_kyoku(h, b, T >> dealer_of(e) & 1, 1);
}

static void abortive_draw(MjoHandle *h, int64_t b, int type)
{
  E *e = &h->env[b];
  clear_result(e);
  e->end_type = (uint8_t)type;
  finish_kyoku(h, b, 1, 1);
}

/* next seat draws, or the wall is exhausted */
static void advance(MjoHandle *h, int64_t b)
{
  E *e = &h->env[b];
  if (e->live_left == 0) { exhaustive_draw(h, b); return; }
  draw_live(h, e, (e->last_discarder + 1) & 3);
  turn_mask(h, e);
}

/* indicators of earlier open / added kans that wait to be turned are turned now */
static void turn_pending_indicators(E *e)
{
  e->n_dora = (uint8_t)(e->n_dora + e->dora_pending);
  e->dora_pending = 0;
}

/* the replacement draw that completes any kan; `open` = a kan from a discard or a tile added to a pon */
static void finish_kan(MjoHandle *h, int64_t b, int open)
{
  E *e = &h->env[b];
  int s = e->cur;
  e->kan_by[s]++;
  /* Reading (the paper names the rule set, section 3.2, not this detail): by default the new indicator is shown at
   * once for every kan type.  With MJO_F_KANDORA_LATE only a concealed kan shows it at once; after an open or
   * added kan it is turned when the seat discards (before anyone answers that discard) or declares another kan,
   * so a win on the replacement tile does not count it. */
  if ((h->rules.flags & MJO_F_KANDORA_LATE) && open) e->dora_pending++;
  else e->n_dora++;
  int id = e->wall[122 + e->n_kan];
  e->n_kan++;
  e->live_left--;
  clear_first_turn_and_ippatsu(e);
  e->drawn = (uint8_t)take_tile(h, e, s, id);
  e->rinshan = 1;
  e->kakan_tile = 255;
  turn_mask(h, e);
}

/* The discard was not won on: a pending riichi is established and paid for;
 * then the abortive draws that are judged on a surviving discard.
 * Returns 1 when the kyoku ended here. */
static int settle_discard(MjoHandle *h, int64_t b)
{
  E *e = &h->env[b];
  int d = e->last_discarder;
  if (e->riichi_pending) {
    e->score[d] -= 1000; e->delta[d] -= 1000;
    e->kyotaku++;
    e->riichi[d] = e->riichi_pending;      /* 2 when declared in the first go-around without calls */
    e->ippatsu[d] = 1;
    e->riichi_idx[d] = (uint8_t)(e->n_river[d] - 1);
    e->riichi_pending = 0;
  }
  if (h->rules.flags & MJO_F_ABORT) {
    if (e->same_wind_cnt == 4) { abortive_draw(h, b, 5); return 1; }
    if (e->riichi[0] && e->riichi[1] && e->riichi[2] && e->riichi[3]) { abortive_draw(h, b, 6); return 1; }
    if (e->n_kan == 4 && e->kan_by[0] != 4 && e->kan_by[1] != 4 && e->kan_by[2] != 4 && e->kan_by[3] != 4) {
      abortive_draw(h, b, 7); return 1;
    }
  }
  return 0;
}

/* what seat o may do about the tile `code` just discarded by d */
static void response_options(const MjoHandle *h, E *e, int o, int d, int code, uint64_t m[2])
{
  int k = t_kind(code);
  m[0] = m[1] = 0;
  e->hand[o][k]++;
  int shape = mjo_is_complete(e->hand[o], e->n_meld[o]);
  e->hand[o][k]--;
  if (shape) {
    int ok = 0;
    if (!furiten(e, o)) {
      MjoHandResult r;
      eval_seat(h, e, o, k, 0, 0, &r);
      ok = r.yaku_ok;
    }
    if (ok) set_bit(m, MJO_A_RON);
    else if (e->riichi[o]) e->furiten_riichi[o] = 1;
    else e->furiten_temp[o] = 1;
  }
  if (!e->riichi[o] && e->live_left > 0) {
    int total = concealed_total(e, o);
    int red_held = is_five(k) && (e->hand_red[o] >> (k / 9) & 1);
    if (total - e->hand[o][k] > 0) {                  /* something else is left to discard */
      if (nonred(e, o, k) >= 2) set_bit(m, MJO_A_PON);
      if (red_held && nonred(e, o, k) >= 1) set_bit(m, MJO_A_PON_RED);
    }
    if (e->hand[o][k] >= 3 && e->n_kan < 4) set_bit(m, MJO_A_MINKAN);
    if (o == ((d + 1) & 3) && is_suited(k)) {
      int r = k % 9;
      /* pos 0: called tile lowest, 1: middle, 2: highest */
      for (int pos = 0; pos < 3; pos++) {
        int lo = r - pos;                              /* rank of the lowest tile of the run */
        if (lo < 0 || lo > 6) continue;
        int base = k - pos, a = -1, c2 = -1;
        for (int t = 0; t < 3; t++) if (t != pos) { if (a < 0) a = base + t; else c2 = base + t; }
        if (e->hand[o][a] == 0 || e->hand[o][c2] == 0) continue;
        int extra = -1;                                /* kind that may not be discarded besides k */
        if (pos == 0 && r + 3 <= 8) extra = k + 3;
        if (pos == 2 && r - 3 >= 0) extra = k - 3;
        int left = total - 2 - e->hand[o][k] - (extra >= 0 ? e->hand[o][extra] : 0);
        if (left <= 0) continue;
        int five = is_five(a) ? a : is_five(c2) ? c2 : -1;
        if (nonred(e, o, a) >= 1 && nonred(e, o, c2) >= 1) set_bit(m, MJO_A_CHI_L + pos);
        if (five >= 0 && (e->hand_red[o] >> (five / 9) & 1)) set_bit(m, MJO_A_CHI_L_RED + pos);
      }
    }
  }
  if (m[0] | m[1]) set_bit(m, MJO_A_PASS);
}

/* seat s discards the tile (kind k, red flag) */
static void discard(MjoHandle *h, int64_t b, int s, int k, int red)
{
  E *e = &h->env[b];
  turn_pending_indicators(e);
  e->hand[s][k]--;
  if (red) e->hand_red[s] &= (uint8_t)~(1 << (k / 9));
  /* A seat never discards more than 30 times in a kyoku: between two discards of one seat the turn goes once round the
   * table (4 seats); a live draw moves it by one seat, a claim by at most three; there are at most 70 live draws and
   * 16 claims (4 melds per seat), so 4 (n - 1) <= 70 + 3 * 16 gives n <= 30.  The 32 entries are enough. */
  assert(e->n_river[s] < 32);
  e->river[s][e->n_river[s]++] = (uint8_t)(k | red << 6);
  e->discarded_kinds[s] |= 1ull << k;
  e->furiten_temp[s] = 0;
  if (e->riichi[s] && e->ippatsu[s]) e->ippatsu[s] = 0;
  /* four-winds tracker: discards made while the first go-around is unbroken */
  if (e->first_turn[s] && e->same_wind_cnt != 255) {
    if (is_wind(k) && (e->same_wind_cnt == 0 || k == e->first_wind)) { e->first_wind = (uint8_t)k; e->same_wind_cnt++; }
    else e->same_wind_cnt = 255;
  }
  e->first_turn[s] = 0;
  e->kuikae[0] = e->kuikae[1] = 255;
  refresh_waits(e, s);
  e->last_discard = (uint8_t)(k | red << 6);
  e->last_discarder = (uint8_t)s;
  e->drawn = 255;

  int any = 0;
  uint64_t m[4][2];
  memset(m, 0, sizeof m);
  for (int o = 0; o < 4; o++) if (o != s) {
    response_options(h, e, o, s, e->last_discard, m[o]);
    if (m[o][0] | m[o][1]) any |= 1 << o;
  }
  if (any) {
    clear_masks(e);
    e->phase = MJO_RESPOND;
    e->actor_mask = (uint8_t)any;
    memcpy(e->mask, m, sizeof m);
    return;
  }
  if (settle_discard(h, b)) return;
  advance(h, b);
}

static void remove_from_hand(E *e, int s, int k, int n_nonred, int take_red)
{
  e->hand[s][k] -= (uint8_t)(n_nonred + take_red);
  if (take_red) e->hand_red[s] &= (uint8_t)~(1 << (k / 9));
}

static void do_call(MjoHandle *h, int64_t b, int s, int a)
{
  E *e = &h->env[b];
  int d = e->last_discarder, k = t_kind(e->last_discard), cred = t_red(e->last_discard);
  int from_rel = (d - s) & 3;
  e->river[d][e->n_river[d] - 1] |= 0x80;
  clear_first_turn_and_ippatsu(e);
  e->cur = (uint8_t)s;
  e->drawn = 255;
  e->rinshan = 0;
  int j = e->n_meld[s]++;
  if (a == MJO_A_PON || a == MJO_A_PON_RED) {
    int tr = a == MJO_A_PON_RED;
    remove_from_hand(e, s, k, tr ? 1 : 2, tr);
    e->meld[s][j] = m_make(M_PON, k, from_rel, 0, tr || cred, cred);
    e->kuikae[0] = (uint8_t)k; e->kuikae[1] = 255;
    turn_mask(h, e);
  } else if (a == MJO_A_MINKAN) {
    int tr = is_five(k) && (e->hand_red[s] >> (k / 9) & 1);
    remove_from_hand(e, s, k, tr ? 2 : 3, tr);
    e->meld[s][j] = m_make(M_MINKAN, k, from_rel, 0, tr || cred, cred);
    refresh_waits(e, s);
    finish_kan(h, b, 1);
  } else {
    int pos = (a - MJO_A_CHI_L) % 3, tr = a >= MJO_A_CHI_L_RED;
    int base = k - pos;
    for (int t = 0; t < 3; t++) if (t != pos) {
      int kk = base + t, r = tr && is_five(kk);
      remove_from_hand(e, s, kk, r ? 0 : 1, r);
    }
    e->meld[s][j] = m_make(M_CHI, base, from_rel, pos, tr || cred, cred);
    e->kuikae[0] = (uint8_t)k;
    e->kuikae[1] = 255;
    if (pos == 0 && k % 9 + 3 <= 8) e->kuikae[1] = (uint8_t)(k + 3);
    if (pos == 2 && k % 9 - 3 >= 0) e->kuikae[1] = (uint8_t)(k - 3);
    turn_mask(h, e);
  }
}

/* Seats other than s that can win on kind k of a kan that s has just declared get RON and PASS in m; returns
 * them as a bit set.  A seat whose hand the tile completes but that may not win on it becomes furiten.
 * `orphans_only`: only the thirteen orphans count (the tile of a concealed kan, MJO_F_ANKAN_ROB). */
static int offer_rob(MjoHandle *h, E *e, int s, int k, int orphans_only, uint64_t m[4][2])
{
  int any = 0;
  for (int o = 0; o < 4; o++) if (o != s) {
    e->hand[o][k]++;
    int shape = orphans_only ? (e->n_meld[o] == 0 && thirteen_orphans(e->hand[o])) : mjo_is_complete(e->hand[o], e->n_meld[o]);
    e->hand[o][k]--;
    if (!shape) continue;
    int ok = 0;
    if (!furiten(e, o)) {
      MjoHandResult r;
      eval_seat(h, e, o, k, 0, 1, &r);
      ok = r.yaku_ok;
    }
    if (ok) { set_bit(m[o], MJO_A_RON); set_bit(m[o], MJO_A_PASS); any |= 1 << o; }
    else if (e->riichi[o]) e->furiten_riichi[o] = 1;
    else e->furiten_temp[o] = 1;
  }
  return any;
}

/* KAN action on the own turn: concealed kan with four in hand, otherwise a
 * tile added to an own pon (which the other seats may rob). */
static void own_kan(MjoHandle *h, int64_t b, int k)
{
  E *e = &h->env[b];
  int s = e->cur;
  turn_pending_indicators(e);
  if (e->hand[s][k] == 4) {
    int tr = is_five(k) && (e->hand_red[s] >> (k / 9) & 1);
    remove_from_hand(e, s, k, tr ? 3 : 4, tr);
    e->meld[s][e->n_meld[s]++] = m_make(M_ANKAN, k, 0, 0, tr, 0);
    e->drawn = 255;
    refresh_waits(e, s);
    /* Reading (section 3.2 names the rule set, not this detail), with MJO_F_ANKAN_ROB: a hand that waits for this
     * tile as thirteen orphans may win on it; the offer uses the phase of the added kan, the tile code carries
     * bit 7 to tell the two apart, and a pass lets the kan go on. */
    if ((h->rules.flags & MJO_F_ANKAN_ROB) && is_yaochu(k)) {
      uint64_t m[4][2];
      memset(m, 0, sizeof m);
      int any = offer_rob(h, e, s, k, 1, m);
      if (any) {
        e->kakan_tile = (uint8_t)(k | 0x80);
        clear_masks(e);
        e->phase = MJO_RESPOND_KAKAN;
        e->actor_mask = (uint8_t)any;
        memcpy(e->mask, m, sizeof m);
        return;
      }
    }
    finish_kan(h, b, 0);
    return;
  }
  int tr = is_five(k) && (e->hand_red[s] >> (k / 9) & 1);
  remove_from_hand(e, s, k, tr ? 0 : 1, tr);
  for (int j = 0; j < e->n_meld[s]; j++)
    if (m_type(e->meld[s][j]) == M_PON && m_kind(e->meld[s][j]) == k) {
      uint16_t m = e->meld[s][j];
      m = (uint16_t)((m & ~7) | M_KAKAN);
      if (tr) m |= 1 << 13;
      e->meld[s][j] = m;
    }
  e->kakan_tile = (uint8_t)(k | tr << 6);
  e->drawn = 255;
  refresh_waits(e, s);
  uint64_t m[4][2];
  memset(m, 0, sizeof m);
  int any = offer_rob(h, e, s, k, 0, m);
  if (any) {
    clear_masks(e);
    e->phase = MJO_RESPOND_KAKAN;
    e->actor_mask = (uint8_t)any;
    memcpy(e->mask, m, sizeof m);
    return;
  }
  finish_kan(h, b, 1);
}

static void mark_passed_ron(E *e)
{
  for (int s = 0; s < 4; s++) if ((e->actor_mask >> s & 1) && get_bit(e->mask[s], MJO_A_RON)) {
    if (e->riichi[s]) e->furiten_riichi[s] = 1; else e->furiten_temp[s] = 1;
  }
}

/* The action history of the observation (section 3.2, "Observation Space"): every public action of the kyoku in
 * the order it took effect -- discards, kans, riichi, wins and the nine-terminals draw by the seat to move; the
 * wins on a discard or kan tile in turn order from the seat that gave it; otherwise the one claim (pon, kan, chi)
 * that took the discard.  Passes and draws are not public and are not recorded.  Reading: the paper names the
 * history but not its content; this is what the other players can see. */
static void hist_push(E *e, int s, int a)
{
  if (e->n_hist < 128) e->hist[e->n_hist++] = (uint16_t)(a | s << 8);
}

static void step_env(MjoHandle *h, int64_t b, const int8_t a[4])
{
  E *e = &h->env[b];
  memset(e->delta, 0, sizeof e->delta);
  e->illegal_seat = 255;
  if (e->terminated) return;
  /* an action outside the mask ends the game at once (section 3.2) */
  for (int s = 0; s < 4; s++) if (e->actor_mask >> s & 1) {
    if (a[s] < 0 || a[s] >= MJO_NUM_ACTIONS || !get_bit(e->mask[s], a[s])) {
      e->illegal_seat = (uint8_t)s;
      clear_result(e);
      e->end_type = 9;
      e->terminated = 1;
      e->phase = MJO_TERMINAL;
      clear_masks(e);
      return;
    }
  }
  if (e->phase == MJO_TURN) {
    int s = e->cur, act = a[s];
    hist_push(e, s, act);
    if (act < MJO_A_DISCARD_RED) discard(h, b, s, act, 0);
    else if (act < MJO_A_KAN) discard(h, b, s, 4 + 9 * (act - MJO_A_DISCARD_RED), 1);
    else if (act < MJO_A_RIICHI) own_kan(h, b, act - MJO_A_KAN);
    else if (act == MJO_A_RIICHI) { e->riichi_pending = e->first_turn[s] ? 2 : 1; turn_mask(h, e); }
    else if (act == MJO_A_TSUMO) win(h, b, 1 << s, 1, -1, t_kind(e->drawn), 0);
    else abortive_draw(h, b, 4);                       /* nine terminals */
  } else if (e->phase == MJO_RESPOND) {
    int d = e->last_discarder, ronners = 0, n_ron = 0;
    for (int s = 0; s < 4; s++) if ((e->actor_mask >> s & 1) && a[s] == MJO_A_RON) { ronners |= 1 << s; n_ron++; }
    for (int j = 1; j < 4; j++) if (ronners >> ((d + j) & 3) & 1) hist_push(e, (d + j) & 3, MJO_A_RON);
    if (n_ron == 3 && (h->rules.flags & MJO_F_ABORT)) { abortive_draw(h, b, 8); return; }
    if (n_ron) { win(h, b, ronners, 0, d, t_kind(e->last_discard), 0); return; }
    mark_passed_ron(e);
    int caller = -1, call = 0;
    for (int s = 0; s < 4; s++) if ((e->actor_mask >> s & 1) && a[s] >= MJO_A_PON && a[s] <= MJO_A_MINKAN) { caller = s; call = a[s]; }
    if (caller < 0) {
      int nx = (d + 1) & 3;
      if ((e->actor_mask >> nx & 1) && a[nx] >= MJO_A_CHI_L && a[nx] <= MJO_A_CHI_H_RED) { caller = nx; call = a[nx]; }
    }
    if (settle_discard(h, b)) return;
    if (caller >= 0) hist_push(e, caller, call);
    if (caller >= 0) do_call(h, b, caller, call);
    else advance(h, b);
  } else if (e->phase == MJO_RESPOND_KAKAN) {
    int ronners = 0;
    for (int s = 0; s < 4; s++) if ((e->actor_mask >> s & 1) && a[s] == MJO_A_RON) ronners |= 1 << s;
    for (int j = 1; j < 4; j++) if (ronners >> ((e->cur + j) & 3) & 1) hist_push(e, (e->cur + j) & 3, MJO_A_RON);
    if (ronners) { win(h, b, ronners, 0, e->cur, t_kind(e->kakan_tile), 1); return; }
    mark_passed_ron(e);
    finish_kan(h, b, !(e->kakan_tile & 0x80));
  }
}

/* ------------------------------------------------------------------- API */

int mjo_create(MjoHandle **out, int64_t B, uint64_t seed, const MjoRules *rules)
{
  if (!out || !rules || B <= 0 || seed >> 32 || rules->mode > 2) return -1;
  MjoHandle *h = (MjoHandle *)calloc(1, sizeof *h);
  if (!h) return -2;
  h->env = (E *)calloc((size_t)B, sizeof(E));
  if (!h->env) { free(h); return -2; }
  h->B = B; h->seed = (uint32_t)seed; h->rules = *rules; h->step = 0;
  for (int64_t b = 0; b < B; b++) {
    E *e = &h->env[b];
    e->illegal_seat = 255; e->loser = 255;
    new_game(h, b);
  }
  *out = h;
  return 0;
}

int mjo_step(MjoHandle *h, const int8_t *actions)
{
  for (int64_t b = 0; b < h->B; b++) step_env(h, b, actions + 4 * b);
  h->step++;
  return 0;
}

int mjo_legal_mask(const MjoHandle *h, uint64_t *mask)
{
  for (int64_t b = 0; b < h->B; b++) memcpy(mask + 8 * b, h->env[b].mask, 64);
  return 0;
}

/* reward: the point change of the last step; the float view is points/1000,
 * and the illegal-action penalty for the offending seat (section 3.2). */
int mjo_reward(const MjoHandle *h, int32_t *delta, float *reward, uint8_t *terminated)
{
  for (int64_t b = 0; b < h->B; b++) {
    const E *e = &h->env[b];
    for (int s = 0; s < 4; s++) {
      if (delta) delta[4 * b + s] = e->delta[s];
      if (reward) reward[4 * b + s] = e->illegal_seat == s ? h->rules.illegal_penalty : (float)e->delta[s] * 0.001f;
    }
    if (terminated) terminated[b] = e->terminated;
  }
  return 0;
}

int mjo_reset_done(MjoHandle *h)
{
  for (int64_t b = 0; b < h->B; b++) if (h->env[b].terminated) {
    h->env[b].episode++;
    h->env[b].kyoku_serial++;
    new_game(h, b);
  }
  return 0;
}

/* uniform choice over the legal mask: key (seed, env_id), counter
 * (step_lo, step_hi, seat, 1); the mulhi(r0, n)-th set bit in ascending id */
int mjo_sample_random(MjoHandle *h, int8_t *actions)
{
  for (int64_t b = 0; b < h->B; b++) {
    const E *e = &h->env[b];
    for (int s = 0; s < 4; s++) {
      int n = 0;
      for (int a = 0; a < MJO_NUM_ACTIONS; a++) n += get_bit(e->mask[s], a);
      actions[4 * b + s] = -1;
      if (n == 0) continue;
      uint32_t ctr[4] = { (uint32_t)h->step, (uint32_t)(h->step >> 32), (uint32_t)s, 1 };
      uint32_t key[2] = { h->seed, h->rules.env_id_base + (uint32_t)b }, r[4];
      mjo_philox4x32_10(ctr, key, r);
      int pick = (int)mulhi32(r[0], (uint32_t)n);
      for (int a = 0; a < MJO_NUM_ACTIONS; a++) if (get_bit(e->mask[s], a)) {
        if (pick == 0) { actions[4 * b + s] = (int8_t)a; break; }
        pick--;
      }
    }
  }
  return 0;
}

int mjo_step_random(MjoHandle *h, int32_t n_steps, int auto_reset)
{
  int8_t *a = (int8_t *)malloc((size_t)h->B * 4);
  if (!a) return -2;
  for (int32_t t = 0; t < n_steps; t++) {
    mjo_sample_random(h, a);
    mjo_step(h, a);
    if (auto_reset) mjo_reset_done(h);
  }
  free(a);
  return 0;
}

int mjo_export(const MjoHandle *h, int64_t lo, int64_t n, MjoEnv *out)
{
  if (lo < 0 || n < 0 || lo + n > h->B) return -1;
  memcpy(out, h->env + lo, (size_t)n * sizeof(E));
  return 0;
}
int mjo_import(MjoHandle *h, int64_t lo, int64_t n, const MjoEnv *in)
{
  if (lo < 0 || n < 0 || lo + n > h->B) return -1;
  memcpy(h->env + lo, in, (size_t)n * sizeof(E));
  return 0;
}
int mjo_deal_from_wall(MjoHandle *h, int64_t b, const uint8_t wall[136])
{
  if (b < 0 || b >= h->B) return -1;
  memcpy(h->env[b].wall, wall, 136);
  deal(h, b, 0);
  return 0;
}
uint64_t mjo_step_count(const MjoHandle *h) { return h->step; }
void mjo_destroy(MjoHandle *h) { if (h) { free(h->env); free(h); } }
size_t mjo_sizeof_env(void) { return sizeof(E); }

/* Token observation (see MjoTokenObs). */
static uint8_t tile_token(int kind, int red) { return (uint8_t)(red ? 34 + kind / 9 : kind); }
int mjo_observe_tokens(const MjoHandle *h, MjoTokenObs *out)
{
  for (int64_t b = 0; b < h->B; b++) {
    const E *e = &h->env[b];
    for (int me = 0; me < 4; me++) {
      MjoTokenObs *o = &out[b * 4 + me];
      memset(o, 255, sizeof *o);
      int n = 0;
      for (int k = 0; k < 34; k++) {
        int cnt = e->hand[me][k];
        int red = (k % 9 == 4 && k < 27 && (e->hand_red[me] >> (k / 9) & 1)) ? 1 : 0;
        if (red) { o->hand[n++] = tile_token(k, 1); cnt--; }
        for (int i = 0; i < cnt; i++) o->hand[n++] = tile_token(k, 0);
      }
      o->n_hand = (uint8_t)n;
      o->shanten = (int8_t)mjo_shanten(e->hand[me], e->n_meld[me]);
      o->drawn = (e->phase == MJO_TURN && e->cur == me && e->drawn != 255) ? tile_token(e->drawn & 63, e->drawn >> 6 & 1) : 255;
      o->phase = e->phase;
      o->cur = e->phase == MJO_TURN ? (uint8_t)((e->cur - me) & 3) : 255;
      o->last_discarder = e->last_discarder == 255 ? 255 : (uint8_t)((e->last_discarder - me) & 3);
      o->last_discard = e->last_discard == 255 ? 255 : tile_token(e->last_discard & 63, e->last_discard >> 6 & 1);
      o->kyoku = e->kyoku; o->honba = e->honba; o->kyotaku = e->kyotaku;
      o->dealer = (uint8_t)((dealer_of(e) - me) & 3);
      o->live_left = e->live_left; o->n_dora = e->n_dora;
      for (int i = 0; i < 5; i++)
        o->dora[i] = i < e->n_dora ? tile_token(e->wall[126 + i] >> 2, is_red_id(h, e->wall[126 + i])) : 255;
      for (int rel = 0; rel < 4; rel++) {
        int s = (me + rel) & 3;
        o->n_meld[rel] = e->n_meld[s]; o->n_river[rel] = e->n_river[s];
        o->riichi[rel] = e->riichi[s]; o->riichi_idx[rel] = e->riichi_idx[s];
        o->score[rel] = e->score[s];
        for (int j = 0; j < 4; j++) o->meld[rel][j] = j < e->n_meld[s] ? e->meld[s][j] : 0;
        for (int i = 0; i < 32; i++) {
          if (i >= e->n_river[s]) { o->river[rel][i] = 255; continue; }
          int t = e->river[s][i];
          o->river[rel][i] = (uint8_t)(tile_token(t & 63, t >> 6 & 1) | (t & 0x80));
        }
      }
      o->n_hist = e->n_hist;
      memset(o->zero_, 0, sizeof o->zero_);
      for (int i = 0; i < e->n_hist; i++)
        o->hist[i] = (uint16_t)((e->hist[i] & 0xFF) | (((e->hist[i] >> 8) - me) & 3) << 8);
    }
  }
  return 0;
}

/* Observation, one stack of 56 planes over the 34 kinds per seat, entries 0/1,
 * seen from that seat (rel 0 self, 1 next, 2 across, 3 previous). */
int mjo_observe(const MjoHandle *h, uint8_t *obs)
{
  for (int64_t b = 0; b < h->B; b++) {
    const E *e = &h->env[b];
    int dealer = dealer_of(e);
    for (int me = 0; me < 4; me++) {
      uint8_t (*P)[34] = (uint8_t (*)[34])(obs + ((size_t)b * 4 + me) * 56 * 34);
      memset(P, 0, 56 * 34);
      for (int k = 0; k < 34; k++)
        for (int c = 1; c <= 4; c++) if (e->hand[me][k] >= c) P[c - 1][k] = 1;
      for (int su = 0; su < 3; su++) if (e->hand_red[me] >> su & 1) P[4][9 * su + 4] = 1;
      int ind_cnt[34] = {0};
      for (int i = 0; i < e->n_dora; i++) {
        ind_cnt[e->wall[126 + i] >> 2]++;
        if (is_red_id(h, e->wall[126 + i])) P[41][e->wall[126 + i] >> 2] = 1;
      }
      for (int k = 0; k < 34; k++)
        for (int c = 1; c <= 4; c++) if (ind_cnt[k] >= c) P[36 + c][k] = 1;
      for (int rel = 0; rel < 4; rel++) {
        int s = (me + rel) & 3;
        int rc[34] = {0}, mc[34] = {0};
        for (int i = 0; i < e->n_river[s]; i++) {
          int t = e->river[s][i];
          rc[t & 63]++;
          if (t >> 6 & 1) P[41][t & 63] = 1;
        }
        for (int j = 0; j < e->n_meld[s]; j++) {
          for (int k = 0; k < 34; k++) mc[k] += m_count(e->meld[s][j], k);
          if (m_has_red(e->meld[s][j])) {
            int mk = m_kind(e->meld[s][j]);
            P[41][(mk / 9) * 9 + 4] = 1;
          }
        }
        for (int k = 0; k < 34; k++)
          for (int c = 1; c <= 4; c++) {
            if (rc[k] >= c) P[5 + 4 * rel + c - 1][k] = 1;
            if (mc[k] >= c) P[21 + 4 * rel + c - 1][k] = 1;
          }
        if (e->riichi[s]) memset(P[42 + rel], 1, 34);
        for (int i = 0; i < 34; i++) if (e->score[s] >= 2000 * (i + 1)) P[49 + rel][i] = 1;
      }
      P[46][27 + (e->kyoku >> 2)] = 1;
      P[47][27 + ((me - dealer) & 3)] = 1;
      P[48][(dealer - me) & 3] = 1;
      for (int i = 0; i < 18; i++) if (e->live_left >= 4 * (i + 1)) P[53][i] = 1;
      for (int i = 18; i < 26; i++) if (e->honba >= i - 17) P[53][i] = 1;
      for (int i = 26; i < 34; i++) if (e->kyotaku >= i - 25) P[53][i] = 1;
      if (e->phase == MJO_RESPOND) P[54][t_kind(e->last_discard)] = 1;
      if (e->phase == MJO_RESPOND_KAKAN) P[54][t_kind(e->kakan_tile)] = 1;
      if (e->phase == MJO_TURN && e->cur == me && e->drawn != 255) P[55][t_kind(e->drawn)] = 1;
    }
  }
  return 0;
}
