// TEST-ONLY host build of the kernels' per-environment code.
//
// Compiles paper_2605_20577_amd/csrc/mj_*.hpp (the code every HIP kernel runs,
// one lane per environment) with g++ and loops over the environments on the
// CPU, so that the GPU-less test tier can run that logic against the oracle
// and so that it can be put under gdb or a sanitizer.  It is not part of the
// product: the Python package never loads it, and nothing here is reachable
// from libmj.so.
#ifndef MJ_HD
#define MJ_HD inline __attribute__((always_inline))
#endif
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_2605_20577_amd/csrc/mj_canon.hpp"
#include "../../paper_2605_20577_amd/csrc/mj_tables.hpp"

using namespace mj;

struct Sim {
  int64_t B;
  Rules R;
  uint64_t step;
  std::vector<uint64_t> state;
  mjt::SuitTables T;
  Lut L;
};

static Ctx ctx_of(Sim *h, int64_t b)
{
  Ctx c;
  c.e = make_env(h->state.data(), h->B, b);
  c.L = h->L; c.R = h->R; c.env_id = h->R.env_id_base + (uint32_t)b;
  c.need_deal = false; c.need_turn = false; c.live_ptr = -1;
  return c;
}
static void reset_env(Ctx &c, bool first)
{
  if (first) {
    c.e.episode[0] = 0; c.e.serial[0] = 0;
    memset(&c.g, 0, sizeof c.g);
    clear_result(c);
    for (int s = 0; s < 4; s++) DELTA(c, s) = 0;
    c.g.illegal_seat = 255;
  } else { c.e.episode[0]++; c.e.serial[0]++; }
  new_game(c);
  if (c.need_deal) deal(c, true);
  step_finish(c);
}
static uint32_t pack4(const int a[4])
{
  return (uint32_t)(uint8_t)a[0] | (uint32_t)(uint8_t)a[1] << 8 | (uint32_t)(uint8_t)a[2] << 16 | (uint32_t)(uint8_t)a[3] << 24;
}
static void step_and_deal(Ctx &c, const int a[4], int sampled_ron = -1)
{
  step_env(c, pack4(a), sampled_ron);
  if (c.need_deal) deal(c, true);
  step_finish(c);
}

extern "C" {

Sim *hs_create(int64_t B, uint64_t seed, const MjRules *r)
{
  Sim *h = new Sim();
  h->B = B; h->step = 0;
  h->R.flags = r->flags; h->R.env_id_base = r->env_id_base; h->R.start_score = r->start_score;
  h->R.illegal_penalty = r->illegal_penalty; h->R.mode = r->mode; h->R.seed = (uint32_t)seed;
  h->state.assign((size_t)(B * kBytesPerEnv + 7) / 8, 0);
  h->T = mjt::build();
  h->L.rowid = h->T.rowid.data(); h->L.bitmap = h->T.bitmap.data(); h->L.base = h->T.base.data();
  h->L.rowrank = h->T.rowrank.data(); h->L.recs = h->T.recs.data();
  static const std::vector<uint32_t> nb_table = mjt::build_neighbour_table();
  h->L.nb = nb_table.data();
  for (int64_t b = 0; b < B; b++) { Ctx c = ctx_of(h, b); reset_env(c, true); store_glob(c.e, c.g); }
  return h;
}
void hs_destroy(Sim *h) { delete h; }
void hs_table_stats(Sim *h, int *out) { out[0] = h->T.n_keys; out[1] = h->T.n_recs; out[2] = h->T.n_rows; }

void hs_step(Sim *h, const int8_t *actions)
{
  for (int64_t b = 0; b < h->B; b++) {
    Ctx c = ctx_of(h, b);
    load_glob(c.e, c.g);
    int a[4] = {actions[4 * b], actions[4 * b + 1], actions[4 * b + 2], actions[4 * b + 3]};
    step_and_deal(c, a);
    store_glob(c.e, c.g);
  }
  h->step++;
}
void hs_sample(Sim *h, int8_t *actions)
{
  for (int64_t b = 0; b < h->B; b++) {
    Ctx c = ctx_of(h, b);
    for (int s = 0; s < 4; s++)
      actions[4 * b + s] = (int8_t)sample_action(MASK(c, s, 0), MASK(c, s, 1), h->R.seed, c.env_id, h->step, s);
  }
}
void hs_reset_done(Sim *h)
{
  for (int64_t b = 0; b < h->B; b++) {
    Ctx c = ctx_of(h, b);
    load_glob(c.e, c.g);
    if (!c.g.terminated) continue;
    reset_env(c, false);
    store_glob(c.e, c.g);
  }
}
void hs_step_random(Sim *h, int n, int auto_reset)
{
  // as the fused kernel does it: the action history is staged in a column of 136 bytes per environment (bytes at
  // stride B, like the hot arrays here), flushed every kHistFlushEvery steps and at the end; every 64 steps the kernel
  // uses the column for a shuffle, which is a fill with junk here
  std::vector<uint8_t> stage((size_t)137 * h->B, 0xEE);
  for (int64_t b = 0; b < h->B; b++) {
    Ctx c = ctx_of(h, b);
    load_glob(c.e, c.g);
    c.e.hstage = stage.data() + b;
    c.e.hbase = stage.data() + (size_t)136 * h->B + b;
    *c.e.hbase = c.g.hist_len;
    for (int t = 0; t < n; t++) {
      if ((h->step + t) % kHistFlushEvery == 0) {
        hist_flush(c.e, c.g.hist_len);
        if ((h->step + t) % 64 == 0) for (int i = 0; i < 136; i++) c.e.hstage[(int64_t)i * h->B] = 0xEE;
      }
      int a[4], ron_offered = 0;                  // as the fused kernel does it: sampled actions skip the legality check
      for (int s = 0; s < 4; s++) {
        a[s] = sample_action(MASK(c, s, 0), MASK(c, s, 1), h->R.seed, c.env_id, h->step + t, s);
        if ((c.g.actor_mask >> s & 1) && (MASK(c, s, 1) >> (A_RON - 64) & 1)) ron_offered |= 1 << s;
      }
      step_and_deal(c, a, ron_offered);
      if (auto_reset && c.g.terminated) reset_env(c, false);
    }
    hist_flush(c.e, c.g.hist_len);
    store_glob(c.e, c.g);
  }
  h->step += n;
}
void hs_export(Sim *h, int64_t lo, int64_t n, MjEnvCanon *out)
{
  for (int64_t i = 0; i < n; i++) export_env(make_env(h->state.data(), h->B, lo + i), out[i]);
}
void hs_import(Sim *h, int64_t lo, int64_t n, const MjEnvCanon *in)
{
  for (int64_t i = 0; i < n; i++) import_env(make_env(h->state.data(), h->B, lo + i), in[i]);
}
void hs_deal_from_wall(Sim *h, int64_t b, const uint8_t *wall)
{
  Ctx c = ctx_of(h, b);
  load_glob(c.e, c.g);
  for (int i = 0; i < 136; i++) wall_set(c.e, c.g.wall_sel, i, wall[i]);
  deal(c, false);
  store_glob(c.e, c.g);
}
void hs_observe(Sim *h, uint8_t *obs)
{
  for (int64_t b = 0; b < h->B; b++) {
    Env e = make_env(h->state.data(), h->B, b);
    Glob g;
    load_glob(e, g);
    uint64_t S[4][OB_SEAT_WORDS], G[OG_WORDS], red = 0;
    for (int s = 0; s < 4; s++) red |= obs_seat_masks(e, s, S[s]);
    uint32_t dw[2];
    dora_words(e, g.wall_sel, dw);
    obs_env_masks(g, h->R.flags, red, dw, G);
    for (int me = 0; me < 4; me++)
      for (int p = 0; p < 56; p++) {
        uint64_t v = obs_plane(p, me, &S[0][0], e.seatw[me * h->B] & 7u, G) & K_ALL;
        for (int k = 0; k < 34; k++) obs[(((size_t)b * 4 + me) * 56 + p) * 34 + k] = (uint8_t)(v >> k & 1);
      }
  }
}
void hs_observe_tokens(Sim *h, MjTokenObs *out)
{
  static const std::vector<uint32_t> sh_suit = mjt::build_shanten_table(9, true), sh_honor = mjt::build_shanten_table(7, false);
  for (int64_t b = 0; b < h->B; b++) {
    Env e = make_env(h->state.data(), h->B, b);
    Glob g;
    load_glob(e, g);
    for (int me = 0; me < 4; me++) token_obs(e, g, me, h->R.flags, sh_suit.data(), sh_honor.data(), out[b * 4 + me]);
  }
}
int hs_shanten(Sim *h, const uint8_t *hand, int n_meld)
{
  (void)h;
  static const std::vector<uint32_t> sh_suit = mjt::build_shanten_table(9, true), sh_honor = mjt::build_shanten_table(7, false);
  uint32_t hw[4] = {0, 0, 0, 0};
  for (int k = 0; k < 34; k++) { int su = suit_of(k); hw[su] |= (uint32_t)hand[k] << (3 * rank_of(k, su)); }
  return shanten_of(sh_suit.data(), sh_honor.data(), hw[0], hw[1], hw[2], hw[3], n_meld);
}
void hs_eval_hands(Sim *h, int64_t n, const MjHandQuery *in, MjHandResult *out)
{
  for (int64_t i = 0; i < n; i++) {
    const MjHandQuery &q = in[i];
    HandIn hi;
    for (int su = 0; su < 4; su++) {
      uint32_t hw = 0;
      int nr = su == 3 ? 7 : 9;
      for (int r = 0; r < nr; r++) {
        uint32_t cnt = q.hand[(su == 3 ? 27 : 9 * su) + r];
        hw |= (cnt > 7 ? 7u : cnt) << (3 * r);
      }
      hi.h[su] = hw;
    }
    hi.meldw = (uint64_t)q.meld[0] | (uint64_t)q.meld[1] << 16 | (uint64_t)q.meld[2] << 32 | (uint64_t)q.meld[3] << 48;
    hi.n_meld = q.n_meld; hi.win = q.win_kind; hi.flags = q.flags; hi.riichi = q.riichi;
    hi.seat_wind = q.seat_wind; hi.round_wind = q.round_wind; hi.n_ind = q.n_ind; hi.n_aka = q.n_aka; hi.kuitan = q.kuitan;
    for (int j = 0; j < 5; j++) { hi.ind[j] = q.ind[j]; hi.ura[j] = q.ura[j]; }
    HandOut ho;
    eval_hand(&h->L, hi, ho);
    MjHandResult r;
    memset(&r, 0, sizeof r);
    r.yaku = ho.yaku; r.points = ho.points; r.han = (uint8_t)ho.han; r.fu = (uint8_t)ho.fu;
    r.yakuman_units = (uint8_t)ho.units; r.shape_ok = (uint8_t)ho.shape_ok; r.yaku_ok = (uint8_t)ho.yaku_ok;
    r.n_dora = (uint8_t)ho.n_dora; r.n_ura = (uint8_t)ho.n_ura; r.n_aka = (uint8_t)ho.n_aka;
    out[i] = r;
  }
}
uint64_t hs_waits(Sim *h, const uint8_t *hand, const uint16_t *meld, int n_meld)
{
  uint32_t hw[4] = {0, 0, 0, 0};
  for (int k = 0; k < 34; k++) { int su = suit_of(k); hw[su] |= (uint32_t)hand[k] << (3 * rank_of(k, su)); }
  uint64_t mw = 0;
  for (int j = 0; j < 4; j++) mw |= (uint64_t)meld[j] << (16 * j);
  return waits_of(&h->L, hw[0], hw[1], hw[2], hw[3], mw, n_meld) & K_ALL;
}

uint64_t hs_tenpai_discards(Sim *h, const uint8_t *hand, const uint16_t *meld, int n_meld)
{
  uint32_t hw[4] = {0, 0, 0, 0};
  for (int k = 0; k < 34; k++) { int su = suit_of(k); hw[su] |= (uint32_t)hand[k] << (3 * rank_of(k, su)); }
  uint64_t mw = 0;
  for (int j = 0; j < 4; j++) mw |= (uint64_t)meld[j] << (16 * j);
  return tenpai_discards_of(&h->L, hw[0], hw[1], hw[2], hw[3], mw, n_meld, true);
}

}  // extern "C"
