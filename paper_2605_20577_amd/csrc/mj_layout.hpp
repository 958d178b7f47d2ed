// Structure-of-arrays layout of the environment state in HBM.
//
// For B environments every field is an array over b, so the lanes of a
// wavefront (16, 32 or 64 consecutive environments, see mj_lib.hip) touch
// consecutive addresses.
// Sections, in this order, each array of length B:
//   u64 hot : discarded_kinds[4] waits[4] mask[8] meld[4] tenpai_discards   (21 arrays)
//   u64 cold: yaku[4] result[4] next_waits[4]                               (12 arrays)
//   u32 hot : score[4] delta[4] episode serial hand[16] seatw[4]            (30 arrays)
//   u32 cold: gain[4] glob[7] wall[2][34] (two buffers of 136 tile ids, four per word: the current wall and
//             the next one) next_serial next_hand[16] next_red (the next deal, made ahead)     (97 arrays)
//   u8  cold: river[128] (arrays over b like the rest); then history[B][128] u16 (action | seat << 8): the history
//             is one ROW of 256 bytes PER ENVIRONMENT, not arrays over b, so that the token observation reads a quarter
//             of it with sixteen word loads (rivers as rows were tried as well: the plane observation kernel lost 17 %)
// = 1,156 bytes per environment, 288 of them hot.  The "next" arrays are not part of the logical state: they are
// a pure function of (seed, env id, kyoku_serial + 1), valid when next_serial says so; tenpai_discards is a cache
// (a function of the hand of the seat to move, valid when its top bit is set).  The step kernels copy the
// hot arrays of their block into LDS, run there, and copy them back.
#pragma once
#include "mj_core.hpp"

namespace mj {

constexpr int kHotU64 = 21, kColdU64 = 12, kHotU32 = 30, kColdU32 = 97, kU8Arrays = 384;
constexpr int kU64Arrays = kHotU64 + kColdU64, kU32Arrays = kHotU32 + kColdU32;
constexpr int64_t kBytesPerEnv = 8 * kU64Arrays + 4 * kU32Arrays + kU8Arrays;
constexpr int kHotBytesPerEnv = 8 * kHotU64 + 4 * kHotU32;

MJ_HD uint64_t *state_u64(void *state, int64_t B) { (void)B; return (uint64_t *)state; }
MJ_HD uint32_t *state_u32(void *state, int64_t B) { return (uint32_t *)((uint64_t *)state + (int64_t)kU64Arrays * B); }
MJ_HD uint8_t *state_u8(void *state, int64_t B) { return (uint8_t *)(state_u32(state, B) + (int64_t)kU32Arrays * B); }

MJ_HD void set_hot(Env &e, uint64_t *q, uint32_t *w, int64_t hs)
{
  e.hs = hs;
  e.dk = q; e.waits = q + 4 * hs; e.mask = q + 8 * hs; e.meld = q + 16 * hs; e.tdisc = q + 20 * hs;
  e.score = (int32_t *)w; e.delta = (int32_t *)(w + 4 * hs); e.episode = w + 8 * hs; e.serial = w + 9 * hs;
  e.hand = w + 10 * hs; e.seatw = w + 26 * hs;
}
// view of environment b with every field in HBM
MJ_HD Env make_env(void *state, int64_t B, int64_t b)
{
  Env e;
  e.n = B;
  uint64_t *q = state_u64(state, B) + b;
  uint32_t *w = state_u32(state, B) + b;
  set_hot(e, q, w, B);
  e.yaku = q + (int64_t)kHotU64 * B; e.resw = q + (int64_t)(kHotU64 + 4) * B;
  e.gain = (int32_t *)(w + (int64_t)kHotU32 * B); e.glob = w + (int64_t)(kHotU32 + 4) * B;
  e.wallw = w + (int64_t)(kHotU32 + 11) * B;
  e.nserial = w + (int64_t)(kHotU32 + 79) * B; e.nexth = w + (int64_t)(kHotU32 + 80) * B;
  e.nextred = w + (int64_t)(kHotU32 + 96) * B; e.nextwaits = q + (int64_t)(kHotU64 + 8) * B;
  e.river = state_u8(state, B) + b;
  e.hist = (uint16_t *)(state_u8(state, B) + (int64_t)128 * B) + b * 128;
  e.hstage = nullptr; e.hbase = nullptr;
  return e;
}

MJ_HD void load_glob(const Env &e, Glob &g)
{
  uint32_t w[7];
#pragma unroll
  for (int i = 0; i < 7; i++) w[i] = e.glob[(int64_t)i * e.n];
  __builtin_memcpy(&g, w, 28);
}
MJ_HD void store_glob(const Env &e, const Glob &g)
{
  uint32_t w[7];
  __builtin_memcpy(w, &g, 28);
#pragma unroll
  for (int i = 0; i < 7; i++) e.glob[(int64_t)i * e.n] = w[i];
}

}  // namespace mj
