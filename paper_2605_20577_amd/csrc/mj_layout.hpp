// Structure-of-arrays layout of the environment state in HBM.
//
// For B environments every field is an array over b, so the 64 lanes of a
// wavefront (64 consecutive environments) touch consecutive addresses.
// Sections, in this order, each array of length B:
//   u64: discarded_kinds[4] waits[4] mask[8] yaku[4] meld[4] result[4]      (28 arrays)
//   u32: score[4] delta[4] gain[4] episode serial hand[16] seatw[4] glob[7] (41 arrays)
//   u8 : wall[136] river[128]                                               (264 arrays)
// = 652 bytes per environment.
#pragma once
#include "mj_core.hpp"

namespace mj {

constexpr int kU64Arrays = 28, kU32Arrays = 41, kU8Arrays = 264;
constexpr int64_t kBytesPerEnv = 8 * kU64Arrays + 4 * kU32Arrays + kU8Arrays;

MJ_HD Env make_env(void *state, int64_t B, int64_t b)
{
  Env e;
  e.n = B;
  uint64_t *q = (uint64_t *)state + b;
  e.dk = q; e.waits = q + 4 * B; e.mask = q + 8 * B; e.yaku = q + 16 * B; e.meld = q + 20 * B; e.resw = q + 24 * B;
  uint32_t *w = (uint32_t *)((uint64_t *)state + (int64_t)kU64Arrays * B) + b;
  e.score = (int32_t *)w; e.delta = (int32_t *)(w + 4 * B); e.gain = (int32_t *)(w + 8 * B);
  e.episode = w + 12 * B; e.serial = w + 13 * B; e.hand = w + 14 * B; e.seatw = w + 30 * B; e.glob = w + 34 * B;
  uint8_t *y = (uint8_t *)((uint32_t *)((uint64_t *)state + (int64_t)kU64Arrays * B) + (int64_t)kU32Arrays * B) + b;
  e.wall = y; e.river = y + 136 * B;
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
