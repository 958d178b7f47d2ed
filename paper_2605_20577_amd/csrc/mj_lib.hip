// libmj: HIP kernels (gfx950) and the C ABI of include/mj.h.
//
// Step kernels (k_rollout, k_step, k_new_games) map one lane to one environment, with LPW = 16 or 32 (or 64)
// environments per wavefront and the remaining lanes idle: the step is bound by instruction issue along divergent
// paths, so narrower wavefronts and two of them per SIMD run faster than full ones.  A block of 128 lanes (two
// wavefronts) stages into LDS the probe part of the per-suit pattern table (11 KB), the hot state arrays of its
// environments (288 B each, structure of arrays, see mj_layout.hpp) and a 136-byte shuffle column per environment;
// it runs its steps there and writes the hot arrays back.  Walls are shuffled ahead of time, every lane for itself
// on its LDS column; a deal that finds no wall ready is done by the whole wavefront for one environment at a time
// (ballot over the lanes that need it, 34 lanes run Philox, the wall sits in one vector register and the swaps are
// readlane / select pairs).  Between two shuffles the fused kernel uses an environment's shuffle column as a ring
// that collects the entries of its action history, written to HBM every 32 steps.  The observation writers build bit planes / token records per environment in LDS and
// then stream them out with all lanes, 16 bytes per lane.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstddef>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/mj.h"
#include "mj_canon.hpp"
#include "mj_tables.hpp"

using namespace mj;

static_assert(sizeof(MjTokenObs) == 496, "token record");
static_assert(sizeof(MjEnvCanon) == 1000, "canonical record layout");
static_assert(sizeof(MjHandQuery) == 64 && sizeof(MjHandResult) == 24, "hand records");
static_assert(sizeof(Glob) == 28, "control bytes");

namespace {

constexpr int kBlock = 128;              // lanes per block of the step kernels
constexpr int kAuxBlock = 256;           // lanes per block of the helper kernels

struct DevTables {
  const uint8_t *probe;                  // global: rowid[kRowIdBytes] followed by bitmap[rows * 20]
  const uint16_t *base, *rowrank;
  const uint32_t *recs;
  const uint32_t *nb;                    // neighbours of every suit pattern (7.8 MB, read through L2)
  int probe_bytes;                       // multiple of 16
};
constexpr int kRowIdBytes = 3136;        // 3125 row ids padded to a multiple of 16
#ifndef MJ_OCC
#define MJ_OCC 2                         // waves per SIMD the register budget of the stepping kernels is sized for
#endif
constexpr int kRefillEvery = 64;         // steps between refills of the walls made ahead of time
#ifndef MJ_STEP_REFILL
#define MJ_STEP_REFILL 32
#endif
constexpr int kStepRefillEvery = MJ_STEP_REFILL;   // the same for the one-step kernels
static_assert(kRefillEvery % kHistFlushEvery == 0, "the history's staging ring is empty when the shuffle takes its column");

// A step kernel may leave lanes of each wavefront idle: with LPW (lanes per wave) of 32 or 16 the same batch
// occupies 2x or 4x as many wavefronts, which lets a SIMD overlap the LDS / memory latency of one wavefront
// with the instructions of another and shrinks the set of divergent paths per wavefront.  The step is bound by
// dependent-access latency, not by lane count, so small batches run faster that way.
// LDS of a step kernel: probe tables | hot u64 arrays | hot u32 arrays | 136 wall bytes per env | one byte per env
// (between two shuffles the wall bytes of an environment stage its action history, see hist_push; the last byte
// says where the staged entries start)
__host__ __device__ inline int envs_per_block(int lpw) { return (kBlock / 64) * lpw; }
__host__ __device__ inline size_t step_lds_bytes(int probe_bytes, int lpw)
{
  return (size_t)probe_bytes + (size_t)envs_per_block(lpw) * (kHotBytesPerEnv + 136 + 1);
}

struct BlockMem {
  Lut L;                                 // table pointers: the probe tables in LDS, the records in HBM.  Held by value
                                         // (in registers) so that the probes compile to LDS reads, not flat loads.
  uint64_t *hq;                          // [kHotU64][envs per block]
  uint32_t *hw;                          // [kHotU32][envs per block]
  uint8_t *col;                          // this lane's column of the [136][envs per block] shuffle area
  uint8_t *hbase;                        // this lane's byte of the [envs per block] area behind the shuffle area
  int epb, idx;                          // envs per block; this lane's env slot in the block
  bool lane_on;                          // this lane carries an environment
};

// The probe tables go from global memory to the block's LDS in two halves, so that a kernel can put its own loads
// between them: table_fetch starts the loads (all in flight together), table_commit writes them to LDS.  A caller
// that loads its hot state in between pays one memory round trip for both.
constexpr int kTableChunks = 6;          // 16-byte chunks per lane: 6 x 128 lanes x 16 B = 12 KB >= the probe tables
struct TableRegs { uint4 v[kTableChunks]; };
__device__ __forceinline__ TableRegs table_fetch(const DevTables &T)
{
  TableRegs r;
  const uint4 *src = (const uint4 *)T.probe;
  const int n = T.probe_bytes / 16;
#pragma unroll
  for (int k = 0; k < kTableChunks; k++) {
    const int i = (int)threadIdx.x + k * kBlock;
    r.v[k] = i < n ? src[i] : make_uint4(0, 0, 0, 0);
  }
  return r;
}
__device__ __forceinline__ void table_commit(const DevTables &T, uint8_t *lds, const TableRegs &r)
{
  uint4 *dst = (uint4 *)lds;
  const int n = T.probe_bytes / 16;
#pragma unroll
  for (int k = 0; k < kTableChunks; k++) {
    const int i = (int)threadIdx.x + k * kBlock;
    if (i < n) dst[i] = r.v[k];
  }
}
// carve up the block's LDS (no memory traffic)
template <int LPW>
__device__ __forceinline__ BlockMem carve_block(const DevTables &T, uint8_t *lds)
{
  BlockMem m;
  m.epb = envs_per_block(LPW);
  m.idx = (int)(threadIdx.x >> 6) * LPW + (int)(threadIdx.x & 63);
  m.lane_on = (threadIdx.x & 63) < LPW;
  m.hq = (uint64_t *)(lds + T.probe_bytes);
  m.hw = (uint32_t *)(lds + T.probe_bytes + (size_t)m.epb * 8 * kHotU64);
  m.L.rowid = lds;
  m.L.bitmap = (const uint32_t *)(lds + kRowIdBytes);
  m.L.base = T.base; m.L.rowrank = T.rowrank; m.L.recs = T.recs; m.L.nb = T.nb;
  m.col = lds + T.probe_bytes + (size_t)m.epb * kHotBytesPerEnv + m.idx;
  m.hbase = lds + T.probe_bytes + (size_t)m.epb * (kHotBytesPerEnv + 136) + m.idx;
  return m;
}
// ... and copy the probe tables in (ends with a block barrier)
template <int LPW>
__device__ __forceinline__ BlockMem stage_block(const DevTables &T, uint8_t *lds)
{
  BlockMem m = carve_block<LPW>(T, lds);
  const TableRegs r = table_fetch(T);
  table_commit(T, lds, r);
  __syncthreads();
  return m;
}
// the per-lane environment view: hot fields in LDS, cold fields in HBM
__device__ __forceinline__ Env block_env(const BlockMem &m, void *state, int64_t B, int64_t b)
{
  Env e = make_env(state, B, b);
  set_hot(e, m.hq + m.idx, m.hw + m.idx, m.epb);
  return e;
}
__device__ __forceinline__ void load_hot(const BlockMem &m, void *state, int64_t B, int64_t b)
{
  const uint64_t *gq = state_u64(state, B) + b;
  const uint32_t *gw = state_u32(state, B) + b;
#pragma unroll
  for (int f = 0; f < kHotU64; f++) m.hq[f * m.epb + m.idx] = gq[(int64_t)f * B];
#pragma unroll
  for (int f = 0; f < kHotU32; f++) m.hw[f * m.epb + m.idx] = gw[(int64_t)f * B];
}
__device__ __forceinline__ void store_hot(const BlockMem &m, void *state, int64_t B, int64_t b)
{
  uint64_t *gq = state_u64(state, B) + b;
  uint32_t *gw = state_u32(state, B) + b;
#pragma unroll
  for (int f = 0; f < kHotU64; f++) gq[(int64_t)f * B] = m.hq[f * m.epb + m.idx];
#pragma unroll
  for (int f = 0; f < kHotU32; f++) gw[(int64_t)f * B] = m.hw[f * m.epb + m.idx];
}

// Deal for every lane of the wavefront that needs one.  All 64 lanes must call this together.
// One environment at a time, with values that are uniform over the wavefront:
//   - 34 lanes run Philox (counter word 1 = lane) and turn their four words into four swap targets;
//   - the wall lives in ONE vector register, four tile ids per lane in lanes 0..33; instead of doing the 135 swaps
//     of the Fisher-Yates pass one after the other, every position is traced back through them on its own lane
//     (compare / select against swap targets read by readlane; no memory and no long dependent chain in the loop);
//   - lanes 0..33 store their word of the wall to HBM; lanes 0..3 collect the 13 tiles of one seat wind each into
//     packed hand words (lane permutes) and compute the waits of the four hands side by side;
//   - the owner lane writes the results into its state and takes the dealer's first draw.

__device__ __forceinline__ void deal_wave(Ctx &c, bool need, void *state, int64_t B, int64_t b)
{
  const int lane = threadIdx.x & 63;
  unsigned long long pending = __ballot(need ? 1 : 0);
  const uint32_t my_serial = need ? c.e.serial[0] : 0u;
  const uint32_t my_kyoku = c.g.kyoku;
  const uint32_t b_lo = (uint32_t)b, b_hi = (uint32_t)((uint64_t)b >> 32);
  const bool red_rules = (c.R.flags & F_RED) != 0;
  while (pending) {
    const int src = __builtin_ctzll(pending);
    pending &= pending - 1;
    const uint32_t serial = __builtin_amdgcn_readlane(my_serial, src);
    const uint32_t env_id = __builtin_amdgcn_readlane(c.env_id, src);
    const int dealer = (int)(__builtin_amdgcn_readlane(my_kyoku, src) & 3u);
    const int64_t bsrc = (int64_t)(((uint64_t)__builtin_amdgcn_readlane(b_hi, src) << 32) | __builtin_amdgcn_readlane(b_lo, src));
    // swap targets: lane j holds k[4j .. 4j+3]; position 135 is never swapped (target = itself)
    uint32_t kv0 = 0, kv1 = 0, kv2 = 0, kv3 = 0;
    if (lane < 34) {
      uint32_t r[4];
      philox(serial, (uint32_t)lane, 0, 0, c.R.seed, env_id, r);
      const int i = 4 * lane;
      kv0 = i + mulhi(r[0], (uint32_t)(136 - i));
      kv1 = i + 1 + mulhi(r[1], (uint32_t)(135 - i));
      kv2 = i + 2 + mulhi(r[2], (uint32_t)(134 - i));
      kv3 = i + 3 < 135 ? i + 3 + mulhi(r[3], (uint32_t)(133 - i)) : (uint32_t)(i + 3);
    }
    // The permutation without doing the swaps one after the other: position i is final after swap i, which puts
    // there what stood at k_i just before; what stood at a position q > j before swap j is what stood at j before it
    // if q = k_j, else what stood at q.  So every position is traced back on its own -- q = k_i, then for j = i - 1
    // down to 0: q = j where q = k_j -- to the tile id it started as (the wall starts as 0..135).  Lane L < 34 traces
    // positions 4L..4L+3 (their k_i are its own four values; position 135 is never swapped as "i": k = 135); the only
    // value carried through the 135 steps is q, the k_j come from registers by readlane.
    uint32_t q0 = kv0, q1 = kv1, q2 = kv2, q3 = kv3;
    const uint32_t i0 = 4u * (uint32_t)lane;
    for (int jj = 33; jj >= 0; jj--) {
#pragma unroll
      for (int t = 3; t >= 0; t--) {
        const uint32_t j = 4u * (uint32_t)jj + (uint32_t)t;
        if (j >= 135u) continue;
        const uint32_t kj = __builtin_amdgcn_readlane(t == 0 ? kv0 : t == 1 ? kv1 : t == 2 ? kv2 : kv3, jj);
        q0 = (j < i0 && q0 == kj) ? j : q0;
        q1 = (j < i0 + 1u && q1 == kj) ? j : q1;
        q2 = (j < i0 + 2u && q2 == kj) ? j : q2;
        q3 = (j < i0 + 3u && q3 == kj) ? j : q3;
      }
    }
    // the wall: ids of positions 4*lane .. 4*lane+3 in the four bytes of lane's word
    const uint32_t wv = lane < 34 ? (q0 | q1 << 8 | q2 << 16 | q3 << 24) : 0u;
    // the wall goes to HBM, one word per lane
    const int sel = (int)__builtin_amdgcn_readlane((uint32_t)c.g.wall_sel, src);
    if (lane < 34) (state_u32(state, B) + (int64_t)(kHotU32 + 11 + 34 * sel) * B + bsrc)[(int64_t)lane * B] = wv;
    // 4 x 13 tiles -> packed hand words: lane j < 4 collects the hand of seat wind j (its tiles come from the other
    // lanes' wall words by a lane permute; every lane takes part, lanes >= 4 repeat the work of lane & 3) and then
    // computes that hand's waits.  Field 3k of a 102-bit accumulator counts kind k, as in refill_next_wall.
    uint32_t h0, h1, h2, h3, reds = 0;
    {
      const int j = lane & 3;
      uint64_t lo = 0, hi = 0;
#pragma unroll 1                          // rolled on purpose: unrolled, the thirteen permutes in flight cost the kernel
      for (int t = 0; t < 13; t++) {          // registers on a path that is rare (measured 1.7 % of the rollout's rate)
        const int i = 13 * j + t;
        const uint32_t id = ((uint32_t)__shfl((int)wv, i >> 2) >> (8 * (i & 3))) & 255u;
        const uint32_t kind = id >> 2;
        if (kind < 21) lo += 1ull << (3 * kind); else hi += 1ull << (3 * (kind - 21));
        if (red_rules && (id == 16u || id == 52u || id == 88u)) reds |= 1u << (kind / 9);
      }
      h0 = (uint32_t)lo & 0x7FFFFFFu; h1 = (uint32_t)(lo >> 27) & 0x7FFFFFFu;
      h2 = (uint32_t)(lo >> 54) | ((uint32_t)hi & 0x3FFFFu) << 9; h3 = (uint32_t)(hi >> 18);
    }
    uint64_t wt = 0;
    if (lane < 4) wt = waits_of(&c.L, h0, h1, h2, h3, 0, 0);
    const uint32_t wt_lo = (uint32_t)wt, wt_hi = (uint32_t)(wt >> 32);
    const uint32_t first_id = (__builtin_amdgcn_readlane(wv, 13) >> 0) & 255u;        // wall[52]
    if (lane == src) {
      deal_reset(c);
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const int s = (dealer + j) & 3;
        HW(c, s, 0) = __builtin_amdgcn_readlane(h0, j); HW(c, s, 1) = __builtin_amdgcn_readlane(h1, j);
        HW(c, s, 2) = __builtin_amdgcn_readlane(h2, j); HW(c, s, 3) = __builtin_amdgcn_readlane(h3, j);
        SW(c, s) |= __builtin_amdgcn_readlane(reds, j);
        WAITS(c, s) = (uint64_t)__builtin_amdgcn_readlane(wt_hi, j) << 32 | __builtin_amdgcn_readlane(wt_lo, j);
      }
      // the dealer's first draw (wall[52]) without going through HBM
      c.g.draw_ptr = 53; c.g.live_left = 69; c.g.kanflags &= (uint8_t)~1u;
      c.g.drawn = (uint8_t)take_tile(c, dealer, (int)first_id);
      c.need_deal = false;
      c.need_turn = true;
    }
  }
}

// Walls are made ahead of time: the wall of a deal depends only on (seed, env id, kyoku_serial), so each lane
// shuffles the wall of its NEXT deal every kRefillEvery steps, all lanes side by side, deals it into four
// hands and computes their waits; the deal itself then only copies about 60 words.  (A deal that finds no wall ready, e.g. the second deal inside one interval, falls back to
// the wave-cooperative shuffle above.)  Plain per-lane Fisher-Yates on a byte column in LDS.
__device__ __forceinline__ void refill_next_wall(Ctx &c, uint8_t *col, int stride, uint32_t target_serial)
{
  for (int i = 0; i < 136; i++) col[i * stride] = (uint8_t)i;
  for (int j = 0; j < 34; j++) {
    uint32_t r[4];
    philox(target_serial, (uint32_t)j, 0, 0, c.R.seed, c.env_id, r);
#pragma unroll
    for (int t = 0; t < 4; t++) {
      const int i = 4 * j + t;
      if (i >= 135) break;
      const int k = i + (int)mulhi(r[t], (uint32_t)(136 - i));
      const uint8_t x = col[i * stride], y = col[k * stride];
      col[i * stride] = y; col[k * stride] = x;
    }
  }
  for (int j = 0; j < 34; j++) {
    const uint32_t w = (uint32_t)col[(4 * j) * stride] | (uint32_t)col[(4 * j + 1) * stride] << 8 |
                       (uint32_t)col[(4 * j + 2) * stride] << 16 | (uint32_t)col[(4 * j + 3) * stride] << 24;
    c.e.wallw[(int64_t)((1 - c.g.wall_sel) * 34 + j) * c.e.n] = w;
  }
  // the four dealt hands (by seat wind j) and their waits, so that the deal itself is only a copy.
  // Field 3k of a 102-bit accumulator counts kind k: kinds 0..20 in `lo`, 21..33 in `hi`.
  const bool red_rules = (c.R.flags & F_RED) != 0;
  uint32_t reds = 0;
#pragma unroll 1
  for (int j = 0; j < 4; j++) {
    uint64_t lo = 0, hi = 0;
#pragma unroll
    for (int t = 0; t < 13; t++) {
      const uint32_t id = col[(13 * j + t) * stride];
      const uint32_t kind = id >> 2;
      if (kind < 21) lo += 1ull << (3 * kind); else hi += 1ull << (3 * (kind - 21));
      if (red_rules && (id == 16u || id == 52u || id == 88u)) reds |= 1u << (3 * j + kind / 9);
    }
    const uint32_t h0 = (uint32_t)lo & 0x7FFFFFFu, h1 = (uint32_t)(lo >> 27) & 0x7FFFFFFu;
    const uint32_t h2 = (uint32_t)(lo >> 54) | ((uint32_t)hi & 0x3FFFFu) << 9, h3 = (uint32_t)(hi >> 18);
    c.e.nexth[(int64_t)(4 * j) * c.e.n] = h0; c.e.nexth[(int64_t)(4 * j + 1) * c.e.n] = h1;
    c.e.nexth[(int64_t)(4 * j + 2) * c.e.n] = h2; c.e.nexth[(int64_t)(4 * j + 3) * c.e.n] = h3;
    c.e.nextwaits[(int64_t)j * c.e.n] = waits_of(&c.L, h0, h1, h2, h3, 0, 0);
  }
  c.e.nextred[0] = reds;
  c.e.nserial[0] = target_serial;
}

// the deal of a lane whose next deal is ready: copies only
__device__ __forceinline__ void deal_from_next(Ctx &c)
{
  const int64_t n = c.e.n;
  uint32_t hw[16];
  uint64_t wt[4];
#pragma unroll
  for (int i = 0; i < 16; i++) hw[i] = c.e.nexth[(int64_t)i * n];
#pragma unroll
  for (int j = 0; j < 4; j++) wt[j] = c.e.nextwaits[(int64_t)j * n];
  const uint32_t reds = c.e.nextred[0];
  c.g.wall_sel ^= 1;                                        // the spare wall becomes the wall: no copy
  const uint32_t first = c.e.wallw[(int64_t)(c.g.wall_sel * 34 + 13) * n] & 255u;      // wall[52]
  deal_reset(c);
  const int dealer = dealer_of(c);
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const int s = (dealer + j) & 3;
#pragma unroll
    for (int q = 0; q < 4; q++) HW(c, s, q) = hw[4 * j + q];
    SW(c, s) |= (reds >> (3 * j)) & 7u;
    WAITS(c, s) = wt[j];
  }
  c.g.draw_ptr = 53; c.g.live_left = 69; c.g.kanflags &= (uint8_t)~1u;
  c.g.drawn = (uint8_t)take_tile(c, dealer, (int)first);
  c.need_deal = false;
  c.need_turn = true;
}

// every deal of a step: the ready ones lane by lane, the others through the wave-cooperative shuffle
__device__ __forceinline__ void deal_stage(Ctx &c, bool active, void *state, int64_t B, int64_t b)
{
  const bool need = active && c.need_deal;
  const bool ready = need && c.e.nserial[0] == c.e.serial[0];
  MJ_RB(dn, ready);
  if (ready) deal_from_next(c);
  MJ_RE(dn, PR_DEAL_NEXT);
  MJ_RB(dw, need && !ready);
  deal_wave(c, need && !ready, state, B, b);
  MJ_RE(dw, PR_DEAL_WAVE);
}

__device__ __forceinline__ void reset_env(Ctx &c, bool first)
{
  if (first) {
    c.e.episode[0] = 0; c.e.serial[0] = 0;
    __builtin_memset(&c.g, 0, sizeof c.g);
    clear_result(c);
#pragma unroll
    for (int s = 0; s < 4; s++) DELTA(c, s) = 0;
    c.g.illegal_seat = 255;
  } else {
    c.e.episode[0]++; c.e.serial[0]++;
  }
  new_game(c);
}

// mode 0: first initialisation of every env; mode 1: restart of the terminated ones (a block without a
// terminated env leaves before it stages anything)
template <int LPW>
__global__ void __launch_bounds__(kBlock, MJ_OCC) k_new_games(void *state, int64_t B, Rules R, DevTables T, int mode)
{
  extern __shared__ __align__(16) uint8_t lds[];
  if (mode == 1) {
    const int idx = (int)(threadIdx.x >> 6) * LPW + (int)(threadIdx.x & 63);
    const int64_t b0 = (int64_t)blockIdx.x * envs_per_block(LPW) + idx;
    int term = 0;
    if ((threadIdx.x & 63) < LPW && b0 < B) term = (int)(make_env(state, B, b0).glob[0] >> 24 & 0xFFu);   // Glob::terminated
    if (!__syncthreads_or(term)) return;
  }
  BlockMem m = carve_block<LPW>(T, lds);
  const int64_t b = (int64_t)blockIdx.x * m.epb + m.idx;
  const bool active = m.lane_on && b < B;
  Ctx c;
  c.e = block_env(m, state, B, active ? b : 0); c.L = m.L; c.R = R; c.env_id = R.env_id_base + (uint32_t)b;
  c.need_deal = false; c.need_turn = false; c.live_ptr = -1;
  bool touched = false;
  const TableRegs tr = table_fetch(T);
  if (active && mode == 1) { load_hot(m, state, B, b); load_glob(c.e, c.g); }     // with the tables: one round trip
  table_commit(T, lds, tr);
  __syncthreads();
  if (active) {
    if (mode == 0) {
      reset_env(c, true); touched = true;
      refill_next_wall(c, m.col, m.epb, 0);          // every lane deals now: make the first walls side by side
    } else if (c.g.terminated) { reset_env(c, false); touched = true; }
  }
  deal_stage(c, active, state, B, b);
  if (touched) { step_finish(c); store_hot(m, state, B, b); store_glob(c.e, c.g); }
  if (mode == 0 && active) refill_next_wall(c, m.col, m.epb, 1);
}

#ifdef MJ_PROFILE
__device__ long long mj_kstep_prof[4096][8];      // profiling builds only: time stamps of the last k_step launch
__device__ unsigned long long mj_kstep_regions[2048][3 * PR_N];   // ... and its region counters, per block
#endif
// what a step can hand back besides the new state (any pointer may be null)
struct StepOut {
  uint64_t *mask;          // [B][4][2] legal actions of the state after the step (after the restart, if any)
  int32_t *delta;          // [B][4] point changes of this step
  float *reward;           // [B][4] the same as reward (points / 1000, or the penalty for an illegal action)
  uint8_t *terminated;     // [B] the game ended with this step (or had ended before)
};

template <int LPW>
__global__ void __launch_bounds__(kBlock, MJ_OCC) k_step(void *state, int64_t B, Rules R, DevTables T, const int8_t *actions, int refill,
                                                 int auto_reset, StepOut out)
{
  extern __shared__ __align__(16) uint8_t lds[];
#ifdef MJ_PROFILE
  long long pt[8];
  for (int i = threadIdx.x; i < 3 * PR_N; i += blockDim.x) mj_prof[i] = 0;
  __syncthreads();
  pt[0] = wall_clock64();
#define MJ_PT(i) pt[i] = wall_clock64()
#else
#define MJ_PT(i) ((void)0)
#endif
  BlockMem m = carve_block<LPW>(T, lds);
  const int64_t b = (int64_t)blockIdx.x * m.epb + m.idx;
  const bool active = m.lane_on && b < B;
  Ctx c;
  c.e = block_env(m, state, B, active ? b : 0); c.L = m.L; c.R = R; c.env_id = R.env_id_base + (uint32_t)b;
  c.need_deal = false; c.need_turn = false; c.live_ptr = -1;
  // the tables, the hot state and the control bytes come in with one memory round trip
  const TableRegs tr = table_fetch(T);
  uint32_t acts = 0;
  if (active) {
    load_hot(m, state, B, b);
    load_glob(c.e, c.g);
    acts = ((const uint32_t *)actions)[b];
  }
  table_commit(T, lds, tr);
  __syncthreads();
  MJ_PT(1);
  if (active) {
    if (refill && c.e.nserial[0] != c.e.serial[0] + 1) refill_next_wall(c, m.col, m.epb, c.e.serial[0] + 1);
    MJ_PT(2);
    step_env(c, acts);
    MJ_PT(3);
    // the step's own results go out before a finished game is started again
    if (out.delta) ((int4 *)out.delta)[b] = make_int4(DELTA(c, 0), DELTA(c, 1), DELTA(c, 2), DELTA(c, 3));
    if (out.reward) {
      float r[4];
#pragma unroll
      for (int s = 0; s < 4; s++) r[s] = c.g.illegal_seat == s ? R.illegal_penalty : (float)DELTA(c, s) * 0.001f;
      ((float4 *)out.reward)[b] = make_float4(r[0], r[1], r[2], r[3]);
    }
    if (out.terminated) out.terminated[b] = c.g.terminated;
    if (auto_reset && c.g.terminated) reset_env(c, false);
  }
  MJ_PT(4);
  deal_stage(c, active, state, B, b);
  MJ_PT(5);
  if (active) {
    step_finish(c);
    MJ_PT(6);
    if (out.mask) {
#pragma unroll
      for (int s = 0; s < 4; s++) {
        ulonglong2 w;
        w.x = MASK(c, s, 0); w.y = MASK(c, s, 1);
        ((ulonglong2 *)out.mask)[b * 4 + s] = w;
      }
    }
    store_hot(m, state, B, b);
    store_glob(c.e, c.g);
  }
#ifdef MJ_PROFILE
  MJ_PT(7);
  // 10 ns ticks per wavefront: in, staged, refilled, stepped, (outputs), dealt, mask, stored
  if ((threadIdx.x & 63) == 0 && blockIdx.x < 2048) {
    long long *o = mj_kstep_prof[blockIdx.x * 2 + (threadIdx.x >> 6)];
    for (int i = 0; i < 8; i++) o[i] = active ? pt[i] : 0;
  }
  __syncthreads();
  if (blockIdx.x < 2048)
    for (int i = threadIdx.x; i < 3 * PR_N; i += blockDim.x) mj_kstep_regions[blockIdx.x][i] = mj_prof[i];
#endif
#undef MJ_PT
}

// the random policy for every acting seat of the lane's environment, packed as four signed bytes
// (also notes, in ron_offered, the seats whose mask offers a win: the step needs that and skips its own look at the
// masks when the actions come from here)
__device__ __forceinline__ uint32_t sample_actors(Ctx &c, uint64_t step, int &ron_offered)
{
  uint32_t acts = 0xFFFFFFFFu, am = c.g.actor_mask;
  ron_offered = 0;
  while (am) {
    int s = __builtin_ctz(am);
    am &= am - 1;
    const uint64_t m0 = MASK(c, s, 0), m1 = MASK(c, s, 1);
    if (m1 >> (A_RON - 64) & 1) ron_offered |= 1 << s;
    int a = sample_action(m0, m1, c.R.seed, c.env_id, step, s);
    acts = (acts & ~(0xFFu << (8 * s))) | ((uint32_t)(uint8_t)(int8_t)a << (8 * s));
  }
  return acts;
}

// n_steps of { sample, step, optional reset } without leaving the kernel: environments never interact
template <int LPW>
__global__ void __launch_bounds__(kBlock, MJ_OCC) k_rollout(void *state, int64_t B, Rules R, DevTables T, uint64_t step0,
                                                    int n_steps, int auto_reset, int64_t env_lo, int64_t env_hi)
{
  extern __shared__ __align__(16) uint8_t lds[];
  BlockMem m = carve_block<LPW>(T, lds);
  const int64_t b = env_lo + (int64_t)blockIdx.x * m.epb + m.idx;      // the launch covers environments [env_lo, env_hi)
  const bool active = m.lane_on && b < env_hi;
  Ctx c;
  c.e = block_env(m, state, B, active ? b : 0); c.L = m.L; c.R = R; c.env_id = R.env_id_base + (uint32_t)b;
  c.need_deal = false; c.need_turn = false; c.live_ptr = -1;
  const TableRegs tr = table_fetch(T);
  if (active) { load_hot(m, state, B, b); load_glob(c.e, c.g); }
  table_commit(T, lds, tr);
  // the action history is staged in the lane's shuffle column (hist_push): empty now, flushed before every shuffle
  // and at the end
  if (active) { c.e.hstage = m.col; c.e.hbase = m.hbase; *m.hbase = c.g.hist_len; }
  __syncthreads();
#ifdef MJ_PROFILE
  for (int i = threadIdx.x; i < 3 * PR_N; i += blockDim.x) mj_prof[i] = 0;
  __syncthreads();
#endif
  for (int t = 0; t < n_steps; t++) {
    uint32_t acts = 0;
    MJ_RB(loop, true);
    // The stride of the cold arrays is made opaque once per step: otherwise every address "array + k * stride" is
    // computed before the loop and kept in a register pair for the whole launch (dozens of pairs, many of them
    // spilled to scratch memory and fetched back one by one on the rare paths that use them).
    { int64_t stride = c.e.n; asm volatile("" : "+s"(stride)); c.e.n = stride; }
    if (active) {
      MJ_RB(rf, (step0 + t) % kRefillEvery == 0 && c.e.nserial[0] != c.e.serial[0] + 1);
      if ((step0 + t) % kHistFlushEvery == 0) {
        hist_flush(c.e, c.g.hist_len);                 // the shuffle needs the column that stages the history
        if ((step0 + t) % kRefillEvery == 0 && c.e.nserial[0] != c.e.serial[0] + 1)
          refill_next_wall(c, m.col, m.epb, c.e.serial[0] + 1);
      }
      MJ_RE(rf, PR_REFILL);
      int ron_offered;
      MJ_RB(sa, true);
      acts = sample_actors(c, step0 + t, ron_offered);
      MJ_RE(sa, PR_SAMPLE);
      MJ_RB(st, true);
      step_env<1>(c, acts, ron_offered);
      MJ_RE(st, PR_STEP);
      MJ_RB(rs, auto_reset && c.g.terminated);
      if (auto_reset && c.g.terminated) reset_env(c, false);
      MJ_RE(rs, PR_RESET);
    }
    MJ_RB(dl, active && c.need_deal);
    deal_stage(c, active, state, B, b);
    MJ_RE(dl, PR_DEAL);
    MJ_RB(fin, active && c.need_turn);
    if (active) step_finish(c);
    MJ_RE(fin, PR_FINISH);
    MJ_RE(loop, PR_LOOP);
  }
#ifdef MJ_PROFILE
  __syncthreads();
  if (blockIdx.x == 7 && threadIdx.x == 0 && n_steps >= 128) {
    static const char *const nm[PR_N] = {"LOOP", "REFILL", "SAMPLE", "STEP", "RESET", "DEAL", "DEAL_NEXT", "DEAL_WAVE", "FINISH",
      "S0", "S1_TURN", "DISCARD", "KAN", "DECL", "S1_RESP", "CALL", "S2", "W_SHORT", "W_FACTS", "W_REFRESH", "WF_CAND",
      "WF_SPECIAL", "S3", "S3_RON", "WIN", "ABORT", "EXH", "DRAW", "KANDRAW", "TM_FACTS", "TM_EXACT", "TP_STD", "TP_OWN",
      "TP_SPECIAL", "TM_TSUMO", "TM_RIICHI", "TM_BITS", "EVAL"};
    // two wavefronts per block: cycles and entries are summed over both, so divide by 2 x steps for "per wave-step"
    for (int i = 0; i < PR_N; i++)
      printf("PROF %-10s cyc/wave-step %8.1f  entries/wave-step %6.3f  lanes/entry %5.2f  cyc/entry %8.1f\n", nm[i],
             (double)mj_prof[3 * i] / (2.0 * n_steps), (double)mj_prof[3 * i + 1] / (2.0 * n_steps),
             mj_prof[3 * i + 1] ? (double)mj_prof[3 * i + 2] / (double)mj_prof[3 * i + 1] : 0.0,
             mj_prof[3 * i + 1] ? (double)mj_prof[3 * i] / (double)mj_prof[3 * i + 1] : 0.0);
  }
#endif
  if (active) {
    hist_flush(c.e, c.g.hist_len);
    store_hot(m, state, B, b); store_glob(c.e, c.g);
  }
}

// test / scripting aid: give env b the wall in `wall` and deal the current kyoku again from it
__global__ void __launch_bounds__(kBlock, MJ_OCC) k_deal_from_wall(void *state, int64_t B, Rules R, DevTables T, int64_t b,
                                                           const uint8_t *wall)
{
  extern __shared__ __align__(16) uint8_t lds[];
  BlockMem m = stage_block<64>(T, lds);
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  Ctx c;
  c.e = make_env(state, B, b); c.L = m.L; c.R = R; c.env_id = R.env_id_base + (uint32_t)b;
  c.need_deal = false; c.need_turn = false; c.live_ptr = -1;
  load_glob(c.e, c.g);
  for (int i = 0; i < 136; i++) wall_set(c.e, c.g.wall_sel, i, wall[i]);
  deal(c, false);
  store_glob(c.e, c.g);
}

__global__ void __launch_bounds__(kAuxBlock) k_sample(void *state, int64_t B, Rules R, uint64_t step, int8_t *actions)
{
  int64_t b = (int64_t)blockIdx.x * kAuxBlock + threadIdx.x;
  if (b >= B) return;
  Env e = make_env(state, B, b);
  uint32_t packed = 0;
#pragma unroll
  for (int s = 0; s < 4; s++) {
    int a = sample_action(e.mask[(2 * s) * B], e.mask[(2 * s + 1) * B], R.seed, R.env_id_base + (uint32_t)b, step, s);
    packed |= (uint32_t)(uint8_t)(int8_t)a << (8 * s);
  }
  ((uint32_t *)actions)[b] = packed;
}

__global__ void __launch_bounds__(kAuxBlock) k_legal_mask(void *state, int64_t B, uint64_t *out)
{
  int64_t i = (int64_t)blockIdx.x * kAuxBlock + threadIdx.x;      // one thread per (b, word)
  if (i >= 8 * B) return;
  int64_t b = i >> 3;
  int w = (int)(i & 7);
  const uint64_t *mask = (const uint64_t *)state + 8 * B;
  out[i] = mask[(int64_t)w * B + b];
}

__global__ void __launch_bounds__(kAuxBlock) k_reward(void *state, int64_t B, float penalty, int32_t *delta, float *reward,
                                                   uint8_t *terminated)
{
  int64_t b = (int64_t)blockIdx.x * kAuxBlock + threadIdx.x;
  if (b >= B) return;
  Env e = make_env(state, B, b);
  Glob g;
  load_glob(e, g);
  int32_t d[4];
#pragma unroll
  for (int s = 0; s < 4; s++) d[s] = e.delta[s * B];
  if (delta) ((int4 *)delta)[b] = make_int4(d[0], d[1], d[2], d[3]);
  if (reward) {
    float r[4];
#pragma unroll
    for (int s = 0; s < 4; s++) r[s] = g.illegal_seat == s ? penalty : (float)d[s] * 0.001f;
    ((float4 *)reward)[b] = make_float4(r[0], r[1], r[2], r[3]);
  }
  if (terminated) terminated[b] = g.terminated;
}

__global__ void __launch_bounds__(kAuxBlock) k_standings(void *state, int64_t B, int32_t *score, uint8_t *rank)
{
  int64_t b = (int64_t)blockIdx.x * kAuxBlock + threadIdx.x;
  if (b >= B) return;
  Env e = make_env(state, B, b);
  if (score) ((int4 *)score)[b] = make_int4(e.score[0], e.score[B], e.score[2 * B], e.score[3 * B]);
  if (rank) {
    uint32_t r = 0;
#pragma unroll
    for (int s = 0; s < 4; s++) r |= sw_get(e.seatw[s * B], SW_RANK, 2) << (8 * s);
    ((uint32_t *)rank)[b] = r;
  }
}

__global__ void __launch_bounds__(kAuxBlock) k_export(void *state, int64_t B, int64_t lo, int64_t n, MjEnvCanon *out)
{
  int64_t i = (int64_t)blockIdx.x * kAuxBlock + threadIdx.x;
  if (i >= n) return;
  MjEnvCanon o;
  export_env(make_env(state, B, lo + i), o);
  out[i] = o;
}
__global__ void __launch_bounds__(kAuxBlock) k_import(void *state, int64_t B, int64_t lo, int64_t n, const MjEnvCanon *in)
{
  int64_t i = (int64_t)blockIdx.x * kAuxBlock + threadIdx.x;
  if (i >= n) return;
  MjEnvCanon o = in[i];
  import_env(make_env(state, B, lo + i), o);
}

__global__ void __launch_bounds__(kAuxBlock, MJ_OCC) k_eval_hands(DevTables T, int64_t n, const MjHandQuery *in, MjHandResult *out)
{
  extern __shared__ __align__(16) uint8_t lds[];
  {
    const uint4 *src = (const uint4 *)T.probe;
    uint4 *dst = (uint4 *)lds;
    for (int j = threadIdx.x; j < T.probe_bytes / 16; j += blockDim.x) dst[j] = src[j];
    __syncthreads();
  }
  Lut Lv;
  Lv.rowid = lds; Lv.bitmap = (const uint32_t *)(lds + kRowIdBytes);
  Lv.base = T.base; Lv.rowrank = T.rowrank; Lv.recs = T.recs; Lv.nb = T.nb;
  const Lut *L = &Lv;
  int64_t i = (int64_t)blockIdx.x * kAuxBlock + threadIdx.x;
  if (i >= n) return;
  const uint32_t *qw = (const uint32_t *)(in + i);
  uint32_t w[16];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    uint4 v = ((const uint4 *)qw)[j];
    w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
  }
  MjHandQuery q;
  __builtin_memcpy(&q, w, 64);
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
  eval_hand(L, hi, ho);
  MjHandResult r;
  r.yaku = ho.yaku; r.points = ho.points; r.han = (uint8_t)ho.han; r.fu = (uint8_t)ho.fu;
  r.yakuman_units = (uint8_t)ho.units; r.shape_ok = (uint8_t)ho.shape_ok; r.yaku_ok = (uint8_t)ho.yaku_ok;
  r.n_dora = (uint8_t)ho.n_dora; r.n_ura = (uint8_t)ho.n_ura; r.n_aka = (uint8_t)ho.n_aka;
  r.pad_[0] = r.pad_[1] = r.pad_[2] = r.pad_[3] = 0;
  out[i] = r;
}

// Observation writer.  Blocks stay resident and take groups of kObsEnvs environments in order from a device counter
// (ctr[0]; ctr[1] counts the blocks that have left, and the last one sets both back to zero), so launches of one
// handle must not overlap.  For each group:
//  0. everything the group's planes are made from (seat words, hands, melds, scores, control bytes, the two wall
//     words with the dora indicators of either wall buffer, all 128 river rows) is read with ONE round of loads,
//     every lane a few words, whatever the rivers' lengths, and put into LDS; the loads of the NEXT group are issued
//     before this group's stores, so they travel while the stores drain.  The kernel is bound by its stores, and a
//     load queues behind the stores of the compute unit's other blocks: with the four to six dependent rounds of
//     loads that reading "length, then that many tiles" takes, a launch that follows a step (state not in the
//     memory-side cache) took 1.80 ms against 1.39 ms for a launch that follows another observation;
//  1. 4 lanes per env build the per-seat masks from LDS, then one lane per env the env masks;
//  2. one lane per (env, viewer) concatenates the 56 planes of 34 bits into a 1904-bit string (LDS, over the raw copy);
//  3. all lanes expand bits to bytes, 16 bytes per store, consecutive lanes on consecutive addresses.
constexpr int kObsEnvs = 32;             // 49 KB of LDS per block; 16 per group reached 3.9 TB/s, 32 reach 5.2 TB/s
constexpr int kObsBits = 56 * 34;                 // 1904
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kObsWords = 60;                     // u32 words per (env, viewer), 1920 bits
constexpr int kObsStride = 33;                    // elements between two rows of the raw copy in LDS
constexpr int kObsRawRows = 35;                   // u32 rows: seat words 0..3, hands 4..19, scores 20..23, control 24..30,
                                                  // wall words 31, 32 of buffer 0 and of buffer 1: 31..34
struct ObsRaw {
  uint64_t meld[4][kObsStride];
  uint32_t w[kObsRawRows][kObsStride];
  uint8_t river[128][kObsStride];
};
// what one lane holds of a group between its loads and their way into LDS
struct ObsFetch { uint32_t w[5]; uint64_t meld; uint32_t riv[4]; };

__device__ __forceinline__ void obs_fetch(void *state, int64_t B, int64_t base, int nenv, int tid, ObsFetch &f)
{
  const Env e = make_env(state, B, base);
#pragma unroll
  for (int k = 0; k < 5; k++) {
    const int idx = tid + kAuxBlock * k, r = idx >> 5, el = idx & 31;
    const uint32_t *row = r < 4    ? e.seatw + (int64_t)r * B
                          : r < 20 ? e.hand + (int64_t)(r - 4) * B
                          : r < 24 ? (const uint32_t *)e.score + (int64_t)(r - 20) * B
                          : r < 31 ? e.glob + (int64_t)(r - 24) * B
                                   : e.wallw + (int64_t)(((r - 31) >> 1) * 34 + 31 + ((r - 31) & 1)) * B;
    f.w[k] = (r < kObsRawRows && el < nenv) ? row[el] : 0u;
  }
  f.meld = (tid < 128 && (tid & 31) < nenv) ? e.meld[(int64_t)(tid >> 5) * B + (tid & 31)] : 0ull;
  if ((B & 3) == 0) {
    // rows start on a word boundary, and a group that is not full still has a multiple of four environments
#pragma unroll
    for (int k = 0; k < 4; k++) {
      const int idx = tid + kAuxBlock * k, r = idx >> 3, q = idx & 7;
      f.riv[k] = 4 * q < nenv ? *(const uint32_t *)(e.river + (int64_t)r * B + 4 * q) : 0xFFFFFFFFu;
    }
  } else {
#pragma unroll
    for (int k = 0; k < 4; k++) {
      const int idx = tid + kAuxBlock * k, r = idx >> 3, q = idx & 7;
      uint32_t v = 0;
#pragma unroll
      for (int j = 0; j < 4; j++) v |= (uint32_t)(4 * q + j < nenv ? e.river[(int64_t)r * B + 4 * q + j] : 255) << (8 * j);
      f.riv[k] = v;
    }
  }
}
__device__ __forceinline__ void obs_commit(ObsRaw &raw, int tid, const ObsFetch &f)
{
#pragma unroll
  for (int k = 0; k < 5; k++) {
    const int idx = tid + kAuxBlock * k, r = idx >> 5, el = idx & 31;
    if (r < kObsRawRows) raw.w[r][el] = f.w[k];
  }
  if (tid < 128) raw.meld[tid >> 5][tid & 31] = f.meld;
#pragma unroll
  for (int k = 0; k < 4; k++) {
    const int idx = tid + kAuxBlock * k, r = idx >> 3, q = idx & 7;
#pragma unroll
    for (int j = 0; j < 4; j++) raw.river[r][4 * q + j] = (uint8_t)(f.riv[k] >> (8 * j));
  }
}
// view of environment el of the raw copy, for the code that reads a state through an Env
__device__ __forceinline__ Env obs_view(ObsRaw &raw, int el)
{
  Env v = {};
  v.n = kObsStride; v.hs = kObsStride;
  v.seatw = &raw.w[0][el]; v.hand = &raw.w[4][el]; v.score = (int32_t *)&raw.w[20][el]; v.glob = &raw.w[24][el];
  v.meld = &raw.meld[0][el]; v.river = &raw.river[0][el];
  return v;
}

__global__ void __launch_bounds__(kAuxBlock) k_observe(void *state, int64_t B, uint32_t rule_flags, uint8_t *obs, unsigned *ctr)
{
  __shared__ uint64_t S[kObsEnvs][4][OB_SEAT_WORDS];
  __shared__ uint64_t G[kObsEnvs][OG_WORDS];
  __shared__ uint64_t R[kObsEnvs][4];
  __shared__ uint32_t own_red[kObsEnvs][4];
  __shared__ union ObsShared { uint32_t bits[kObsEnvs][4][kObsWords]; ObsRaw raw; } U;   // raw is dead once S and G are made
  __shared__ unsigned next_group;
  static_assert(sizeof(ObsRaw) <= sizeof(uint32_t) * kObsEnvs * 4 * kObsWords, "the raw copy fits under the bit strings");
  const int tid = threadIdx.x;
  const int64_t n_groups = (B + kObsEnvs - 1) / kObsEnvs;
  // The counter's value g stands for environments (n_groups - 1 - g) * 32 ..: from the end of the batch down, so that a
  // launch that follows a step starts with the environments that the step wrote last (what the memory-side cache
  // still holds): 1.60 -> 1.57 ms at B = 2^20.
  if (tid == 0) next_group = atomicAdd(&ctr[0], 1u);
  __syncthreads();
  int64_t grp = next_group;
  ObsFetch f;
  if (grp < n_groups) {
    const int64_t base = (n_groups - 1 - grp) * kObsEnvs;
    obs_fetch(state, B, base, (int)((B - base) < kObsEnvs ? (B - base) : kObsEnvs), tid, f);
  }
  while (grp < n_groups) {
    const int64_t base = (n_groups - 1 - grp) * kObsEnvs;
    const int nenv = (int)((B - base) < kObsEnvs ? (B - base) : kObsEnvs);
    unsigned taken = 0;
    if (tid == 0) taken = atomicAdd(&ctr[0], 1u);      // the group after this one; its answer is needed only below
    obs_commit(U.raw, tid, f);
    __syncthreads();
    if (tid < 4 * nenv) {
      int el = tid >> 2, s = tid & 3;
      Env e = obs_view(U.raw, el);
      uint64_t m[OB_SEAT_WORDS];
      R[el][s] = obs_seat_masks(e, s, m);
#pragma unroll
      for (int i = 0; i < OB_SEAT_WORDS; i++) S[el][s][i] = m[i];
      own_red[el][s] = e.seatw[s * kObsStride] & 7u;
    }
    __syncthreads();
    if (tid < nenv) {
      Env e = obs_view(U.raw, tid);
      Glob g;
      load_glob(e, g);
      const uint32_t dw[2] = {U.raw.w[31 + 2 * g.wall_sel][tid], U.raw.w[32 + 2 * g.wall_sel][tid]};
      uint64_t m[OG_WORDS];
      obs_env_masks(g, rule_flags, R[tid][0] | R[tid][1] | R[tid][2] | R[tid][3], dw, m);
#pragma unroll
      for (int i = 0; i < OG_WORDS; i++) G[tid][i] = m[i];
    }
    __syncthreads();
    if (tid < 4 * nenv) {
      int el = tid >> 2, me = tid & 3;
      uint32_t *out = U.bits[el][me];
      uint64_t acc = 0;
      int fill = 0, wpos = 0;                 // fill stays even and <= 30 before each plane is added
      for (int p = 0; p < 56; p++) {
        uint64_t v = obs_plane(p, me, &S[el][0][0], own_red[el][me], G[el]) & K_ALL;
        acc |= v << fill;
        fill += 34;
        while (fill >= 32) { out[wpos++] = (uint32_t)acc; acc >>= 32; fill -= 32; }
      }
      while (wpos < kObsWords) { out[wpos++] = (uint32_t)acc; acc = 0; }
    }
    if (tid == 0) next_group = taken;
    __syncthreads();
    const int64_t nxt = next_group;
    if (nxt < n_groups) {
      const int64_t nb = (n_groups - 1 - nxt) * kObsEnvs;
      obs_fetch(state, B, nb, (int)((B - nb) < kObsEnvs ? (B - nb) : kObsEnvs), tid, f);
    }
    // 7616 bytes per env = 476 stores of 16 bytes; 16 bytes = 16 bits of the string
    const int per_env = 4 * kObsBits / 16;
    u32x4 *dst = (u32x4 *)(obs + (size_t)base * 4 * kObsBits);
    for (int i = tid; i < nenv * per_env; i += kAuxBlock) {
      int el = i / per_env, j = i - el * per_env;          // j-th 16-byte group of env el
      int me = j / (kObsBits / 16), q = j - me * (kObsBits / 16);
      uint32_t word = U.bits[el][me][q >> 1];
      uint32_t v = (q & 1) ? word >> 16 : word & 0xFFFFu;
      u32x4 o;
      o.x = ((v & 0xFu) * 0x00204081u) & 0x01010101u;
      o.y = (((v >> 4) & 0xFu) * 0x00204081u) & 0x01010101u;
      o.z = (((v >> 8) & 0xFu) * 0x00204081u) & 0x01010101u;
      o.w = (((v >> 12) & 0xFu) * 0x00204081u) & 0x01010101u;
      // one 16-byte streaming store: the tensor is written once and not read back by this kernel
      __builtin_nontemporal_store(o, &dst[i]);
    }
    __syncthreads();       // the bit strings and next_group have been read by every lane
    grp = nxt;
  }
  // the last block to leave rearms both counters for the next launch
  if (tid == 0 && atomicAdd(&ctr[1], 1u) == gridDim.x - 1) { atomicExch(&ctr[0], 0u); atomicExch(&ctr[1], 0u); }
}

// Token observation.  One lane per (environment, seat).  What the four viewers of a game share is computed once:
// lane (env, s) turns seat s's river into token bytes in LDS; as viewer s, it writes the first 96 bytes of its record
// (own hand, shanten number, scalars, the seats' words rotated to it) into LDS, and stages a quarter of the game's
// action history (two entries per word, absolute
// seats).  The block then streams the records out, one record per wavefront and iteration, consecutive lanes on
// consecutive words: 24 words from the record head, 32 from the four rivers picked by relative seat, 4 for the
// length of the history, 64 of history with the seats turned to the viewer.
constexpr int kTokEnvs = kAuxBlock / 4;           // 64 environments per block
constexpr int kTokHead = 96;                      // bytes of MjTokenObs before river[][]
constexpr int kTokHeadStride = 100, kTokRivStride = 36;   // LDS strides: an odd number of words, so that the lanes of a
                                                          // wavefront (consecutive environments) fall into different banks
constexpr int kTokHistStride = 65;                // words per game in the LDS copy of the history (odd, as above)
static_assert(offsetof(MjTokenObs, river) == kTokHead && offsetof(MjTokenObs, n_hist) == kTokHead + 128 &&
              offsetof(MjTokenObs, hist) == kTokHead + 144 && sizeof(MjTokenObs) == kTokHead + 144 + 256, "token record layout");
__global__ void __launch_bounds__(kAuxBlock) k_observe_tokens(void *state, int64_t B, uint32_t rule_flags, const uint32_t *sh_suit,
                                                           const uint32_t *sh_honor, MjTokenObs *out)
{
  __shared__ __align__(4) uint8_t head[4][kTokEnvs][kTokHeadStride];       // [viewer][env]
  __shared__ __align__(4) uint8_t riv[4][kTokEnvs][kTokRivStride];         // [seat][env]
  __shared__ uint32_t p_hist[kTokEnvs][kTokHistStride];                    // two entries per word: action | seat << 8
  __shared__ uint32_t p_nhist[kTokEnvs];
  const int tid = threadIdx.x;
  const int64_t base = (int64_t)blockIdx.x * kTokEnvs;
  const int nenv = (int)((B - base) < kTokEnvs ? (B - base) : kTokEnvs);
  // lanes of a wavefront take consecutive environments of one seat, so that state reads are coalesced
  const int s = tid / nenv, el = tid - s * nenv;
  const bool on = tid < 4 * nenv;
  Env e = make_env(state, B, base + (on ? el : 0));
  // MjTokenObs is used as a view of the record head only: nothing below touches river[][]
  MjTokenObs &o = *(MjTokenObs *)head[on ? s : 0][on ? el : 0];
  if (on) {
    tok_river(e, s, riv[s][el]);
    // the four seats' public words, read by each of the game's four lanes (the repeats are cache hits): 52 KB of LDS
    // instead of 56 KB lets three blocks share a compute unit
    uint32_t sw[4];
    int32_t sc[4];
    uint64_t ml[4];
#pragma unroll
    for (int t = 0; t < 4; t++) { sw[t] = e.seatw[t * B]; sc[t] = e.score[t * B]; ml[t] = e.meld[t * B]; }
    Glob g;
    load_glob(e, g);
    tok_own(e, s, sh_suit, sh_honor, o);
    tok_env(e, g, s, rule_flags, o);
    // entries 32 s .. 32 s + 31 of the history: sixteen words of the environment's row, two entries each
    const int nh = g.hist_len;
    if (s == 0) p_nhist[el] = (uint32_t)nh;
    uint32_t hv[16];
#pragma unroll
    for (int j = 0; j < 16; j++) hv[j] = row_word(e.hist + 32 * s, j);              // all sixteen loads in flight together
#pragma unroll
    for (int j = 0; j < 16; j++) {
      const int i0 = 32 * s + 2 * j;
      const uint32_t lo = i0 < nh ? hv[j] & 0xFFFFu : 0xFFFFu, hi = i0 + 1 < nh ? hv[j] >> 16 : 0xFFFFu;
      p_hist[el][16 * s + j] = lo | hi << 16;
    }
    tok_seats(sw, sc, ml, s, o);
  }
  __syncthreads();
  // out: wavefront `me` writes the records of viewer `me`, two games per iteration; each half of the wavefront streams
  // one record of 31 chunks of 16 bytes (6 from the record head, 8 from the four rivers picked by relative seat, 1 with
  // the length of the history, 16 of history), lane by lane on consecutive addresses; a lane's source is a fixed LDS
  // address plus a stride per game
  static_assert(sizeof(MjTokenObs) == 31 * 16 && kAuxBlock / 64 == 4, "token record chunks");
  const int lane = tid & 63, me = tid >> 6, ch = lane & 31;
  const bool live = ch < 31, is_len = ch == 14, is_hist = ch > 14;
  const uint8_t *src = &head[me][0][16 * (ch < 6 ? ch : 0)];
  int stride = kTokHeadStride;
  if (ch >= 6 && ch < 14) { src = &riv[(me + ((ch - 6) >> 1)) & 3][0][16 * ((ch - 6) & 1)]; stride = kTokRivStride; }
  if (is_hist && live) { src = (const uint8_t *)&p_hist[0][4 * (ch - 15)]; stride = 4 * kTokHistStride; }
  // a history word as this viewer sees it: seats turned, unused entries left at 0xFFFF
  const uint32_t sub = 0x00040004u - (uint32_t)me * 0x00010001u;
  auto turned = [&](uint32_t x) {
    uint32_t y = (x & 0x00FF00FFu) | (((x >> 8 & 0x00030003u) + sub) & 0x00030003u) << 8;
    if ((x & 0xFFu) == 0xFFu) y |= 0x0000FFFFu;
    if ((x >> 16 & 0xFFu) == 0xFFu) y |= 0xFFFF0000u;
    return y;
  };
  u32x4 *dst = (u32x4 *)(out + base * 4 + me) + ch;
#pragma unroll 2
  for (int env = lane >> 5; env < nenv; env += 2) {
    const uint32_t *p = (const uint32_t *)(src + env * stride);
    u32x4 v;
    v.x = p[0]; v.y = p[1]; v.z = p[2]; v.w = p[3];
    if (is_hist) { v.x = turned(v.x); v.y = turned(v.y); v.z = turned(v.z); v.w = turned(v.w); }
    if (is_len) { v.x = p_nhist[env]; v.y = 0u; v.z = 0u; v.w = 0u; }
    if (live) __builtin_nontemporal_store(v, dst + (size_t)env * (4 * sizeof(MjTokenObs) / 16));
  }
}

}  // namespace

// ------------------------------------------------------------------ host side
struct MjHandle {
  int64_t B;
  Rules R;
  MjRules rules;
  uint64_t step;
  void *d_state, *d_scratch;
  DevTables T;
  const uint32_t *sh_suit, *sh_honor;    // block tables of the shanten number (device)
  unsigned *obs_ctr;                     // work counters of the observation writer (device, zero between launches)
  int n_cu;
  size_t lds_bytes, probe_bytes;
  int lpw;
  hipEvent_t ev[2];
  int ev_steps;
  bool ev_valid;
};

namespace {

const mjt::SuitTables &tables()
{
  static const mjt::SuitTables t = mjt::build();
  return t;
}
const std::vector<uint32_t> &sh_suit_table()
{
  static const std::vector<uint32_t> t = mjt::build_shanten_table(9, true);
  return t;
}
const std::vector<uint32_t> &nb_table()
{
  static const std::vector<uint32_t> t = mjt::build_neighbour_table();
  return t;
}
const std::vector<uint32_t> &sh_honor_table()
{
  static const std::vector<uint32_t> t = mjt::build_shanten_table(7, false);
  return t;
}
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
struct ScratchLayout { size_t probe, base, rowrank, recs, nb, sh_suit, sh_honor, counters, total, probe_bytes; };
ScratchLayout scratch_layout()
{
  const mjt::SuitTables &t = tables();
  ScratchLayout s;
  s.probe = 0;
  s.probe_bytes = t.rowid.size() + t.bitmap.size() * 4;
  s.base = align256(s.probe_bytes);
  s.rowrank = align256(s.base + t.base.size() * 2);
  s.recs = align256(s.rowrank + t.rowrank.size() * 2);
  s.nb = align256(s.recs + t.recs.size() * 4);
  s.sh_suit = align256(s.nb + nb_table().size() * 4);
  s.sh_honor = align256(s.sh_suit + sh_suit_table().size() * 4);
  s.counters = align256(s.sh_honor + sh_honor_table().size() * 4);
  s.total = s.counters + 256;
  return s;
}
size_t scratch_bytes_impl() { return scratch_layout().total; }
inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kAuxBlock - 1) / kAuxBlock); }
inline unsigned step_blocks(int64_t n, int lpw) { int e = envs_per_block(lpw); return (unsigned)((n + e - 1) / e); }
// lanes per wave for a batch: fill the machine's wave slots (256 CUs x 4 SIMDs x 2 resident waves of this kernel)
inline int pick_lpw(int64_t B)
{
  const char *ov = std::getenv("MJ_LPW");
  if (ov) { int v = std::atoi(ov); if (v == 64 || v == 32 || v == 16) return v; }
  if (B >= 2048 * 32) return 32;        // also for larger batches: 64 per wavefront leaves room for one wavefront
                                        // per SIMD only (LDS), measured slower at every batch size
  return 16;
}
#define MJ_LAUNCH_STEP(kern, h, st, ...) MJ_LAUNCH_STEP_N(kern, h, st, (h)->B, __VA_ARGS__)
#define MJ_LAUNCH_STEP_N(kern, h, st, n_envs, ...)                                                               \
  do {                                                                                                           \
    size_t lds_ = step_lds_bytes((int)(h)->probe_bytes, (h)->lpw);                                               \
    unsigned nb_ = step_blocks((n_envs), (h)->lpw);                                                              \
    if ((h)->lpw == 64) kern<64><<<nb_, kBlock, lds_, st>>>(__VA_ARGS__);                                        \
    else if ((h)->lpw == 32) kern<32><<<nb_, kBlock, lds_, st>>>(__VA_ARGS__);                                   \
    else kern<16><<<nb_, kBlock, lds_, st>>>(__VA_ARGS__);                                                       \
  } while (0)
inline int check(hipError_t e) { return e == hipSuccess ? MJ_OK : MJ_E_HIP; }

// ---- tables for callers that can not allocate (mj_eval_hands_static) ----------------------------------------
// A copy of the per-suit pattern tables (probe part and records, without the shanten block tables) in a file-scope
// device array: every GPU the library runs on holds its own copy at its own address until the process ends.  In
// host code the array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr size_t kStaticScratchBytes = 384 * 1024;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 16;
struct StaticTables { bool ready; DevTables T; };
StaticTables g_static[kMaxDevices];
std::mutex g_static_mu;

// the tables of the CURRENT device, uploaded on first use (a synchronous copy from a host image)
int static_tables(const DevTables **out)
{
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MJ_E_HIP;
  if (dev < 0 || dev >= kMaxDevices) return MJ_E_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_static_mu);
  StaticTables &st = g_static[dev];
  if (!st.ready) {
    const mjt::SuitTables &t = tables();
    const ScratchLayout sl = scratch_layout();
    const size_t need = sl.nb;                            // everything before the neighbour and shanten tables
    if (need > kStaticScratchBytes || (sl.probe_bytes & 15)) return MJ_E_UNSUPPORTED;
    uint8_t *ptr = nullptr;
    if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MJ_E_HIP;
    std::vector<uint8_t> img(need, 0);
    std::memcpy(img.data() + sl.probe, t.rowid.data(), t.rowid.size());
    std::memcpy(img.data() + sl.probe + t.rowid.size(), t.bitmap.data(), t.bitmap.size() * 4);
    std::memcpy(img.data() + sl.base, t.base.data(), t.base.size() * 2);
    std::memcpy(img.data() + sl.rowrank, t.rowrank.data(), t.rowrank.size() * 2);
    std::memcpy(img.data() + sl.recs, t.recs.data(), t.recs.size() * 4);
    if (hipMemcpy(ptr, img.data(), need, hipMemcpyHostToDevice) != hipSuccess) return MJ_E_HIP;
    st.T.probe = ptr + sl.probe;
    st.T.base = (const uint16_t *)(ptr + sl.base);
    st.T.rowrank = (const uint16_t *)(ptr + sl.rowrank);
    st.T.recs = (const uint32_t *)(ptr + sl.recs);
    st.T.nb = nullptr;                                    // the hand evaluator does not search for tenpai
    st.T.probe_bytes = (int)sl.probe_bytes;
    st.ready = true;
  }
  *out = &st.T;
  return MJ_OK;
}

}  // namespace

extern "C" {

const char *mj_strerror(int code)
{
  switch (code) {
    case MJ_OK: return "ok";
    case MJ_E_ARG: return "bad argument";
    case MJ_E_HIP: return "HIP call or kernel launch failed";
    case MJ_E_NOMEM: return "host allocation failed";
    case MJ_E_UNSUPPORTED: return "device cannot run the kernels";
    case MJ_E_RANGE: return "size beyond the entry point's stated maximum";
    default: return "unknown error";
  }
}

size_t mj_state_bytes(int64_t B, const MjRules *rules)
{
  if (B <= 0 || !rules) return 0;
  return (size_t)B * (size_t)kBytesPerEnv;
}
size_t mj_scratch_bytes(int64_t B, const MjRules *rules)
{
  if (B <= 0 || !rules) return 0;
  return scratch_bytes_impl();
}

int mj_init(MjHandle **out, void *d_state, void *d_scratch, int64_t B, uint64_t seed, const MjRules *rules, void *stream)
{
  if (!out || !d_state || !d_scratch || !rules || B <= 0 || (seed >> 32) || rules->mode > 2) return MJ_E_ARG;
  if (((uintptr_t)d_state & 15) || ((uintptr_t)d_scratch & 15)) return MJ_E_ARG;
  MjHandle *h = new (std::nothrow) MjHandle();
  if (!h) return MJ_E_NOMEM;
  h->B = B; h->rules = *rules; h->step = 0; h->d_state = d_state; h->d_scratch = d_scratch;
  h->R.flags = rules->flags; h->R.env_id_base = rules->env_id_base; h->R.start_score = rules->start_score;
  h->R.illegal_penalty = rules->illegal_penalty; h->R.mode = rules->mode; h->R.seed = (uint32_t)seed;
  h->ev_valid = false; h->ev_steps = 0;
  const mjt::SuitTables &t = tables();
  const ScratchLayout sl = scratch_layout();
  if (t.rowid.size() != (size_t)kRowIdBytes || (sl.probe_bytes & 15) || sl.probe_bytes > (size_t)kTableChunks * kBlock * 16) {
    delete h;
    return MJ_E_UNSUPPORTED;
  }
  int dev = 0, lds_max = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
      hipDeviceGetAttribute(&h->n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || h->n_cu <= 0) { delete h; return MJ_E_HIP; }
  h->lpw = pick_lpw(B);
  h->lds_bytes = step_lds_bytes((int)sl.probe_bytes, 64);
  h->probe_bytes = sl.probe_bytes;
  if ((size_t)lds_max < h->lds_bytes) { delete h; return MJ_E_UNSUPPORTED; }
  hipStream_t st = (hipStream_t)stream;
  // table image in the caller's scratch buffer
  std::vector<uint8_t> img(sl.total, 0);
  std::memcpy(img.data() + sl.probe, t.rowid.data(), t.rowid.size());
  std::memcpy(img.data() + sl.probe + t.rowid.size(), t.bitmap.data(), t.bitmap.size() * 4);
  std::memcpy(img.data() + sl.base, t.base.data(), t.base.size() * 2);
  std::memcpy(img.data() + sl.rowrank, t.rowrank.data(), t.rowrank.size() * 2);
  std::memcpy(img.data() + sl.recs, t.recs.data(), t.recs.size() * 4);
  std::memcpy(img.data() + sl.nb, nb_table().data(), nb_table().size() * 4);
  std::memcpy(img.data() + sl.sh_suit, sh_suit_table().data(), sh_suit_table().size() * 4);
  std::memcpy(img.data() + sl.sh_honor, sh_honor_table().data(), sh_honor_table().size() * 4);
  int rc = check(hipMemcpyAsync(d_scratch, img.data(), sl.total, hipMemcpyHostToDevice, st));
  if (rc == MJ_OK) rc = check(hipStreamSynchronize(st));       // the host image goes away
  char *sc = (char *)d_scratch;
  h->T.probe = (const uint8_t *)(sc + sl.probe);
  h->T.base = (const uint16_t *)(sc + sl.base);
  h->T.rowrank = (const uint16_t *)(sc + sl.rowrank);
  h->T.recs = (const uint32_t *)(sc + sl.recs);
  h->T.nb = (const uint32_t *)(sc + sl.nb);
  h->T.probe_bytes = (int)sl.probe_bytes;
  h->sh_suit = (const uint32_t *)(sc + sl.sh_suit);
  h->sh_honor = (const uint32_t *)(sc + sl.sh_honor);
  h->obs_ctr = (unsigned *)(sc + sl.counters);
  if (rc == MJ_OK) { const DevTables *unused; rc = static_tables(&unused); }   // for mj_eval_hands_static on this device
  if (rc == MJ_OK) rc = check(hipEventCreate(&h->ev[0]));
  if (rc == MJ_OK) rc = check(hipEventCreate(&h->ev[1]));
  if (rc != MJ_OK) { delete h; return rc; }
  MJ_LAUNCH_STEP(k_new_games, h, st, d_state, B, h->R, h->T, 0);
  rc = check(hipGetLastError());
  if (rc != MJ_OK) { delete h; return rc; }
  *out = h;
  return MJ_OK;
}

int mj_step(MjHandle *h, const int8_t *d_actions, void *stream)
{
  if (!h || !d_actions || ((uintptr_t)d_actions & 3)) return MJ_E_ARG;
  MJ_LAUNCH_STEP(k_step, h, (hipStream_t)stream, h->d_state, h->B, h->R, h->T, d_actions, (int)(h->step % kStepRefillEvery == 0), 0,
                 StepOut{nullptr, nullptr, nullptr, nullptr});
  h->step++;
  return check(hipGetLastError());
}

int mj_step_full(MjHandle *h, const int8_t *d_actions, int auto_reset, uint64_t *d_mask, int32_t *d_delta, float *d_reward,
                 uint8_t *d_terminated, void *stream)
{
  if (!h || !d_actions || ((uintptr_t)d_actions & 3) || ((uintptr_t)d_mask & 15) || ((uintptr_t)d_delta & 15) ||
      ((uintptr_t)d_reward & 15))
    return MJ_E_ARG;
  MJ_LAUNCH_STEP(k_step, h, (hipStream_t)stream, h->d_state, h->B, h->R, h->T, d_actions, (int)(h->step % kStepRefillEvery == 0),
                 auto_reset ? 1 : 0, StepOut{d_mask, d_delta, d_reward, d_terminated});
  h->step++;
  return check(hipGetLastError());
}

int mj_legal_mask(const MjHandle *h, uint64_t *d_mask, void *stream)
{
  if (!h || !d_mask) return MJ_E_ARG;
  k_legal_mask<<<blocks_for(8 * h->B), kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, d_mask);
  return check(hipGetLastError());
}

int mj_observe(const MjHandle *h, uint8_t *d_obs, void *stream)
{
  if (!h || !d_obs || ((uintptr_t)d_obs & 15)) return MJ_E_ARG;
  int64_t groups = (h->B + kObsEnvs - 1) / kObsEnvs;
  // three blocks fit a compute unit (LDS); they take the groups of 32 games in order from a counter, so that the
  // blocks in flight write one compact, advancing window of the tensor (measured: 5.8 TB/s against 5.3 TB/s with
  // one block per group in launch order)
  const int64_t resident = (int64_t)h->n_cu * 3;
  unsigned grid = (unsigned)(groups < resident ? groups : resident);
  k_observe<<<grid, kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, h->R.flags, d_obs, h->obs_ctr);
  return check(hipGetLastError());
}

int mj_observe_tokens(const MjHandle *h, MjTokenObs *d_out, void *stream)
{
  if (!h || !d_out || ((uintptr_t)d_out & 15)) return MJ_E_ARG;
  const unsigned grid = (unsigned)((h->B + kTokEnvs - 1) / kTokEnvs);
  k_observe_tokens<<<grid, kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, h->R.flags, h->sh_suit, h->sh_honor, d_out);
  return check(hipGetLastError());
}

int mj_reward(const MjHandle *h, int32_t *d_delta, float *d_reward, uint8_t *d_terminated, void *stream)
{
  if (!h || ((uintptr_t)d_delta & 15) || ((uintptr_t)d_reward & 15)) return MJ_E_ARG;
  k_reward<<<blocks_for(h->B), kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, h->R.illegal_penalty, d_delta, d_reward,
                                                                 d_terminated);
  return check(hipGetLastError());
}

int mj_standings(const MjHandle *h, int32_t *d_score, uint8_t *d_rank, void *stream)
{
  if (!h || ((uintptr_t)d_score & 15) || ((uintptr_t)d_rank & 3)) return MJ_E_ARG;
  if (h->B == 0) return MJ_OK;
  k_standings<<<blocks_for(h->B), kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, d_score, d_rank);
  return check(hipGetLastError());
}

int mj_reset_done(MjHandle *h, void *stream)
{
  if (!h) return MJ_E_ARG;
  MJ_LAUNCH_STEP(k_new_games, h, (hipStream_t)stream, h->d_state, h->B, h->R, h->T, 1);
  return check(hipGetLastError());
}

int mj_sample_random(const MjHandle *h, int8_t *d_actions, void *stream)
{
  if (!h || !d_actions || ((uintptr_t)d_actions & 3)) return MJ_E_ARG;
  k_sample<<<blocks_for(h->B), kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, h->R, h->step, d_actions);
  return check(hipGetLastError());
}

int mj_step_random(MjHandle *h, int32_t n_steps, int auto_reset, int write_obs, uint8_t *d_obs, void *stream)
{
  if (!h || n_steps < 0 || (write_obs && (!d_obs || ((uintptr_t)d_obs & 15)))) return MJ_E_ARG;
  if (n_steps == 0) return MJ_OK;
  hipStream_t st = (hipStream_t)stream;
  int rc = check(hipEventRecord(h->ev[0], st));
  if (rc != MJ_OK) return rc;
  if (!write_obs) {
    // environments never interact, so many steps run inside one launch; chunked to bound a launch's duration.
    // Long launches matter at B = 65,536: all 2,048 wavefronts are resident at once, a launch ends with its
    // slowest wavefront, and the spread of per-wavefront work shrinks with the number of steps (measured:
    // 128 / 256 / 512 / 1024 / 2048 steps per launch = 6.26 / 6.44 / 6.58 / 6.67 / 6.69 G env steps/s on an earlier
    // build, 1024 / 2048 / 4096 = 7.13 / 7.19 / 7.23 G on this one).  4,096 steps of 65,536 games take 37 ms; larger
    // batches get proportionally shorter launches.  MJ_CHUNK overrides the length for experiments.
    int chunk = MJ_ROLLOUT_CHUNK;
    while (chunk > 256 && (int64_t)chunk * h->B > (int64_t)MJ_ROLLOUT_CHUNK * 131072) chunk /= 2;
    if (const char *cv = std::getenv("MJ_CHUNK")) { int v = std::atoi(cv); if (v > 0) chunk = v; }
    // A batch of up to six times what the machine holds at once (4 blocks per compute unit) can go out in slices of
    // that size (the last one smaller), one launch each.  Measured in units of one full slice's time: a single launch
    // over x slices' worth of games takes about x + 0.5 (x = 2 / 3 / 4: 2.6 / 3.5 / 4.3; B = 131,072: 5.3 G env
    // steps/s) and only from x = 6 on about x; sliced launches take ceil(x), however small the last slice is
    // (B = 131,072: 7.0 G).  So slices are used when the last one is more than half full.
    const int64_t resident = (int64_t)h->n_cu * 4 * envs_per_block(h->lpw);
    const int64_t tail = h->B % resident;
    const bool slices = h->lpw == 32 && h->B <= 6 * resident && (tail == 0 || 2 * tail > resident);
    const int64_t per_slice = slices ? resident : h->B;
    for (int t = 0; t < n_steps && rc == MJ_OK; t += chunk) {
      int n = n_steps - t < chunk ? n_steps - t : chunk;
      for (int64_t lo = 0; lo < h->B && rc == MJ_OK; lo += per_slice) {
        const int64_t hi = lo + per_slice < h->B ? lo + per_slice : h->B;
        MJ_LAUNCH_STEP_N(k_rollout, h, st, hi - lo, h->d_state, h->B, h->R, h->T, h->step + t, n, auto_reset, lo, hi);
        rc = check(hipGetLastError());
      }
    }
  } else {
    for (int t = 0; t < n_steps && rc == MJ_OK; t++) {
      MJ_LAUNCH_STEP(k_rollout, h, st, h->d_state, h->B, h->R, h->T, h->step + t, 1, auto_reset, (int64_t)0, h->B);
      rc = check(hipGetLastError());
      if (rc == MJ_OK) rc = mj_observe(h, d_obs, stream);
    }
  }
  if (rc != MJ_OK) return rc;
  h->step += (uint64_t)n_steps;
  rc = check(hipEventRecord(h->ev[1], st));
  h->ev_valid = rc == MJ_OK;
  h->ev_steps = n_steps;
  return rc;
}

int mj_export(const MjHandle *h, int64_t env_lo, int64_t n, MjEnvCanon *d_out, void *stream)
{
  if (!h || env_lo < 0 || n < 0 || env_lo + n > h->B) return MJ_E_ARG;
  if (n == 0) return MJ_OK;
  if (!d_out) return MJ_E_ARG;
  k_export<<<blocks_for(n), kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, env_lo, n, d_out);
  return check(hipGetLastError());
}
int mj_import(MjHandle *h, int64_t env_lo, int64_t n, const MjEnvCanon *d_in, void *stream)
{
  if (!h || env_lo < 0 || n < 0 || env_lo + n > h->B) return MJ_E_ARG;
  if (n == 0) return MJ_OK;
  if (!d_in) return MJ_E_ARG;
  k_import<<<blocks_for(n), kAuxBlock, 0, (hipStream_t)stream>>>(h->d_state, h->B, env_lo, n, d_in);
  return check(hipGetLastError());
}

int mj_eval_hands(const MjHandle *h, int64_t n, const MjHandQuery *d_in, MjHandResult *d_out, void *stream)
{
  if (!h || n < 0) return MJ_E_ARG;
  if (n == 0) return MJ_OK;                               // an empty batch needs no buffers
  if (!d_in || !d_out || ((uintptr_t)d_in & 15) || ((uintptr_t)d_out & 7)) return MJ_E_ARG;
  k_eval_hands<<<blocks_for(n), kAuxBlock, h->probe_bytes, (hipStream_t)stream>>>(h->T, n, d_in, d_out);
  return check(hipGetLastError());
}

int mj_eval_hands_static(int64_t n, const MjHandQuery *d_in, MjHandResult *d_out, void *stream)
{
  if (n < 0 || n > MJ_EVAL_STATIC_MAX_HANDS) return MJ_E_RANGE;
  if (n == 0) return MJ_OK;
  if (!d_in || !d_out || ((uintptr_t)d_in & 15) || ((uintptr_t)d_out & 7)) return MJ_E_ARG;
  const DevTables *T = nullptr;
  int rc = static_tables(&T);          // ready since mj_init on this device, otherwise uploaded now
  if (rc != MJ_OK) return rc;
  k_eval_hands<<<blocks_for(n), kAuxBlock, T->probe_bytes, (hipStream_t)stream>>>(*T, n, d_in, d_out);
  return check(hipGetLastError());
}

int mj_deal_from_wall(MjHandle *h, int64_t b, const uint8_t *d_wall, void *stream)
{
  if (!h || !d_wall || b < 0 || b >= h->B) return MJ_E_ARG;
  k_deal_from_wall<<<1, kBlock, h->lds_bytes, (hipStream_t)stream>>>(h->d_state, h->B, h->R, h->T, b, d_wall);
  return check(hipGetLastError());
}

uint64_t mj_step_count(const MjHandle *h) { return h ? h->step : 0; }
int mj_set_step_count(MjHandle *h, uint64_t steps)
{
  if (!h) return MJ_E_ARG;
  h->step = steps;
  return MJ_OK;
}

float mj_last_step_kernel_ms(MjHandle *h)
{
  if (!h || !h->ev_valid || h->ev_steps <= 0) return -1.0f;
  if (hipEventSynchronize(h->ev[1]) != hipSuccess) return -1.0f;
  float ms = 0;
  if (hipEventElapsedTime(&ms, h->ev[0], h->ev[1]) != hipSuccess) return -1.0f;
  return ms / (float)h->ev_steps;
}

#ifdef MJ_PROFILE
int mj_prof_read_kstep(long long *h_out /*[4096][8]*/)
{
  return check(hipMemcpyFromSymbol(h_out, HIP_SYMBOL(mj_kstep_prof), sizeof(long long) * 4096 * 8));
}
int mj_prof_read_kstep_regions(unsigned long long *h_out /*[2048][3 * n]*/, int *n_regions)
{
  *n_regions = PR_N;
  return check(hipMemcpyFromSymbol(h_out, HIP_SYMBOL(mj_kstep_regions), sizeof(unsigned long long) * 2048 * 3 * PR_N));
}
#endif

int mj_destroy(MjHandle *h)
{
  if (!h) return MJ_E_ARG;
  (void)hipEventDestroy(h->ev[0]);
  (void)hipEventDestroy(h->ev[1]);
  delete h;
  return MJ_OK;
}

}  // extern "C"
