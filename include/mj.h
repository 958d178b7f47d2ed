/*
 * mj.h -- C ABI of libmj: the batched four-player Riichi Mahjong environment
 * step on one AMD MI355X (gfx950), hand-written HIP kernels.
 *
 * The operations are those of the paper's environment (section 3.1: a State
 * holding hands, scores, winds, melds and masks, advanced by init / step in
 * the Pgx style; section 3.2: rule sets, game modes, discrete action ids,
 * legal_action_mask, illegal action => termination with a penalty,
 * ego-centric observation; section 4.1: batched steps under a random policy).
 *
 * Conventions for every entry point
 *   - returns 0 on success, a negative MJ_E_* code otherwise (mj_strerror
 *     gives the text); nothing throws, errno is not used;
 *   - every `d_` pointer is DEVICE memory owned by the caller and valid on
 *     the device of `stream`; the library allocates no device memory;
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream);
 *     kernels are enqueued and the call returns without synchronising, so a
 *     fault inside a kernel surfaces on a later call or synchronise;
 *   - B environments; seats 0..3 per environment; action ids and the state
 *     record are described below.  All arithmetic is integer; the only float
 *     is the optional reward view.
 */
#ifndef MJ_H
#define MJ_H
#include <stdint.h>
#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* error codes */
#define MJ_OK            0
#define MJ_E_ARG        -1   /* bad argument (NULL, B <= 0, seed >= 2^32, mode > 2, range) */
#define MJ_E_HIP        -2   /* a HIP call or kernel launch failed */
#define MJ_E_NOMEM      -3   /* host allocation of the handle failed */
#define MJ_E_UNSUPPORTED -4  /* the device cannot run the kernels (LDS too small) */
#define MJ_E_RANGE      -5   /* a size beyond the stated maximum of the entry point */

/* rule flags (section 3.2, "Rules") */
#define MJ_F_RED      1u     /* red fives: tile ids 16, 52, 88 */
#define MJ_F_ABORT    2u     /* abortive draws */
#define MJ_F_KUITAN   4u     /* open tanyao */
#define MJ_F_MULTIRON 8u     /* reserved, multiple ron is always on */
#define MJ_F_ENDGAME 16u     /* end of game by points (east / half): the last regular kyoku ends the game only if
                                somebody has 30,000; otherwise at most one more round is played, ending after any
                                kyoku that leaves somebody at 30,000; a dealer who repeats in the last regular
                                kyoku or later ends the game when alone in the lead with 30,000 */
#define MJ_F_KANDORA_LATE 32u /* the indicator of an open kan or of a tile added to a pon is turned when the seat
                                discards (before the discard is answered) or declares another kan, so a win on the
                                replacement tile does not count it; a concealed kan still turns it at once.
                                Off: every kan turns its indicator at once */
#define MJ_F_NAGASHI 64u      /* at an exhaustive draw a seat whose river holds terminals and honors only, none of
                                them claimed, is paid as for a self-drawn mangan (no counter bonus, deposits stay,
                                no payments for tenpai); end_type 10, winners = the seats paid.  Off: no such payment */
#define MJ_F_ANKAN_ROB 128u   /* a hand waiting as thirteen orphans may win on the tile of a concealed kan: the offer
                                uses phase 2 like an added kan, kakan_tile carries bit 7 (0x80) then, and a pass lets
                                the kan go on.  Off: a concealed kan can not be robbed */
#define MJ_F_PAO 256u         /* liability: when all three dragon sets (all four wind sets) of a winner are exposed and
                                the last one exposed was claimed from a discard, that discarder pays the whole of
                                that yakuman and the counter bonus on a self-draw, and half of it (the discarder of
                                the winning tile the other half, the counter bonus and any further yakuman) on a
                                ron off somebody else.  Off: no liability */
#define MJ_RULES_NORED (MJ_F_KUITAN | MJ_F_MULTIRON)
#define MJ_RULES_RED   (MJ_F_RED | MJ_F_ABORT | MJ_F_KUITAN | MJ_F_MULTIRON)

typedef struct MjRules {
  uint32_t flags;
  uint32_t env_id_base;      /* global id of env 0: Philox key word 1 is env_id_base + b */
  int32_t  start_score;      /* 25000 */
  float    illegal_penalty;  /* -1.0f: section 3.2, "Action Space" */
  uint8_t  mode;             /* 0 single, 1 east, 2 half: section 3.2, "Game Modes" */
  uint8_t  pad[3];
} MjRules;

/* action ids (section 3.2 lists the categories; the numbering is this library's) */
enum {
  MJ_A_DISCARD = 0,          /* 0..33  discard a non-red copy of kind k          (phase TURN) */
  MJ_A_DISCARD_RED = 34,     /* 34..36 discard the red 5m / 5p / 5s              (TURN) */
  MJ_A_KAN = 37,             /* 37..70 concealed kan of kind k, or add to a pon  (TURN) */
  MJ_A_RIICHI = 71, MJ_A_TSUMO = 72, MJ_A_KYUUSHU = 73,
  MJ_A_RON = 74,             /* RESPOND, RESPOND_KAKAN */
  MJ_A_PON = 75, MJ_A_PON_RED = 76, MJ_A_MINKAN = 77,
  MJ_A_CHI_L = 78, MJ_A_CHI_M = 79, MJ_A_CHI_H = 80,          /* called tile is low / middle / high */
  MJ_A_CHI_L_RED = 81, MJ_A_CHI_M_RED = 82, MJ_A_CHI_H_RED = 83, /* the five taken from the hand is the red one */
  MJ_A_PASS = 84, MJ_NUM_ACTIONS = 85
};
enum { MJ_PHASE_TURN = 0, MJ_PHASE_RESPOND = 1, MJ_PHASE_RESPOND_KAKAN = 2, MJ_PHASE_TERMINAL = 3 };

/* Canonical per-environment record written by mj_export / read by mj_import
 * (array of structures, 1000 bytes, no padding between fields).
 * Tile kinds 0..33 (1m..9m, 1p..9p, 1s..9s, E S W N, white green red); tile
 * ids 0..135, kind = id >> 2.  "tile code" = kind | red << 6, 255 = none.
 * meld word: type(3: 1 chi 2 pon 3 open kan 4 concealed kan 5 added kan) |
 * kind << 3 (lowest kind for chi) | from_rel << 9 | called_pos << 11 |
 * has_red << 13 | called_is_red << 14.  river byte: kind | red << 6 |
 * called_away << 7. */
typedef struct MjEnvCanon {
  uint64_t discarded_kinds[4];   /* 34-bit sets */
  uint64_t waits[4];             /* 34-bit sets, valid while the seat holds 13 - 3*melds tiles */
  uint64_t mask[4][2];           /* legal actions: bit a of word a >> 6 */
  uint64_t yaku[4];              /* last result, per winner */
  int32_t  score[4];
  int32_t  delta[4];             /* point change applied by the last step */
  int32_t  gain[4];              /* last result: amount credited to each winner */
  uint32_t episode, kyoku_serial;
  uint16_t meld[4][4];
  uint16_t hist[128];            /* the kyoku's public actions in the order they took effect: action | seat << 8
                                    (passes and draws are not recorded); entries from n_hist on are 0 */
  uint8_t  wall[136];
  uint8_t  hand[4][34];
  uint8_t  river[4][32];
  uint8_t  hand_red[4], n_meld[4], n_river[4], riichi_idx[4], riichi[4],
           ippatsu[4], first_turn[4], furiten_temp[4], furiten_riichi[4],
           kan_by[4], final_rank[4];
  uint8_t  han[4], fu[4], yakuman_units[4], r_dora[4], r_ura[4], r_aka[4];
  uint8_t  kyoku, honba, kyotaku, terminated;
  uint8_t  draw_ptr, n_kan, live_left, n_dora;
  uint8_t  drawn, phase, cur, actor_mask, riichi_pending, rinshan,
           last_discard, last_discarder, kakan_tile, kuikae[2],
           first_wind, same_wind_cnt, illegal_seat;
  uint8_t  end_type, winners, loser, tenpai_mask;
  uint8_t  dora_pending;         /* kan indicators not turned yet (MJ_F_KANDORA_LATE) */
  uint8_t  n_hist;               /* entries of hist in use (at most 128; later actions of a kyoku are dropped) */
} MjEnvCanon;

/* one hand to evaluate (64 bytes) and its value (24 bytes) */
typedef struct MjHandQuery {
  uint16_t meld[4];
  uint8_t  hand[34];        /* concealed counts INCLUDING the winning tile */
  uint8_t  n_meld, win_kind;
  uint8_t  flags;           /* bit0 tsumo, 1 ippatsu, 2 rinshan, 3 chankan, 4 haitei, 5 houtei, 6 first turn */
  uint8_t  riichi;          /* 0, 1, 2 = double */
  uint8_t  seat_wind, round_wind;
  uint8_t  n_ind;           /* revealed dora indicators, 0..5 */
  uint8_t  ind[5], ura[5];  /* indicator kinds */
  uint8_t  n_aka;           /* red fives among the tiles */
  uint8_t  kuitan;
  uint8_t  pad_[3];
} MjHandQuery;
typedef struct MjHandResult {
  uint64_t yaku;            /* bits 0..29 yaku, 32..43 yakuman */
  int32_t  points;          /* total received by the winner, without honba and sticks */
  uint8_t  han, fu, yakuman_units, shape_ok, yaku_ok, n_dora, n_ura, n_aka;
  uint8_t  pad_[4];
} MjHandResult;

/* Token observation of one (environment, viewer) pair, 496 bytes (section
 * 3.2, "Observation Space": a structured observation for sequence models --
 * hand indices, the action history, scalar properties such as the shanten
 * number and the scores -- ego-centric; the field layout is
 * this library's).  Seats are relative to the viewer: 0 self, 1 next, 2 across,
 * 3 previous.  A tile token is its kind 0..33, or 34 / 35 / 36 for the red
 * 5m / 5p / 5s; 255 pads.  A river entry is token | called_away << 7.  Meld
 * words are those of MjEnvCanon (unused slots 0). */
typedef struct MjTokenObs {
  uint8_t  hand[14];        /* own concealed tiles, ascending kind, the red five before the plain fives */
  uint8_t  n_hand;
  int8_t   shanten;         /* of the own hand: -1 complete, 0 tenpai, .. 6 (customary block formula, tile
                               availability not considered; melds count as sets) */
  uint8_t  drawn;           /* the tile the viewer has just drawn, 255 otherwise */
  uint8_t  phase, cur, last_discarder, last_discard;    /* cur: the seat to move in phase TURN, else 255 */
  uint8_t  kyoku, honba, kyotaku, dealer, live_left, n_dora;
  uint8_t  dora[5];         /* revealed indicators */
  uint8_t  n_meld[4], n_river[4], riichi[4], riichi_idx[4];
  int32_t  score[4];
  uint16_t meld[4][4];
  uint8_t  river[4][32];
  uint8_t  n_hist;          /* public actions of the kyoku so far */
  uint8_t  zero_[15];
  uint16_t hist[128];       /* in the order they took effect: action id | relative seat << 8 (discards, kans, riichi,
                               wins, claims; no passes, no draws); unused entries 0xFFFF */
} MjTokenObs;

typedef struct MjHandle MjHandle;   /* host object: B, seed, rules, step counter, pointers into the caller's buffers */

const char *mj_strerror(int code);

/* Bytes of device memory the caller must provide for B environments (state,
 * structure of arrays) and for the tables (the per-suit decomposition table
 * image).  0 on bad arguments. */
size_t mj_state_bytes(int64_t B, const MjRules *rules);
size_t mj_scratch_bytes(int64_t B, const MjRules *rules);

/* init (section 3.1): builds the per-suit table on the host, uploads it to
 * d_scratch, then for every env shuffles the wall (Philox4x32-10 keyed
 * (seed, env_id), counter (kyoku_serial, j, 0, 0)), deals East-1 with seat 0
 * as dealer and start_score points each, draws for the dealer and fills the
 * legal masks.  d_state / d_scratch must stay alive and untouched by the
 * caller until mj_destroy.  seed must be < 2^32. */
int mj_init(MjHandle **out, void *d_state, void *d_scratch, int64_t B, uint64_t seed,
            const MjRules *rules, void *stream);

/* step (section 3.1 / 3.2): d_actions[b][s] is the action of seat s; every
 * seat whose mask is non-empty acts in the same call (responses to a discard
 * are simultaneous; ron > pon/kan > chi), other entries are ignored.  An
 * action outside the mask ends that game at once (end_type 9); its penalty
 * appears in mj_reward's float view.  A finished kyoku pays, rotates and is
 * followed by the next deal inside the same step unless the game is over.
 * Terminated envs stay frozen until mj_reset_done.  Increments the handle's
 * step counter, which keys the random policy. */
int mj_step(MjHandle *h, const int8_t *d_actions /*[B][4]*/, void *stream);

/* The same step, handing back in the same launch what an agent loop reads after
 * it (section 3.1: step returns the state with rewards, termination flags and
 * the next legal_action_mask).  Every output pointer may be NULL.  d_delta,
 * d_reward (as mj_reward) and d_terminated describe THIS step.  With auto_reset
 * a game that this step ended (or that had ended before) is started again as by
 * mj_reset_done before d_mask is written, so d_mask always belongs to the state
 * the next actions are for; without it, ended games keep an empty mask.
 * d_mask, d_delta, d_reward must be 16-byte aligned. */
int mj_step_full(MjHandle *h, const int8_t *d_actions /*[B][4]*/, int auto_reset,
                 uint64_t *d_mask /*[B][4][2]*/, int32_t *d_delta /*[B][4]*/, float *d_reward /*[B][4]*/,
                 uint8_t *d_terminated /*[B]*/, void *stream);

/* legal_action_mask (section 3.2): d_mask[b][s][w], bit a of word a >> 6; all
 * zero for seats that do not act and for terminated envs. */
int mj_legal_mask(const MjHandle *h, uint64_t *d_mask /*[B][4][2]*/, void *stream);

/* observation (section 3.2, ego-centric; this library's plane layout):
 * d_obs[b][seat][56][34], bytes 0/1, seen from `seat`.  The kernel hands out
 * its work through counters in d_scratch: two mj_observe calls on one handle
 * must be ordered (same stream, or an event between them). */
int mj_observe(const MjHandle *h, uint8_t *d_obs /*[B][4][56][34]*/, void *stream);

/* token observation (section 3.2, see MjTokenObs): d_out[b][seat], seen from
 * `seat`.  d_out must be 16-byte aligned. */
int mj_observe_tokens(const MjHandle *h, MjTokenObs *d_out /*[B][4]*/, void *stream);

/* rewards of the last step: point change per seat, optional float view
 * (points / 1000, or the illegal-action penalty for the offending seat,
 * section 3.2), and the terminated flag.  Any of the three may be NULL. */
int mj_reward(const MjHandle *h, int32_t *d_delta /*[B][4]*/, float *d_reward /*[B][4]*/,
              uint8_t *d_terminated /*[B]*/, void *stream);

/* standings (section 4.2 evaluates agents by their average rank over whole
 * games): current points per seat and, for a terminated env, each seat's final
 * rank 0..3 (0 = first; equal points: the lower seat number is ahead).  Ranks of
 * an env that has not terminated are those of its previous game.  Either
 * pointer may be NULL. */
int mj_standings(const MjHandle *h, int32_t *d_score /*[B][4]*/, uint8_t *d_rank /*[B][4]*/, void *stream);

/* auto-reset: every terminated env starts a new game (episode + 1, a new wall
 * with kyoku_serial + 1, start_score points, East-1). */
int mj_reset_done(MjHandle *h, void *stream);

/* random legal policy (section 4.1): per acting seat, Philox keyed
 * (seed, env_id) with counter (step_lo, step_hi, seat, 1) picks the
 * mulhi(r0, n)-th set bit of the mask; -1 for seats that do not act. */
int mj_sample_random(const MjHandle *h, int8_t *d_actions /*[B][4]*/, void *stream);

/* fused benchmark path: n_steps times { sample, step, reset if auto_reset,
 * write d_obs if write_obs }.  Equivalent to the unfused calls, state by
 * state.  d_obs may be NULL when write_obs is 0.  Without observations up to
 * MJ_ROLLOUT_CHUNK steps run inside one kernel launch (environments never
 * interact; fewer for batches above 131,072 games, so that a launch stays
 * below about 0.1 s); with observations every step is one step launch plus
 * one observation launch. */
#define MJ_ROLLOUT_CHUNK 4096
int mj_step_random(MjHandle *h, int32_t n_steps, int auto_reset, int write_obs, uint8_t *d_obs, void *stream);

/* canonical records of envs [env_lo, env_lo + n) to / from DEVICE memory */
int mj_export(const MjHandle *h, int64_t env_lo, int64_t n, MjEnvCanon *d_out, void *stream);
int mj_import(MjHandle *h, int64_t env_lo, int64_t n, const MjEnvCanon *d_in, void *stream);

/* hand-evaluation micro-batch: value of n hands (best interpretation under
 * the order points, han, fu, yaku mask).  Needs only the tables of `h`. */
int mj_eval_hands(const MjHandle *h, int64_t n, const MjHandQuery *d_in, MjHandResult *d_out, void *stream);

/* The same evaluation for callers that can not allocate and hold no handle: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The tables the kernel reads (the per-suit pattern table, about
 * 370 KB) live in a device array that is part of the library image, one copy per GPU, kept until the process
 * ends; no workspace argument, no handle.  The call allocates nothing: no hipMalloc, no hipFree, no allocating
 * library routine.  d_in / d_out as for mj_eval_hands (device memory, 16- and 8-byte aligned), n at most
 * MJ_EVAL_STATIC_MAX_HANDS (MJ_E_RANGE beyond it; the tables do not grow with n, the limit is that of one launch).
 * The tables of a GPU are uploaded by the first mj_init on that GPU; if none has run there, the first call of this
 * entry point uploads them itself with one synchronous copy (so THAT call must not sit inside a graph capture).
 * The kernel only reads the array, so calls on one GPU may overlap each other; they must not overlap that first
 * upload. */
#define MJ_EVAL_STATIC_MAX_HANDS ((int64_t)1 << 24)
int mj_eval_hands_static(int64_t n, const MjHandQuery *d_in, MjHandResult *d_out, void *stream);

/* scripting / test aid: env b receives the 136 tile ids at d_wall (a
 * permutation of 0..135, not checked) as its wall and the current kyoku is
 * dealt again from it, without shuffling: hands, first draw, masks. */
int mj_deal_from_wall(MjHandle *h, int64_t b, const uint8_t *d_wall /*[136]*/, void *stream);

/* steps taken since mj_init, and its setter: the counter keys the random
 * policy, so a run resumed from mj_export / mj_import records continues the
 * same trajectory once the counter is restored as well (checkpoint / resume). */
uint64_t mj_step_count(const MjHandle *h);
int mj_set_step_count(MjHandle *h, uint64_t steps);
/* timing aid for benchmarks: average duration in milliseconds of the step
 * kernels launched by the last mj_step_random call, measured with HIP events
 * on `stream`; synchronises the stream.  < 0 if nothing was recorded. */
float mj_last_step_kernel_ms(MjHandle *h);

int mj_destroy(MjHandle *h);

#ifdef __cplusplus
}
#endif
#endif
