/*
 * mjo.h -- CPU ORACLE for the batched Riichi Mahjong environment step.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, single-threaded,
 * obviously-correct statement of what one environment step computes (paper
 * section 3.2 "RL Environment Design": rules, game modes, action space,
 * legal_action_mask, illegal-action termination; section 3.1 names the State
 * contents: hands, scores, winds, melds, masks; section 4.1 gives the
 * random-policy benchmark protocol).  It uses recursion over the hand, no
 * lookup tables, no blocking and no reordering.  It shares no code, header or
 * table with the HIP library; only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load it.
 *
 * The paper states THAT standard four-player East-South Riichi rules are
 * implemented but not the rule text, the action numbering, the reward or the
 * observation layout; every such reading taken here is listed in the design
 * document of the repository and summarised at each function in mjo.c.
 *
 * Parity status: Philox, shuffle, agari, fu/han/points and the phase-machine
 * invariants are pinned by tests (known-answer vectors, brute force, closed
 * forms, conservation laws).  Agreement with the paper's own implementation
 * (validated by its authors against Tenhou logs that are not available here)
 * is "parity unpinned".
 */
#ifndef MJO_H
#define MJO_H
#include <stdint.h>
#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* rule flag bits */
#define MJO_F_RED      1u   /* red fives: tile ids 16, 52, 88 */
#define MJO_F_ABORT    2u   /* abortive draws */
#define MJO_F_KUITAN   4u   /* open tanyao */
#define MJO_F_MULTIRON 8u   /* reserved: multiple ron is always on */
#define MJO_F_ENDGAME 16u   /* end of game by points: 30,000 to finish, one extra round, the leading dealer may stop */
#define MJO_F_NAGASHI 64u     /* a river of unclaimed terminals and honors is paid as a mangan at an exhaustive draw */
#define MJO_F_ANKAN_ROB 128u  /* thirteen orphans may win on the tile of a concealed kan */
#define MJO_F_PAO 256u        /* liability for feeding the last exposed set of the three dragons / four winds */
#define MJO_F_KANDORA_LATE 32u /* the indicator of an open or added kan is turned with the next discard or kan, not at once */

typedef struct MjoRules {
  uint32_t flags;
  uint32_t env_id_base;     /* global id of env 0 (Philox key word 1 = base + b) */
  int32_t  start_score;     /* 25000 */
  float    illegal_penalty; /* -1.0 (section 3.2, action space) */
  uint8_t  mode;            /* 0 single, 1 east, 2 half (section 3.2, game modes) */
  uint8_t  pad[3];
} MjoRules;

/* phases */
enum { MJO_TURN = 0, MJO_RESPOND = 1, MJO_RESPOND_KAKAN = 2, MJO_TERMINAL = 3 };

/* action ids (A = 85) */
enum {
  MJO_A_DISCARD = 0,       /* 0..33 discard a non-red copy of kind k */
  MJO_A_DISCARD_RED = 34,  /* 34..36 discard red 5m/5p/5s */
  MJO_A_KAN = 37,          /* 37..70 ankan / kakan of kind k */
  MJO_A_RIICHI = 71, MJO_A_TSUMO = 72, MJO_A_KYUUSHU = 73, MJO_A_RON = 74,
  MJO_A_PON = 75, MJO_A_PON_RED = 76, MJO_A_MINKAN = 77,
  MJO_A_CHI_L = 78, MJO_A_CHI_M = 79, MJO_A_CHI_H = 80,
  MJO_A_CHI_L_RED = 81, MJO_A_CHI_M_RED = 82, MJO_A_CHI_H_RED = 83,
  MJO_A_PASS = 84, MJO_NUM_ACTIONS = 85
};

/* One environment, all logical state.  Field order is by descending
 * alignment so the struct has no internal padding (sizeof == 1000). */
typedef struct MjoEnv {
  uint64_t discarded_kinds[4];
  uint64_t waits[4];
  uint64_t mask[4][2];
  uint64_t yaku[4];
  int32_t  score[4];
  int32_t  delta[4];
  int32_t  gain[4];
  uint32_t episode, kyoku_serial;
  uint16_t meld[4][4];
  uint16_t hist[128];     /* the kyoku's public actions in order: action | seat << 8; entries from n_hist on are 0 */
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
  uint8_t  dora_pending;  /* kan indicators not turned yet (MJO_F_KANDORA_LATE) */
  uint8_t  n_hist;        /* entries of hist in use */
} MjoEnv;

/* hand-evaluation query / result (the 2^20-hand micro-batch) */
typedef struct MjoHandQuery {
  uint16_t meld[4];
  uint8_t  hand[34];      /* concealed counts INCLUDING the winning tile */
  uint8_t  n_meld, win_kind;
  uint8_t  flags;         /* bit0 tsumo, 1 ippatsu, 2 rinshan, 3 chankan, 4 haitei, 5 houtei, 6 first turn */
  uint8_t  riichi;        /* 0, 1, 2 = double */
  uint8_t  seat_wind, round_wind;
  uint8_t  n_ind;         /* revealed dora indicators 0..5 */
  uint8_t  ind[5], ura[5];
  uint8_t  n_aka;         /* red fives in hand + melds */
  uint8_t  kuitan;
  uint8_t  pad_[3];
} MjoHandQuery;           /* 64 bytes */

typedef struct MjoHandResult {
  uint64_t yaku;
  int32_t  points;        /* total received, without honba and sticks */
  uint8_t  han, fu, yakuman_units, shape_ok, yaku_ok, n_dora, n_ura, n_aka;
  uint8_t  pad_[4];
} MjoHandResult;          /* 24 bytes */

typedef struct MjoHandle MjoHandle;

/* pins / building blocks exposed for the tests */
/* Token observation of one (environment, viewer) pair, 496 bytes (paper
 * section 3.2: a structured observation for sequence models -- hand indices,
 * the action history, scalar properties such as the shanten number and the
 * scores -- ego-centric).  Seats are relative to the
 * viewer: 0 self, 1 next, 2 across, 3 previous.  A tile token is its kind
 * 0..33, or 34 / 35 / 36 for the red 5m / 5p / 5s; 255 pads.  A river entry is
 * token | called_away << 7.  Meld words are those of MjoEnv. */
typedef struct MjoTokenObs {
  uint8_t  hand[14];      /* own concealed tiles, ascending kind, the red five before the plain fives */
  uint8_t  n_hand;
  int8_t   shanten;       /* of the own hand: -1 complete, 0 tenpai, .. 6 */
  uint8_t  drawn;         /* the tile the viewer has just drawn, 255 otherwise */
  uint8_t  phase, cur, last_discarder, last_discard;   /* relative seats (255 none), token */
  uint8_t  kyoku, honba, kyotaku, dealer, live_left, n_dora;
  uint8_t  dora[5];       /* revealed indicators */
  uint8_t  n_meld[4], n_river[4], riichi[4], riichi_idx[4];
  int32_t  score[4];
  uint16_t meld[4][4];
  uint8_t  river[4][32];
  uint8_t  n_hist;        /* public actions of the kyoku so far */
  uint8_t  zero_[15];
  uint16_t hist[128];     /* in order: action id | relative seat << 8; unused entries 0xFFFF */
} MjoTokenObs;

void mjo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void mjo_shuffle_wall(uint32_t seed, uint32_t env_id, uint32_t kyoku_serial, uint8_t wall[136]);
int  mjo_is_complete(const uint8_t hand[34], int n_meld);
uint64_t mjo_waits_of(const uint8_t hand[34], const uint16_t meld[4], int n_meld);
int  mjo_shanten(const uint8_t hand[34], int n_meld);   /* -1 complete, 0 tenpai, ... (section 3.2, observation scalars) */
void mjo_eval_hand(const MjoHandQuery *q, MjoHandResult *r);

/* environment API (host pointers everywhere) */
int  mjo_create(MjoHandle **out, int64_t B, uint64_t seed, const MjoRules *rules);
int  mjo_step(MjoHandle *h, const int8_t *actions /*[B][4]*/);
int  mjo_legal_mask(const MjoHandle *h, uint64_t *mask /*[B][4][2]*/);
int  mjo_observe(const MjoHandle *h, uint8_t *obs /*[B][4][56][34]*/);
int  mjo_reward(const MjoHandle *h, int32_t *delta /*[B][4]*/, float *reward /*[B][4] or NULL*/,
                uint8_t *terminated /*[B]*/);
int  mjo_reset_done(MjoHandle *h);
int  mjo_sample_random(MjoHandle *h, int8_t *actions /*[B][4]*/);
int  mjo_step_random(MjoHandle *h, int32_t n_steps, int auto_reset);
int  mjo_export(const MjoHandle *h, int64_t env_lo, int64_t n, MjoEnv *out);
int  mjo_import(MjoHandle *h, int64_t env_lo, int64_t n, const MjoEnv *in);
/* replace env b's wall by the given permutation and deal the current kyoku again from it */
int  mjo_deal_from_wall(MjoHandle *h, int64_t b, const uint8_t wall[136]);
int  mjo_observe_tokens(const MjoHandle *h, MjoTokenObs *out /*[B][4]*/);
uint64_t mjo_step_count(const MjoHandle *h);
void mjo_destroy(MjoHandle *h);
size_t mjo_sizeof_env(void);

#ifdef __cplusplus
}
#endif
#endif
