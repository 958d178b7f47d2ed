"""Batched Riichi Mahjong environment step on AMD MI355X (gfx950): Python binding of libmj.

The binding only marshals arguments: PyTorch provides device memory and the stream, every step of the
environment runs in the HIP kernels of libmj.so (C ABI in include/mj.h).
"""
from .binding import (ENV_DTYPE, MODE_EAST, MODE_HALF, MODE_SINGLE, NUM_ACTIONS, ROLLOUT_CHUNK, QUERY_DTYPE, RESULT_DTYPE, TOKEN_DTYPE, RULES_NORED,
                      RULES_RED, F_ABORT, F_ANKAN_ROB, F_ENDGAME, F_KANDORA_LATE, F_KUITAN, F_NAGASHI, F_PAO, F_RED, MahjongEnv, MjRules, lib, mj_deal_from_wall, mj_destroy, mj_eval_hands, mj_eval_hands_static,
                      mj_export, mj_import, mj_init, mj_legal_mask, mj_observe, mj_observe_tokens, mj_reset_done, mj_reward,
                      mj_sample_random, mj_scratch_bytes, mj_standings, mj_state_bytes, mj_step, mj_step_full, mj_step_random, mj_strerror)

__all__ = ["MahjongEnv", "MjRules", "lib"]
