"""Whole-game evaluation of per-seat policies on the batched environment (paper section 4.2: an agent is rated
by its average rank over many games against three fixed opponents; equal players average 2.5).

The environment runs in libmj (mj_legal_mask / mj_observe / mj_step / mj_reward / mj_standings /
mj_reset_done); a policy is any callable on device tensors, so a PyTorch model plugs in directly:

    policy(mask, obs) -> actions
      mask     bool  [B, 85]       legal actions of this seat (all False where the seat does not act)
      obs      uint8 [B, 56, 34]   the seat's observation planes, or None unless the policy sets `needs_obs = True`
      actions  int   [B]           an action id per game; ignored where the seat does not act
"""
import torch

from .binding import NUM_ACTIONS


def mask_to_bool(mask_words):
    """[B, 4, 2] 64-bit mask words (as int64) -> bool [B, 4, 85]"""
    m = mask_words.view(torch.int64)
    bit = torch.arange(64, device=m.device, dtype=torch.int64)
    bits = ((m.unsqueeze(-1) >> bit) & 1).to(torch.bool)            # [B, 4, 2, 64]
    return bits.reshape(m.shape[0], 4, 128)[:, :, :NUM_ACTIONS]


def lowest_legal(mask, obs=None):
    """the legal action with the smallest id (a fixed, deterministic opponent)"""
    return mask.to(torch.uint8).argmax(dim=1)


def highest_legal(mask, obs=None):
    """the legal action with the largest id: takes every win, call and pass before any discard"""
    return (NUM_ACTIONS - 1) - mask.flip(1).to(torch.uint8).argmax(dim=1)


class UniformRandom:
    """uniform over the legal actions, from its own seeded generator"""

    def __init__(self, seed, device="cuda:0"):
        self.gen = torch.Generator(device=device)
        self.gen.manual_seed(seed)

    def __call__(self, mask, obs=None):
        score = torch.rand(mask.shape, generator=self.gen, device=mask.device)
        return torch.where(mask, score, torch.full_like(score, -1.0)).argmax(dim=1)


def play(env, policies, n_games):
    """Plays until n_games games have finished (games run B at a time, a finished game is replaced by a new one
    at once; the first n_games to finish are counted).  Returns a dict with the mean rank (1 = first .. 4) and
    mean final points per seat, the rank counts [4 seats][4 ranks], and the number of batched steps taken."""
    assert len(policies) == 4
    B, dev = env.B, env.device
    need_obs = any(getattr(p, "needs_obs", False) for p in policies)
    rank_count = torch.zeros((4, 4), dtype=torch.int64, device=dev)
    score_sum = torch.zeros(4, dtype=torch.int64, device=dev)
    done, steps = 0, 0
    actions = torch.empty((B, 4), dtype=torch.int8, device=dev)
    while done < n_games:
        mask = mask_to_bool(env.legal_mask())
        obs = env.observe() if need_obs else None
        for s, pol in enumerate(policies):
            a = pol(mask[:, s], obs[:, s] if need_obs else None)
            acts = mask[:, s].any(dim=1)
            actions[:, s] = torch.where(acts, a.to(torch.int8), torch.full_like(a, -1, dtype=torch.int8))
        env.step(actions)
        steps += 1
        _, _, term = env.reward()
        idx = torch.nonzero(term).flatten()
        if idx.numel():
            idx = idx[: n_games - done]                              # lowest env ids first: the count is exact
            score, rank = env.standings()
            r = rank[idx].to(torch.int64)                            # [n, 4]
            for s in range(4):
                rank_count[s] += torch.bincount(r[:, s], minlength=4)
            score_sum += score[idx].to(torch.int64).sum(dim=0)
            done += int(idx.numel())
            env.reset_done()
    rc = rank_count.cpu().double()
    mean_rank = (rc * torch.arange(1, 5, dtype=torch.float64)).sum(dim=1) / rc.sum(dim=1)
    return {"games": done, "steps": steps, "mean_rank": mean_rank.tolist(),
            "mean_score": (score_sum.cpu().double() / done).tolist(), "rank_count": rank_count.cpu().tolist()}


def one_vs_three(env, agent, opponent, n_games):
    """the agent on seat 0 against three copies of the opponent; returns play()'s dict (mean_rank[0] is the
    figure of section 4.2)"""
    return play(env, [agent, opponent, opponent, opponent], n_games)
