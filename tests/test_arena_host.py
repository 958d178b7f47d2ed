"""host-side pieces of the evaluation harness (tensor marshalling only; the games themselves need the GPU tier)"""
import numpy as np
import torch

from paper_2605_20577_amd import arena


def test_mask_words_to_bool_and_fixed_policies():
    rng = np.random.default_rng(1)
    words = rng.integers(0, 2**63, size=(50, 4, 2), dtype=np.uint64) | (rng.integers(0, 2, size=(50, 4, 2), dtype=np.uint64) << np.uint64(63))
    words[:, :, 1] &= np.uint64((1 << 21) - 1)                      # 85 actions: bits 64..84
    words[3, 2] = 0
    want = ((words[..., None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(bool).reshape(50, 4, 128)[:, :, :85]
    got = arena.mask_to_bool(torch.from_numpy(words.view(np.int64)))
    assert got.shape == (50, 4, 85) and np.array_equal(got.numpy(), want)
    m = got[:, 1]
    lo, hi = arena.lowest_legal(m).numpy(), arena.highest_legal(m).numpy()
    for b in range(50):
        ids = np.flatnonzero(want[b, 1])
        assert lo[b] == ids[0] and hi[b] == ids[-1]
    pick = arena.UniformRandom(7, device="cpu")(m).numpy()
    assert all(want[b, 1, pick[b]] for b in range(50))
