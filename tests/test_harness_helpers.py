"""CPU checks of the helpers the GPU parity tests lean on."""
import numpy as np
import torch

from oracle import mtla_oracle as O
from tests import harness as H


def test_bf16_round_is_round_to_nearest_even():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(50000) * 3, rng.standard_normal(1000) * 1e-3, [0.0, -0.0, 1.0, 255.5, 256.5]])
    got = H.bf16_round(x)
    want = torch.from_numpy(x).float().bfloat16().double().numpy()
    assert np.array_equal(got, want)
    assert H.bf16_round(np.array([1.00390625]))[0] == 1.0          # 1 + 2^-8: a tie, the even neighbour is 1
    assert H.bf16_round(np.array([1.01171875]))[0] == 1.015625     # 1 + 3 * 2^-8: a tie, the even neighbour is 1 + 2^-6
    assert np.all(np.abs(got - x) <= 2.0 ** -8 * np.abs(x) + 1e-40)


def test_stored_cache_rounds_the_latent_slots_only():
    c = O.LatentCache(4, 2, 2)
    c.append(np.array([1.00390625, 2.0, 3.1, -0.3]), np.array([0.5, 0.25]), 1.0)
    c.append(np.array([1.0, 1.0, 1.0, 1.0]), np.array([0.75, 0.125]), 0.5)
    s = H.stored_cache(c)
    assert s.i == c.i == 2 and s.n_slots == 1
    assert np.array_equal(s.C[0], H.bf16_round(c.C[0])) and not np.array_equal(s.C[0], c.C[0])
    assert np.array_equal(s.KR[0], c.KR[0])
    c.C[0][0] = 99.0                                                  # a copy, not a view
    assert s.C[0][0] != 99.0
