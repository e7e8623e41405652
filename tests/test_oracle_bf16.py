"""Pins for the oracle's bfloat16 rounding: torch's own conversion (a library
routine written by someone else) and hand-built halfway cases."""
import numpy as np
import torch

from oracle import round_to_bf16


def _torch_bf16(x):
    # torch rounds float32 -> bfloat16 to nearest even; feed it float32-exact inputs
    return torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).double().numpy()


def test_matches_torch_on_float32_inputs():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32).astype(np.float64)
    assert np.array_equal(round_to_bf16(x), _torch_bf16(x))


def test_halfway_cases_round_to_even():
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: even neighbour is 1.
    assert round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd) and 1+2^-6 (even).
    assert round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # just above / below halfway, distinguishable only in float64
    assert round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    assert round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8 - 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    # carry into the exponent
    assert round_to_bf16(np.array([2.0 - 2.0 ** -9]))[0] == 2.0
    assert round_to_bf16(np.array([-(2.0 - 2.0 ** -9)]))[0] == -2.0


def test_fixed_points_and_specials():
    grid = torch.arange(-2 ** 15, 2 ** 15, dtype=torch.int32).to(torch.int16).view(torch.bfloat16).double().numpy()
    finite = grid[np.isfinite(grid)]
    assert np.array_equal(round_to_bf16(finite), finite)          # idempotent on the grid
    out = round_to_bf16(np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, 3.5e38]))
    assert out[0] == 0 and out[1] == 0 and np.signbit(out[1])
    assert out[2] == np.inf and out[3] == -np.inf and np.isnan(out[4])
    assert out[5] == 0.0 and out[6] == np.inf
    sub = np.array([2.0 ** -130, 3 * 2.0 ** -134, 2.0 ** -127 + 2.0 ** -134])
    assert np.array_equal(round_to_bf16(sub), _torch_bf16(sub))
