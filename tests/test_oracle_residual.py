"""Pins for the oracle's rounding to storage and the cached-activation reuse step."""
import numpy as np

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import synth


def bf16_values(bits):
    return O.widen(np.asarray(bits, dtype=np.uint16))


def test_narrow_to_bf16_is_the_nearest_value_with_ties_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000),
                        [0.0, -0.0, 1.0, -1.0, 2.0 ** -126, 2.0 ** -133, 3 * 2.0 ** -134, 1e-45]])
    got = O.narrow(x, np.zeros(1, np.uint16))
    # brute force: among the bfloat16 neighbours (bit pattern -1, 0, +1) none is closer
    for xi, gi in zip(x, got):
        cand = [int(gi) + d for d in (-1, 0, 1) if 0 <= (int(gi) & 0x7fff) + d < 0x7f80]
        vals = bf16_values(cand)
        best = np.min(np.abs(vals - xi))
        assert abs(bf16_values([gi])[0] - xi) == best
    # exact ties go to the even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.narrow(np.array([1.0 + 2.0 ** -8]), np.zeros(1, np.uint16))[0] == 0x3f80
    assert O.narrow(np.array([1.0 + 3 * 2.0 ** -8]), np.zeros(1, np.uint16))[0] == 0x3f82
    # just above the tie rounds up although float32 rounding first would have hidden it
    assert O.narrow(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]), np.zeros(1, np.uint16))[0] == 0x3f81


def test_narrow_agrees_with_the_generator_on_float32_inputs_and_round_trips():
    rng = np.random.default_rng(1)
    x32 = (rng.standard_normal(5000) * 3).astype(np.float32)
    assert np.array_equal(O.narrow(x32.astype(np.float64), np.zeros(1, np.uint16)),
                          synth.f32_to_bf16_bits(x32))
    bits = rng.integers(0, 0x7f80, 5000).astype(np.uint16)        # every finite positive pattern
    assert np.array_equal(O.narrow(O.widen(bits), bits), bits)
    assert O.narrow(np.array([0.1]), np.zeros(1, np.float32)).dtype == np.float32


def test_residual_apply_hand_worked():
    # two chunks of two elements, float32: chunk 1 is recomputed, chunk 0 reused
    x = np.array([[1.0, 2.0], [10.0, 20.0]], np.float32)
    y = np.array([[12.5, 19.0]], np.float32)                       # compact row 0 <-> chunk 1
    res = np.array([[0.5, -0.25], [7.0, 7.0]], np.float32)
    new_res, out = O.residual_apply(x, y, res, [1])
    assert new_res.tolist() == [[0.5, -0.25], [2.5, -1.0]]
    assert out.tolist() == [[1.5, 1.75], [12.5, 19.0]]


def test_residual_round_trip_and_all_recompute():
    rng = np.random.default_rng(2)
    x = synth.to_storage(rng.standard_normal((3, 64)).astype(np.float32), "bf16")
    y = synth.to_storage(rng.standard_normal((3, 64)).astype(np.float32), "bf16")
    res0 = np.zeros_like(x)
    res, out = O.residual_apply(x, y, res0, [0, 1, 2])
    assert np.array_equal(out, y)
    # reuse on the same input reproduces the output up to the two roundings of the cache
    _, out2 = O.residual_apply(x, None, res, [])
    err = np.abs(O.widen(out2) - O.widen(y))
    assert err.max() <= 2.0 ** -7 * np.maximum(np.abs(O.widen(y)), np.abs(O.widen(res))).max()
    # compact rows follow the ascending recompute list, not the chunk number
    res1, out1 = O.residual_apply(x, y[:2], res0, [0, 2])
    assert np.array_equal(out1[2], y[1]) and np.array_equal(out1[0], y[0])
    assert np.array_equal(out1[1], O.narrow(O.widen(x[1]), x))      # zero cache: input unchanged
    assert np.array_equal(res1[1], res0[1])


def test_uniform_policy_reduces_to_the_chunkwise_one_for_a_single_chunk():
    rng = np.random.default_rng(3)
    xp = rng.standard_normal((1, 512)).astype(np.float32)
    acc_u, acc_c = 0.0, np.zeros(1)
    for tick in range(12):
        xc = (xp + 0.02 * rng.standard_normal(xp.shape)).astype(np.float32)
        u = O.uniform_decide(xc, xp, [tick], 3, 0.05, acc_u)
        c = O.chunk_decide(xc, xp, np.array([tick], np.int32), 3, 0.05, acc_c)
        assert u["mask"].tolist() == c["mask"].tolist()
        assert np.isclose(u["acc"], c["acc"][0], rtol=1e-15)
        acc_u, acc_c, xp = u["acc"], c["acc"], xc
