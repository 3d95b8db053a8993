"""Shared assertions of the GPU parity tests."""
import numpy as np

# Importance mass (Eq. (9)) against the float64 oracle.  Both precisions compute the scores
# from exactly representable inputs with float32 accumulation, a float32 exp2 and a float32
# normaliser, so every element carries a relative error of about 1e-6 for unit-scale logits
# (measured: 5e-7 to 1e-6) that grows with the size of the logits (7e-6 at three times the
# scale); the bounds leave more than an order of magnitude above that for heavy-tailed keys.  The per-head L1 norm is kept beside the
# element-wise bound at the tolerance the method's own statement gives it.
MASS_RTOL = {"bf16": 5e-4, "f32": 2e-4}
MASS_L1 = {"bf16": 1e-2, "f32": 1e-5}


def assert_mass_close(got, ref, dtype, where=""):
    """got, ref: [H_k, L] (any float type).  Element-wise |got - ref| <= rtol * ref + 1e-6 / L,
    non-negative, rows summing to 1, per-head L1 within the stated tolerance, and the largest
    entries at the same positions."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (where, got.shape, ref.shape)
    L = ref.shape[1]
    assert np.all(np.isfinite(got)) and np.all(got >= 0), where
    assert np.allclose(got.sum(axis=1), 1.0, atol=1e-4), (where, got.sum(axis=1))
    rel_l1 = np.abs(got - ref).sum(axis=1) / ref.sum(axis=1)
    assert rel_l1.max() <= MASS_L1[dtype], (where, rel_l1.max())
    bound = MASS_RTOL[dtype] * ref + 1e-6 / L
    excess = np.abs(got - ref) - bound
    worst = np.unravel_index(np.argmax(excess), excess.shape)
    assert excess[worst] <= 0, (where, "element", worst, got[worst], ref[worst])
    # the keys the selection cares most about: the top entries sit where the oracle has them
    k = min(8, L)
    for h in range(ref.shape[0]):
        top_ref = np.argsort(-ref[h], kind="stable")[:k]
        floor = ref[h][top_ref[-1]] * (1 - 4 * MASS_RTOL[dtype])
        top_got = np.argsort(-got[h], kind="stable")[:k]
        assert np.all(ref[h][top_got] >= floor), (where, h, top_got, top_ref)
        assert abs(got[h].max() - ref[h].max()) <= MASS_RTOL[dtype] * ref[h].max(), (where, h)
