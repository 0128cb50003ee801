"""The seeded input generators: deterministic, storage-exact, shaped as documented."""
import numpy as np
import pytest

from paper_2602_10056_amd import workloads as wl


@pytest.mark.parametrize("cfg,ov", [(1, {}), (2, dict(batch=1, q_heads=2, kv_heads=2, n=256)),
                                    (3, dict(q_heads=2, kv_heads=2, n=512)), (4, dict(q_heads=4, kv_heads=2, n=512)),
                                    (5, dict(q_heads=1, kv_heads=1, n=1024)),
                                    (6, dict(q_heads=2, kv_heads=2, n=1024)), (7, dict(batch=2)),
                                    (8, dict(batch=1))])
def test_make_is_deterministic_and_storage_exact(cfg, ov):
    a, b = wl.make(cfg, **ov), wl.make(cfg, **ov)
    s = a["shape"]
    for k in ("Q", "K", "V", "u"):
        np.testing.assert_array_equal(a[k], b[k])
    assert a["Q"].shape == (s.batch, s.q_heads, s.m, s.d) and a["K"].shape == (s.batch, s.kv_heads, s.n, s.d)
    assert a["V"].shape == (s.batch, s.kv_heads, s.n, s.dv)
    if cfg == 7:
        assert (s.m, s.n, s.d, s.dv, s.r, s.bins) == (4096, 1024, 64, 256, 96, 8)
    assert a["u"].shape == (s.problems, s.r) and a["u"].min() >= 0 and a["u"].max() < 1
    if s.dtype == "bf16":
        for k in ("Q", "K", "V"):
            wl.bf16_bits(a[k])            # raises if a value is not bf16-representable
    assert not np.array_equal(a["K"][0, 0], a["V"][0, 0])
    assert s.bins == {6: 16, 7: 8, 8: 224}.get(cfg, 1) and s.n % s.bins == 0 and s.r % s.bins == 0


def test_bins_must_divide_length_and_rank():
    with pytest.raises(ValueError):
        wl.shape(6, n=1000)
    with pytest.raises(ValueError):
        wl.shape(2, bins=3)
    assert wl.shape(2, bins=4).bins == 4


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -3.3, 1e-3])
    r = wl.round_to_storage(x, "bf16")
    np.testing.assert_array_equal(r[:4], [1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6])
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    assert wl.bf16_bits(r).dtype == np.uint16


def test_recipes_have_the_documented_structure():
    w = wl.make(5, q_heads=1, kv_heads=1, n=4096)
    nrm = np.linalg.norm(w["K"][0, 0].astype(np.float64), axis=1)
    np.testing.assert_allclose(nrm[:16], 4 * np.sqrt(128), rtol=0.01)          # sink keys
    assert abs(np.log(nrm[16:] / np.sqrt(128)).std() - 0.5) < 0.05             # log-normal norms
    w = wl.make(2, batch=1, q_heads=1, kv_heads=1, n=2048)
    sv = np.linalg.svd(w["K"][0, 0].astype(np.float64), compute_uv=False)
    assert sv[31] > 3 * sv[32]                                                  # rank 32 plus small noise
    w = wl.make(4, q_heads=4, kv_heads=1, n=64)
    assert w["shape"].group == 4
    # rotary rotation preserves row norms
    g = np.random.default_rng([104, 0, 0, 0])
    raw = g.standard_normal((64, 128))
    np.testing.assert_allclose(np.linalg.norm(w["K"][0, 0], axis=1), np.linalg.norm(raw, axis=1), rtol=0.01)
