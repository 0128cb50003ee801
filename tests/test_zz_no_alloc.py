"""wildcat_query_radius_static -- the entry point that allocates nothing -- against wildcat_query_radius, through the
C ABI: two calls in a row on the same device, the second with a smaller input (the library's scratch keeps the first
call's contents), then the size limit."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2602_10056_amd as wc                      # noqa: E402
from paper_2602_10056_amd import workloads as wl       # noqa: E402


def _q(shape, dtype, seed):
    rng = np.random.default_rng(seed)
    q = wl.round_to_storage(rng.standard_normal(shape) * rng.uniform(0.5, 2.0, shape[:2] + (1, 1)), dtype)
    t = torch.from_numpy(q).to(torch.device("cuda:0"))
    return (t.to(torch.bfloat16) if dtype == "bf16" else t).contiguous(), q


def test_static_scratch_entry_point_equals_the_workspace_one():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    wc.load_library()
    dev = torch.device("cuda:0")
    big = torch.empty(8 * (4096 + 64), dtype=torch.uint8, device=dev)
    # first call: 24 query heads in groups of 3, several workgroups per head; second call: fewer heads, fewer rows,
    # another storage type; third: a single short head
    for shape, kv, dtype, seed in (((2, 12, 3000, 64), 4, "bf16", 1), ((1, 4, 700, 128), 2, "f32", 2),
                                   ((1, 1, 5, 64), 1, "bf16", 3)):
        Q, q64 = _q(shape, dtype, seed)
        ref_ws = wc.query_radius(Q, kv_heads=kv, workspace=big)        # per-workgroup maxima in a caller's workspace
        ref_at = wc.query_radius(Q, kv_heads=kv)                       # atomic maxima
        out = torch.full((shape[0], kv), -1.0, dtype=torch.float64, device=dev)
        got = wc.query_radius_static(Q, kv_heads=kv, out=out)
        torch.cuda.synchronize()
        assert got.data_ptr() == out.data_ptr()
        assert torch.equal(got, ref_ws) and torch.equal(got, ref_at)
        nrm = np.sqrt((q64.astype(np.float64) ** 2).sum(-1)).reshape(shape[0], kv, -1).max(-1)
        np.testing.assert_allclose(got.cpu().numpy(), nrm, rtol=1e-14)
    # odd row width: the path without scratch, same answer
    Q, _ = _q((1, 2, 100, 40), "f32", 4)
    assert torch.equal(wc.query_radius_static(Q, kv_heads=1), wc.query_radius(Q, kv_heads=1))


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    wc.load_library()
    lib = wc.load_library()
    dev = torch.device("cuda:0")
    Q = torch.zeros((1, 4097, 1, 64), dtype=torch.bfloat16, device=dev)
    out = torch.zeros((1, 4097), dtype=torch.float64, device=dev)
    o = wc._opts(1, 4097, 4097, 1, 0, wc.WILDCAT_BF16, None)
    rc = lib.wildcat_query_radius_static(Q.data_ptr(), 1, 64, ctypes.byref(o), out.data_ptr())
    assert rc == -5 and b"scratch" in lib.wildcat_strerror(rc)
    with pytest.raises(wc.WildcatError):
        wc.query_radius_static(Q)
    # the ordinary entry point takes the same shape
    assert wc.query_radius(Q).shape == (1, 4097)
