"""Host-side checks of libwildcat that need no GPU: the library loads, exports every symbol the header
declares, validates arguments before launching anything, and its uniform stream is the documented one."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2602_10056_amd as wc
from oracle import wildcat_oracle as wo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(wc.LIB_PATH), reason="libwildcat.so not built")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "wildcat.h")).read()
    declared = set(re.findall(r"^(?:int|size_t|const char \*)\s*(wildcat_[a-z_0-9]+)\(", header, flags=re.M))
    assert declared == set(wc.EXPORTS)
    lib = wc.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert wc.version() >= 100


def test_struct_layout_matches_header_order():
    header = open(os.path.join(ROOT, "include", "wildcat.h")).read()
    body = header[header.index("typedef struct {", header.index("Options.")):header.index("} wildcat_opts;")]
    names = re.findall(r"\b(\w+);\s*(?:/\*|$)", body, flags=re.M)
    assert names == [f[0] for f in wc._Opts._fields_]
    body = header[header.index("typedef struct {", header.index("compressed cache")):header.index("} wildcat_coreset;")]
    names = re.findall(r"\*(\w+);", body)
    assert names == [f[0] for f in wc._Coreset._fields_]


def test_strerror():
    lib = wc.load_library()
    texts = {lib.wildcat_strerror(c).decode() for c in (0, -1, -2, -3, -4, -99)}
    assert len(texts) == 6 and all(texts)


def test_uniform_stream_equals_the_documented_generator():
    for seed in (0, 1234567, 2 ** 63 + 5):
        np.testing.assert_array_equal(wc.draw_uniforms(seed, 257), wo.splitmix_uniforms(seed, 257))
    assert wc.load_library().wildcat_draw_uniforms(1, -1, None) == -1


def test_workspace_bytes():
    a = wc.workspace_bytes(4096, 64, 128, batch=4, kv_heads=8)
    b = wc.workspace_bytes(8192, 64, 128, batch=4, kv_heads=8)
    assert 0 < a < b and a % 256 == 0
    # dominated by the fp64 history P * n * r * 8
    assert a >= 32 * 4096 * 128 * 8
    assert wc.workspace_bytes(100, 64, 101) == 0            # r > n
    assert wc.workspace_bytes(100, 0, 10) == 0
    assert wc.workspace_bytes(100, 64, 10, dtype=7) == 0
    assert wc.workspace_bytes(100000, 64, 5000) == 0        # rank limit of this build
    # bins: B problems of n/B keys and r/B pivots each -- the history shrinks by B
    c = wc.workspace_bytes(4096, 64, 128, batch=4, kv_heads=8, bins=16)
    assert 0 < c < a / 4
    assert wc.workspace_bytes(4096, 64, 128, bins=3) == 0   # B must divide n and r
    assert wc.workspace_bytes(100000, 64, 5000, bins=4) > 0  # the rank limit applies per bin
    # fast mode: fp32 history rows halve the dominant term
    e = wc.workspace_bytes(4096, 64, 128, batch=4, kv_heads=8, history="f32")
    assert a - e == 32 * 4096 * 128 * 4                      # exactly the 4 bytes saved per history entry


def test_entry_points_reject_bad_arguments_before_launching():
    lib = wc.load_library()
    o = wc._Opts()
    c = wc._Coreset()
    one = ctypes.c_void_p(8)          # never dereferenced: validation fails first
    assert lib.wildcat_compress_kv(None, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, None, ctypes.byref(c)) == -1
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1   # no r_q
    o.r_q = 8
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1   # null outputs
    for f, _ in wc._Coreset._fields_:
        setattr(c, f, 8)
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -2   # no workspace
    o.workspace, o.workspace_bytes = 256, 16
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -2   # too small
    o.workspace, o.workspace_bytes = 264, 1 << 40
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -2   # misaligned
    assert lib.wildcat_compress_kv(one, one, 128, 64, 129, 0, ctypes.byref(o), ctypes.byref(c)) == -1  # r > n
    o.bins = 3
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1   # 3 !| n, r
    o.bins = 4
    assert lib.wildcat_compress_kv(one, one, 128, 64, 18, 0, ctypes.byref(o), ctypes.byref(c)) == -1   # 4 | n, 4 !| r
    o.bins, o.tau_length = 4, 2
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1   # bad switch
    o.bins, o.tau_length = -1, 0
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1
    o.bins = 0
    o.history = 2
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1   # unknown mode
    o.history = 0
    o.q_heads, o.kv_heads = 6, 4
    assert lib.wildcat_compress_kv(one, one, 128, 64, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -1   # 6 % 4
    o.q_heads, o.kv_heads = 0, 0
    assert lib.wildcat_compress_kv(one, one, 128, 512, 16, 0, ctypes.byref(o), ctypes.byref(c)) == -4  # d too wide
    assert lib.wildcat_wtd_attn(None, ctypes.byref(c), one, 16, 64, 16, ctypes.byref(o)) == -1
    assert lib.wildcat_wtd_attn(one, ctypes.byref(c), one, 0, 64, 16, ctypes.byref(o)) == -1
    o.dtype = 3
    assert lib.wildcat_wtd_attn(one, ctypes.byref(c), one, 16, 64, 16, ctypes.byref(o)) == -1
    assert lib.wildcat_query_radius(one, 0, 64, ctypes.byref(o), one) == -1


def test_library_shares_the_hip_runtime_of_torch():
    """Loaded before torch, the library would bring a second HIP runtime into the process (the system's, next to
    the one torch ships) and launch on a runtime that has no device.  load_library() imports torch first."""
    import subprocess, sys
    code = (
        "import paper_2602_10056_amd as wc\n"
        "wc.load_library()\n"
        "import torch\n"
        "paths = {l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l}\n"
        "print(len(paths))\n"
    )
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.strip().splitlines()[-1] == "1"


# ---------------------------------------------------------------------------------- launch form of the selection loop
MI355X = dict(compute_units=256, occ_resident_keys=2, occ_streamed_keys=4)   # what the loop kernels reach on that device


def test_loop_plan_headline_and_long_context_shapes():
    """Pure host logic (no device is touched when compute_units > 0): which launch form the selection loop takes."""
    # headline shape: 8 problems x 64 slabs of 512 keys = 512 workgroups = 2 per compute unit, keys in registers
    p = wc.loop_plan(32768, 128, 512, kv_heads=8, **MI355X)
    assert p == dict(driver=1, keys_per_thread=2, slabs=64, problems_per_launch=8, launches=1, keys_in_registers=1,
                     workgroups_per_cu=2, reserved=0)
    # twice / four times the length: the problems run in groups that keep the keys in registers
    p = wc.loop_plan(65536, 128, 512, kv_heads=8, **MI355X)
    assert (p["driver"], p["problems_per_launch"], p["launches"], p["keys_in_registers"]) == (1, 4, 2, 1)
    p = wc.loop_plan(131072, 128, 1024, kv_heads=8, **MI355X)
    assert (p["driver"], p["problems_per_launch"], p["launches"], p["keys_in_registers"]) == (1, 2, 4, 1)
    assert p["workgroups_per_cu"] == 2
    # uneven split: 3 problems per launch would be 3 + 3 + 2; balanced groups of at most 3
    p = wc.loop_plan(131072 // 2 * 3 // 3, 128, 64, kv_heads=7, **MI355X)
    assert p["problems_per_launch"] * p["launches"] >= 7 and p["problems_per_launch"] * 128 <= 512
    # one problem whose slabs exceed even the streamed-keys capacity: one launch per step
    p = wc.loop_plan(1 << 20, 128, 64, kv_heads=1, **MI355X)
    assert p["slabs"] == 2048 and p["driver"] == 0 and p["launches"] == 1
    # ... and one that fits only with streamed keys
    p = wc.loop_plan(1 << 19, 128, 64, kv_heads=1, **MI355X)
    assert (p["driver"], p["keys_in_registers"], p["launches"]) == (1, 0, 1)


def test_loop_plan_honours_the_loop_driver_option_and_small_shapes():
    # the caller's opt-out for shared devices
    p = wc.loop_plan(32768, 128, 512, kv_heads=8, loop="steps", **MI355X)
    assert p["driver"] == 0
    # a single step needs no loop at all unless the problem is one slab
    assert wc.loop_plan(32768, 128, 1, kv_heads=8, **MI355X)["driver"] == 0
    assert wc.loop_plan(200, 64, 1, kv_heads=8, **MI355X)["driver"] == 2
    # one slab per problem: a workgroup alone with its problem, any number of problems in one launch
    p = wc.loop_plan(4096, 64, 64, kv_heads=8, bins=16, dtype=wc.WILDCAT_BF16, **MI355X)
    assert p["slabs"] == 1 and p["driver"] == 2 and p["launches"] == 1 and p["problems_per_launch"] == 128
    # many tiny problems: a wavefront per problem; few of them: only on request
    assert wc.loop_plan(3136, 64, 224, batch=8, bins=224, dtype=wc.WILDCAT_F32, **MI355X)["driver"] == 3
    assert wc.loop_plan(3136, 64, 224, batch=1, bins=224, dtype=wc.WILDCAT_F32, **MI355X)["driver"] == 2
    assert wc.loop_plan(3136, 64, 224, batch=1, bins=224, dtype=wc.WILDCAT_F32, loop="wave", **MI355X)["driver"] == 3
    assert wc.loop_plan(4096, 64, 64, kv_heads=8, bins=16, loop="wave", **MI355X)["driver"] == 2   # 256 keys: too many for a wave
    # a device that cannot hold a single workgroup of the loop kernel
    assert wc.loop_plan(32768, 128, 512, kv_heads=8, compute_units=256, occ_resident_keys=0,
                        occ_streamed_keys=0)["driver"] == 0
    # widths whose keys do not fit the registers fall back to streamed keys: fp32 storage, d = 128, two keys per thread
    p = wc.loop_plan(32768, 128, 64, kv_heads=8, dtype=wc.WILDCAT_F32, **MI355X)
    assert p["driver"] == 1 and p["keys_in_registers"] == 0


def test_loop_plan_binned_long_sequence_keeps_keys_in_registers_when_four_workgroups_fit():
    """128 bins x 8 slabs (workload 6).  With the loop kernel of few-step loops at four workgroups per compute unit
    all 1024 slabs are resident with their keys in registers; at two per compute unit the plan weighs a second
    launch (7 us more per step) against re-reading all keys every step (10 us) and splits the bins in two groups."""
    shape = dict(kv_heads=8, bins=16, dtype=wc.WILDCAT_BF16)
    p = wc.loop_plan(65536, 64, 64, compute_units=256, occ_resident_keys=4, occ_streamed_keys=4, **shape)
    assert (p["driver"], p["slabs"], p["problems_per_launch"], p["launches"], p["keys_in_registers"],
            p["workgroups_per_cu"]) == (1, 8, 128, 1, 1, 4)
    p = wc.loop_plan(65536, 64, 64, compute_units=256, occ_resident_keys=2, occ_streamed_keys=4, **shape)
    assert (p["driver"], p["problems_per_launch"], p["launches"], p["keys_in_registers"]) == (1, 64, 2, 1)
    # ... and streams them where no workgroup with keys in registers fits at all
    p = wc.loop_plan(65536, 64, 64, compute_units=256, occ_resident_keys=0, occ_streamed_keys=4, **shape)
    assert (p["driver"], p["launches"], p["keys_in_registers"]) == (1, 1, 0)


def test_loop_plan_rejects_bad_arguments():
    lib = wc.load_library()
    o = wc._Opts()
    out = (ctypes.c_int32 * 8)()
    assert lib.wildcat_loop_plan(128, 64, 16, ctypes.byref(o), 256, 2, 4, None) == -1
    assert lib.wildcat_loop_plan(128, 64, 129, ctypes.byref(o), 256, 2, 4, out) == -1      # r > n
    assert lib.wildcat_loop_plan(128, 64, 16, ctypes.byref(o), 256, -1, 4, out) == -1
    o.loop_driver = 3
    assert lib.wildcat_loop_plan(128, 64, 16, ctypes.byref(o), 256, 2, 4, out) == -1       # unknown driver
    o.loop_driver = 0
    o.bins = 3
    assert lib.wildcat_loop_plan(128, 64, 16, ctypes.byref(o), 256, 2, 4, out) == -1
