#!/usr/bin/env python3
"""Benchmark of the WildCat hot path on one MI355X.

A "step" is one pass of the whole path -- query radius, CompressKV (prologue, RPNys selection loop,
Gram pass, core solve, gather) and WtdAttn -- over one batch of synthetic attention inputs that are
already resident in HBM.  Workload: 32 query heads sharing 8 key/value heads, n = m = 32768, d = 128,
r = 512, bf16 storage (rotary-rotated Gaussian inputs), the shape the headline metric is quoted on.

Prints ONE JSON line: tokens/s of the whole path, the roofline of the dominant kernel (the RPNys step
kernel, HBM-bound, timed with HIP events on the launch stream; `frac` on algorithmic bytes, `frac_traffic` on
the HBM bytes a counter run measured for the same launch), the WtdAttn MFMA rate, the float64 CPU oracle timed
on the host cores, exact attention at the same shape for context, the same path at n = 32K / 64K / 128K
(`scaling_in_n`) and the binned regime of Sec. 2.5 (`binned`: workload 6 with exact attention beside it).
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense MFMA rate, the same for bf16 and fp16 operands


class HipEvents:
    """Raw hipEvent_t pairs (the library records them on its launch stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        if self.hip.hipEventCreate(ctypes.byref(ev)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return ev

    def elapsed_ms(self, a, b):
        if self.hip.hipEventSynchronize(b) != 0:
            raise RuntimeError("hipEventSynchronize failed")
        ms = ctypes.c_float()
        if self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)


def step_loop_bytes(P, n, d, r, es, single_launch, hs=8):
    """Algorithmic HBM bytes of the RPNys selection loop.  Per step i and key: the i earlier Cholesky entries of
    that key (hs i; hs = 8 bytes, 4 in the fp32-history fast mode), the new entry (hs), and p written for the other
    workgroups plus read back during the pivot search (16).  The key rows (d * es per key) are read once when the
    loop is one persistent launch that keeps them in registers, and once per step when the loop is one launch per
    step."""
    key_reads = 1 if single_launch else r
    return float(P) * n * (key_reads * d * es + r * (hs + 16) + float(hs) * r * (r - 1) / 2.0)


def device_workload_cfg4(s, dev, tdt):
    """Workload 4's recipe (N(0,1) entries, rotary rotation of Q and K by position, N(0,1) values, uniforms in
    [0, 1)) drawn on the device with a seeded generator: the sweep over n needs the distribution, not the
    oracle's exact numbers, and NumPy takes a minute for the 128K point."""
    import torch
    g = torch.Generator(device=dev)
    g.manual_seed(s.data_seed * 1000003 + s.n)

    def rope(x):
        n, d = x.shape[-2], x.shape[-1]
        j = torch.arange(d // 2, device=dev, dtype=torch.float64)
        ang = torch.arange(n, device=dev, dtype=torch.float64)[:, None] * (10000.0 ** (-2.0 * j / d))[None, :]
        c, sn = torch.cos(ang).float(), torch.sin(ang).float()
        out = torch.empty_like(x)
        out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * sn
        out[..., 1::2] = x[..., 0::2] * sn + x[..., 1::2] * c
        return out

    Q = rope(torch.randn((s.batch, s.q_heads, s.m, s.d), generator=g, device=dev)).to(tdt)
    K = rope(torch.randn((s.batch, s.kv_heads, s.n, s.d), generator=g, device=dev)).to(tdt)
    V = torch.randn((s.batch, s.kv_heads, s.n, s.dv), generator=g, device=dev).to(tdt)
    u = torch.rand((s.problems, s.r), generator=g, device=dev, dtype=torch.float64)
    return Q, K, V, u


def timed_pass(wc, torch, s, Q, K, V, u, history, reps=3):
    """ms of the whole path (query radius, CompressKV, WtdAttn) on resident inputs: one warm-up, then `reps` passes."""
    es = 1 if s.dtype == "bf16" else 0
    ws = torch.empty(wc.workspace_bytes(s.n, s.d, s.r, s.batch, s.kv_heads, s.dv, es, s.bins, history),
                     dtype=torch.uint8, device=Q.device)
    out = torch.empty((s.batch, s.q_heads, s.m, s.dv), dtype=Q.dtype, device=Q.device)

    def one():
        cs = wc.compress_kv(K, V, s.r, wc.query_radius(Q, s.kv_heads, workspace=ws), uniforms=u, workspace=ws,
                            bins=s.bins, history=history)
        wc.wtd_attn(Q, cs, out=out)

    one()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        one()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def exact_attention_ms(torch, s, Q, K, V, reps=3):
    import torch.nn.functional as F
    Kx = K.repeat_interleave(s.group, dim=1) if s.group > 1 else K
    Vx = V.repeat_interleave(s.group, dim=1) if s.group > 1 else V
    for _ in range(2):
        F.scaled_dot_product_attention(Q, Kx, Vx)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        F.scaled_dot_product_attention(Q, Kx, Vx)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def cpu_baseline(w, budget_heads):
    """The float64 oracle, as it stands, on the host cores; whole kv heads of the benchmark workload."""
    import numpy as np
    from oracle import wildcat_oracle as wo
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        threads = os.cpu_count() or 1
    s = w["shape"]
    t0 = time.perf_counter()
    done = 0
    for h in range(budget_heads):
        Qg = w["Q"][0, h * s.group:(h + 1) * s.group].astype(np.float64)
        wo.wildcat(Qg, w["K"][0, h].astype(np.float64), w["V"][0, h].astype(np.float64), s.beta, s.r, w["u"][h],
                   bins=s.bins)
        done += 1
        if time.perf_counter() - t0 > 20.0:
            break
    dt = time.perf_counter() - t0
    tokens_per_s = s.batch * s.n / (dt * s.kv_heads / done)
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{done} of {s.kv_heads} kv heads (each with its {s.group} query heads) of the same workload, "
                      f"full n={s.n}, r={s.r}; {dt:.1f} s of float64 NumPy; scaled to all heads"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cfg", type=int, default=4, help="workload catalogue entry (4 = headline shape)")
    ap.add_argument("--history", choices=("f64", "f32"), default="f64",
                    help="precision of the selection loop's history rows (f32 = the fast mode; default f64)")
    ap.add_argument("--loop", choices=("auto", "steps"), default="auto",
                    help="selection loop driver (steps = one launch per step; for profiling the two forms)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-exact", action="store_true")
    ap.add_argument("--sweep-n", action="store_true",
                    help="'scaling_in_n' from n = 4K up (default: 32K, 64K, 128K), inputs from the NumPy recipe")
    ap.add_argument("--no-sweep", action="store_true", help="leave out 'scaling_in_n' and 'binned'")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives): use --gpus 1")

    import numpy as np
    import torch
    import paper_2602_10056_amd as wc
    from paper_2602_10056_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    wc.load_library()
    dev = torch.device("cuda:0")
    w = wl.make(args.cfg)
    s = w["shape"]
    tdt = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    es = 2 if s.dtype == "bf16" else 4
    Q, K, V = (torch.from_numpy(w[k]).to(dev).to(tdt).contiguous() for k in ("Q", "K", "V"))
    u = torch.from_numpy(w["u"]).to(dev)
    ws = torch.empty(wc.workspace_bytes(s.n, s.d, s.r, s.batch, s.kv_heads, s.dv, 1 if s.dtype == "bf16" else 0, s.bins,
                                        args.history), dtype=torch.uint8, device=dev)
    out = torch.empty((s.batch, s.q_heads, s.m, s.dv), dtype=tdt, device=dev)
    hev = HipEvents()
    loop_ev = [(hev.create(), hev.create()) for _ in range(args.steps)]
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]

    def one_step(k=None):
        ev = loop_ev[k] if k is not None else None
        if k is not None:
            marks[k][0].record()
        r_q = wc.query_radius(Q, s.kv_heads, workspace=ws)
        if k is not None:
            marks[k][1].record()
        cs = wc.compress_kv(K, V, s.r, r_q, uniforms=u, workspace=ws, loop_events=ev, bins=s.bins,
                            history=args.history, loop=args.loop)
        if k is not None:
            marks[k][2].record()
        wc.wtd_attn(Q, cs, out=out)
        if k is not None:
            marks[k][3].record()
        return cs

    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        cs = one_step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    loop_ms = float(np.mean([hev.elapsed_ms(a, b) for a, b in loop_ev]))
    ph = np.array([[m[i].elapsed_time(m[i + 1]) for i in range(3)] for m in marks]).mean(axis=0)
    P = s.problems
    plan = wc.loop_plan(s.n, s.d, s.r, s.batch, s.kv_heads, s.dv, 1 if s.dtype == "bf16" else 0, s.bins, args.history,
                        args.loop)
    single = plan["driver"] != 0
    launches = plan["launches"] * (1 if single else s.r // s.bins)
    # with bins the loop is P * B independent problems of n / B keys and r / B steps
    loop_bytes = step_loop_bytes(P * s.bins, s.n // s.bins, s.d, s.r // s.bins, es, bool(plan["keys_in_registers"]),
                                 8 if args.history == "f64" else 4)
    achieved = loop_bytes / (loop_ms * 1e-3) / 1e9
    # HBM bytes of the same launch from the rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE scaled by a copy kernel of
    # known size); the file says which launch form it was measured on
    traffic = traffic_source = None
    tfile = os.path.join(ROOT, "profiles", "rpnys_loop_traffic.json")
    if os.path.exists(tfile) and args.cfg == 4 and args.history == "f64":
        with open(tfile) as f:
            rec = json.load(f).get("single_launch" if single else "per_step", {})
        if rec.get("launches") == launches:
            traffic = rec.get("hbm_bytes_per_launch")
            traffic_source = "profiles/rpnys_loop_traffic.json (summary: profiles/rpnys_loop_cfg4_hbm_traffic.md)"
    attn_flops = float(s.batch * s.q_heads) * s.m * (2.0 * s.r * (s.d + s.dv) + 2.0 * s.r)
    attn_tflops = attn_flops / (ph[2] * 1e-3) / 1e12

    res = {
        "metric": "WildCat attention tokens/sec + HBM/MFMA % of peak vs exact attn at n=32K",
        "value": s.batch * s.n / (dt / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": f"{s.name}: batch {s.batch} x {s.q_heads} query heads / {s.kv_heads} kv heads, "
                               f"n={s.n}, m={s.m}, d={s.d}, d_v={s.dv}, r={s.r}, B={s.bins}, {s.dtype} storage; selection loop in fp64{' with fp32 history rows (fast mode)' if args.history == 'f32' else ''}, "
                               f"WtdAttn on MFMA (bf16 scores, fp16 value product) with fp32 accumulation",
                   "uniform_seed": s.uniform_seed, "data_seed": s.data_seed},
        "phases_ms": {"query_radius": float(ph[0]), "compress_kv": float(ph[1]), "rpnys_loop": loop_ms,
                      "wtd_attn": float(ph[2])},
        "roofline": {"kernel": ("k_rpnys_persistent (RPNys selection loop, all %d steps in one launch)" % (s.r // s.bins)) if single
                               else "k_step (RPNys selection loop, one launch per step)", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "frac_traffic": (traffic / (loop_ms / launches * 1e-3) / 1e9 / HBM_PEAK_GBS) if traffic else None,
                     "launches": launches, "avg_launch_ms": loop_ms / launches,
                     "algorithmic_bytes_per_launch": loop_bytes / launches,
                     "loop_plan": plan},
        "wtd_attn": {"bound": "mfma", "achieved": attn_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS},
    }

    if not args.no_exact:
        try:
            ems = exact_attention_ms(torch, s, Q, K, V)
            res["exact_attention"] = {"impl": "torch scaled_dot_product_attention (ROCm)", "ms": ems,
                                      "tokens_per_s": s.batch * s.n / (ems * 1e-3)}
        except Exception as e:           # context only; never fatal
            res["exact_attention"] = {"error": str(e)[:200]}

    if not args.no_exact and args.history == "f64":
        # Context: the same pass with the selection loop's history rows stored in fp32 (the library's fast mode), and
        # whether it drew the same pivots as the float64 default just timed.  Not part of `value`.
        try:
            ws32 = torch.empty(wc.workspace_bytes(s.n, s.d, s.r, s.batch, s.kv_heads, s.dv, 1 if s.dtype == "bf16" else 0,
                                                  s.bins, "f32"), dtype=torch.uint8, device=dev)

            def fast_step():
                r_q = wc.query_radius(Q, s.kv_heads, workspace=ws32)
                c32 = wc.compress_kv(K, V, s.r, r_q, uniforms=u, workspace=ws32, bins=s.bins, history="f32")
                wc.wtd_attn(Q, c32, out=out)
                return c32

            for _ in range(2):
                c32 = fast_step()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(3):
                c32 = fast_step()
            torch.cuda.synchronize()
            fms = (time.perf_counter() - t1) / 3 * 1e3
            res["fast_mode"] = {"history": "f32", "ms_per_step": fms, "tokens_per_s": s.batch * s.n / (fms * 1e-3),
                                "same_pivots_as_f64": bool(torch.equal(c32.idx, cs.idx))}
            del ws32
        except Exception as e:           # context only; never fatal
            res["fast_mode"] = {"error": str(e)[:200]}

    if not args.no_sweep:
        del Q, K, V, ws, out
        torch.cuda.empty_cache()
        # ---- the same path at other n (r fixed): near-linear means a flat us/token column ----
        sweep = []
        on_device = args.cfg == 4 and not args.sweep_n
        ns = ((4096, 8192, 16384) if args.sweep_n else ()) + (32768, 65536, 131072) \
            + ((262144,) if args.sweep_n and s.bins > 1 else ())
        for n2 in ns:
            s2 = wl.shape(args.cfg, n=n2)
            if on_device:
                Q2, K2, V2, u2 = device_workload_cfg4(s2, dev, tdt)
            else:
                w2 = wl.make(args.cfg, n=n2)
                Q2, K2, V2 = (torch.from_numpy(w2[k]).to(dev).to(tdt).contiguous() for k in ("Q", "K", "V"))
                u2 = torch.from_numpy(w2["u"]).to(dev)
                del w2
            ms2 = timed_pass(wc, torch, s2, Q2, K2, V2, u2, args.history)
            p2 = wc.loop_plan(n2, s2.d, s2.r, s2.batch, s2.kv_heads, s2.dv, 1 if es == 2 else 0, s2.bins, args.history)
            sweep.append({"n": n2, "ms": ms2, "tokens_per_s": s2.batch * n2 / (ms2 * 1e-3), "us_per_token": ms2 * 1e3 / n2,
                          "loop_driver": p2["driver"], "loop_launches": p2["launches"] * (1 if p2["driver"] else s2.r // s2.bins),
                          "keys_in_registers": bool(p2["keys_in_registers"])})
            del Q2, K2, V2, u2
            torch.cuda.empty_cache()
        res["scaling_in_n"] = {"workload": f"{s.name} recipe at other n, r={s.r} fixed"
                                           + (" (inputs drawn on the device, same distributions)" if on_device else ""),
                               "points": sweep}
        # ---- the binned regime (Sec. 2.5), the setting of the paper's FlashAttention-2 comparison ----
        try:
            w6 = wl.make(6)
            s6 = w6["shape"]
            Q6, K6, V6 = (torch.from_numpy(w6[k]).to(dev).to(torch.bfloat16).contiguous() for k in ("Q", "K", "V"))
            u6 = torch.from_numpy(w6["u"]).to(dev)
            # (fifty passes: a pass is a dozen launches of a few microseconds, and over fewer the figure is the
            # pipeline's fill and drain, not its rate)
            ms6 = timed_pass(wc, torch, s6, Q6, K6, V6, u6, args.history, reps=50)
            # streaming roof: Q, K and V each read twice (R_Q before the temperature and again in WtdAttn; the key
            # mean before the kernel columns; the value range before the Gram pass) and the output written once
            tensor_bytes = float(s6.batch) * s6.n * 2
            roof_bytes = (2 * s6.q_heads * s6.d + 2 * s6.kv_heads * s6.d + 2 * s6.kv_heads * s6.dv
                          + s6.q_heads * s6.dv) * tensor_bytes
            roof_ms = roof_bytes / (HBM_PEAK_GBS * 1e9) * 1e3
            binned = {"workload": f"{s6.name}: {s6.kv_heads} heads, n={s6.n}, d={s6.d}, r={s6.r}, B={s6.bins}, bf16",
                      "ms": ms6, "tokens_per_s": s6.batch * s6.n / (ms6 * 1e-3),
                      "streaming_roof_bytes": roof_bytes, "streaming_roof_ms": roof_ms, "frac_of_roof": roof_ms / ms6}
            if not args.no_exact:
                ems6 = exact_attention_ms(torch, s6, Q6, K6, V6)
                binned["exact_attention"] = {"impl": "torch scaled_dot_product_attention (ROCm)", "ms": ems6,
                                             "tokens_per_s": s6.batch * s6.n / (ems6 * 1e-3)}
            res["binned"] = binned
            del Q6, K6, V6, u6, w6
        except Exception as e:           # context only; never fatal
            res["binned"] = {"error": str(e)[:200]}

    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, s.kv_heads)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
