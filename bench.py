#!/usr/bin/env python3
"""Benchmark of the WildCat hot path on one MI355X.

A "step" is one pass of the whole path -- query radius, CompressKV (prologue, RPNys selection loop,
Gram pass, core solve, gather) and WtdAttn -- over one batch of synthetic attention inputs that are
already resident in HBM.  Workload: 32 query heads sharing 8 key/value heads, n = m = 32768, d = 128,
r = 512, bf16 storage (rotary-rotated Gaussian inputs), the shape the headline metric is quoted on.

Prints ONE JSON line: tokens/s of the whole path, the roofline of the dominant kernel (the RPNys step
kernel, HBM-bound, timed with HIP events on the launch stream), the WtdAttn MFMA rate, the float64 CPU
oracle timed on the host cores, and exact attention at the same shape for context.
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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-exact", action="store_true")
    ap.add_argument("--sweep-n", action="store_true",
                    help="also time the path at n = 4K ... 128K (same recipe, r fixed) and add it as 'scaling_in_n'")
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
                            history=args.history)
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
    single = wc.rpnys_single_launch(s.n, s.d, s.r, s.batch, s.kv_heads, s.dv, 1 if s.dtype == "bf16" else 0, s.bins,
                                    args.history)
    launches = 1 if single else s.r // s.bins
    # with bins the loop is P * B independent problems of n / B keys and r / B steps
    loop_bytes = step_loop_bytes(P * s.bins, s.n // s.bins, s.d, s.r // s.bins, es, single,
                                 8 if args.history == "f64" else 4)
    achieved = loop_bytes / (loop_ms * 1e-3) / 1e9
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "rpnys_loop_traffic.json")
    if os.path.exists(tfile) and args.cfg == 4 and args.history == "f64":
        with open(tfile) as f:
            traffic = json.load(f).get("single_launch" if single else "per_step", {}).get("hbm_bytes_per_launch")
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
                     "traffic": traffic, "launches": launches, "avg_launch_ms": loop_ms / launches,
                     "algorithmic_bytes_per_launch": loop_bytes / launches},
        "wtd_attn": {"bound": "mfma", "achieved": attn_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS},
    }

    if not args.no_exact:
        try:
            import torch.nn.functional as F
            Kx = K.repeat_interleave(s.group, dim=1)
            Vx = V.repeat_interleave(s.group, dim=1)
            for _ in range(2):
                F.scaled_dot_product_attention(Q, Kx, Vx)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(3):
                F.scaled_dot_product_attention(Q, Kx, Vx)
            b.record()
            torch.cuda.synchronize()
            ems = a.elapsed_time(b) / 3
            res["exact_attention"] = {"impl": "torch scaled_dot_product_attention (ROCm)", "ms": ems,
                                      "tokens_per_s": s.batch * s.n / (ems * 1e-3)}
            del Kx, Vx
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

    if args.sweep_n:
        del Q, K, V, ws, out
        torch.cuda.empty_cache()
        sweep = []
        for n2 in (4096, 8192, 16384, 32768, 65536, 131072) + ((262144,) if s.bins > 1 else ()):
            w2 = wl.make(args.cfg, n=n2)
            s2 = w2["shape"]
            Q2, K2, V2 = (torch.from_numpy(w2[k]).to(dev).to(tdt).contiguous() for k in ("Q", "K", "V"))
            u2 = torch.from_numpy(w2["u"]).to(dev)
            ws2 = torch.empty(wc.workspace_bytes(n2, s2.d, s2.r, s2.batch, s2.kv_heads, s2.d, 1 if es == 2 else 0,
                                                 s2.bins, args.history), dtype=torch.uint8, device=dev)

            def pass2():
                cs2 = wc.compress_kv(K2, V2, s2.r, wc.query_radius(Q2, s2.kv_heads, workspace=ws2), uniforms=u2, workspace=ws2,
                                     bins=s2.bins, history=args.history)
                return wc.wtd_attn(Q2, cs2)

            pass2()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(3):
                pass2()
            b.record()
            torch.cuda.synchronize()
            ms2 = a.elapsed_time(b) / 3
            sweep.append({"n": n2, "ms": ms2, "tokens_per_s": s2.batch * n2 / (ms2 * 1e-3), "us_per_token": ms2 * 1e3 / n2,
                          "single_launch_loop": wc.rpnys_single_launch(n2, s2.d, s2.r, s2.batch, s2.kv_heads, s2.d,
                                                                      1 if es == 2 else 0, s2.bins, args.history)})
            del Q2, K2, V2, ws2, w2
            torch.cuda.empty_cache()
        res["scaling_in_n"] = sweep

    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, s.kv_heads)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
