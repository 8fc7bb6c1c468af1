#!/usr/bin/env python3
"""Benchmark of the VMoBA hot path on one MI355X.

A step = one attention layer, forward and backward, through the whole path:
partition(K,V) -> select -> attn_fwd -> attn_bwd.  Only the keys and values are rearranged (Eq. 1);
Q is read where the caller has it and O, dO, dQ stay in the caller's token order, dK and dV return
to it through the partition's row map, so the step has no inverse-partition or partition(dO) call
(--permute-q: the variant that also moves Q into block order).  Steps cycle through the 1D / 2D / 3D
partitions (layer l uses kind l mod 3), so a multiple of 3 steps covers the cycle evenly.  Inputs are synthetic (blurred noise
on the 480p latent grid 21x30x52, 12 heads x 128, bf16) and resident in HBM before timing.

Prints ONE JSON line.  `value` is effective TFLOP/s of the whole step: 14 * D * (sum over
selected (query, block) pairs of the block length) per layer, divided by the wall time of the
step -- selected work only, no credit for recompute, padding or the dense work avoided.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak (published)
HBM_PEAK_GBS = 8000.0              # MI355X HBM3E peak (published)
# HBM bytes per launch of the MFMA kernels at the 480p workload (mean over the 1d/2d/3d partitions, tau = 0.25),
# from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in profiles/layer_480p_tau025_hbm_traffic_pmc.md
# (FETCH_SIZE scaled by 1.992, WRITE_SIZE by 1.000: the factors kernels of known traffic give in the same runs).
MEASURED_TRAFFIC_BYTES_480P = {"attn_fwd_tile": 1.969e9, "attn_bwd_dq_tile": 2.952e9, "attn_bwd_dkv": 3.121e9}
METRIC = "VMoBA attn fwd+bwd ms/layer + effective TFLOP/s (%MFMA peak), 480p shape"


class Hip:
    """The few HIP runtime calls the benchmark needs for raw events."""

    def __init__(self):
        self.lib = C.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.lib.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.lib.hipEventDestroy.argtypes = [C.c_void_p]

    def event(self):
        e = C.c_void_p()
        rc = self.lib.hipEventCreate(C.byref(e))
        assert rc == 0, rc
        return e.value

    def elapsed_ms(self, a, b):
        ms = C.c_float()
        rc = self.lib.hipEventElapsedTime(C.byref(ms), C.c_void_p(a), C.c_void_p(b))
        assert rc == 0, rc
        return ms.value


def selected_key_sum(plan):
    """sum over selected (query, block) pairs of L_j, over all heads (host, after a sync)."""
    blk_ptr = plan.blk_ptr.cpu().numpy().astype(np.int64)
    L = np.diff(plan.blk_off.cpu().numpy().astype(np.int64))
    cnt = np.diff(blk_ptr, axis=1)
    return int((cnt * L[None, :]).sum()), int(cnt.sum())


def cpu_baseline(Q, K, V, dO, cfg, part, tau, rows=16384):
    """The CPU oracle on head 0: selection over the whole head, masked attention forward and
    backward on every (S/rows)-th query row; time scaled to the whole head."""
    from oracle import vmoba_oracle as vo
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    T, H, W = cfg["grid"]
    bt, bh, bw, chunk = part
    D = Q.shape[-1]
    scale = 1.0 / math.sqrt(D)
    t0 = time.perf_counter()
    perm, inv, off = vo.partition_index(T, H, W, bt, bh, bw, chunk)
    Qp, Kp, Vp, dOp = (vo.gather_rows(x[:, :, :1], perm)[0, 0] for x in (Q, K, V, dO))
    sel = vo.select_blocks(Qp, Kp, off, tau, scale)
    t_sel = time.perf_counter() - t0
    S = Qp.shape[0]
    step = max(1, S // rows)
    idx = np.arange(0, S, step)
    t0 = time.perf_counter()
    vo.masked_attention_fwd(Qp[idx], Kp, Vp, sel["mask"][idx], off, scale)
    vo.masked_attention_bwd(Qp[idx], Kp, Vp, sel["mask"][idx], off, scale, dOp[idx])
    t_att = time.perf_counter() - t0
    L = np.diff(off).astype(np.int64)
    keysum_head = int((sel["mask"].sum(0).astype(np.int64) * L).sum())
    est = t_sel + t_att * (S / len(idx))
    return {"value": 14.0 * D * keysum_head / est / 1e12, "unit": "TFLOP/s (effective, fwd+bwd)",
            "cores": int(cores), "kind": "oracle",
            "sample": f"head 0 of {Q.shape[2]}, 3D partition: selection on the whole head ({t_sel:.1f} s) + float64 masked "
                      f"attention fwd+bwd on {len(idx)} of {S} query rows ({t_att:.1f} s), scaled to the head: {est:.1f} s/head",
            "seconds_per_head_est": est}


def sweep(args):
    """Sequence-length sweep in the shape of the paper's latency-vs-length figure (Fig. 1b): the 480p frame
    (30 x 52 latent tokens) with 9..72 latent frames, 12 heads x 128, the three partitions of the 480p
    workload, tau = 0.25, sparse layer fwd+bwd (all steps) next to PyTorch's dense attention fwd+bwd."""
    import numpy as np
    import torch
    from paper_2506_23858_amd import binding as vb, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    Hh, D, dtype = 12, 128, torch.bfloat16
    frames = [int(x) for x in args.sweep_frames.split(",")]
    points = []
    for T in frames:
        grid = (T, 30, 52)
        S = T * 30 * 52
        t_gen = time.perf_counter()
        ts = [torch.from_numpy(synth.to_bf16_grid(synth.blurred_noise(7000 + 10 * T + i, grid, Hh, D, 2.0))).to("cuda").to(dtype)
              for i in range(4)]
        Q, K, V, dO = ts
        print(f"[sweep] T={T} S={S}: inputs in {time.perf_counter() - t_gen:.1f} s", file=sys.stderr, flush=True)
        pt = {"frames": T, "tokens": S, "kinds": {}}
        for kind, (block, chunk) in {"1d": ((0, 0, 0), 1560), "2d": ((1, 15, 26), 0), "3d": ((3, 15, 13), 0)}.items():
            nb = S // 1560 if chunk else -(-T // block[0]) * 2 * (52 // block[2])
            if nb > 512:
                pt["kinds"][kind] = None          # more key blocks than the library's mask words hold
                continue
            p = vb.LayerPlan(1, Hh, D, grid, block, chunk, args.tau, dtype, q_in_place=True)
            p.forward(Q, K, V); p.backward(dO)
            torch.cuda.synchronize()
            assert int(p.dev_status.item()) == 0
            reps = 4
            t = time.perf_counter()
            for _ in range(reps):
                p.forward(Q, K, V); p.backward(dO)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t) * 1e3 / reps
            keysum, pairs = selected_key_sum(p)
            pt["kinds"][kind] = {"ms_per_layer": ms, "n_blocks": p.nb, "selected_pair_fraction": pairs / (Hh * S * p.nb),
                                 "effective_tflops": 14.0 * D * keysum / (ms * 1e-3) / 1e12}
            del p
            torch.cuda.empty_cache()
        done = [v["ms_per_layer"] for v in pt["kinds"].values() if v]
        pt["sparse_ms_mean_over_kinds"] = sum(done) / len(done)
        q, k, v = (x.permute(0, 2, 1, 3).detach().clone().requires_grad_(True) for x in (Q, K, V))
        g = dO.permute(0, 2, 1, 3).contiguous()
        def sdpa():
            torch.nn.functional.scaled_dot_product_attention(q, k, v).backward(g)
            q.grad = k.grad = v.grad = None
        sdpa()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(2):
            sdpa()
        torch.cuda.synchronize()
        pt["torch_sdpa_fwd_bwd_ms"] = (time.perf_counter() - t) * 1e3 / 2
        pt["speedup_vs_torch_sdpa"] = pt["torch_sdpa_fwd_bwd_ms"] / pt["sparse_ms_mean_over_kinds"]
        points.append(pt)
        print(f"[sweep] {json.dumps(pt)}", file=sys.stderr, flush=True)
        del q, k, v, g, Q, K, V, dO, ts
        torch.cuda.empty_cache()
    lt = np.log([p["tokens"] for p in points])
    fit = {"dense_exponent": float(np.polyfit(lt, np.log([p["torch_sdpa_fwd_bwd_ms"] for p in points]), 1)[0]),
           "sparse_exponent": float(np.polyfit(lt, np.log([p["sparse_ms_mean_over_kinds"] for p in points]), 1)[0])}
    print(json.dumps({"metric": "sequence-length sweep: VMoBA layer fwd+bwd ms vs dense (torch SDPA) ms", "tau": args.tau,
                      "heads": Hh, "D": D, "dtype": "bf16", "data": "synthetic", "points": points,
                      "log_log_slope": fit}))


def tau_sweep(args):
    """Threshold sweep of one configuration (the long-sequence stress shape asks for tau = 0.1 .. 0.75): inputs are
    generated once; per tau and partition kind a whole layer fwd+bwd is timed, with the selected-pair fraction,
    the token sparsity and the effective TFLOP/s on the selected blocks."""
    import torch
    from paper_2506_23858_amd import binding as vb, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    Hh, D = cfg["heads"], cfg["D"]
    dtype = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    t_gen = time.perf_counter()
    Q, K, V, dO = (torch.from_numpy(x).to("cuda").to(dtype).contiguous() for x in synth.make_qkv(args.config))
    t_gen = time.perf_counter() - t_gen
    print(f"[tau-sweep] {args.config}: inputs in {t_gen:.1f} s", file=sys.stderr, flush=True)
    S = Q.shape[1]
    kinds = [k for k in args.kinds.split(",") if k in cfg["partitions"]]
    points = []
    for tau in [float(x) for x in args.tau_sweep.split(",")]:
        for kind in kinds:
            bt, bh, bw, chunk = cfg["partitions"][kind]
            p = vb.LayerPlan(1, Hh, D, cfg["grid"], (bt, bh, bw), chunk, tau, dtype, q_in_place=True)
            p.forward(Q, K, V); p.backward(dO)
            torch.cuda.synchronize()
            assert int(p.dev_status.item()) == 0
            reps, times = 3, []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                p.forward(Q, K, V); p.backward(dO)
                b.record()
                torch.cuda.synchronize()
                times.append(a.elapsed_time(b))
            keysum, pairs = selected_key_sum(p)
            ms = float(np.median(times))
            pt = {"tau": tau, "kind": kind, "n_blocks": p.nb, "ms_per_layer_median": ms, "ms_per_layer_min": float(min(times)),
                  "selected_pair_fraction": pairs / (Hh * S * p.nb), "token_sparsity": keysum / (Hh * S * S),
                  "empty_row_fraction": float((p.row_ptr[:, 1:] == p.row_ptr[:, :-1]).float().mean().item()),
                  "effective_tflops": 14.0 * D * keysum / (ms * 1e-3) / 1e12,
                  "frac_of_bf16_mfma_peak": 14.0 * D * keysum / (ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
            points.append(pt)
            print(f"[tau-sweep] {json.dumps(pt)}", file=sys.stderr, flush=True)
            del p
            torch.cuda.empty_cache()
    print(json.dumps({"metric": "threshold sweep: VMoBA layer fwd+bwd, whole path", "config": args.config,
                      "workload": f"grid {cfg['grid']}, {Hh} heads x {D}", "tokens": S, "dtype": "bf16", "data": "synthetic",
                      "input_generation_s": round(t_gen, 1), "points": points}))


def probe_atomics(args):
    """Why dQ is not formed inside the dK/dV kernel with atomics: the atomic traffic of that design alone (no matrix
    work), per partition of the 480p workload at the measured list densities, against the dQ path it would replace."""
    import torch
    from paper_2506_23858_amd import binding as vb

    torch.cuda.set_device(0)
    S, heads = 32760, 12
    dq = torch.zeros(heads, S, 128, dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(7)
    points = []
    for name, nb, L, frac in (("3d", 56, 585, 0.144), ("2d", 84, 390, 0.167), ("1d", 21, 1560, 0.209)):
        cnt = int(frac * S)
        lists = torch.from_numpy(np.stack([np.sort(rng.choice(S, cnt, replace=False)) for _ in range(64)]).astype(np.int32)).cuda()
        runs = nb * (-(-L // 128))
        best = 1e9
        for _ in range(4):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            vb.vmoba_probe_atomic_rows(dq, lists, cnt, S, runs, heads)
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b))
        nbytes = runs * heads * cnt * 512.0
        points.append({"partition": name, "runs": runs, "heads": heads, "list_rows": cnt, "atomic_GB": nbytes / 1e9,
                       "ms": best, "TBps": nbytes / best / 1e9})
    print(json.dumps({"metric": "float32 atomic row adds of a dQ-inside-dK/dV design, 480p tau=0.25 list densities",
                      "points": points}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="480p")
    ap.add_argument("--tau", type=float, default=0.25)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense comparators")
    ap.add_argument("--kinds", default="1d,2d,3d")
    ap.add_argument("--no-extras", action="store_true", help="skip the copy-rate probe and the tau = 0.5 run (profiling runs)")
    ap.add_argument("--input-sets", type=int, default=3, help="copies of the inputs the steps rotate over")
    ap.add_argument("--kv-in-place", action="store_true",
                    help="rearrange nothing: K and V are read where the caller has them through the partition's row map")
    ap.add_argument("--permute-q", action="store_true",
                    help="also rearrange Q into block order (default: only K and V move, as in the paper's Eq. 1)")
    ap.add_argument("--sweep", action="store_true", help="sequence-length sweep instead of the benchmark line")
    ap.add_argument("--sweep-frames", default="9,15,21,36,48,72")
    ap.add_argument("--tau-sweep", default="", help="comma-separated thresholds: time a whole layer per tau and kind instead")
    ap.add_argument("--probe-atomics", action="store_true", help="time the atomic traffic of a dQ-inside-dK/dV design instead")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; --gpus must be 1 (the path shards by head, see DESIGN.md)",
              file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        return sweep(args)
    if args.probe_atomics:
        return probe_atomics(args)
    if args.tau_sweep:
        return tau_sweep(args)

    import torch
    from paper_2506_23858_amd import binding as vb, synth

    if not os.path.exists(vb.LIB_PATH):
        raise SystemExit("libvmoba.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda"
    torch.cuda.set_device(0)
    hip = Hip()
    cfg = synth.CONFIGS[args.config]
    Hh, D = cfg["heads"], cfg["D"]
    dtype = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    t_gen = time.perf_counter()
    Qn, Kn, Vn, dOn = synth.make_qkv(args.config)
    t_gen = time.perf_counter() - t_gen
    Q, K, V, dO = (torch.from_numpy(x).to(dev).to(dtype).contiguous() for x in (Qn, Kn, Vn, dOn))
    S = Q.shape[1]
    # Rotating input sets: the same values at N_SETS different addresses, one set per step in turn, so that no step
    # finds its inputs in the 256 MB last-level cache from the step before (4 tensors of ~100 MB per set at 480p;
    # identical values keep the selection, and with it the counted work, the same for every step).
    N_SETS = max(1, args.input_sets)
    sets = [(Q, K, V, dO)] + [tuple(t.clone() for t in (Q, K, V, dO)) for _ in range(N_SETS - 1)]
    kinds = [k for k in args.kinds.split(",") if k in cfg["partitions"]]
    plans = {}
    for kind in kinds:
        bt, bh, bw, chunk = cfg["partitions"][kind]
        plans[kind] = vb.LayerPlan(1, Hh, D, cfg["grid"], (bt, bh, bw), chunk, args.tau, dtype, fused_io=True,
                                   q_in_place=not args.permute_q, kv_in_place=args.kv_in_place)

    def step(i):
        p = plans[kinds[i % len(kinds)]]
        q, k, v, g = sets[i % N_SETS]
        p.forward(q, k, v)
        p.backward(g)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    for p in plans.values():
        assert int(p.dev_status.item()) == 0

    # ---- timed region: exactly `steps` steps, kernel events on the launch stream
    SLOTS = {0: "attn_fwd_tile", 1: "attn_bwd_dq_tile", 2: "attn_bwd_dkv"}
    ev = {s: [(hip.event(), hip.event()) for _ in range(args.steps)] for s in SLOTS}
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # step boundaries, same stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_ev[0].record()
    for i in range(args.steps):
        for s in SLOTS:
            vb.vmoba_profile_events(s, *ev[s][i])
        step(i)
        step_ev[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for s in SLOTS:
        vb.vmoba_profile_events(s, None, None)
    total_s = t1 - t0
    ms_per_step = total_s * 1e3 / args.steps
    step_ms = [step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(args.steps)]

    # ---- work accounting (selected blocks only)
    keysum, pairs = {}, {}
    for kind, p in plans.items():
        keysum[kind], pairs[kind] = selected_key_sum(p)
    step_kinds = [kinds[i % len(kinds)] for i in range(args.steps)]
    flops_total = sum(14.0 * D * keysum[k] for k in step_kinds)
    value = flops_total / total_s / 1e12

    # ---- dominant kernel and its roofline
    kflops = {0: 4.0, 1: 2.0, 2: 8.0}     # algorithmic FLOP per (pair, key, channel): fwd 2 GEMMs; dQ 1; S,dP,dV,dK 4
    ktime = {s: [hip.elapsed_ms(a, b) for a, b in ev[s]] for s in SLOTS}
    dom = max(SLOTS, key=lambda s: sum(ktime[s]))
    dom_flops = sum(kflops[dom] * D * keysum[k] for k in step_kinds)
    dom_ms = sum(ktime[dom])
    achieved = dom_flops / (dom_ms * 1e-3) / 1e12
    traffic = None
    if args.config == "480p" and abs(args.tau - 0.25) < 1e-9 and kinds == ["1d", "2d", "3d"]:
        traffic = MEASURED_TRAFFIC_BYTES_480P.get(SLOTS[dom])
    def by_kind(vals):      # median and minimum of a per-step series, per partition kind (the kinds differ in work)
        return {k: {"median_ms": float(np.median([v for v, sk in zip(vals, step_kinds) if sk == k])),
                    "min_ms": float(min(v for v, sk in zip(vals, step_kinds) if sk == k))} for k in kinds if k in step_kinds}

    roofline = {"bound": "mfma", "kernel": SLOTS[dom], "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / BF16_MFMA_PEAK_TFLOPS, "traffic": traffic,
                "avg_launch_ms": dom_ms / args.steps,
                "all_kernels": {SLOTS[s]: {"avg_launch_ms": sum(ktime[s]) / args.steps,
                                           "tflops": sum(kflops[s] * D * keysum[k] for k in step_kinds) / (sum(ktime[s]) * 1e-3) / 1e12,
                                           "per_kind": by_kind(ktime[s])}
                                for s in SLOTS}}
    # ---- what the matrix cores of this GPU sustain with nothing but matrix instructions in flight (measured here,
    # at the clock the chip holds under that load), next to the published peak the fractions above are taken against
    try:
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        wgs = 2 * torch.cuda.get_device_properties(0).multi_processor_count        # two wavefronts per SIMD
        best = 0.0
        for _ in range(4):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            flop = vb.vmoba_probe_mfma(20000, wgs, sink)
            b.record()
            torch.cuda.synchronize()
            best = max(best, flop / (a.elapsed_time(b) * 1e-3) / 1e12)
        roofline["measured_mfma_ceiling_tflops"] = best
        roofline["measured_mfma_ceiling_note"] = ("independent v_mfma_f32_32x32x16_bf16 only, two wavefronts per SIMD, best of 4 launches "
                                                  "(vmoba_probe_mfma); `peak` is the published figure, this is the measured one")
        roofline["frac_of_measured_ceiling"] = achieved / best
    except Exception as e:
        roofline["measured_mfma_ceiling_error"] = repr(e)[:120]

    # ---- per-call breakdown (outside the timed region), per kind
    BREAKDOWN_REPS = 7

    def timed_calls(p):
        # the attention calls read dO and write O, dQ, dK, dV in the caller's token order (row map = perm);
        # BREAKDOWN_REPS passes over the rotating input sets, median and minimum per call
        names = ["partition", "select", "attn_fwd", "attn_bwd"]
        series = {n: [] for n in names}
        for rep in range(BREAKDOWN_REPS):
            q, k, v, g = sets[rep % N_SETS]
            fns = [lambda: p.partition(q, k, v), p.select, p.attn_fwd, lambda: p.attn_bwd(g)]
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(fns) + 1)]
            evs[0].record()
            for f, e in zip(fns, evs[1:]):
                f()
                e.record()
            torch.cuda.synchronize()
            for i, n in enumerate(names):
                series[n].append(evs[i].elapsed_time(evs[i + 1]))
        return ({n: float(np.median(v)) for n, v in series.items()}, {n: float(min(v)) for n, v in series.items()})

    timed = {kind: timed_calls(p) for kind, p in plans.items()}
    breakdown = {kind: t[0] for kind, t in timed.items()}
    breakdown_min = {kind: t[1] for kind, t in timed.items()}
    # memory-bound steps: algorithmic bytes / time of the call
    es = 2 if dtype == torch.bfloat16 else 4
    row_bytes = S * Hh * D * es
    mem_steps = {}
    n_part = 0 if args.kv_in_place else 3 if args.permute_q else 2          # tensors the partition call moves: (Q,) K, V
    for kind, bd in breakdown.items():
        nbk = plans[kind].nb
        sel_bytes = 2 * row_bytes + Hh * S * nbk * 4 + Hh * S * ((nbk + 31) // 32) * 4 + 3 * 4 * pairs[kind]
        mem_steps[kind] = {
            "partition_GBps": n_part * 2 * row_bytes / (bd["partition"] * 1e-3) / 1e9,
            "partition_GBps_best": n_part * 2 * row_bytes / (breakdown_min[kind]["partition"] * 1e-3) / 1e9,
            "partition_tensors": n_part,
            "select_GBps": sel_bytes / (bd["select"] * 1e-3) / 1e9,
            "select_GBps_best": sel_bytes / (breakdown_min[kind]["select"] * 1e-3) / 1e9,
            "select_algorithmic_bytes": sel_bytes}
    empty_rows = {kind: float((p.row_ptr[:, 1:] == p.row_ptr[:, :-1]).float().mean().item()) for kind, p in plans.items()}
    per_kind = {kind: {"ms_per_layer": sum(b.values()),
                       "selected_pair_fraction": pairs[kind] / (Hh * S * plans[kind].nb),
                       "empty_row_fraction": empty_rows[kind],
                       "token_sparsity": keysum[kind] / (Hh * S * S),
                       "n_blocks": plans[kind].nb,
                       "attn_fwd_bwd_tflops": 14.0 * D * keysum[kind] / ((b["attn_fwd"] + b["attn_bwd"]) * 1e-3) / 1e12}
                for kind, b in breakdown.items()}

    out = {"metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16" if dtype == torch.bfloat16 else "f32", "data": "synthetic",
           "config": {"workload": f"{args.config}: grid {cfg['grid']}, {Hh} heads x {D}, tau={args.tau}, "
                                  f"layer cycle {'/'.join(kinds)}, fwd+bwd per layer", "tokens": S,
                      "input_generation_s": round(t_gen, 1)},
           "frac_of_bf16_mfma_peak": value / BF16_MFMA_PEAK_TFLOPS,
           "ms_per_step_median": float(np.median(step_ms)), "ms_per_step_min": float(min(step_ms)),
           "ms_per_step_by_kind": by_kind(step_ms), "input_sets_rotated": N_SETS,
           "roofline": roofline, "per_kind": per_kind, "breakdown_ms": breakdown, "breakdown_min_ms": breakdown_min,
           "breakdown_note": f"per call: median and minimum of {BREAKDOWN_REPS} passes over the rotating input sets",
           "memory_bound_steps": dict(mem_steps, hbm_peak_GBps=HBM_PEAK_GBS,
                                      note="algorithmic bytes (permute: read+write of every row; select: K and Q read once, "
                                           "P, mask and the three lists written once) over the call's median time; "
                                           "*_best over its minimum; inputs rotate over the sets")}

    # ---- measured copy ceiling (plain device-to-device copy of 1 GiB, read + write counted)
    try:
        if args.no_extras:
            raise RuntimeError("skipped (--no-extras)")
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["memory_bound_steps"]["measured_copy_GBps"] = 2 * 5 * (1 << 30) / (time.perf_counter() - t) / 1e9
        del src, dst
    except Exception as e:
        out["memory_bound_steps"]["measured_copy_error"] = repr(e)[:100]

    # ---- the second threshold of the workload (tau = 0.5), 3D partition, a few steps
    if abs(args.tau - 0.5) > 1e-9 and "3d" in cfg["partitions"] and not args.no_extras:
        try:
            bt, bh, bw, chunk = cfg["partitions"]["3d"]
            p5 = vb.LayerPlan(1, Hh, D, cfg["grid"], (bt, bh, bw), chunk, 0.5, dtype, q_in_place=not args.permute_q, kv_in_place=args.kv_in_place)
            p5.forward(Q, K, V); p5.backward(dO)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(3):
                p5.forward(Q, K, V); p5.backward(dO)
            torch.cuda.synchronize()
            ms5 = (time.perf_counter() - t) * 1e3 / 3
            ks5, pr5 = selected_key_sum(p5)
            out["tau_0.5_3d"] = {"ms_per_layer": ms5, "effective_tflops": 14.0 * D * ks5 / (ms5 * 1e-3) / 1e12,
                                 "selected_pair_fraction": pr5 / (Hh * S * p5.nb)}
            del p5
            torch.cuda.empty_cache()
        except Exception as e:
            out["tau_0.5_3d"] = {"error": repr(e)[:200]}

    # ---- dense comparators on the same GPU
    if not args.no_dense:
        dense = {}
        try:
            q, k, v = (x.permute(0, 2, 1, 3).detach().clone().requires_grad_(True) for x in (Q, K, V))
            g = dO.permute(0, 2, 1, 3).contiguous()
            def sdpa():
                o = torch.nn.functional.scaled_dot_product_attention(q, k, v)
                o.backward(g)
                q.grad = k.grad = v.grad = None
            sdpa()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(3):
                sdpa()
            torch.cuda.synchronize()
            dense["torch_sdpa_fwd_bwd_ms"] = (time.perf_counter() - t) * 1e3 / 3
            del q, k, v, g
        except Exception as e:   # comparator only; never part of the product path
            dense["torch_sdpa_error"] = repr(e)[:200]
        try:
            kind0 = "1d" if "1d" in plans else kinds[0]
            bt, bh, bw, chunk = cfg["partitions"][kind0]
            for p in plans.values():
                p.ws_attn = None
            torch.cuda.empty_cache()
            pd = vb.LayerPlan(1, Hh, D, cfg["grid"], (bt, bh, bw), chunk, 1.0, dtype, q_in_place=not args.permute_q, kv_in_place=args.kv_in_place)
            pd.forward(Q, K, V); pd.backward(dO)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(2):
                pd.forward(Q, K, V); pd.backward(dO)
            torch.cuda.synchronize()
            dense["this_library_tau1_fwd_bwd_ms"] = (time.perf_counter() - t) * 1e3 / 2
            dense["this_library_tau1_tflops"] = 14.0 * D * Hh * S * S / (dense["this_library_tau1_fwd_bwd_ms"] * 1e-3) / 1e12
            del pd
        except Exception as e:
            dense["tau1_error"] = repr(e)[:200]
        if "torch_sdpa_fwd_bwd_ms" in dense:
            dense["speedup_vs_torch_sdpa"] = dense["torch_sdpa_fwd_bwd_ms"] / ms_per_step
        out["dense"] = dense

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(Qn, Kn, Vn, dOn, cfg, cfg["partitions"]["3d"], args.tau)
    else:
        out["cpu_baseline"] = None
    out["paper_context"] = ("paper reports whole-model numbers on NVIDIA H800 only: 2.92x FLOPs / 1.48x latency (training, "
                            "55-56K tokens), 2.40x / 1.35x (720p inference); at this 33K-token shape its sparse path "
                            "breaks even with dense (1.01x)")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
