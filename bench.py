#!/usr/bin/env python3
"""Benchmark of the SparseD hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: full attention (emitting the row log-sum-exp), pattern selection (pooled scores +
per-row top-k), and block-sparse attention with the selected pattern. The default workload is the
64k long-context configuration the headline metric is quoted on. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload long64k] [--no-schedule] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_F32_TFLOPS = 157.3     # fp32 matrix peak
PEAK_HBM_GBS = 8000.0


def _flops(cfg, keep):
    dense = 4.0 * cfg.B * cfg.Hq * cfg.L * cfg.L * cfg.d
    sparse = 4.0 * cfg.B * cfg.Hq * cfg.nqb * keep * cfg.bq * cfg.bk * cfg.d
    select = 2.0 * cfg.B * cfg.Hq * cfg.L * cfg.L * cfg.d      # one algorithmic QK^T (statistics come from the dense call)
    return dense, select, sparse


def _kernel_source_digest():
    """sha256 (first 16 hex digits) over the sources of the attention kernels: what a counter run was measured on."""
    import hashlib
    h = hashlib.sha256()
    for f in ("attn_bf16.hip", "tile_bf16.hpp", "kernels.hpp"):
        with open(os.path.join(ROOT, "paper_2509_24014_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def _traffic_from_profiles(workload_name):
    """HBM bytes per launch of the sparse kernel from the committed counter summary (FETCH_SIZE / WRITE_SIZE runs
    cannot be taken inside this process), with the digest of the kernel sources it was measured on: a figure taken
    on other sources than the ones running now is reported as stale, not as this run's traffic."""
    path = os.path.join(ROOT, "profiles", f"attn_sparse_{workload_name}_hbm_traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f)
    except Exception:
        return None, None
    now = _kernel_source_digest()
    info = {"file": os.path.relpath(path, ROOT), "measured_on_sources": rec.get("kernel_source_digest"),
            "sources_now": now, "stale": rec.get("kernel_source_digest") != now}
    return (None if info["stale"] else rec.get("traffic_bytes_per_launch")), info


def cpu_baseline(cfg, q, k, v, index, keep, budget_s=15.0):
    """The fp64 oracle, as it stands, timed on this machine's host cores on a bounded sample of the same workload."""
    import numpy as np

    import oracle

    rng = np.random.default_rng(0)
    group = cfg.Hq // cfg.Hkv
    t_sparse = t_dense = 0.0
    n_sparse = n_dense = 0
    t0 = time.perf_counter()
    heads = [int(h) for h in rng.permutation(cfg.Hq)]
    for h in heads:
        if time.perf_counter() - t0 > budget_s:
            break
        qh = q[:, h:h + 1].float().cpu()
        kh = k[:, h // group:h // group + 1].float().cpu()
        vh = v[:, h // group:h // group + 1].float().cpu()
        rp = index.row_ptr[:, h:h + 1].cpu().numpy()
        ci = index.col_idx[:, h:h + 1].cpu().numpy()
        for I in [int(x) for x in rng.permutation(cfg.nqb)[:16]]:
            if time.perf_counter() - t0 > budget_s:
                break
            a = time.perf_counter()
            oracle.attn_sparse_rows(qh, kh, vh, rp, ci, cfg.bq, cfg.bk, 0, 0, I, I + 1)
            t_sparse += time.perf_counter() - a
            n_sparse += 1
        for I in [int(x) for x in rng.permutation(cfg.nqb)[:2]]:
            if time.perf_counter() - t0 > budget_s:
                break
            a = time.perf_counter()
            oracle.attn_dense_rows(qh, kh, vh, 0, 0, I * cfg.bq, (I + 1) * cfg.bq)
            t_dense += time.perf_counter() - a
            n_dense += 1
    unit_sparse = 4.0 * keep * cfg.bq * cfg.bk * cfg.d
    unit_dense = 4.0 * cfg.bq * cfg.L * cfg.d
    out = {
        "value": (n_sparse * unit_sparse / t_sparse / 1e12) if t_sparse > 0 else None,
        "unit": "TFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"{n_sparse} (head, query-block) units of sparse attention and {n_dense} of dense attention "
                  f"from the same {cfg.name} tensors, fp64, {t_sparse + t_dense:.1f} s of CPU work",
        "dense_tflops": (n_dense * unit_dense / t_dense / 1e12) if t_dense > 0 else None,
        "sparse_ms_full_tensor_extrapolated": (t_sparse / n_sparse * cfg.B * cfg.Hq * cfg.nqb * 1e3) if n_sparse else None,
        "dense_ms_full_tensor_extrapolated": (t_dense / n_dense * cfg.B * cfg.Hq * cfg.nqb * 1e3) if n_dense else None,
    }
    return out


def _sclk_while(fn, seconds=2.5):
    """Shader clock in MHz as `rocm-smi --showclocks` reports it while fn() runs back to back; None if unreadable.

    The published matrix peak assumes 2400 MHz; under its power limit the chip runs these kernels slower.
    """
    import re
    import shutil
    import subprocess
    import threading
    import torch
    smi = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
    stop = threading.Event()
    dev = torch.cuda.current_device()

    def work():
        torch.cuda.set_device(dev)
        while not stop.is_set():
            fn()
            torch.cuda.synchronize()

    th = threading.Thread(target=work, daemon=True)
    th.start()
    vals = []
    try:
        time.sleep(0.7)
        t0 = time.time()
        while time.time() - t0 < seconds:
            out = subprocess.run([smi, "--showclocks"], capture_output=True, text=True, timeout=15).stdout
            m = re.search(r"sclk clock level:[^(]*\((\d+)Mhz\)", out)
            if not m:
                break
            vals.append(int(m.group(1)))
    except Exception:
        pass
    finally:
        stop.set()
        th.join()
    return round(sum(vals) / len(vals)) if vals else None


def _select_bytes(cfg, keep):
    """Algorithmic bytes of one selection call that reuses the dense call's statistics."""
    esz = 2 if cfg.dtype == "bf16" else 4
    qk = (cfg.B * cfg.Hq + cfg.B * cfg.Hkv) * cfg.L * cfg.d * esz
    lse = cfg.B * cfg.Hq * cfg.L * 4
    index = cfg.B * cfg.Hq * (cfg.nqb * keep + cfg.nqb + 1) * 4
    return qk + lse + index


def per_workload_block(sd, workload, torch, names, seed, peak):
    """Per-call times of the other named workloads (not the headline step; each timed with HIP events on the launch
    stream after a warm-up call), and the whole T-step schedule where the workload has one."""
    dev = torch.device("cuda:0")

    def timed(fn, reps):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    block = {}
    for name in names:
        cfg = workload.get_config(name)
        keep = sd.kept_blocks(cfg.rho, cfg.nkb)
        inp = workload.make_inputs(cfg, seed=seed, device=dev)
        q, k, v = inp.rounded()
        out = torch.empty_like(q)
        lse = torch.empty(cfg.B, cfg.Hq, cfg.L, dtype=torch.float32, device=dev)
        ws = torch.empty(sd.select_workspace_bytes(q, cfg.bq, cfg.bk), dtype=torch.uint8, device=dev)
        index = sd.BlockIndex(torch.empty(cfg.B, cfg.Hq, cfg.nqb + 1, dtype=torch.int32, device=dev),
                              torch.empty(cfg.B, cfg.Hq, cfg.nqb * keep, dtype=torch.int32, device=dev), cfg.bq, cfg.bk, cfg.nkb)
        reps = 20 if cfg.L <= 16384 else 5
        dense_ms = timed(lambda: sd.attn_dense(q, k, v, out=out), reps)
        sd.attn_dense(q, k, v, out=out, lse_out=lse)
        select_ms = timed(lambda: sd.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho, lse_in=lse, workspace=ws, index=index), reps)
        select_own_ms = timed(lambda: sd.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho, workspace=ws, index=index), reps)
        sparse_ms = timed(lambda: sd.attn_sparse(q, k, v, index, out=out), 4 * reps)
        f_dense, f_select, f_sparse = _flops(cfg, keep)
        rec = {"config": {"B": cfg.B, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "L": cfg.L, "d": cfg.d, "block_q": cfg.bq, "block_k": cfg.bk,
                          "rho": cfg.rho, "kept_blocks": keep},
               "ms_per_call": {"dense": dense_ms, "select": select_ms, "select_with_own_statistics": select_own_ms, "sparse": sparse_ms},
               "frac_of_peak": {"dense": f_dense / (dense_ms * 1e-3) / 1e12 / peak,
                                "select_one_qkT": f_select / (select_ms * 1e-3) / 1e12 / peak,
                                "sparse_executed": f_sparse / (sparse_ms * 1e-3) / 1e12 / peak}}
        if cfg.T > 1:
            def run_schedule(**kw):
                src = workload.make_inputs(cfg, seed=seed, device=dev)
                layer = sd.SparseDLayer(cfg.T, 0.0, cfg.bq, cfg.bk, cfg.rho, **kw)
                evs = []
                for t in range(cfg.T):
                    qq, kk, vv = src.rounded()
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    layer.step(qq, kk, vv, t, out=out)
                    b.record()
                    evs.append((a, b))
                    src.advance()
                torch.cuda.synchronize()
                return sum(a.elapsed_time(b) for a, b in evs), layer

            total, layer = run_schedule(n_dense=cfg.n_dense)
            rec["schedule"] = {"T": cfg.T, "n_dense": cfg.n_dense, "total_attention_ms": total, "dense_only_ms": cfg.T * dense_ms,
                               "speedup_measured": cfg.T * dense_ms / total,
                               "expected_if_sparse_as_efficient_as_dense":
                                   cfg.T / (cfg.n_dense + (cfg.T - cfg.n_dense) * keep / cfg.nkb + select_ms / dense_ms),
                               "calls": layer.calls}
            # the paper's ablation rows (Table 2) on the same kernels: sparse from the first step, and a fresh
            # selection at every sparse step (no handed-over statistics: the one-pass selection)
            for mode, kw in (("no_skipping", {"n_dense": 0}),
                             ("no_sparse_reusing", {"n_dense": cfg.n_dense, "reselect_every_step": True})):
                ms, lay = run_schedule(**kw)
                rec["schedule"][mode] = {"total_attention_ms": ms, "calls": lay.calls}
        block[name] = rec
        del inp, q, k, v, out, lse, ws, index
        print(f"[bench] workload {name} done", file=sys.stderr, flush=True)
    return block


def index_ablation(sd, torch, cfg, q, k, v, index, keep):
    """The sparse kernel on the same tensors with other block indices of the same row length: separates what the
    selected pattern's memory locality costs (against an index whose every K/V copy hits L2) from what a query
    block costs beyond its tiles (rows of other lengths with the all-L2 index)."""
    dev = q.device
    out = torch.empty_like(q)
    H, nqb, nkb = cfg.Hq, cfg.nqb, cfg.nkb

    def timed(ix, rows_keep):
        # the host builds each index while the GPU idles and its clock falls back: warm up for a few tens of
        # milliseconds before timing, or the first rows of the table come out slow
        reps = max(5, min(40, int(40 * keep / max(rows_keep, 1))))
        for _ in range(reps):
            sd.attn_sparse(q, k, v, ix, out=out)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            sd.attn_sparse(q, k, v, ix, out=out)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        fl = 4.0 * cfg.B * H * nqb * rows_keep * cfg.bq * cfg.bk * cfg.d
        return {"ms": ms, "tflops_executed": fl / (ms * 1e-3) / 1e12}

    def regular(cols_of_row, kp):  # the same rows for every head
        rp = (torch.arange(nqb + 1, dtype=torch.int32) * kp).repeat(cfg.B, H, 1).to(dev)
        ci = cols_of_row.to(torch.int32).reshape(1, 1, nqb * kp).repeat(cfg.B, H, 1).contiguous().to(dev)
        return sd.BlockIndex(rp, ci, cfg.bq, cfg.bk, nkb)

    res = {"selected_pattern": timed(index, keep)}
    first = torch.arange(keep).repeat(nqb, 1)
    res["same_blocks_for_every_row_all_L2_hits"] = timed(regular(first, keep), keep)
    g = torch.Generator().manual_seed(1)
    rnd = torch.stack([torch.sort(torch.randperm(nkb, generator=g)[:keep])[0] for _ in range(nqb)])
    res["uniform_random_blocks"] = timed(regular(rnd, keep), keep)
    centre = (torch.arange(nqb) * cfg.bq // cfg.bk - keep // 2).clamp(min=0, max=nkb - keep)
    res["diagonal_window"] = timed(regular(centre[:, None] + torch.arange(keep)[None, :], keep), keep)
    res["row_length_sweep_all_L2_hits"] = {}
    for kp in (keep // 4, keep // 2, keep, 2 * keep, 4 * keep):
        if 1 <= kp <= nkb:
            res["row_length_sweep_all_L2_hits"][str(kp)] = timed(regular(torch.arange(kp).repeat(nqb, 1), kp), kp)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="long64k")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-schedule", action="store_true", help="skip the full T-step schedule run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-clock", action="store_true", help="do not sample the shader clock under load")
    ap.add_argument("--no-per-workload", action="store_true",
                    help="skip the per-call times of the other named workloads (4k, 16k, 32k-GQA) appended to the headline line")
    ap.add_argument("--index-ablation", action="store_true",
                    help="also time the sparse kernel on other block indices of the same row length (all-L2, random, window)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy, the known-size reference for FETCH_SIZE / WRITE_SIZE runs")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards by head with no exchange; "
              "no multi-GPU figure is produced). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2509_24014_amd as sd
    import workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    sd.load_library(build_if_missing=True)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = workload.get_config(args.workload)
    keep = sd.kept_blocks(cfg.rho, cfg.nkb)
    inp = workload.make_inputs(cfg, seed=args.seed, device=dev)
    q, k, v = inp.rounded()
    out = torch.empty_like(q)
    lse = torch.empty(cfg.B, cfg.Hq, cfg.L, dtype=torch.float32, device=dev)
    ws = torch.empty(sd.select_workspace_bytes(q, cfg.bq, cfg.bk), dtype=torch.uint8, device=dev)
    index = sd.BlockIndex(torch.empty(cfg.B, cfg.Hq, cfg.nqb + 1, dtype=torch.int32, device=dev),
                          torch.empty(cfg.B, cfg.Hq, cfg.nqb * keep, dtype=torch.int32, device=dev), cfg.bq, cfg.bk, cfg.nkb)

    def one_step(ev=None):
        # the switch step of Algorithm 1: full attention (also emitting the row log-sum-exp that the
        # selection reuses), pattern selection, then one sparse-attention call with the new pattern
        if ev:
            ev[0].record()
        sd.attn_dense(q, k, v, out=out, lse_out=lse)
        if ev:
            ev[1].record()
        sd.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho, lse_in=lse, workspace=ws, index=index)
        if ev:
            ev[2].record()
        sd.attn_sparse(q, k, v, index, out=out)
        if ev:
            ev[3].record()

    def time_call(fn, reps):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)  # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(events[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    dense_lse_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    select_ms = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps
    sparse_ms = sum(e[2].elapsed_time(e[3]) for e in events) / args.steps
    ms_per_step = wall_ms / args.steps
    # the dense call of an ordinary (non-switch) step does not emit the log-sum-exp
    dense_ms = time_call(lambda: sd.attn_dense(q, k, v, out=out), max(1, min(args.steps, 5)))
    # selection when the caller has no log-sum-exp to hand over (own statistics pass included)
    select_alone_ms = time_call(lambda: sd.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho, workspace=ws, index=index), 1)

    f_dense, f_select, f_sparse = _flops(cfg, keep)
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    tf = lambda fl, ms: fl / (ms * 1e-3) / 1e12  # noqa: E731
    sparse_tf, dense_tf, select_tf = tf(f_sparse, sparse_ms), tf(f_dense, dense_ms), tf(f_select, select_ms)

    T, n_dense = cfg.T, cfg.n_dense
    sched = None
    if T > 1:
        derived = (T * dense_ms) / (n_dense * dense_ms + select_ms + (T - n_dense) * sparse_ms)
        expected = T / (n_dense + (T - n_dense) * keep / cfg.nkb + select_ms / dense_ms)
        sched = {"T": T, "n_dense": n_dense, "speedup_from_call_times": derived, "expected_if_sparse_as_efficient_as_dense": expected}
        if not args.no_schedule:
            # the real thing: all T calls of Algorithm 1 with drifting inputs; only the attention calls are timed
            layer = sd.SparseDLayer(T, 0.0, cfg.bq, cfg.bk, cfg.rho, n_dense=n_dense)
            inp2 = workload.make_inputs(cfg, seed=args.seed, device=dev)
            evs = []
            for t in range(T):
                qq, kk, vv = inp2.rounded()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                layer.step(qq, kk, vv, t, out=out)
                b.record()
                evs.append((a, b))
                inp2.advance()
                if t % 64 == 63:
                    torch.cuda.synchronize()
                    print(f"[bench] schedule step {t + 1}/{T}", file=sys.stderr, flush=True)
            torch.cuda.synchronize()
            total_ms = sum(a.elapsed_time(b) for a, b in evs)
            sched.update({"total_attention_ms": total_ms, "dense_only_ms": T * dense_ms, "speedup_measured": T * dense_ms / total_ms,
                          "calls": layer.calls})
            del inp2

    traffic, traffic_info = _traffic_from_profiles(cfg.name)
    result = {
        "metric": "ms/layer-call + executed TFLOP/s (% bf16 MFMA peak) for sparse attn at 64k; schedule speedup",
        "value": sparse_tf,
        "unit": "TFLOP/s (executed, sparse attention)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "L": cfg.L, "d": cfg.d,
                   "block_q": cfg.bq, "block_k": cfg.bk, "rho": cfg.rho, "kept_blocks": keep, "step": "dense+select+sparse"},
        "ms_per_call": {"dense": dense_ms, "dense_with_lse": dense_lse_ms, "select": select_ms,
                        "select_with_own_statistics": select_alone_ms, "sparse": sparse_ms},
        "tflops": {"dense": dense_tf, "select_one_qkT": select_tf, "sparse_executed": sparse_tf,
                   "sparse_dense_equivalent": tf(f_dense, sparse_ms)},
        "pct_of_peak": {"dense": 100 * dense_tf / peak, "sparse_executed": 100 * sparse_tf / peak, "select_one_qkT": 100 * select_tf / peak},
        "schedule": sched,
        "roofline": {"kernel": "attn_sparse", "bound": "mfma", "achieved": sparse_tf, "peak": peak, "unit": "TFLOP/s",
                     "frac": sparse_tf / peak, "traffic": traffic, "traffic_provenance": traffic_info},
        "roofline_dense": {"kernel": "attn_dense", "bound": "mfma", "achieved": dense_tf, "peak": peak, "unit": "TFLOP/s",
                           "frac": dense_tf / peak},
        "roofline_select": {"kernel": "select_pattern (pooled scores + top-k, statistics reused)", "bound": "mfma",
                            "achieved": select_tf, "peak": peak, "unit": "TFLOP/s", "frac": select_tf / peak,
                            # the same call as memory traffic: Q and K read once, row statistics read, index written
                            "hbm_algorithmic_GBps": _select_bytes(cfg, keep) / (select_ms * 1e-3) / 1e9},
    }
    if cfg.dtype == "bf16":
        # What the matrix cores sustain on their own (no LDS, no vector work): all-zero operands reach the published
        # peak, operands with random signs and mantissas make the chip settle at a lower clock. The second figure is
        # the ceiling for any kernel that multiplies real data; `frac` above stays relative to the published peak.
        zero_tf, rand_tf = sd.probe_mfma_bf16(False), sd.probe_mfma_bf16(True)
        result["mfma_rate_measured"] = {"unit": "TFLOP/s", "zero_operands": zero_tf, "random_operands": rand_tf,
                                        "kernel": "bf16 32x32x16 matrix instructions only, operands in registers"}
        # The same matrix instructions issued the way an attention loop issues them (58 vector instructions per 16 matrix
        # instructions, a quarter of them exp2: probe setting 4; operands read from LDS) but with no dependencies, barriers
        # or global loads: the ceiling for the attention kernels; and the pooling mix (7 vector instructions per matrix
        # instruction: half the matrix work per exponential), for which the nearest probe settings are 6 and 8.
        mix = {"mfma_plus_4_vector": sd.probe_mix_bf16(4, False), "mfma_plus_4_vector_plus_lds_operands": sd.probe_mix_bf16(4, True),
               "mfma_plus_6_vector_plus_lds_operands": sd.probe_mix_bf16(6, True),
               "mfma_plus_8_vector_plus_lds_operands": sd.probe_mix_bf16(8, True)}
        result["mfma_rate_measured"]["attention_like_mix_random_operands"] = mix
        for key, val in (("roofline", sparse_tf), ("roofline_dense", dense_tf), ("roofline_select", select_tf)):
            result[key]["frac_of_measured_rate_random_operands"] = val / rand_tf
        for key, val in (("roofline", sparse_tf), ("roofline_dense", dense_tf)):
            result[key]["frac_of_attention_mix_ceiling"] = val / mix["mfma_plus_4_vector_plus_lds_operands"]
        result["roofline_select"]["frac_of_pooling_mix_ceiling"] = select_tf / (
            0.5 * (mix["mfma_plus_6_vector_plus_lds_operands"] + mix["mfma_plus_8_vector_plus_lds_operands"]))
        # The vector unit on its own: what the softmax side (one fma, one exp2, one add per logit, plus the running
        # maximum and the bf16 conversion in attention) costs if nothing else ran.
        fma_g, exp_g = sd.probe_valu_f32("fma"), sd.probe_valu_f32("exp2")
        logits = cfg.B * cfg.Hq * cfg.L * cfg.L
        result["valu_rate_measured"] = {"unit": "1e9 lane-operations/s", "fma_f32": fma_g, "exp2_f32": exp_g,
                                        "exp2_cost_in_fma": fma_g / exp_g,
                                        "vector_only_ms": {"dense_3.5_ops_plus_exp_per_logit": logits * (3.5 / fma_g + 1.0 / exp_g) * 1e-6,
                                                           "pooled_scores_2_ops_plus_exp_per_logit": logits * (2.0 / fma_g + 1.0 / exp_g) * 1e-6},
                                        "matrix_only_ms_at_random_operand_rate": {"dense": f_dense / rand_tf * 1e-9,
                                                                                  "pooled_scores": f_select / rand_tf * 1e-9}}
    under_profiler = "rocprof" in os.environ.get("LD_PRELOAD", "") or any(key.startswith("ROCPROF") for key in os.environ)
    if not args.no_clock and not under_profiler:
        result["shader_clock_mhz"] = {"at_published_peak": 2400,
                                      "during_attn_dense": _sclk_while(lambda: sd.attn_dense(q, k, v, out=out)),
                                      "during_attn_sparse": _sclk_while(lambda: sd.attn_sparse(q, k, v, index, out=out))}
    if args.index_ablation:
        result["index_ablation"] = index_ablation(sd, torch, cfg, q, k, v, index, keep)
    if not args.no_per_workload and cfg.name == "long64k":
        result["per_workload"] = per_workload_block(sd, workload, torch, ("llada4k", "llada16k", "dream32k"), args.seed, peak)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, q, k, v, index, keep)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
