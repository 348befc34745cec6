#!/usr/bin/env python3
"""Benchmark of the Blossom attention hot path on one MI355X.

One step = one pass of the whole path over one batch of seeded synthetic input that is
already resident in HBM: block selection, fused forward (saving what backward needs) and
backward.  The headline value is valid tokens per second of that step.  The same JSON line
carries the stage times, the forward-only rate (the quantity the L=8192 target is stated
on), a roofline object for the dominant kernel, the same-style dense causal kernel and the
CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4]
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

import numpy as np

# HBM-side bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a plain copy of known size (FETCH_SIZE x2.000, WRITE_SIZE x1.000); the commands and the
# raw readings are in profiles/cfg4_hbm_traffic.txt.  Other workloads: not measured (null).
MEASURED_TRAFFIC_BYTES = {
    ("cfg4", "fwd"): 562362246, ("cfg4", "fwd_saving_for_bwd"): 1113369366, ("cfg4", "bwd_gate"): 1006265795,
    ("cfg4", "bwd_dq"): 916631857, ("cfg4", "bwd_dkv"): 1078798472, ("cfg4", "select"): 276989981,
}

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA
FP32_VALU_PEAK_TFLOPS = 157.3   # 256 CU x 4 SIMD x 64 FLOP/clk x 2.4 GHz


def algorithmic_pairs(w, valid_len, sel):
    """Unmasked (query, key) pairs of the two branches, from the selection lists (integer
    bookkeeping only; no attention arithmetic)."""
    L, b, win, NB = w.L, w.block, w.window, w.NB
    lt = st = dense = 0
    blk_lo = np.arange(NB) * b
    blk_hi = np.minimum(blk_lo + b, L)
    for r in range(w.B):
        n = int(valid_len[r])
        p0 = L - n
        if n == 0:
            continue
        i = np.arange(p0, L)
        if w.stis_block == 0:
            st += int(np.minimum(win, i - p0 + 1).sum()) * w.H
        else:
            # all of Eq. 15, causal: the window and the last-block term are suffixes of [p0, i]; the
            # blocks at power-of-two block distances lie below them and are disjoint
            sb = w.stis_block
            lo = np.maximum(p0, i - win + 1)
            lo = np.where(i >= L - sb, np.minimum(lo, max(p0, L - sb)), lo)
            cnt = i - lo + 1
            bq = i // sb
            e2 = 0
            while (1 << e2) <= int(bq.max()):
                bk = bq - (1 << e2)
                k_lo = np.maximum(bk * sb, p0)
                k_hi = np.minimum(np.minimum((bk + 1) * sb - 1, L - 1), lo - 1)
                cnt = cnt + np.where(bk >= 0, np.clip(k_hi - k_lo + 1, 0, None), 0)
                e2 += 1
            st += int(cnt.sum()) * w.H
        dense += n * (n + 1) // 2 * w.H
        vcount = np.clip(blk_hi - np.maximum(blk_lo, p0), 0, None)          # valid positions per block
        first = np.maximum(blk_lo, p0)
        diag = vcount * (vcount + 1) // 2                                    # causal pairs inside a block
        s = sel[r]                                                           # [H,NB,k]
        mask = s >= 0
        I = np.broadcast_to(np.arange(NB)[None, :, None], s.shape)
        off = mask & (s != I)
        kv = np.where(off, vcount[np.clip(s, 0, NB - 1)], 0).sum(-1)         # keys in selected past blocks
        has_diag = (mask & (s == I)).any(-1)
        lt += int((kv * vcount[None, :]).sum() + (has_diag * diag[None, :]).sum())
        del first
    return lt, st, dense


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4", help="cfg1..cfg5 (shapes of the five parity configs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--input-sets", type=int, default=3,
                    help="independent seeded input sets the timed steps rotate over, so that a small workload is not "
                         "served from the 256 MB last-level cache (one set with --stage and --graph)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step (select + forward + backward) in a HIP graph once and time its replays")
    ap.add_argument("--shape", default="",
                    help="overrides of the workload's fields, e.g. B=32,H=8,L=2000,len_lo=2000,len_hi=2000 "
                         "(the efficiency-study shapes of the paper's Appendix B); the JSON line names them")
    ap.add_argument("--stis-block", type=int, default=0,
                    help="0: short-term mask = causal window (default); N >= 1: all of Eq. 15 with mask block N")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--stage", choices=["select", "fwd", "fwd_save", "bwd", "bwd_gate", "bwd_dq", "bwd_dkv", "dense", "serve",
                                        "copy"],
                    default=None,
                    help="profiling aid: run only this stage --steps times (after the others ran once) "
                         "and print its average time; the headline line is not produced")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(every (row, head) pair is independent in selection, forward and backward: rows shard over GPUs "
              "with no exchange in forward and one small all-reduce of the gate gradients in backward).",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_13368_amd import binding as B
    from paper_2512_13368_amd.inputs import WORKLOADS, bf16_bits, make_inputs, with_shape

    w = WORKLOADS[args.workload]
    if args.stis_block:
        w = with_shape(w, stis_block=args.stis_block)
    if args.shape:
        kv = dict(t.split("=") for t in args.shape.split(","))
        w = with_shape(w, name=w.name + "*", **{k_: int(v_) for k_, v_ in kv.items()})
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n_sets = 1 if (args.stage or args.graph) else max(1, args.input_sets)
    xs = [make_inputs(w, input_set=i, want_dO=True) for i in range(n_sets)]
    x = xs[0]  # the per-kernel passes, the pair counts and the CPU baseline use the first set

    def up(a):
        if w.dtype == "bf16":
            return torch.from_numpy(bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    sets = [(up(xi.Q), up(xi.K), up(xi.V), up(xi.dO), torch.from_numpy(xi.valid_len).to(dev)) for xi in xs]
    Q, K, V, dO, vl = sets[0]
    gw = torch.from_numpy(x.gate_w).to(dev)
    gb = torch.from_numpy(x.gate_b).to(dev)
    dt = B.F32 if w.dtype == "fp32" else B.BF16
    stis = dict(stis_mode=int(w.stis_block > 0), stis_block=w.stis_block)
    p = B.Params(w.B, w.H, w.L, w.d, w.block, w.topk, w.window, dt, save_for_bwd=1, **stis)
    p_nosave = B.Params(w.B, w.H, w.L, w.d, w.block, w.topk, w.window, dt, save_for_bwd=0, **stis)
    p_serve = B.Params(w.B, w.H, w.L, w.d, w.block, w.topk, w.window, dt, save_for_bwd=0, last_block_only=1, **stis)

    # all buffers are allocated once, outside the timed region
    tdt = torch.float32 if w.dtype == "fp32" else torch.bfloat16
    shp = (w.B, w.H, w.L, w.d)
    sel = torch.empty((w.B, w.H, w.NB, w.topk), dtype=torch.int32, device=dev)
    mk = lambda: torch.empty(shp, dtype=tdt, device=dev)
    mk32 = lambda: torch.empty(shp, dtype=torch.float32, device=dev)
    fo = B.FwdOut(mk(), mk32(), mk32(), torch.empty(shp[:3], dtype=torch.float32, device=dev),
                  torch.empty(shp[:3], dtype=torch.float32, device=dev))
    fo_nosave = B.FwdOut(fo.O)
    bo = B.BwdOut(mk(), mk(), mk(), torch.empty((w.H, 2 * w.d), dtype=torch.float32, device=dev),
                  torch.empty((w.H,), dtype=torch.float32, device=dev))
    ws_sel = torch.empty(max(1, B.workspace_bytes(p, B.WS_SELECT)), dtype=torch.uint8, device=dev)
    ws_bwd = torch.empty(max(1, B.workspace_bytes(p, B.WS_BWD)), dtype=torch.uint8, device=dev)
    O_dense = mk()

    def step(i=0):
        Qi, Ki, Vi, dOi, vli = sets[i % n_sets]
        B.select_blocks(p, Qi, Ki, vli, sel=sel, ws=ws_sel)
        B.attn_fwd(p, Qi, Ki, Vi, vli, sel, gw, gb, out=fo)
        B.attn_bwd(p, Qi, Ki, Vi, vli, sel, gw, gb, fo, dOi, out=bo, ws=ws_bwd)

    if args.stage:
        step()  # every buffer a later stage reads is filled once
        fn = {"select": lambda: B.select_blocks(p, Q, K, vl, sel=sel, ws=ws_sel),
              "fwd": lambda: B.attn_fwd(p_nosave, Q, K, V, vl, sel, gw, gb, out=fo_nosave),
              "fwd_save": lambda: B.attn_fwd(p, Q, K, V, vl, sel, gw, gb, out=fo),
              "bwd": lambda: B.attn_bwd(p, Q, K, V, vl, sel, gw, gb, fo, dO, out=bo, ws=ws_bwd),
              "bwd_gate": lambda: B.attn_bwd(p, Q, K, V, vl, sel, gw, gb, fo, dO, out=bo, ws=ws_bwd,
                                             stages=B.BWD_GATE),
              "bwd_dq": lambda: B.attn_bwd(p, Q, K, V, vl, sel, gw, gb, fo, dO, out=bo, ws=ws_bwd,
                                           stages=B.BWD_DQ),
              "bwd_dkv": lambda: B.attn_bwd(p, Q, K, V, vl, sel, gw, gb, fo, dO, out=bo, ws=ws_bwd,
                                            stages=B.BWD_DKV),
              "dense": lambda: B.dense_causal_fwd(p, Q, K, V, vl, O=O_dense),
              # serving: selection and forward of the last query block only (the scored position)
              "serve": lambda: (B.select_blocks(p_serve, Q, K, vl, sel=sel, ws=ws_sel),
                                B.attn_fwd(p_serve, Q, K, V, vl, sel, gw, gb, out=fo_nosave)),
              # a plain device copy of one [B,H,L,d] tensor: calibrates the HBM byte counters
              "copy": lambda: O_dense.copy_(Q)}[args.stage]
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        print(json.dumps({"stage": args.stage, "workload": w.name, "steps": args.steps,
                          "avg_ms": round(e0.elapsed_time(e1) / args.steps, 4)}))
        return

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        # the library allocates nothing and never synchronises: the step is captured as it is
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        run_step = lambda i: graph.replay()
        run_step(0)
        torch.cuda.synchronize()

    # ---- timed region: exactly K steps ----
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    # ---- per-kernel times with HIP events on the launch stream (separate passes) ----
    def timed(fn, reps):
        ev0 = torch.cuda.Event(enable_timing=True)
        ev1 = torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps

    reps = max(3, args.steps)
    bwd = lambda st: B.attn_bwd(p, Q, K, V, vl, sel, gw, gb, fo, dO, out=bo, ws=ws_bwd, stages=st)
    ms = {
        "select": timed(lambda: B.select_blocks(p, Q, K, vl, sel=sel, ws=ws_sel), reps),
        "fwd": timed(lambda: B.attn_fwd(p_nosave, Q, K, V, vl, sel, gw, gb, out=fo_nosave), reps),
        "fwd_saving_for_bwd": timed(lambda: B.attn_fwd(p, Q, K, V, vl, sel, gw, gb, out=fo), reps),
        "bwd_gate": timed(lambda: bwd(B.BWD_GATE), reps),
        "bwd_inverse_list": timed(lambda: bwd(B.BWD_INVERSE), reps),
        "bwd_dq": timed(lambda: bwd(B.BWD_DQ), reps),
        "bwd_dkv": timed(lambda: bwd(B.BWD_DKV), reps),
        "bwd": timed(lambda: bwd(B.BWD_ALL), reps),
    }
    ms_dense = None
    if not args.no_dense:
        ms_dense = timed(lambda: B.dense_causal_fwd(p, Q, K, V, vl, O=O_dense), max(2, reps // 4))

    # ---- algorithmic work (pairs from the selection lists; bytes = tensors touched once) ----
    sel_h = sel.cpu().numpy()
    nnz_lt, nnz_st, nnz_dense = algorithmic_pairs(w, x.valid_len, sel_h)
    pairs = nnz_lt + nnz_st
    tokens = int(x.valid_len.sum())
    tokens_timed = sum(int(xs[i % n_sets].valid_len.sum()) for i in range(args.steps))  # over the timed steps
    sz = 4 if w.dtype == "fp32" else 2
    tensor = float(w.B) * w.H * w.L * w.d
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else FP32_VALU_PEAK_TFLOPS
    # kernel -> (flops, bytes): contractions each kernel has to produce per unmasked pair (2d flops
    # each) and tensors it has to read or write once
    work = {
        "fwd": (4.0 * w.d * pairs, 4 * tensor * sz),                                  # QK^T, PV | Q,K,V,O
        "fwd_saving_for_bwd": (4.0 * w.d * pairs, 4 * tensor * sz + 2 * tensor * 4),  # + o_lt, o_st fp32
        "bwd_dq": (6.0 * w.d * pairs, 5 * tensor * sz),                               # S, dP, dQ | Q,K,V,dO,dQ
        "bwd_dkv": (8.0 * w.d * pairs, 6 * tensor * sz),                              # S, dP, dV, dK | Q,K,V,dO,dK,dV
        "bwd_gate": (0.0, tensor * (sz + 8)),                                         # dO, o_lt, o_st
        "select": (0.0, 2 * tensor * sz),                                             # Q, K
    }

    def roofline(kernel):
        flops, nbytes = work[kernel]
        t = ms[kernel] * 1e-3
        t_mfma = flops / (mfma_peak * 1e12)
        t_hbm = nbytes / (HBM_PEAK_GBS * 1e9)
        if t_mfma >= t_hbm:
            a = flops / t / 1e12
            r = {"bound": "mfma", "achieved": round(a, 2), "peak": mfma_peak, "unit": "TFLOP/s",
                 "frac": round(a / mfma_peak, 4)}
        else:
            a = nbytes / t / 1e9
            r = {"bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": round(a / HBM_PEAK_GBS, 4)}
        r.update({"traffic": None if w.stis_block else MEASURED_TRAFFIC_BYTES.get((w.name, kernel)), "kernel": kernel, "avg_launch_ms": round(ms[kernel], 4),
                  "algorithmic_gflop": round(flops / 1e9, 2), "algorithmic_mb": round(nbytes / 1e6, 1)})
        return r

    step_kernels = ["select", "fwd_saving_for_bwd", "bwd_gate", "bwd_dq", "bwd_dkv"]
    dominant = max(step_kernels, key=lambda k_: ms[k_])
    out = {
        "metric": "sparse-attn fwd+bwd tokens/sec (select + forward + backward per step)",
        "value": round(tokens_timed / (wall), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype if w.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} L={w.L} d={w.d} b={w.block} k={w.topk} "
                               f"w={w.window} {w.dtype}, lens U[{w.len_lo},{w.len_hi}] left-padded, seed {w.seed}"
                               + (f", short-term mask = all of Eq. 15 with mask block {w.stis_block}" if w.stis_block else ""),
                   "tokens_per_step": tokens, "unmasked_pairs_lt": nnz_lt, "unmasked_pairs_st": nnz_st,
                   "launch": "hip graph replay" if args.graph else "stream", "input_sets": n_sets},
        "kernels_ms": {k_: round(v, 4) for k_, v in ms.items()},
        "fwd_tokens_per_s": round(tokens / ((ms["select"] + ms["fwd"]) * 1e-3), 1),
        "roofline": roofline(dominant),
        "roofline_fwd": roofline("fwd"),
        "roofline_all": {k_: roofline(k_)["frac"] for k_ in ("fwd", "fwd_saving_for_bwd", "bwd_dq", "bwd_dkv",
                                                              "bwd_gate", "select")},
    }
    if ms_dense is not None:
        flops_dense = 4.0 * w.d * nnz_dense
        out["dense_causal"] = {"ms": round(ms_dense, 4), "tokens_per_s": round(tokens / (ms_dense * 1e-3), 1),
                               "tflops": round(flops_dense / (ms_dense * 1e-3) / 1e12, 2),
                               "sparse_fwd_speedup": round(ms_dense / (ms["select"] + ms["fwd"]), 3)}

    # ---- CPU oracle on a bounded sample of the same workload (reported, not a target) ----
    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.num_threads()
        total_pairs = w.B * w.H

        def run_oracle(n_pairs):
            prs = np.linspace(0, total_pairs - 1, n_pairs).astype(np.int32)
            t0 = time.perf_counter()
            sel_ref = oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk, bh_list=prs)
            sel_ref = np.where(sel_ref == -2, -1, sel_ref)
            oracle.attn_fwd(x.Q, x.K, x.V, x.valid_len, sel_ref, x.gate_w, x.gate_b, w.block, w.topk, w.window,
                            bh_list=prs, stis_block=w.stis_block)
            oracle.attn_bwd(x.Q, x.K, x.V, x.valid_len, sel_ref, x.gate_w, x.gate_b, x.dO, w.block, w.topk,
                            w.window, bh_list=prs, stis_block=w.stis_block)
            dt_ = time.perf_counter() - t0
            toks = float(sum(int(x.valid_len[int(bh) // w.H]) for bh in prs)) / w.H
            return dt_, toks

        n_pairs = min(total_pairs, threads)
        cpu_s, sample_tokens = run_oracle(n_pairs)
        if cpu_s < 8.0 and n_pairs < total_pairs:  # aim at about 15 s of CPU work
            n_pairs = min(total_pairs, max(n_pairs + 1, int(n_pairs * 15.0 / max(cpu_s, 1e-3))))
            cpu_s, sample_tokens = run_oracle(n_pairs)
        cpu_model = "unknown"
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        out["cpu_baseline"] = {"value": round(sample_tokens / cpu_s, 2), "unit": "tokens/s",
                               "cores": threads, "cpu": cpu_model, "kind": "oracle",
                               "sample": f"{n_pairs} of {total_pairs} (row, head) pairs, select+fwd+bwd, "
                                         f"{cpu_s:.1f} s; tokens counted as pairs/H * valid_len"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
