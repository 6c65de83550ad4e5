#!/usr/bin/env python3
"""Benchmark of the Ecco hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
  ecco_kv_append (1 new token x 8 sequences x 32 heads, K and V)           -- encoder
  ecco_decode                on the 8192 x 28672 projection (70B class)     -- standalone decode
  ecco_decode_gemv batch 1   on the same projection                         -- THE METRIC
  ecco_decode_gemv batch 8, batch 16
  ecco_kv_attend             8 x 32 heads x 4096 cached tokens
The headline workload is the largest single-GPU configuration (--workload proj70b, the default); the fused GEMV
on the smaller matrices (4096 x 4096, 11008 x 4096, 4096 x 11008) is timed the same way after the step and
reported as further rows of the same line (rows.proj7b_gemv1, rows.mlp_up_gemv16, ...).
Every call reads a different copy of its compressed input (the copies rotate through > 1 GiB), so
no launch finds its blocks in the 256 MB last-level cache.  Inputs are resident in HBM before
the timed region.  The K timed steps are recorded into one HIP graph and replayed once, so the GPU
runs them back to back (launching each call from Python costs more than the short kernels take);
per-kernel durations come from HIP events on the launch stream around a replayed graph of that call
over all its rotating copies.  `value` is the fused batch-1 decode-GEMV rate on compressed bytes
read (68 B per group: 64 B payload + 4 B meta).

Prints ONE JSON line.  `--gpus` above 1 is refused: this build runs on a single GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
BYTES_PER_GROUP = 68   # 64-byte payload + 4-byte meta word
# HBM bytes per launch of the fused batch-1 kernel.  These are NOT measured by this program: they come from two
# rocprofv3 --pmc runs of it (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, each scaled by what the same counter
# reads for a plain copy of known size); the JSON line names the summary file beside the figure (roofline.traffic_from).
MEASURED_TRAFFIC = {
    "proj7b": {"bytes": int((4465.6 * 1.994 + 16.0) * 1024), "from": "profiles/bench_step_proj7b.md"},
    "proj70b": {"bytes": int((61376.5 * 1.9994 + 32.0) * 1024), "from": "profiles/bench_default_proj70b.md"},
}
# Which resource the fused batch-1 kernel saturates on the headline workload, from the SQ counters of the same summary
# (not measured by this program either): share of the kernel's cycles in which a compute unit's LDS pipeline is active,
# and LDS / VALU issue cycles per wavefront and decoded value.
OBSERVED_LIMIT = {
    "proj70b": {"resource": "LDS gather rate (table reads with bank conflicts), not HBM", "lds_pipeline_active_frac": 0.827,
                "lds_cycles_per_wave_value": 8.8, "valu_cycles_per_wave_value": 7.3, "from": "profiles/bench_default_proj70b.md"},
}
WEIGHT_WORKLOADS = {"proj7b": ("proj7b", 0), "mlp_up": ("mlp", 0), "mlp_down": ("mlp", 1), "proj70b": ("proj70b", 0)}


def cpu_baseline(m, blocks_np, meta_np, rows, cols, x_np, w_np=None, budget_s=12.0):
    """The oracle's decode + GEMV (double accumulation) on the same matrix, repeated for about budget_s seconds."""
    from oracle import oracle as O
    threads = O.set_threads(os.cpu_count() or 1)
    gpr = cols // 128
    cent, lens = m.centroids, m.code_lens

    def run(nrows):
        t0 = time.perf_counter()
        O.gemv(cent, lens, blocks_np[: nrows * gpr], meta_np[: nrows * gpr], nrows, cols, x_np.view(np.uint16))
        return time.perf_counter() - t0

    probe_rows = min(rows, 8 * threads)
    t_probe = run(probe_rows)
    nrows = int(min(rows, max(probe_rows, probe_rows * budget_s / max(t_probe, 1e-6))))
    passes, spent = 0, 0.0
    while spent < budget_s and passes < 1000:
        spent += run(nrows)
        passes += 1
    groups = nrows * gpr
    per_pass = spent / passes
    # one thread, on a slice: about two seconds
    O.set_threads(1)
    rows1 = max(1, min(rows, nrows // max(threads, 1)))
    t1, n1 = 0.0, 0
    while t1 < 2.0 and n1 < 50:
        t1 += run(rows1)
        n1 += 1
    O.set_threads(threads)
    # the oracle's standalone decoder and encoder on all threads, about three seconds each, on the first groups
    # of the same matrix (rates on the same byte accounting as the GPU rows)
    extra = {}

    def timed(fn, n0, total, budget=3.0):
        n = min(total, n0)
        t0 = time.perf_counter()
        fn(n)
        t = time.perf_counter() - t0
        n = int(min(total, max(n, n * budget / max(t, 1e-6))))
        t0 = time.perf_counter()
        fn(n)
        return n, time.perf_counter() - t0

    total_groups = rows * gpr
    n, t = timed(lambda n: O.decode(cent, lens, blocks_np[:n], meta_np[:n]), 64 * threads, total_groups)
    extra["decode"] = {"groups": n, "seconds": t, "GBps_total_traffic": n * (BYTES_PER_GROUP + 256) / t / 1e9}
    if w_np is not None:
        wg = w_np.reshape(-1, 128).view(np.uint16)
        n, t = timed(lambda n: O.encode(cent, lens, wg[:n]), 16 * threads, total_groups)
        extra["encode"] = {"groups": n, "seconds": t, "groups_per_s": n / t}
    cpu = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    cpu = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"value": groups * BYTES_PER_GROUP / per_pass / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"oracle_gemv batch 1 on the first {nrows} of {rows} rows of the same matrix ({groups} groups), "
                      f"{passes} passes, {spent:.1f} s in all",
            "gemv_per_s_equiv": 1.0 / (per_pass * rows / nrows),
            "single_thread_GBps": rows1 * gpr * BYTES_PER_GROUP / (t1 / n1) / 1e9, "cpu": cpu, "host_cpus": os.cpu_count(),
            "other_oracle_legs": extra}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="launch every call from Python with its own event pair instead of replaying a HIP graph")
    ap.add_argument("--only", default="", help="comma list of rows to run (kv_append,decode,gemv1,gemv8,gemv16,kv_attend; "
                    "on request only: kv_append_minmax, encode, encode_minmax -- the bulk encoders run over the K cache -- "
                    "act_encode, act_decode -- the 2x activation codec on 32768 x 4096 activations -- and pb_encode, pb_decode, pb_gemv1 -- the self-contained "
                    "block format on the workload's weight matrix)")
    ap.add_argument("--kv-batch", type=int, default=0, help="sequences of the KV rows (default: the workload's 8)")
    ap.add_argument("--kv-tokens", type=int, default=0, help="tokens per sequence of the KV rows (default: the workload's 4096)")
    ap.add_argument("--gqa-group", type=int, default=4, help="query heads per key/value head of the kv_attend_gqa row (on request: --only kv_attend_gqa)")
    ap.add_argument("--gqa-splits", type=int, default=0, help="token splits of the kv_attend_gqa row (0: enough to give every compute unit a workgroup)")
    ap.add_argument("--selector-quality", action="store_true",
                    help="add the reconstruction error of the min/max pattern selector against the least-squared-error search on the K and V caches")
    ap.add_argument("--kv-patterns", type=int, default=0, help="shared patterns of the K and V models (default: the KV workload's 64; the paper's online compressor uses 16)")
    ap.add_argument("--workload", default="proj70b", choices=["proj7b", "mlp_up", "mlp_down", "proj70b"],
                    help="the matrix of the step and of the headline value (default: the largest single-GPU configuration)")
    ap.add_argument("--also", default="proj7b,mlp_up,mlp_down",
                    help="comma list of further matrices whose fused GEMV is timed after the step and reported as extra rows "
                         "(batch 1 on all, batch 8 and 16 on the MLP pair); empty for none")
    ap.add_argument("--sweep", action="store_true", help="add an ecco_decode sweep over block counts 2^14..2^22 (as far as the workload has blocks)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (every box has one); run with --gpus 1")

    import torch

    import paper_2505_06901_amd as E
    from paper_2505_06901_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    only = set(filter(None, args.only.split(",")))

    def want(row):
        return not only or row in only

    # ---- weights --------------------------------------------------------------------------------
    wname, which = WEIGHT_WORKLOADS[args.workload]
    cfg = W.CONFIGS[wname]
    rows, cols = cfg["shapes"][which]
    w = W.config_weight(wname, which)
    m = E.ecco_model_to_device(E.ecco_fit_patterns(w, cfg["S"], 12, cfg["seeds"][which]), 0)
    blocks0, meta0 = E.ecco_encode(m, torch.from_numpy(w).to(dev))
    torch.cuda.synchronize()
    n_groups = rows * cols // 128
    raw_frac = float(((meta0 >> 22) & 1).float().mean())
    copy_bytes = n_groups * BYTES_PER_GROUP
    n_copies = max(2, min(256, int(np.ceil((1.25 * 2**30) / copy_bytes))))
    wb = [blocks0] + [blocks0.clone() for _ in range(n_copies - 1)]
    wm = [meta0] + [meta0.clone() for _ in range(n_copies - 1)]
    xs = {b: torch.from_numpy(W.activation(b, cols, cfg["x_seed"])).to(dev) for b in (1, 8, 16)}
    ys = {b: torch.empty((b, rows), dtype=torch.float32, device=dev) for b in (1, 8, 16)}
    dec_out = torch.empty((n_groups, 128), dtype=torch.float16, device=dev)

    # ---- KV cache ---------------------------------------------------------------------------------
    kc = W.CONFIGS["kv"]
    B, H, T = args.kv_batch or kc["batch"], kc["heads"], args.kv_tokens or kc["tokens"]
    extra_rows = [r for r in ("kv_append_minmax", "encode", "encode_minmax", "kv_attend_gqa") if r in only]
    pb_rows = [r for r in ("pb_encode", "pb_decode", "pb_gemv1") if r in only]
    act_rows = [r for r in ("act_encode", "act_decode") if r in only]
    if act_rows:
        act_rows.append("copy_reference")  # a plain device copy of the same FP16 tensor: the practical HBM ceiling beside the codec
    kv_needed = want("kv_append") or want("kv_attend") or bool(extra_rows) or args.selector_quality
    if kv_needed:
        k, v = W.kv_cache(B, H, T, 128, kc["seeds"][0])
        cal = kc["calib_tokens"]
        kv_S = args.kv_patterns or kc["S"]
        mk = E.ecco_model_to_device(E.ecco_fit_patterns(k[:, :, :cal], kv_S, 12, kc["seeds"][0]), 0)
        mv = E.ecco_model_to_device(E.ecco_fit_patterns(v[:, :, :cal], kv_S, 12, kc["seeds"][0] + 1), 0)
        k_dev = torch.from_numpy(k).to(dev)
        kb0, km0 = E.ecco_encode(mk, k_dev)
        vb0, vm0 = E.ecco_encode(mv, torch.from_numpy(v).to(dev))
        selector_quality = None
        if args.selector_quality:
            selector_quality = {}
            for name, model, src, fb, fm in (("K", mk, k_dev, kb0, km0), ("V", mv, torch.from_numpy(v).to(dev), vb0, vm0)):
                x = src.reshape(-1, 128).float()
                mb, mm = E.ecco_encode_minmax(model, src)
                err_full = (E.ecco_decode(model, fb, fm).float() - x).square().sum(dim=1)
                err_mm = (E.ecco_decode(model, mb, mm).float() - x).square().sum(dim=1)
                power = x.square().sum().item()
                selector_quality[name] = {
                    "rel_mse_least_squares": err_full.sum().item() / power, "rel_mse_minmax": err_mm.sum().item() / power,
                    "mse_ratio": err_mm.sum().item() / err_full.sum().item(),
                    "same_pattern_fraction": float((((fm >> 16) & 63) == ((mm >> 16) & 63)).float().mean()),
                    "raw_block_fraction_least_squares": float(((fm >> 22) & 1).float().mean()),
                    "raw_block_fraction_minmax": float(((mm >> 22) & 1).float().mean())}
                del x, mb, mm, err_full, err_mm
        if not ("encode" in only or "encode_minmax" in only):
            del k_dev
        else:
            enc_blocks, enc_meta = torch.empty_like(kb0), torch.empty_like(km0)
        kv_copies = 10  # 10 x 143 MB of compressed K+V
        kbs = [kb0.view(B, H, T, 64)] + [kb0.view(B, H, T, 64).clone() for _ in range(kv_copies - 1)]
        kms = [km0.view(B, H, T)] + [km0.view(B, H, T).clone() for _ in range(kv_copies - 1)]
        vbs = [vb0.view(B, H, T, 64)] + [vb0.view(B, H, T, 64).clone() for _ in range(kv_copies - 1)]
        vms = [vm0.view(B, H, T)] + [vm0.view(B, H, T).clone() for _ in range(kv_copies - 1)]
        q = torch.from_numpy(W.activation(B * H, 128, kc["q_seed"]).reshape(B, H, 128)).to(dev)
        k_new = torch.from_numpy(np.ascontiguousarray(k[:, :, T - 1])).to(dev)
        v_new = torch.from_numpy(np.ascontiguousarray(v[:, :, T - 1])).to(dev)
        seq_full = torch.full((B,), T, dtype=torch.int32, device=dev)
        seq_app = torch.full((B,), T - 1, dtype=torch.int32, device=dev)  # append overwrites the last slot
        attn_out = torch.empty((B, H, 128), dtype=torch.float32, device=dev)
        if "kv_attend_gqa" in only:
            # the same H query heads over H / group key/value heads: the caches of the first H / group heads of every sequence
            grp = args.gqa_group
            Hkv = H // grp
            gqa_splits = args.gqa_splits or E.ecco_kv_attend_gqa_splits(0, B, Hkv, T)
            take = lambda a: [x[:, :Hkv].contiguous() for x in a]
            gkb, gkm, gvb, gvm = take(kbs), take(kms), take(vbs), take(vms)
            n_ws = (B * H * gqa_splits * 130 * 4) if gqa_splits > 1 else 16
            gqa_ws = torch.empty((n_ws,), dtype=torch.uint8, device=dev)
        del k, v
    torch.cuda.synchronize()

    # ---- the self-contained block format on the same weight matrix ------------------------------------------------------
    if pb_rows:
        pbm = E.ecco_pb_model_to_device(E.ecco_pb_fit(w, cfg["S"], cfg["seeds"][which]), 0)
        w_dev = torch.from_numpy(w).to(dev)
        pb_blocks = [E.ecco_pb_encode(pbm, w_dev) for _ in range(min(n_copies, 64))]
        pb_out = torch.empty((n_groups, 128), dtype=torch.float16, device=dev)
        pb_dec = E.ecco_pb_decode(pbm, pb_blocks[0]).float()
        wf = w_dev.float().reshape(-1, 128)
        pb_info = {"rel_mse": float((pb_dec - wf).square().sum() / wf.square().sum()),
                   "rel_mse_other_format": float((E.ecco_decode(m, blocks0, meta0).float() - wf).square().sum() / wf.square().sum()),
                   "texp": pbm.texp}
        del pb_dec, wf
    torch.cuda.synchronize()

    # ---- activations for the 2x codec: 32768 tokens x 4096 channels, N(0,1) times a per-channel magnitude ----------
    if act_rows:
        act_tokens, act_hidden = 32768, 4096
        base = torch.from_numpy(W.activation(1024, act_hidden, kc["q_seed"] + 1)).to(dev).float()
        chan = torch.from_numpy((10.0 ** np.random.default_rng(5).uniform(-1, 1, act_hidden)).astype(np.float32)).to(dev)
        act_src = (base.repeat(act_tokens // 1024, 1) * chan).to(torch.float16).contiguous()   # 256 MiB of FP16
        act_groups = act_src.numel() // 64
        act_blocks = E.ecco_act_encode(act_src)                                                  # 128 MiB
        act_dst = torch.empty_like(act_src)
        del base
    torch.cuda.synchronize()

    # ---- the step -----------------------------------------------------------------------------------
    row_names = [r for r in ("kv_append", "decode", "gemv1", "gemv8", "gemv16", "kv_attend") if want(r)] + extra_rows + pb_rows + act_rows
    counter = [0]

    def next_copy(n):
        counter[0] += 1
        return counter[0] % n

    def run_row(row):
        if row == "kv_append":
            c = next_copy(kv_copies)
            E.ecco_kv_append(mk, mv, k_new, v_new, kbs[c], kms[c], vbs[c], vms[c], seq_app, B, H, T)
        elif row == "kv_append_minmax":
            c = next_copy(kv_copies)
            E.ecco_kv_append_minmax(mk, mv, k_new, v_new, kbs[c], kms[c], vbs[c], vms[c], seq_app, B, H, T)
        elif row == "pb_encode":
            E.ecco_pb_encode(pbm, w_dev, pb_blocks[next_copy(len(pb_blocks))])
        elif row == "pb_gemv1":
            E.ecco_pb_decode_gemv(pbm, pb_blocks[next_copy(len(pb_blocks))], rows, cols, xs[1], ys[1])
        elif row == "pb_decode":
            E.ecco_pb_decode(pbm, pb_blocks[next_copy(len(pb_blocks))], pb_out)
        elif row == "act_encode":
            E.ecco_act_encode(act_src, act_blocks)
        elif row == "act_decode":
            E.ecco_act_decode(act_blocks, act_dst)
        elif row == "copy_reference":
            act_dst.copy_(act_src)
        elif row == "kv_attend_gqa":
            c = next_copy(kv_copies)
            E.ecco_kv_attend_gqa(mk, mv, q, gkb[c], gkm[c], gvb[c], gvm[c], seq_full, B, H, Hkv, T, gqa_splits, gqa_ws, attn_out)
        elif row == "encode":
            E.ecco_encode(mk, k_dev, enc_blocks, enc_meta)
        elif row == "encode_minmax":
            E.ecco_encode_minmax(mk, k_dev, enc_blocks, enc_meta)
        elif row == "decode":
            c = next_copy(n_copies)
            E.ecco_decode(m, wb[c], wm[c], dec_out)
        elif row in ("gemv1", "gemv8", "gemv16"):
            b = int(row[4:])
            c = next_copy(n_copies)
            E.ecco_decode_gemv(m, wb[c], wm[c], rows, cols, xs[b], ys[b])
        elif row == "kv_attend":
            c = next_copy(kv_copies)
            E.ecco_kv_attend(mk, mv, q, kbs[c], kms[c], vbs[c], vms[c], seq_full, B, H, T, attn_out)

    def step():
        for row in row_names:
            run_row(row)

    def capture(fn):
        """Records fn's launches into a HIP graph (no memset nodes: the library issues kernels only)."""
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    def timed_replays(g, replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    spread = {}  # row -> (median, least, replays, launches per replay) of the per-replay means, graph timing only

    if args.eager:
        # every call bracketed by its own pair of events; the host-side launch path (about 10 us per call from
        # Python) then bounds the short kernels, so these figures are upper bounds on the kernel durations
        events = {r: [] for r in row_names}
        t0 = time.perf_counter()
        for _ in range(args.steps):
            for row in row_names:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                run_row(row)
                e1.record()
                events[row].append((e0, e1))
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms = {r: float(np.mean([a.elapsed_time(b) for a, b in events[r]])) for r in row_names}
    else:
        # the K steps are recorded once into a HIP graph and replayed: the GPU then runs the launches back to back
        # and HIP events on the launch stream see kernel time, not the Python launch path
        def k_steps():
            for _ in range(args.steps):
                step()
        g_steps = capture(k_steps)
        g_steps.replay()  # first replay uploads the graph; not timed
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gpu_ms = timed_replays(g_steps, 1)
        wall = time.perf_counter() - t0
        del g_steps
        # per-row duration: a graph of one launch per rotating copy of that row's input, replayed
        ms = {}
        for row in row_names:
            n = 2 if row.startswith("encode") else 4 if row.startswith("act_") or row == "copy_reference" else len(pb_blocks) if row.startswith("pb_") else kv_copies if row.startswith("kv_") else n_copies
            def one_round(row=row, n=n):
                for _ in range(n):
                    run_row(row)
            g = capture(one_round)
            g.replay()
            torch.cuda.synchronize()
            replays = 2 if row.startswith("encode") else 5 if row.startswith("act_") or row == "copy_reference" else max(5, int(np.ceil(max(args.steps, 100) / n)))
            # every replay (one launch per rotating copy) between its own pair of events: the median and the least
            # replay say how steady the row is (replays of few launches include the host's gap between replays)
            pairs = []
            for _ in range(replays):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                g.replay()
                e1.record()
                pairs.append((e0, e1))
            torch.cuda.synchronize()
            per = [a.elapsed_time(b) / n for a, b in pairs]
            spread[row] = (float(np.median(per)), float(np.min(per)), replays, n)
            # the row's figure: all replays between one pair of events (no host gaps between short replays)
            ms[row] = timed_replays(g, replays) / (replays * n)
            del g

    # ---- what merely reading the same bytes costs: a read-only streaming kernel over the blocks of every rotating copy ----
    stream_ms = None
    if want("gemv1"):
        sink = torch.zeros((256,), dtype=torch.int32, device=dev)
        def read_round():
            for c in range(n_copies):
                E.ecco_read_stream(wb[c], sink)   # the 64-byte payloads: one launch per copy, like the decoder
        if args.eager:
            read_round()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            read_round()
            e1.record()
            torch.cuda.synchronize()
            stream_ms = e0.elapsed_time(e1) / n_copies
        else:
            g = capture(read_round)
            g.replay()
            torch.cuda.synchronize()
            stream_ms = timed_replays(g, 2) / (2 * n_copies)
            del g

    # ---- cache-warm figure for the metric row (same copy every launch), labelled as such --------------
    warm_ms = None
    if want("gemv1"):
        def warm_round():
            for _ in range(50):
                E.ecco_decode_gemv(m, wb[0], wm[0], rows, cols, xs[1], ys[1])
        if args.eager:
            warm_round()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            warm_round()
            e1.record()
            torch.cuda.synchronize()
            warm_ms = e0.elapsed_time(e1) / 50
        else:
            g = capture(warm_round)
            g.replay()
            torch.cuda.synchronize()
            warm_ms = timed_replays(g, 2) / 100
            del g

    # ---- standalone decode over growing block counts (the first n groups of every rotating copy) -----
    sweep = None
    if args.sweep:
        sweep = []
        sw_b, sw_m, sw_out, sw_copies = wb, wm, dec_out, n_copies
        for lg in range(14, 23):
            n = 1 << lg
            if n > n_groups and sw_b is wb:
                if args.workload != "proj70b":
                    break
                # past the end of the matrix: further rows of the same seeded stream, encoded with the same
                # model, behind the matrix's own blocks; four rotating copies (one already exceeds the cache)
                need = 1 << 22
                more_rows = -(-(need - n_groups) * 128 // cols)
                w_more = W.weight_matrix(more_rows, cols, cfg["sigma"], cfg["outlier_frac"], cfg["outlier_mult"],
                                         cfg["seeds"][which], row_start=rows)
                b_more, m_more = E.ecco_encode(m, torch.from_numpy(w_more).to(dev))
                del w_more
                big_b = torch.cat([blocks0, b_more])[:need].contiguous()
                big_m = torch.cat([meta0, m_more])[:need].contiguous()
                del b_more, m_more
                sw_copies = 4
                sw_b = [big_b] + [big_b.clone() for _ in range(sw_copies - 1)]
                sw_m = [big_m] + [big_m.clone() for _ in range(sw_copies - 1)]
                sw_out = torch.empty((need, 128), dtype=torch.float16, device=dev)
                torch.cuda.synchronize()
            def one_round(n=n, sw_b=sw_b, sw_m=sw_m, sw_out=sw_out, sw_copies=sw_copies):
                for c in range(sw_copies):
                    E.ecco_decode(m, sw_b[c][:n], sw_m[c][:n], sw_out[:n])
            if args.eager:
                one_round()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                one_round()
                e1.record()
                torch.cuda.synchronize()
                t_ms = e0.elapsed_time(e1) / sw_copies
            else:
                g = capture(one_round)
                g.replay()
                torch.cuda.synchronize()
                replays = max(1, int(np.ceil(60 / sw_copies)))
                t_ms = timed_replays(g, replays) / (replays * sw_copies)
                del g
            # the same copy every time: its blocks stay in the last-level cache as far as they fit ("warm")
            warm_us = None
            if not args.eager:
                def warm_round(n=n, sw_b=sw_b, sw_m=sw_m, sw_out=sw_out):
                    for _ in range(20):
                        E.ecco_decode(m, sw_b[0][:n], sw_m[0][:n], sw_out[:n])
                g = capture(warm_round)
                g.replay()
                torch.cuda.synchronize()
                warm_us = timed_replays(g, 3) / 60 * 1e3
                del g
            sweep.append({"n_groups": n, "us": t_ms * 1e3, "us_warm": warm_us, "GBps_compressed_read": n * BYTES_PER_GROUP / (t_ms * 1e-3) / 1e9,
                          "GBps_total_traffic": n * (BYTES_PER_GROUP + 256) / (t_ms * 1e-3) / 1e9,
                          "rotating_copies": sw_copies, "beyond_matrix": n > n_groups})

    # ---- the fused GEMV on the other matrices: same rotation through > 1 GiB of copies, same graph timing ----------
    also_rows = {}
    if want("gemv1") and not args.eager:
        for other in filter(None, args.also.split(",")):
            if other == args.workload or other not in WEIGHT_WORKLOADS:
                continue
            oname, owhich = WEIGHT_WORKLOADS[other]
            ocfg = W.CONFIGS[oname]
            orows, ocols = ocfg["shapes"][owhich]
            ow = W.config_weight(oname, owhich)
            om_ = E.ecco_model_to_device(E.ecco_fit_patterns(ow, ocfg["S"], 12, ocfg["seeds"][owhich]), 0)
            ob0, ome0 = E.ecco_encode(om_, torch.from_numpy(ow).to(dev))
            del ow
            o_groups = orows * ocols // 128
            o_bytes = o_groups * BYTES_PER_GROUP
            o_copies = max(2, min(256, int(np.ceil((1.25 * 2**30) / o_bytes))))
            obs = [ob0] + [ob0.clone() for _ in range(o_copies - 1)]
            oms = [ome0] + [ome0.clone() for _ in range(o_copies - 1)]
            for b in ((1, 8, 16) if oname == "mlp" else (1,)):
                ox = torch.from_numpy(W.activation(b, ocols, ocfg["x_seed"])).to(dev)
                oy = torch.empty((b, orows), dtype=torch.float32, device=dev)
                def one_round(b=b, ox=ox, oy=oy):
                    for c in range(o_copies):
                        E.ecco_decode_gemv(om_, obs[c], oms[c], orows, ocols, ox, oy)
                for _ in range(2):
                    one_round()
                g = capture(one_round)
                g.replay()
                torch.cuda.synchronize()
                replays = max(5, int(np.ceil(max(args.steps, 100) / o_copies)))
                t_ms = timed_replays(g, replays) / (replays * o_copies)
                del g
                also_rows[f"{other}_gemv{b}"] = {
                    "ms": t_ms, "GBps_compressed": o_bytes / (t_ms * 1e-3) / 1e9, "pct_hbm_peak": 100.0 * o_bytes / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "gemv_tokens_per_s": b / (t_ms * 1e-3), "shape": [orows, ocols], "n_groups": o_groups, "rotating_copies": o_copies,
                    "raw_block_fraction": float(((ome0 >> 22) & 1).float().mean())}
            del obs, oms, ob0, ome0
            torch.cuda.empty_cache()

    comp_bytes = n_groups * BYTES_PER_GROUP
    rows_out = {}
    for r in row_names:
        d = {"ms": ms[r]}
        if r in spread:
            d["median_ms"], d["min_ms"], d["replays"], d["launches_per_replay"] = spread[r]
        if r.startswith("gemv"):
            b = int(r[4:])
            d["GBps_compressed"] = comp_bytes / (ms[r] * 1e-3) / 1e9
            d["gemv_tokens_per_s"] = b / (ms[r] * 1e-3)
        elif r == "decode":
            d["GBps_total_traffic"] = n_groups * (BYTES_PER_GROUP + 256) / (ms[r] * 1e-3) / 1e9
            d["GBps_compressed"] = comp_bytes / (ms[r] * 1e-3) / 1e9
        elif r.startswith("kv_append"):
            d["groups_per_s"] = 2 * B * H / (ms[r] * 1e-3)
        elif r == "pb_gemv1":
            d["GBps_compressed"] = n_groups * 64 / (ms[r] * 1e-3) / 1e9   # 64-byte blocks, nothing beside them
            d["pct_hbm_peak"] = 100.0 * d["GBps_compressed"] / HBM_PEAK_GBS
            d["gemv_tokens_per_s"] = 1.0 / (ms[r] * 1e-3)
        elif r.startswith("pb_"):
            d["groups_per_s"] = n_groups / (ms[r] * 1e-3)
            d["GBps_total_traffic"] = n_groups * (64 + 256) / (ms[r] * 1e-3) / 1e9   # 64-byte block + 256 bytes of FP16
            d["pct_hbm_peak"] = 100.0 * d["GBps_total_traffic"] / HBM_PEAK_GBS
            d.update(pb_info)
        elif r == "copy_reference":
            d["GBps_total_traffic"] = 2 * act_src.numel() * 2 / (ms[r] * 1e-3) / 1e9
            d["pct_hbm_peak"] = 100.0 * d["GBps_total_traffic"] / HBM_PEAK_GBS
        elif r.startswith("act_"):
            d["groups_per_s"] = act_groups / (ms[r] * 1e-3)
            d["GBps_total_traffic"] = act_groups * 192 / (ms[r] * 1e-3) / 1e9   # 128 B of FP16 + 64 B block per group
            d["pct_hbm_peak"] = 100.0 * d["GBps_total_traffic"] / HBM_PEAK_GBS
        elif r.startswith("encode"):
            d["groups_per_s"] = B * H * T / (ms[r] * 1e-3)
            d["GBps_fp16_in_plus_blocks_out"] = B * H * T * (256 + BYTES_PER_GROUP) / (ms[r] * 1e-3) / 1e9
        elif r == "kv_attend_gqa":
            d["steps_per_s"] = 1.0 / (ms[r] * 1e-3)
            d["GBps_compressed"] = 2 * B * Hkv * T * BYTES_PER_GROUP / (ms[r] * 1e-3) / 1e9
            d["config"] = {"B": B, "Hq": H, "Hkv": Hkv, "T": T, "n_splits": gqa_splits}
        elif r == "kv_attend":
            d["steps_per_s"] = 1.0 / (ms[r] * 1e-3)
            d["GBps_compressed"] = 2 * B * H * T * BYTES_PER_GROUP / (ms[r] * 1e-3) / 1e9
        rows_out[r] = d
    rows_out.update(also_rows)

    metric_row = "gemv1" if want("gemv1") else row_names[0]
    achieved = rows_out[metric_row].get("GBps_compressed", 0.0)
    out = {
        "metric": "fused Ecco decode-GEMV effective GB/s (compressed-bytes-read) and % HBM peak",
        "value": achieved,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",  # the multiply-adds: FP16 operands (decoded weights, activations), FP32 products and sums
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {rows}x{cols} FP16 projection, group 128, S={cfg['S']}, 64-byte blocks; "
                               f"fused ecco_decode_gemv batch 1; other rows of the step: {','.join(row_names)}",
                   "n_groups": n_groups, "compressed_bytes": comp_bytes, "payload_only_GBps": achieved * 64 / 68,
                   "pct_hbm_peak": 100.0 * achieved / HBM_PEAK_GBS, "raw_block_fraction": raw_frac,
                   "rotating_copies": n_copies, "timing": "eager launches" if args.eager else "HIP graph replay", "cache_warm_gemv1_GBps": (comp_bytes / (warm_ms * 1e-3) / 1e9) if warm_ms else None,
                   "read_only_stream_GBps": (n_groups * 64 / (stream_ms * 1e-3) / 1e9) if stream_ms else None,
                   "frac_of_read_only_stream": (achieved / (n_groups * 64 / (stream_ms * 1e-3) / 1e9)) if stream_ms and metric_row == "gemv1" else None},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     # not measured by this run: counter traffic of the same launch from the named rocprofv3 summary
                     "traffic": MEASURED_TRAFFIC.get(args.workload, {}).get("bytes"),
                     "traffic_from": MEASURED_TRAFFIC.get(args.workload, {}).get("from"),
                     "kernel": "gemv_kernel (fused decode-GEMV, batch 1)", "bytes_per_launch": comp_bytes,
                     "avg_launch_ms": ms.get(metric_row),
                     # this run's time in cycles (2.4 GHz) per wavefront and decoded value and compute unit, to set beside
                     # the counter figures of observed_limit
                     "cycles_per_wave_value": (ms[metric_row] * 1e-3 * 2.4e9 / (n_groups * 2.0 / torch.cuda.get_device_properties(dev).multi_processor_count))
                                              if ms.get(metric_row) else None,
                     "observed_limit": OBSERVED_LIMIT.get(args.workload)},
        "rows": rows_out,
        "footprint": {"fp16_bytes": n_groups * 256, "compressed_bytes": comp_bytes, "ratio": 256.0 / BYTES_PER_GROUP,
                      "payload_bytes": n_groups * 64, "meta_bytes": n_groups * 4, "model_blob_bytes": len(E.ecco_model_save(m))},
    }
    if sweep is not None:
        out["decode_sweep"] = sweep
    props = torch.cuda.get_device_properties(dev)
    out["device"] = {"name": props.name, "compute_units": props.multi_processor_count, "memory_bytes": props.total_memory}
    _, clk, width = E.ecco_device_info(0)
    if clk and width:
        # as the runtime reports them (kHz, bits).  The data-sheet 8 TB/s the roofline uses is four transfers per
        # reported clock on this bus (2 GHz x 8192 bit x 4 / 8)
        out["device"].update({"memory_clock_kHz": clk, "memory_bus_bits": width, "GBps_at_4_transfers_per_clock": 4.0 * clk * 1e3 * width / 8 / 1e9})
    if kv_needed:
        out["config"]["kv_patterns"] = kv_S
    if kv_needed and selector_quality is not None:
        out["selector_quality"] = selector_quality
    if not args.no_cpu_baseline and want("gemv1"):
        out["cpu_baseline"] = cpu_baseline(m, blocks0.cpu().numpy(), meta0.cpu().numpy().view(np.uint32), rows, cols,
                                           xs[1].cpu().numpy(), w_np=w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
