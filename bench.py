#!/usr/bin/env python3
"""Benchmark of the wave-index hot path on one MI355X.

One "step" is one decode call of the whole batch (all sequences, all query
heads of one layer) over an index that was built once, on device, before the
timed region; the build itself is timed separately and reported in the same
JSON line.  Inputs (K, V, 16 rotating query sets) are generated on the GPU and
are resident in HBM when timing starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Prints ONE JSON line ("Measurement").
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
N_QUERY_SETS = 16


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def segment_study() -> int:
    """Index build time and recall@100 against the segment length (Evaluation, "Impact of
    Different Segment Sizes"), on one llama-shaped sequence of 128K indexed tokens with one
    centroid per 16 tokens.  The library takes at most 4096 clusters per segment, so the longest
    segment is 64K tokens (two segments); the paper's 128K point (one global k-means) is not
    reachable.  Prints one JSON line of its own."""
    import torch
    from paper_2505_02922_amd import binding as wb
    from paper_2505_02922_amd import synth
    from tests import parity_util as pu

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    wb.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    base = synth.WORKLOADS["llama8b_120k_b16"]
    n_idx = 131072
    wl0 = synth.scaled(base, name="llama8b_128k_b1", B=1, N=n_idx + base.n_sink + base.n_local)
    K, V = synth.make_kv(wl0, device=dev)
    n_q = 8
    queries = [synth.make_queries(wl0, i, device=dev) for i in range(n_q)]
    rows = []
    for L in (1024, 2048, 4096, 8192, 16384, 32768, 65536):
        wl = synth.scaled(wl0, segment_len=L, clusters_per_segment=L // 16)
        ix = wb.alloc_index(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                            wl.segment_len, wl.clusters_per_segment, dev)
        bws = wb.workspace(ix.build_ws_bytes, dev)

        def build():
            wb.wave_index_build(K, V, wl.n_sink, wl.n_local, wl.segment_len,
                                wl.clusters_per_segment, wl.iters, 0, ws=bws, index=ix)

        build()
        torch.cuda.synchronize()
        ms = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            build()
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        r = pu.retrieve_count(wl)
        rec = []
        for q in queries:
            _, _, sel = wb.wave_attention_decode(q, ix, r, want_selected=True)
            torch.cuda.synchronize()
            rec.append(pu.recall_at_gpu(q, ix, sel, wl.Hq, top=100).mean().item())
        rows.append({"segment_len": L, "clusters_per_segment": L // 16, "m": ix.m, "r": r,
                     "build_ms": round(_median(ms), 3),
                     "recall_at_100": round(sum(rec) / len(rec), 4)})
        print(f"segment_len {L}: build {rows[-1]['build_ms']} ms, recall@100 "
              f"{rows[-1]['recall_at_100']}", file=sys.stderr, flush=True)
        del ix, bws
        torch.cuda.empty_cache()
    print(json.dumps({"study": "segment size vs index build time vs recall@100",
                      "config": {"workload": wl0.name, "B": 1, "Hq": wl0.Hq, "Hkv": wl0.Hkv,
                                 "d": wl0.d, "N_indexed": n_idx, "iters": wl0.iters,
                                 "tokens_per_cluster": 16, "query_sets": n_q,
                                 "retrieve_frac": wl0.retrieve_frac},
                      "dtype": wl0.dtype, "data": "synthetic", "rows": rows}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama8b_120k_b16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=32)
    ap.add_argument("--calibrate", action="store_true",
                    help="also run the library's plain copy/read kernels over 1 GiB (profiler runs "
                         "scale their counters by what these read)")
    ap.add_argument("--only", choices=["all", "build", "decode"], default="all",
                    help="build: stop after the index build (for profiler runs); "
                         "decode: build once untimed, then only the decode phase")
    ap.add_argument("--segment-study", action="store_true",
                    help="instead of the benchmark: index build time and recall@100 for segment "
                         "lengths 1K..64K on one 128K-token sequence")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: every (sequence, KV head) unit is independent and "
              "this build has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        return 2

    if args.segment_study:
        return segment_study()

    import numpy as np
    import torch
    from paper_2505_02922_amd import binding as wb
    from paper_2505_02922_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    wb.lib()   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = synth.WORKLOADS[args.workload]
    es = 2 if wl.dtype == "bf16" else 4

    # ---------------- inputs, resident in HBM ----------------
    K, V = synth.make_kv(wl, device=dev)
    queries = [synth.make_queries(wl, i, device=dev) for i in range(N_QUERY_SETS)]
    torch.cuda.synchronize()

    calib = None
    if args.calibrate:
        nb = 1 << 30
        src = torch.empty(nb, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        res = {}
        for name, fn in (("copy", lambda: wb.wave_calibration_copy(dst, src, 8192)),
                         ("read", lambda: wb.wave_calibration_read(src, sink, 8192))):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                fn()
            e1.record()
            torch.cuda.synchronize()
            res[name + "_GBps"] = round((2 if name == "copy" else 1) * nb / (e0.elapsed_time(e1) / 5) / 1e6, 1)
        calib = {"bytes": nb, **res}
        del src, dst

    # ---------------- index build ----------------
    ix = wb.alloc_index(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                        wl.segment_len, wl.clusters_per_segment, dev)
    bws = wb.workspace(ix.build_ws_bytes, dev)

    def build():
        wb.wave_index_build(K, V, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment,
                            wl.iters, 0, ws=bws, index=ix)

    build()
    torch.cuda.synchronize()
    build_ms = []
    for _ in range(3 if args.only != "decode" else 0):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        build()
        e1.record()
        torch.cuda.synchronize()
        build_ms.append(e0.elapsed_time(e1))
    build_prof = {}
    if args.only != "decode":
        wb.wave_profile_enable(True)
        build()
        build_prof = wb.wave_profile_read()
        wb.wave_profile_enable(False)
    plan_full = ix.N_idx // wl.segment_len
    tail = ix.N_idx - plan_full * wl.segment_len
    kk = min(wl.clusters_per_segment, wl.segment_len)
    assign_flops = 2.0 * wl.d * wl.iters * wl.B * wl.Hkv * (
        plan_full * wl.segment_len * kk + tail * min(kk, tail))
    assign_name = "assign_mfma" if wl.dtype == "bf16" else "assign_plain"
    assign_ms, assign_n = build_prof.get(assign_name, (0.0, 0))
    build_info = {
        "ms": round(_median(build_ms), 3) if build_ms else None,
        "assign_flops": assign_flops,
        "assign_ms_per_launch": round(assign_ms / max(assign_n, 1), 4),
        "assign_tflops": round(assign_flops / max(assign_ms, 1e-9) / 1e9, 2),
        "assign_frac_of_bf16_peak": round(assign_flops / max(assign_ms, 1e-9) / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
        "assign_share_of_build": round(assign_ms / max(sum(v[0] for v in build_prof.values()), 1e-9), 3),
        "kernels_ms": {k: round(v[0], 3) for k, v in sorted(build_prof.items())},
    }
    del bws
    torch.cuda.empty_cache()
    if args.only == "build":
        print(json.dumps({"workload": wl.name, "build": build_info}))
        return 0

    # ---------------- decode ----------------
    from tests import parity_util as pu
    r = pu.retrieve_count(wl)
    dws = wb.workspace(wb.decode_workspace_bytes(ix, wl.Hq, r), dev)
    out = torch.empty(wl.B, wl.Hq, wl.d, dtype=torch.float32, device=dev)
    lse = torch.empty(wl.B, wl.Hq, dtype=torch.float32, device=dev)
    sel = torch.empty(wl.B, wl.Hq, max(r, 1), dtype=torch.int32, device=dev)

    def step(i):
        wb.wave_attention_decode(queries[i % N_QUERY_SETS], ix, r, out=out, lse=lse, selected=sel, ws=dws)

    # retrieved tokens per query set (for the algorithmic byte count)
    sizes = ix.sizes.to(torch.int64)                     # [B, Hkv, m]
    retrieved_tokens = []
    for i in range(N_QUERY_SETS):
        step(i)
        torch.cuda.synchronize()
        ids = sel.to(torch.int64)                        # [B, Hq, r], -1 padded
        sz = sizes.repeat_interleave(wl.G, dim=1)        # [B, Hq, m]
        tok = torch.where(ids >= 0, sz.gather(2, ids.clamp(min=0)), torch.zeros_like(ids)).sum()
        retrieved_tokens.append(int(tok))
    mean_tokens = sum(retrieved_tokens) / len(retrieved_tokens)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = e0.elapsed_time(e1) / args.steps

    # per-kernel durations, same loop with the library's event profiler on
    wb.wave_profile_enable(True)
    for i in range(args.profile_steps):
        step(i)
    dec_prof = wb.wave_profile_read()
    wb.wave_profile_enable(False)

    units = wl.B * wl.Hkv
    row = wl.d * es
    meta = 2 * (units * ix.m * row) + units * ix.m * 4      # C and VS once per KV head, sizes
    steady_b = 2 * units * ix.p * row
    gather_b = 2 * mean_tokens * row
    bytes_k = {                      # algorithmic bytes by kernel (either launch split)
        "meta_index": meta, "steady": steady_b, "gather": gather_b, "select_gather": gather_b,
        "select_gather_steady": gather_b + steady_b, "select": 0, "merge": 0,
        "scores": meta // 2, "select_slices+side": steady_b, "select+side": meta // 2,
        "gather+merge": gather_b, "meta_index+steady": meta + steady_b,
    }
    step_bytes = meta + steady_b + gather_b
    kern = {k: v[0] / max(v[1], 1) for k, v in dec_prof.items()}      # ms per launch
    dominant = max(kern, key=kern.get)
    dom_gbs = bytes_k.get(dominant, 0) / (kern[dominant] * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        tk = json.load(open(tpath)).get(wl.name, {}).get(dominant)
        if tk:
            traffic = tk["fetch_bytes"] + tk["write_bytes"]
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(dom_gbs, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
                "traffic": traffic, "bytes_per_launch": int(bytes_k.get(dominant, 0)),
                "ms_per_launch": round(kern[dominant], 5)}
    decode_info = {
        "algorithmic_bytes_per_step": int(step_bytes),
        "step_GBps": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_frac_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "retrieved_tokens_per_step": round(mean_tokens, 1),
        "kernels_ms_per_launch": {k: round(v, 5) for k, v in sorted(kern.items())},
        "kernels_GBps": {k: round(bytes_k.get(k, 0) / (v * 1e-3) / 1e9, 1) for k, v in sorted(kern.items())
                         if bytes_k.get(k, 0)},
        "host_wall_ms_per_step": round(wall_ms / args.steps, 5),
    }

    # ---------------- brute-force full attention on the same inputs (context) ----------------
    fws = wb.workspace(wb.wave_full_attention_workspace(wl.B, wl.Hq, wl.N, wl.d), dev)
    fout, flse = torch.empty_like(out), torch.empty_like(lse)
    nfull = 10
    for i in range(2):
        wb.wave_full_attention_decode(queries[i], K, V, out=fout, lse=flse, ws=fws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(nfull):
        wb.wave_full_attention_decode(queries[i % N_QUERY_SETS], K, V, out=fout, lse=flse, ws=fws)
    e1.record()
    torch.cuda.synchronize()
    full_ms = e0.elapsed_time(e1) / nfull
    full_bytes = 2 * units * wl.N * row
    step(0)
    wb.wave_full_attention_decode(queries[0], K, V, out=fout, lse=flse, ws=fws)
    torch.cuda.synchronize()
    full_info = {
        "ms_per_step": round(full_ms, 4), "bytes_per_step": int(full_bytes),
        "GBps": round(full_bytes / (full_ms * 1e-3) / 1e9, 1),
        "wave_index_speedup": round(full_ms / ms_per_step, 2),
        "max_abs_diff_of_outputs": float((out - fout).abs().max()),
        "rel_l2_diff_of_outputs": float((out - fout).norm() / fout.norm()),
        "note": "brute-force decode attention over all N tokens with this library's own kernel on the "
                "same inputs; the difference of outputs is the approximation error of the method at "
                "this budget on synthetic data, not a parity figure",
    }
    del fws
    # zone budgets (estimation zone restricted to a share of the clusters; untuned launches)
    budgets = []
    for share in (0.0, 0.232):
        e = int(round(share * ix.m))
        bws2 = wb.workspace(wb.wave_attention_decode_budget_workspace(ix, wl.Hq, r, e), dev)
        bout, blse = torch.empty_like(out), torch.empty_like(lse)
        for i in range(2):
            wb.wave_attention_decode_budget(queries[0], ix, r, e, out=bout, lse=blse, ws=bws2)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(10):
            wb.wave_attention_decode_budget(queries[0], ix, r, e, out=bout, lse=blse, ws=bws2)
        e1.record()
        torch.cuda.synchronize()
        budgets.append({"estimated_share_of_clusters": share, "est_clusters": e,
                        "ms_per_step": round(e0.elapsed_time(e1) / 10, 4),
                        "rel_l2_diff_to_full_attention": float((bout - fout).norm() / fout.norm())})
        del bws2
    budgets.append({"estimated_share_of_clusters": "all other clusters", "est_clusters": ix.m - r,
                    "ms_per_step": round(ms_per_step, 4),
                    "rel_l2_diff_to_full_attention": full_info["rel_l2_diff_of_outputs"]})
    full_info["zone_budgets"] = budgets
    # retrieval-zone sweep (the same query set; every other cluster estimated)
    sweep = []
    for frac in (0.0, 0.005, 0.01, 0.018, 0.036, 0.072):
        rr = int(round(frac * ix.m))
        sws = wb.workspace(wb.decode_workspace_bytes(ix, wl.Hq, rr), dev)
        sout, slse = torch.empty_like(out), torch.empty_like(lse)
        for i in range(2):
            wb.wave_attention_decode(queries[0], ix, rr, out=sout, lse=slse, ws=sws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(10):
            wb.wave_attention_decode(queries[0], ix, rr, out=sout, lse=slse, ws=sws)
        e1.record()
        torch.cuda.synchronize()
        sweep.append({"retrieved_share_of_clusters": frac, "r": rr,
                      "ms_per_step": round(e0.elapsed_time(e1) / 10, 4),
                      "rel_l2_diff_to_full_attention": float((sout - fout).norm() / fout.norm())})
        del sws
    full_info["retrieval_sweep"] = sweep

    # ---------------- index update during decoding (context) ----------------
    # One update segment of 1024 new tokens per sequence (the paper's update segment size),
    # 64 clusters, clustered and appended; the grown index is a new set of arrays.
    U_UPD = 1024
    g = torch.Generator(device=dev)
    g.manual_seed(99)
    Kn = torch.randn(wl.B, wl.Hkv, U_UPD, wl.d, generator=g, device=dev).to(wl.torch_dtype())
    Vn = torch.randn(wl.B, wl.Hkv, U_UPD, wl.d, generator=g, device=dev).to(wl.torch_dtype())
    upd_ms = []
    for _ in range(3):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ix2 = wb.wave_index_append(ix, Kn, Vn, wl.n_local, U_UPD, U_UPD // 16, wl.iters, 0)
        e1.record()
        torch.cuda.synchronize()
        upd_ms.append(e0.elapsed_time(e1))
        assert ix2.m == ix.m + U_UPD // 16 and ix2.n_local == wl.n_local
        del ix2
        torch.cuda.empty_cache()
    # the same with room for the new rows in the permuted key/value arrays (row_capacity): the
    # rows are added in place and only the meta index and the steady rows are rewritten
    ixc = wb.alloc_index(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                         wl.segment_len, wl.clusters_per_segment, dev, row_capacity=ix.N_idx + U_UPD,
                         steady_capacity=ix.p + U_UPD)
    bws3 = wb.workspace(ixc.build_ws_bytes, dev)
    wb.wave_index_build(K, V, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment,
                        wl.iters, 0, ws=bws3, index=ixc)
    torch.cuda.synchronize()
    del bws3
    upd_cap_ms = []
    for _ in range(3):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ix2 = wb.wave_index_append(ixc, Kn, Vn, wl.n_local, U_UPD, U_UPD // 16, wl.iters, 0)
        e1.record()
        torch.cuda.synchronize()
        upd_cap_ms.append(e0.elapsed_time(e1))
        assert ix2.k_perm.data_ptr() == ixc.k_perm.data_ptr() and ix2.m == ix.m + U_UPD // 16
        del ix2
    # one new token per sequence (a decode step's own key and value): with room in the steady
    # buffers its rows go behind the window and nothing else is touched
    ixt = ixc
    wb.wave_profile_enable(True)
    for i in range(8):
        ixt = wb.wave_index_append(ixt, Kn[:, :, i:i + 1], Vn[:, :, i:i + 1], wl.n_local, U_UPD,
                                   U_UPD // 16, wl.iters, 0)
        assert ixt.k_steady.data_ptr() == ixc.k_steady.data_ptr() and ixt.p == ix.p + i + 1
    tok_prof = wb.wave_profile_read()
    wb.wave_profile_enable(False)
    tok_ms = [sum(v[0] for v in tok_prof.values()) / 8]
    del ixt, ixc
    torch.cuda.empty_cache()
    update_info = {
        "new_tokens_per_sequence": U_UPD, "update_segment_len": U_UPD, "update_clusters": U_UPD // 16,
        "dense_arrays": {
            "ms": round(_median(upd_ms), 3),
            "share_of_the_decode_steps_it_follows": round(_median(upd_ms) / (U_UPD * ms_per_step), 5),
            "note": "allocates the grown index and copies every old array to its strides"},
        "rows_in_place": {
            "ms": round(_median(upd_cap_ms), 3),
            "share_of_the_decode_steps_it_follows": round(_median(upd_cap_ms) / (U_UPD * ms_per_step), 5),
            "note": "row_capacity leaves room in perm / k_perm / v_perm: new rows go behind the old "
                    "ones, only the meta index and the steady rows are rewritten"},
        "one_token_in_place": {
            "ms": round(_median(tok_ms), 4),
            "share_of_a_decode_step": round(_median(tok_ms) / ms_per_step, 4),
            "note": "steady_capacity leaves room behind the local window: the token's key and value "
                    "rows are written there, every other array is shared with the index before "
                    "(kernel time by the library's event profiler; one small launch)"},
    }
    del Kn, Vn

    # ---------------- CPU baseline: the oracle on a bounded sample ----------------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import wave_oracle as wo
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        sample_units = [(0, h) for h in range(min(wl.Hkv, 2 if wl.N > 200000 else 4))]
        Kh = {u: K[u[0], u[1]].double().cpu().numpy() for u in sample_units}
        Vh = {u: V[u[0], u[1]].double().cpu().numpy() for u in sample_units}
        plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
        t0 = time.perf_counter()
        ref = {u: wo.build_unit(Kh[u], Vh[u], plan, wl.iters, 0, u[0], u[1], wl.dtype)
               for u in sample_units}
        t_build = time.perf_counter() - t0
        nsets = 4
        qh = [queries[i].double().cpu().numpy() for i in range(nsets)]
        heads = [(u, u[1] * wl.G + g) for u in sample_units for g in range(wl.G)]
        t0 = time.perf_counter()
        ref_out = {}
        for i in range(nsets):
            for (u, hq) in heads:
                ref_out[(i, u[0], hq)] = wo.decode_unit(qh[i][u[0], hq], ref[u], r)
        t_dec = time.perf_counter() - t0
        per_head = t_dec / (nsets * len(heads))
        cpu = {"value": round(1.0 / (per_head * wl.B * wl.Hq), 4), "unit": "steps/s", "cores": cores,
               "kind": "oracle",
               "sample": f"{len(heads)} of {wl.B * wl.Hq} (sequence, query head) units x {nsets} "
                         f"query sets, scaled linearly to the whole batch; index of "
                         f"{len(sample_units)} of {units} units built by the oracle first",
               "oracle_build_s_per_unit": round(t_build / len(sample_units), 3),
               "oracle_build_s_whole_batch_extrapolated": round(t_build / len(sample_units) * units, 1),
               "oracle_decode_ms_per_head": round(per_head * 1e3, 3)}
        # parity of the benchmarked configuration on the sampled units
        worst, lworst, same_sel, same_index = 0.0, 0.0, True, True
        for u in sample_units:
            same_index &= bool(np.array_equal(ix.sizes[u[0], u[1]].cpu().numpy(), ref[u].sizes) and
                               np.array_equal(ix.perm[u[0], u[1]].cpu().numpy(), ref[u].perm))
        for i in range(nsets):
            step(i)
            torch.cuda.synchronize()
            o_g, l_g, s_g = out.cpu().numpy(), lse.cpu().numpy(), sel.cpu().numpy()
            for (u, hq) in heads:
                o, l, s = ref_out[(i, u[0], hq)]
                worst = max(worst, float(np.abs(o_g[u[0], hq] - o).max()))
                lworst = max(lworst, abs(float(l_g[u[0], hq]) - l))
                same_sel &= bool(np.array_equal(s_g[u[0], hq][s_g[u[0], hq] >= 0], s))
        parity = {"sampled_heads": len(heads), "query_sets": nsets, "index_equal": same_index,
                  "selected_equal": same_sel, "out_max_abs_err": worst, "lse_max_abs_err": lworst}

    line = {
        "metric": "decode attention steps/sec at 120K ctx" if wl.name == "llama8b_120k_b16"
                  else f"decode attention steps/sec ({wl.name})",
        "value": round(1e3 / ms_per_step, 2), "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "Hq": wl.Hq, "Hkv": wl.Hkv, "d": wl.d, "N": wl.N,
                   "segment_len": wl.segment_len, "clusters_per_segment": wl.clusters_per_segment,
                   "iters": wl.iters, "m": ix.m, "topk_clusters": r, "n_sink": wl.n_sink,
                   "n_local": wl.n_local},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "decode": decode_info,
        "build": build_info,
        "full_attention": full_info,
        "index_update": update_info,
        "parity": parity,
        "calibration": calib,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
