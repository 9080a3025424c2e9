#!/usr/bin/env python3
"""Benchmark of the wave-index hot path on one MI355X.

One "step" is one decode call of the whole batch (all sequences, all query
heads of one layer) over an index that was built once, on device, before the
timed region; the build itself is timed separately and reported in the same
JSON line.  Inputs (K, V, 16 rotating query sets) are generated on the GPU and
are resident in HBM when timing starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Prints ONE JSON line.  The headline workload is the 120K-token x 16-sequence
one; the 1M-token and the Qwen-shaped workloads follow in the same line under
`other_workloads` (decode step, build, sampled parity), each measured the same
way on the same binary.
"""
from __future__ import annotations

import argparse
import dataclasses
import hashlib
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
HEADLINE = "llama8b_120k_b16"
OTHER_WORKLOADS = ("llama8b_1m", "qwen7b_64k_b64")


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def _event_ms(fn, reps):
    """Mean milliseconds of fn() over `reps` calls, by events on torch's current stream (the
    stream the binding launches on)."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def kernel_sources_sha256() -> str:
    """Hash of the kernel sources the library was built from: recorded counter figures are
    only quoted for the sources they were measured on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2505_02922_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".h")):
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()


def recorded_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` from the committed counter runs (profiles/traffic.json),
    or None when they were taken on other kernel sources than the ones present."""
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(tpath):
        return None
    rec = json.load(open(tpath))
    if rec.get("kernel_sources_sha256") != kernel_sources_sha256():
        return None
    tk = rec.get(workload, {}).get(kernel)
    return tk["fetch_bytes"] + tk["write_bytes"] if tk else None


def recall_at_gpu(q, ix, sel, Hq, top=100):
    """recall@top per query head from the device index, with torch ops (a measurement,
    not part of the library): of the `top` indexed tokens with the largest q . K_j, the
    share lying in the head's selected clusters.  q [B,Hq,d], sel [B,Hq,r] (-1 padded).
    Returns a [B,Hq] float tensor."""
    import torch
    B, Hkv = ix.B, ix.Hkv
    G = Hq // Hkv
    out = torch.zeros(B, Hq, device=q.device)
    for b in range(B):
        for h in range(Hkv):
            Kp = ix.k_perm[b, h, :ix.N_idx].float()                       # [N_idx, d]
            off = ix.offsets[b, h].to(torch.int64)                        # [m + 1]
            n = Kp.shape[0]
            k = min(top, n)
            if k == 0:
                out[b, h * G:(h + 1) * G] = 1.0
                continue
            # cluster of every row: offsets are ascending, empty clusters repeat a value
            row_cluster = torch.searchsorted(off, torch.arange(n, device=q.device), right=True) - 1
            for g in range(G):
                hq = h * G + g
                scores = Kp @ q[b, hq].float()
                best = torch.topk(scores, k).indices
                ids = sel[b, hq].to(torch.int64)
                chosen = torch.zeros(ix.m + 1, dtype=torch.bool, device=q.device)
                chosen[ids[ids >= 0]] = True
                out[b, hq] = chosen[row_cluster[best]].float().mean()
    return out


def segment_study() -> int:
    """Index build time and recall@100 against the segment length (Evaluation, "Impact of
    Different Segment Sizes"), on one llama-shaped sequence of 128K indexed tokens with one
    centroid per 16 tokens, from 1K-token segments up to one segment over the whole sequence
    (global k-means, the study's baseline).  Prints one JSON line of its own."""
    import torch
    from paper_2505_02922_amd import binding as wb
    from paper_2505_02922_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    wb.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    base = synth.WORKLOADS[HEADLINE]
    n_idx = 131072
    wl0 = synth.scaled(base, name="llama8b_128k_b1", B=1, N=n_idx + base.n_sink + base.n_local)
    K, V = synth.make_kv(wl0, device=dev)
    n_q = 8
    queries = [synth.make_queries(wl0, i, device=dev) for i in range(n_q)]
    rows = []
    for L in (1024, 2048, 4096, 8192, 16384, 32768, 65536, 131072):
        wl = synth.scaled(wl0, segment_len=L, clusters_per_segment=L // 16)
        try:
            ix = wb.alloc_index(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                                wl.segment_len, wl.clusters_per_segment, dev)
        except wb.WaveError as e:   # more clusters per segment than the library takes
            print(f"segment_len {L}: {e}", file=sys.stderr, flush=True)
            continue
        bws = wb.workspace(ix.build_ws_bytes, dev)

        def build(_=0):
            wb.wave_index_build(K, V, wl.n_sink, wl.n_local, wl.segment_len,
                                wl.clusters_per_segment, wl.iters, 0, ws=bws, index=ix)

        build()
        torch.cuda.synchronize()
        ms = [_event_ms(build, 1) for _ in range(3)]
        r = wl.retrieve_count(ix.m)
        rec = []
        for q in queries:
            _, _, sel = wb.wave_attention_decode(q, ix, r, want_selected=True)
            torch.cuda.synchronize()
            rec.append(recall_at_gpu(q, ix, sel, wl.Hq, top=100).mean().item())
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


# ---------------------------------------------------------------------------------------------
# Phases of the benchmark of one workload
# ---------------------------------------------------------------------------------------------
def build_phase(wb, wl, K, V, dev, timed: bool):
    """Builds the index (once untimed; then 3 timed repeats and one profiled call when `timed`)."""
    import torch
    ix = wb.alloc_index(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                        wl.segment_len, wl.clusters_per_segment, dev)
    bws = wb.workspace(ix.build_ws_bytes, dev)

    def build(_=0):
        wb.wave_index_build(K, V, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment,
                            wl.iters, 0, ws=bws, index=ix)

    build()
    torch.cuda.synchronize()
    if not timed:
        del bws
        torch.cuda.empty_cache()
        return ix, None
    build_ms = [_event_ms(build, 1) for _ in range(3)]
    wb.wave_profile_enable(True)
    build()
    prof = wb.wave_profile_read()
    wb.wave_profile_enable(False)
    plan_full = ix.N_idx // wl.segment_len
    tail = ix.N_idx - plan_full * wl.segment_len
    kk = min(wl.clusters_per_segment, wl.segment_len)
    assign_flops = 2.0 * wl.d * wl.iters * wl.B * wl.Hkv * (
        plan_full * wl.segment_len * kk + tail * min(kk, tail))
    assign_name = "assign_mfma" if wl.dtype == "bf16" else "assign_plain"
    assign_ms, assign_n = prof.get(assign_name, (0.0, 0))
    info = {"ms": round(_median(build_ms), 3), "assign_flops": assign_flops,
            "assign_ms_per_launch": None, "assign_tflops": None, "assign_frac_of_bf16_peak": None,
            "assign_share_of_build": None,
            "kernels_ms": {k: round(v[0], 3) for k, v in sorted(prof.items())}}
    if assign_n > 0 and assign_ms > 0:
        info["assign_ms_per_launch"] = round(assign_ms / assign_n, 4)
        info["assign_tflops"] = round(assign_flops / assign_ms / 1e9, 2)
        info["assign_frac_of_bf16_peak"] = round(assign_flops / assign_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)
        info["assign_share_of_build"] = round(assign_ms / sum(v[0] for v in prof.values()), 3)
    del bws
    torch.cuda.empty_cache()
    return ix, info


class DecodeRun:
    """Buffers and the step function of one workload's decode benchmark."""

    def __init__(self, wb, wl, ix, queries, dev):
        import torch
        self.wb, self.wl, self.ix, self.queries = wb, wl, ix, queries
        self.r = wl.retrieve_count(ix.m)
        self.ws = wb.workspace(wb.decode_workspace_bytes(ix, wl.Hq, self.r), dev)
        self.out = torch.empty(wl.B, wl.Hq, wl.d, dtype=torch.float32, device=dev)
        self.lse = torch.empty(wl.B, wl.Hq, dtype=torch.float32, device=dev)
        self.sel = torch.empty(wl.B, wl.Hq, max(self.r, 1), dtype=torch.int32, device=dev)

    def step(self, i):
        self.wb.wave_attention_decode(self.queries[i % N_QUERY_SETS], self.ix, self.r, out=self.out,
                                      lse=self.lse, selected=self.sel, ws=self.ws)


def decode_phase(run: DecodeRun, steps: int, warmup: int, profile_steps: int):
    """Times `steps` decode steps and returns (ms per step, decode info, roofline of the dominant
    kernel)."""
    import torch
    wb, wl, ix = run.wb, run.wl, run.ix
    es = 2 if wl.dtype == "bf16" else 4
    # retrieved tokens per query set (for the algorithmic byte count)
    sizes = ix.sizes.to(torch.int64)                     # [B, Hkv, m]
    retrieved_tokens = []
    for i in range(N_QUERY_SETS):
        run.step(i)
        torch.cuda.synchronize()
        ids = run.sel.to(torch.int64)                    # [B, Hq, r], -1 padded
        sz = sizes.repeat_interleave(wl.G, dim=1)        # [B, Hq, m]
        tok = torch.where(ids >= 0, sz.gather(2, ids.clamp(min=0)), torch.zeros_like(ids)).sum()
        retrieved_tokens.append(int(tok))
    mean_tokens = sum(retrieved_tokens) / len(retrieved_tokens)
    del sizes

    for i in range(warmup):
        run.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_per_step = _event_ms(run.step, steps)
    wall_ms = (time.perf_counter() - t0) * 1e3

    # per-kernel durations, same loop with the library's event profiler on (HIP events recorded
    # on the launch stream around every kernel)
    wb.wave_profile_enable(True)
    for i in range(profile_steps):
        run.step(i)
    dec_prof = wb.wave_profile_read()
    wb.wave_profile_enable(False)

    units = wl.B * wl.Hkv
    row = wl.d * es
    cbytes = units * ix.m * row                             # centroids (= value sums) once per KV head
    meta = 2 * cbytes + units * ix.m * 4                    # C and VS once per KV head, sizes
    steady_b = 2 * units * ix.p * row
    gather_b = 2 * mean_tokens * row
    bytes_k = {                      # algorithmic bytes by kernel (whichever launches the step uses)
        "meta_index": meta, "steady": steady_b, "gather": gather_b,
        "select_gather_steady": gather_b + steady_b, "select": 0, "merge": 0,
        "scores": cbytes + units * ix.m * 4, "select_slices+side": steady_b, "select+side": cbytes,
        "meta_index+steady": meta + steady_b,
        "scores+steady": cbytes + units * ix.m * 4 + steady_b, "select+estimate+steady": cbytes + steady_b,
        "gather+estimate": gather_b + cbytes,
    }
    step_bytes = meta + steady_b + gather_b
    kern = {k: v[0] / max(v[1], 1) for k, v in dec_prof.items()}      # ms per launch
    roofline = None
    if kern:   # (no per-kernel profile was asked for: --profile-steps 0)
        dominant = max(kern, key=kern.get)
        dom_gbs = bytes_k.get(dominant, 0) / (kern[dominant] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(dom_gbs, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
                    "traffic": recorded_traffic(wl.name, dominant),
                    "traffic_source": "recorded rocprofv3 --pmc runs (profiles/traffic.json), quoted "
                                      "only when taken on the kernel sources present",
                    "bytes_per_launch": int(bytes_k.get(dominant, 0)),
                    "ms_per_launch": round(kern[dominant], 5)}
    info = {
        "ms_per_step": round(ms_per_step, 5),
        "steps_per_s": round(1e3 / ms_per_step, 2),
        "algorithmic_bytes_per_step": int(step_bytes),
        "step_GBps": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_frac_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "retrieved_tokens_per_step": round(mean_tokens, 1),
        "kernels_ms_per_launch": {k: round(v, 5) for k, v in sorted(kern.items())},
        "kernels_GBps": {k: round(bytes_k.get(k, 0) / (v * 1e-3) / 1e9, 1) for k, v in sorted(kern.items())
                         if bytes_k.get(k, 0)},
        "host_wall_ms_per_step": round(wall_ms / steps, 5),
    }
    return ms_per_step, info, roofline


def full_attention_phase(run: DecodeRun, K, V, ms_per_step, dev, sweeps: bool):
    """Brute-force full attention on the same inputs (context), the zone budgets of the paper's
    evaluation, and (sweeps) the retrieval-zone and steady-zone sweeps."""
    import torch
    wb, wl, ix, queries, r = run.wb, run.wl, run.ix, run.queries, run.r
    es = 2 if wl.dtype == "bf16" else 4
    units, row = wl.B * wl.Hkv, wl.d * es
    out, lse = run.out, run.lse
    fws = wb.workspace(wb.wave_full_attention_workspace(wl.B, wl.Hq, wl.N, wl.d), dev)
    fout, flse = torch.empty_like(out), torch.empty_like(lse)

    def full(i):
        wb.wave_full_attention_decode(queries[i % N_QUERY_SETS], K, V, out=fout, lse=flse, ws=fws)

    for i in range(2):
        full(i)
    torch.cuda.synchronize()
    full_ms = _event_ms(full, 10)
    full_bytes = 2 * units * wl.N * row
    run.step(0)
    full(0)
    torch.cuda.synchronize()
    info = {
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
    # zone budgets: estimation zone restricted to a share of the clusters (Evaluation,
    # "Parameters": 23.2 %; 0 = the ablation without estimation)
    cbytes = units * ix.m * row
    budgets = []
    for share in (0.0, 0.232):
        e = int(round(share * ix.m))
        bws2 = wb.workspace(wb.wave_attention_decode_budget_workspace(ix, wl.Hq, r, e), dev)
        bout, blse = torch.empty_like(out), torch.empty_like(lse)

        def bstep(i):
            wb.wave_attention_decode_budget(queries[i % N_QUERY_SETS], ix, r, e, out=bout, lse=blse, ws=bws2)

        for i in range(2):
            bstep(i)
        torch.cuda.synchronize()
        bms = _event_ms(bstep, 32)
        bstep(0)
        torch.cuda.synchronize()
        # algorithmic bytes: centroids and sizes, steady, retrieved rows as in the plain step,
        # and one value-sum row per estimated cluster and query head
        bbytes = (cbytes + units * ix.m * 4 + 2 * units * ix.p * row
                  + 2 * _retrieved_tokens(run) * row + wl.B * wl.Hq * e * row)
        budgets.append({"estimated_share_of_clusters": share, "est_clusters": e,
                        "ms_per_step": round(bms, 4),
                        "algorithmic_bytes_per_step": int(bbytes),
                        "step_frac_of_hbm_peak": round(bbytes / (bms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                        "rel_l2_diff_to_full_attention": float((bout - fout).norm() / fout.norm())})
        del bws2
    budgets.append({"estimated_share_of_clusters": "all other clusters", "est_clusters": ix.m - r,
                    "ms_per_step": round(ms_per_step, 4),
                    "rel_l2_diff_to_full_attention": info["rel_l2_diff_of_outputs"]})
    info["zone_budgets"] = budgets
    if not sweeps:
        return info
    # retrieval-zone sweep (the same query set; every other cluster estimated)
    sweep = []
    for frac in (0.0, 0.005, 0.01, 0.018, 0.036, 0.072):
        rr = int(round(frac * ix.m))
        sws = wb.workspace(wb.decode_workspace_bytes(ix, wl.Hq, rr), dev)
        sout, slse = torch.empty_like(out), torch.empty_like(lse)

        def sstep(i):
            wb.wave_attention_decode(queries[0], ix, rr, out=sout, lse=slse, ws=sws)

        for i in range(2):
            sstep(i)
        torch.cuda.synchronize()
        sms = _event_ms(sstep, 10)
        sweep.append({"retrieved_share_of_clusters": frac, "r": rr, "ms_per_step": round(sms, 4),
                      "rel_l2_diff_to_full_attention": float((sout - fout).norm() / fout.norm())})
        del sws
    info["retrieval_sweep"] = sweep
    return info


def _retrieved_tokens(run: DecodeRun) -> float:
    """Tokens in the clusters the last step selected, summed over all heads."""
    import torch
    ids = run.sel.to(torch.int64)
    sz = run.ix.sizes.to(torch.int64).repeat_interleave(run.wl.G, dim=1)
    return float(torch.where(ids >= 0, sz.gather(2, ids.clamp(min=0)), torch.zeros_like(ids)).sum())


def steady_sweep_phase(wb, wl, K, V, queries, fout, dev):
    """Steady-zone sizes (Evaluation, zone-size sensitivity: 4 sink tokens + 64 local tokens
    against larger windows): the index is rebuilt with each window, r and the estimation as in
    the headline step."""
    import torch
    rows = []
    for n_local in (64, 256, 1024):
        w2 = dataclasses.replace(wl, n_local=n_local)
        ix2, _ = build_phase(wb, w2, K, V, dev, timed=False)
        run2 = DecodeRun(wb, w2, ix2, queries, dev)
        for i in range(2):
            run2.step(i)
        torch.cuda.synchronize()
        ms = _event_ms(run2.step, 32)
        run2.step(0)
        torch.cuda.synchronize()
        rows.append({"n_sink": w2.n_sink, "n_local": n_local, "m": ix2.m, "r": run2.r,
                     "ms_per_step": round(ms, 4),
                     "rel_l2_diff_to_full_attention": float((run2.out - fout).norm() / fout.norm())})
        del run2, ix2
        torch.cuda.empty_cache()
    return rows


def index_update_phase(wb, wl, ix, K, V, ms_per_step, dev):
    """Index update during decoding (context): one update segment of 1024 new tokens per
    sequence (the paper's update segment size), 64 clusters, clustered and appended."""
    import torch
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
    # the same with room for the new rows and clusters (row_capacity, cluster_capacity): they are
    # added in place and only the steady rows are rewritten
    ixc = wb.alloc_index(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                         wl.segment_len, wl.clusters_per_segment, dev, row_capacity=ix.N_idx + U_UPD,
                         steady_capacity=ix.p + U_UPD, cluster_capacity=ix.m + U_UPD // 16)
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
        assert ix2.centroids.data_ptr() == ixc.centroids.data_ptr()
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
    return {
        "new_tokens_per_sequence": U_UPD, "update_segment_len": U_UPD, "update_clusters": U_UPD // 16,
        "dense_arrays": {
            "ms": round(_median(upd_ms), 3),
            "share_of_the_decode_steps_it_follows": round(_median(upd_ms) / (U_UPD * ms_per_step), 5),
            "note": "allocates the grown index and copies every old array to its strides"},
        "rows_in_place": {
            "ms": round(_median(upd_cap_ms), 3),
            "share_of_the_decode_steps_it_follows": round(_median(upd_cap_ms) / (U_UPD * ms_per_step), 5),
            "note": "row_capacity and cluster_capacity leave room in perm / k_perm / v_perm and in the "
                    "meta-index arrays: the new rows and clusters go behind the old ones, only the steady "
                    "rows are rewritten"},
        "one_token_in_place": {
            "ms": round(_median(tok_ms), 4),
            "share_of_a_decode_step": round(_median(tok_ms) / ms_per_step, 4),
            "note": "steady_capacity leaves room behind the local window: the token's key and value "
                    "rows are written there, every other array is shared with the index before "
                    "(kernel time by the library's event profiler; one small launch)"},
    }


def cpu_baseline(run: DecodeRun, K, V, n_units: int, nsets: int):
    """The CPU oracle on a bounded sample of the workload: timed (the reported baseline) and
    compared with the GPU results of the same units (parity of the benchmarked configuration).
    The only part of this file that touches the oracle."""
    import numpy as np
    import torch
    from oracle import wave_oracle as wo
    wl, ix, r, queries = run.wl, run.ix, run.r, run.queries
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    units = wl.B * wl.Hkv
    sample_units = [(0, h) for h in range(min(wl.Hkv, n_units))]
    Kh = {u: K[u[0], u[1]].double().cpu().numpy() for u in sample_units}
    Vh = {u: V[u[0], u[1]].double().cpu().numpy() for u in sample_units}
    plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
    assert wo.retrieve_count(wl.retrieve_frac, plan.m) == r and plan.m == ix.m
    t0 = time.perf_counter()
    ref = {u: wo.build_unit(Kh[u], Vh[u], plan, wl.iters, 0, u[0], u[1], wl.dtype)
           for u in sample_units}
    t_build = time.perf_counter() - t0
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
        for name in ("sizes", "offsets", "perm"):
            same_index &= bool(np.array_equal(getattr(ix, name)[u[0], u[1]].cpu().numpy(),
                                              np.asarray(getattr(ref[u], name))))
        for name in ("centroids", "vsum"):
            same_index &= bool(np.array_equal(getattr(ix, name)[u[0], u[1]].float().cpu().numpy(),
                                              np.asarray(getattr(ref[u], name), dtype=np.float32)))
    for i in range(nsets):
        run.step(i)
        torch.cuda.synchronize()
        o_g, l_g, s_g = run.out.cpu().numpy(), run.lse.cpu().numpy(), run.sel.cpu().numpy()
        for (u, hq) in heads:
            o, l, s = ref_out[(i, u[0], hq)]
            worst = max(worst, float(np.abs(o_g[u[0], hq] - o).max()))
            lworst = max(lworst, abs(float(l_g[u[0], hq]) - l))
            same_sel &= bool(np.array_equal(s_g[u[0], hq][s_g[u[0], hq] >= 0], s))
    parity = {"sampled_heads": len(heads), "query_sets": nsets, "index_equal": same_index,
              "selected_equal": same_sel, "out_max_abs_err": worst, "lse_max_abs_err": lworst}
    return cpu, parity


def other_workload(wb, synth, name, dev, args):
    """Decode step, build and sampled parity of another workload of the benchmark definition."""
    import torch
    wl = synth.WORKLOADS[name]
    print(f"[bench] {name}: inputs", file=sys.stderr, flush=True)
    K, V = synth.make_kv(wl, device=dev)
    queries = [synth.make_queries(wl, i, device=dev) for i in range(N_QUERY_SETS)]
    torch.cuda.synchronize()
    print(f"[bench] {name}: build", file=sys.stderr, flush=True)
    ix, build_info = build_phase(wb, wl, K, V, dev, timed=True)
    run = DecodeRun(wb, wl, ix, queries, dev)
    print(f"[bench] {name}: decode", file=sys.stderr, flush=True)
    ms_per_step, decode_info, roofline = decode_phase(run, args.steps, args.warmup, args.profile_steps)
    full = full_attention_phase(run, K, V, ms_per_step, dev, sweeps=False)
    parity = None
    if not args.no_cpu_baseline:
        print(f"[bench] {name}: oracle on a sample", file=sys.stderr, flush=True)
        _, parity = cpu_baseline(run, K, V, n_units=1 if wl.N > 200000 else 2, nsets=2)
    res = {"config": {"workload": wl.name, "B": wl.B, "Hq": wl.Hq, "Hkv": wl.Hkv, "d": wl.d, "N": wl.N,
                      "m": ix.m, "topk_clusters": run.r, "iters": wl.iters},
           "ms_per_step": round(ms_per_step, 5), "steps_per_s": round(1e3 / ms_per_step, 2),
           "bytes_per_step": decode_info["algorithmic_bytes_per_step"],
           "step_frac_of_hbm_peak": decode_info["step_frac_of_hbm_peak"],
           "dominant_kernel": roofline, "decode": decode_info, "build": build_info,
           "full_attention": full, "parity": parity}
    del run, ix, K, V, queries
    torch.cuda.empty_cache()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the 1M-token and Qwen-shaped workloads that follow the headline one")
    ap.add_argument("--profile-steps", type=int, default=32)
    ap.add_argument("--calibrate", action="store_true",
                    help="also run the library's plain copy/read kernels over 1 GiB (profiler runs "
                         "scale their counters by what these read)")
    ap.add_argument("--only", choices=["all", "build", "decode"], default="all",
                    help="build: stop after the index build (for profiler runs); "
                         "decode: build once untimed, then only the decode phase")
    ap.add_argument("--segment-study", action="store_true",
                    help="instead of the benchmark: index build time and recall@100 for segment "
                         "lengths 1K..128K on one 128K-token sequence")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: every (sequence, KV head) unit is independent and "
              "this build has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        return 2

    if args.segment_study:
        return segment_study()

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
        for name, fn in (("copy", lambda _: wb.wave_calibration_copy(dst, src, 8192)),
                         ("read", lambda _: wb.wave_calibration_read(src, sink, 8192))):
            fn(0)
            torch.cuda.synchronize()
            res[name + "_GBps"] = round((2 if name == "copy" else 1) * nb / _event_ms(fn, 5) / 1e6, 1)
        calib = {"bytes": nb, **res}
        del src, dst

    ix, build_info = build_phase(wb, wl, K, V, dev, timed=args.only != "decode")
    if args.only == "build":
        print(json.dumps({"workload": wl.name, "build": build_info}))
        return 0

    run = DecodeRun(wb, wl, ix, queries, dev)
    ms_per_step, decode_info, roofline = decode_phase(run, args.steps, args.warmup, args.profile_steps)
    if args.only == "decode":
        print(json.dumps({"workload": wl.name, "ms_per_step": round(ms_per_step, 5), "roofline": roofline,
                          "decode": decode_info, "calibration": calib}))
        return 0

    full_info = full_attention_phase(run, K, V, ms_per_step, dev, sweeps=True)
    fout = torch.empty_like(run.out)
    fws = wb.workspace(wb.wave_full_attention_workspace(wl.B, wl.Hq, wl.N, wl.d), dev)
    wb.wave_full_attention_decode(queries[0], K, V, out=fout, lse=torch.empty_like(run.lse), ws=fws)
    torch.cuda.synchronize()
    del fws
    full_info["steady_zone_sweep"] = steady_sweep_phase(wb, wl, K, V, queries, fout, dev)
    del fout
    update_info = index_update_phase(wb, wl, ix, K, V, ms_per_step, dev)

    cpu = parity = None
    if not args.no_cpu_baseline:
        cpu, parity = cpu_baseline(run, K, V, n_units=2 if wl.N > 200000 else 4, nsets=4)

    r, m = run.r, ix.m
    del run, ix, K, V, queries
    torch.cuda.empty_cache()
    others = {}
    if wl.name == HEADLINE and not args.no_other_workloads:
        for name in OTHER_WORKLOADS:
            others[name] = other_workload(wb, synth, name, dev, args)

    line = {
        "metric": "decode attention steps/sec at 120K ctx" if wl.name == HEADLINE
                  else f"decode attention steps/sec ({wl.name})",
        "value": round(1e3 / ms_per_step, 2), "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "Hq": wl.Hq, "Hkv": wl.Hkv, "d": wl.d, "N": wl.N,
                   "segment_len": wl.segment_len, "clusters_per_segment": wl.clusters_per_segment,
                   "iters": wl.iters, "m": m, "topk_clusters": r, "n_sink": wl.n_sink,
                   "n_local": wl.n_local},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "decode": decode_info,
        "build": build_info,
        "full_attention": full_info,
        "index_update": update_info,
        "parity": parity,
        "other_workloads": others,
        "calibration": calib,
        "kernel_sources_sha256": kernel_sources_sha256(),
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
