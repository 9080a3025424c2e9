"""Helpers shared by the GPU parity tests, the smoke check and the benchmark's
CPU-baseline leg: run the oracle on a workload, move an oracle index to the
device, compare results under the stated tolerances."""
from __future__ import annotations

import math
from typing import Dict, List, Tuple

import numpy as np
import torch

from oracle import wave_oracle as wo
from paper_2505_02922_amd import synth

# Attention outputs: bf16 inputs with fp32 accumulation (the benchmark definition's bar).
OUT_MAX_ABS = 2e-3
OUT_REL = 1e-2
# f32 inputs: fp32 accumulation of a few thousand terms.
OUT_MAX_ABS_F32 = 2e-4
TIE_REL = 1e-6


def oracle_build(wl: synth.Workload, K: torch.Tensor, V: torch.Tensor, seed: int = 0,
                 units=None) -> Dict[Tuple[int, int], wo.UnitIndex]:
    """Oracle index of the given (b, h) units (default: all)."""
    plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
    units = units or [(b, h) for b in range(wl.B) for h in range(wl.Hkv)]
    out = {}
    for (b, h) in units:
        out[(b, h)] = wo.build_unit(K[b, h].double().cpu().numpy(), V[b, h].double().cpu().numpy(),
                                    plan, wl.iters, seed, b, h, wl.dtype)
    return out


def retrieve_count(wl: synth.Workload) -> int:
    plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
    if wl.retrieve_abs is not None:
        return wl.retrieve_abs
    return wo.retrieve_count(wl.retrieve_frac, plan.m)


def oracle_index_arrays(wl: synth.Workload, index: Dict[Tuple[int, int], wo.UnitIndex]
                        ) -> Dict[str, torch.Tensor]:
    """Stack the per-unit oracle arrays into the [B, Hkv, ...] layout of the C struct."""
    names = ("centroids", "vsum", "sizes", "offsets", "perm", "k_perm", "v_perm", "k_steady",
             "v_steady")
    out = {}
    for n in names:
        rows = [[np.asarray(getattr(index[(b, h)], n)) for h in range(wl.Hkv)] for b in range(wl.B)]
        arr = np.stack([np.stack(r) for r in rows])
        out[n] = torch.from_numpy(arr.astype(np.int32) if n in ("sizes", "offsets", "perm")
                                  else arr.astype(np.float32))
    return out


def check_outputs(out_gpu: np.ndarray, lse_gpu: np.ndarray, out_ref: np.ndarray, lse_ref: np.ndarray,
                  dtype: str, what: str = "") -> Tuple[float, float]:
    max_abs = float(np.abs(out_gpu - out_ref).max())
    rel = float(np.linalg.norm(out_gpu - out_ref) / max(np.linalg.norm(out_ref), 1e-30))
    lse_err = float(np.abs(lse_gpu - lse_ref).max())
    bar = OUT_MAX_ABS if dtype == "bf16" else OUT_MAX_ABS_F32
    assert max_abs <= bar, f"{what}: max abs error {max_abs} > {bar}"
    assert rel <= OUT_REL, f"{what}: relative error {rel} > {OUT_REL}"
    assert lse_err <= bar + OUT_REL * 1e-2 * np.abs(lse_ref).max(), f"{what}: lse error {lse_err}"
    return max_abs, lse_err


def check_selected(sel_gpu: np.ndarray, sel_ref: np.ndarray, z_ref: np.ndarray, what: str = "") -> int:
    """Selected sets must agree except for clusters whose oracle score ties the
    r-th best oracle score within TIE_REL.  Returns the number of such swaps."""
    g = set(int(x) for x in sel_gpu if x >= 0)
    r = set(int(x) for x in sel_ref)
    assert len(g) == len(r), f"{what}: {len(g)} selected, oracle {len(r)}"
    assert sorted(g) == [int(x) for x in sel_gpu if x >= 0], f"{what}: ids not ascending/unique"
    diff = g ^ r
    if diff:
        zr = min(z_ref[c] for c in r)
        for c in diff:
            tol = TIE_REL * max(abs(z_ref[c]), abs(zr))
            assert abs(z_ref[c] - zr) <= tol, f"{what}: cluster {c} differs outside the tie band"
    return len(diff) // 2


def check_assign(a_gpu: np.ndarray, xhat: np.ndarray, chat: np.ndarray, what: str = "") -> int:
    """Assignments must equal the oracle's except where its two best
    similarities tie within TIE_REL.  Returns the number of tie differences."""
    scores = xhat @ chat.T
    a_ref = np.argmax(scores, axis=1)
    bad = np.nonzero(a_gpu != a_ref)[0]
    for j in bad:
        top = scores[j, a_ref[j]]
        assert abs(top - scores[j, a_gpu[j]]) <= TIE_REL * abs(top), \
            f"{what}: point {j}: gpu {a_gpu[j]} oracle {a_ref[j]} gap {top - scores[j, a_gpu[j]]}"
    return bad.size
