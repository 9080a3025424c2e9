"""Host-side checks of the C-ABI library: it loads, exports what include/wave.h
declares, plans like the oracle lays segments out, refuses bad arguments before
any launch, and draws the same seed points as the oracle.  No GPU needed."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from oracle import wave_oracle as wo
from paper_2505_02922_amd import binding as wb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "wave.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wave_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(wb.EXPORTS), names
    L = wb.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_struct_layout_matches_header():
    # 14 int32 fields, 9 pointers, 5 int32 fields (the index update's and the capacities), padded
    # to the pointers' alignment
    assert ctypes.sizeof(wb.wave_index) == 14 * 4 + 9 * 8 + 5 * 4 + 4
    assert wb.wave_index.centroids.offset == 56
    assert wb.wave_index.appended_segments.offset == 56 + 72


@pytest.mark.parametrize("N0,ns,nl,L,k,n_new,U,ku", [(5000, 4, 64, 1024, 64, 1, 256, 16),
                                                     (5000, 4, 64, 1024, 64, 255, 256, 16),
                                                     (5000, 4, 64, 1024, 64, 256, 256, 16),
                                                     (5000, 4, 64, 1024, 64, 1500, 256, 300),
                                                     (70, 4, 64, 1024, 64, 700, 128, 8),
                                                     (5000, 0, 0, 1024, 64, 600, 128, 8)])
def test_append_plan_matches_oracle_layout(N0, ns, nl, L, k, n_new, U, ku):
    """Host only: the planned dimensions of a grown index against the oracle's bookkeeping,
    once in one step and once in two."""
    c0, _, _, _ = wb.wave_index_plan(torch.bfloat16, 2, 3, 128, N0, ns, nl, L, k)
    L_ = wb.lib()

    def plan(c_old, n):
        c = wb.wave_index()
        sizes = (ctypes.c_size_t * 9)()
        wsb = ctypes.c_size_t(0)
        st = L_.wave_index_append_plan(ctypes.byref(c_old), n, nl, U, ku, ctypes.byref(c), sizes,
                                       ctypes.byref(wsb))
        assert st == 0, st
        return c, list(sizes), wsb.value

    p0 = wo.make_plan(N0, ns, nl, L, k)
    lc0 = N0 - p0.local_start
    F = max(0, (lc0 + n_new - nl) // U)
    c1, sizes, wsb = plan(c0, n_new)
    assert c1.N == N0 + n_new and c1.appended_segments == F
    assert c1.n_local == lc0 + n_new - F * U and c1.p == p0.n_sink + c1.n_local
    assert (c1.S, c1.m, c1.N_idx) == (p0.S + F, p0.m + F * min(ku, U), p0.N_idx + F * U)
    assert sizes[2] == 6 * c1.m * 4 and sizes[5] == 6 * c1.N_idx * 256 and sizes[7] == 6 * c1.p * 256
    assert (wsb > 0) == (F > 0)
    half = n_new // 2
    ca, _, _ = plan(c0, half)
    cb, _, _ = plan(ca, n_new - half)
    assert (cb.N, cb.n_local, cb.S, cb.m, cb.N_idx, cb.appended_segments) == \
           (c1.N, c1.n_local, c1.S, c1.m, c1.N_idx, c1.appended_segments)
    # decode accepts the grown index's dimensions (workspace planning goes through the same checks)
    sizes2 = (ctypes.c_size_t * 9)()
    dws = ctypes.c_size_t(0)
    assert L_.wave_index_plan(ctypes.byref(c1), sizes2, None, 12, 7, ctypes.byref(dws)) == 0 and dws.value > 0
    # another update segment length on an index that already has update segments is refused
    if F > 0:
        c = wb.wave_index()
        st = L_.wave_index_append_plan(ctypes.byref(c1), 5, nl, U + 1, ku, ctypes.byref(c),
                                       (ctypes.c_size_t * 9)(), None)
        assert st == 2


@pytest.mark.parametrize("N,ns,nl,L,k", [(4096, 4, 64, 2048, 128), (32768, 4, 1024, 8192, 512),
                                           (122880, 4, 1024, 8192, 512), (1048576, 4, 1024, 8192, 512),
                                           (50, 4, 64, 2048, 128), (100, 4, 64, 2048, 128),
                                           (700, 0, 0, 256, 300), (513, 1, 0, 256, 16)])
def test_plan_matches_oracle_layout(N, ns, nl, L, k):
    c, sizes, bws, dws = wb.wave_index_plan(torch.bfloat16, 2, 3, 128, N, ns, nl, L, k, Hq=12,
                                            topk_clusters=7)
    p = wo.make_plan(N, ns, nl, L, k)
    assert (c.S, c.m, c.N_idx, c.p) == (p.S, p.m, p.N_idx, p.steady_positions.size)
    u = 6
    assert sizes == [u * p.m * 128 * 2, u * p.m * 128 * 2, u * p.m * 4, u * (p.m + 1) * 4,
                     u * p.N_idx * 4, u * p.N_idx * 128 * 2, u * p.N_idx * 128 * 2,
                     u * c.p * 128 * 2, u * c.p * 128 * 2]
    assert dws > 0 and (bws > 0) == (p.m > 0)


def test_row_capacity_in_the_plan():
    """Room for more permuted rows than the index holds: sizes of perm / k_perm / v_perm follow the
    capacity, too small a capacity is refused, and the plan of an update keeps it while it fits."""
    c, sizes, _, _ = wb.wave_index_plan(torch.bfloat16, 2, 3, 128, 5000, 4, 64, 1024, 64, row_capacity=6000)
    assert c.N_idx == 4932 and c.row_capacity == 6000
    assert sizes[4] == 6 * 6000 * 4 and sizes[5] == sizes[6] == 6 * 6000 * 256
    assert sizes[0] == 6 * c.m * 256                      # the meta index stays dense
    with pytest.raises(wb.WaveError) as e:
        wb.wave_index_plan(torch.bfloat16, 2, 3, 128, 5000, 4, 64, 1024, 64, row_capacity=4000)
    assert e.value.status == 2
    c2, sizes2, _, _ = wb.wave_index_plan(torch.bfloat16, 2, 3, 128, 5000, 4, 64, 1024, 64, steady_capacity=100)
    assert c2.p == 68 and sizes2[7] == sizes2[8] == 6 * 100 * 256
    with pytest.raises(wb.WaveError) as e:
        wb.wave_index_plan(torch.bfloat16, 2, 3, 128, 5000, 4, 64, 1024, 64, steady_capacity=67)
    assert e.value.status == 2
    L_ = wb.lib()
    for n_new, stays in ((32, True), (33, False)):         # 68 + 32 rows fill the room exactly
        cn = wb.wave_index()
        st = L_.wave_index_append_plan(ctypes.byref(c2), n_new, 64, 256, 16, ctypes.byref(cn),
                                       (ctypes.c_size_t * 9)(), None)
        assert st == 0 and cn.p == 68 + n_new and cn.steady_capacity == (100 if stays else 0)
    for n_new, keeps in ((1024, True), (1300, False)):    # 4 or 5 update segments of 256 rows
        cn = wb.wave_index()
        st = L_.wave_index_append_plan(ctypes.byref(c), n_new, 64, 256, 16, ctypes.byref(cn),
                                       (ctypes.c_size_t * 9)(), None)
        assert st == 0 and cn.N_idx == 4932 + 256 * (n_new // 256)
        assert cn.row_capacity == (6000 if keeps else 0), (n_new, cn.row_capacity)


def test_cluster_capacity_in_the_plan():
    """Room for more clusters than the index holds: the four meta-index arrays follow the capacity,
    too small a capacity is refused, and the plan of an update keeps it while the clusters fit."""
    c, sizes, _, _ = wb.wave_index_plan(torch.bfloat16, 2, 3, 128, 5000, 4, 64, 1024, 64, cluster_capacity=400)
    assert c.m == 320 and c.cluster_capacity == 400      # 4 full segments + 836 tokens: 5 x 64 clusters
    assert sizes[0] == sizes[1] == 6 * 400 * 256 and sizes[2] == 6 * 400 * 4 and sizes[3] == 6 * 401 * 4
    assert sizes[5] == 6 * c.N_idx * 256                  # the rows stay dense
    with pytest.raises(wb.WaveError) as e:
        wb.wave_index_plan(torch.bfloat16, 2, 3, 128, 5000, 4, 64, 1024, 64, cluster_capacity=319)
    assert e.value.status == 2
    with pytest.raises(wb.WaveError) as e:
        wb.wave_index_plan(torch.bfloat16, 2, 3, 128, 5000, 4, 64, 1024, 64, cluster_capacity=-1)
    assert e.value.status == 1
    L_ = wb.lib()
    for n_new, keeps in ((1280, True), (1536, False)):    # 5 or 6 update segments of 16 clusters
        cn = wb.wave_index()
        st = L_.wave_index_append_plan(ctypes.byref(c), n_new, 64, 256, 16, ctypes.byref(cn),
                                       (ctypes.c_size_t * 9)(), None)
        assert st == 0 and cn.m == 320 + 16 * (n_new // 256)
        assert cn.cluster_capacity == (400 if keeps else 0), (n_new, cn.cluster_capacity)


def test_status_strings():
    for code in range(7):
        assert len(wb.lib().wave_status_string(code)) > 0


def _plan_struct(**kw):
    args = dict(dtype=torch.bfloat16, B=1, Hkv=2, d=128, N=5000, n_sink=4, n_local=64,
                segment_len=1024, clusters_per_segment=64)
    args.update(kw)
    return wb.wave_index_plan(**args)


def test_plan_rejects_bad_shapes():
    for kw, code in [(dict(d=96), 2), (dict(clusters_per_segment=8193), 2), (dict(B=0), 1),
                     (dict(segment_len=0), 1), (dict(n_sink=-1), 1)]:
        with pytest.raises(wb.WaveError) as e:
            _plan_struct(**kw)
        assert e.value.status == code, kw
    with pytest.raises(wb.WaveError) as e:
        _plan_struct(Hq=5, topk_clusters=3)      # 5 query heads over 2 KV heads
    assert e.value.status == 2
    with pytest.raises(wb.WaveError) as e:
        _plan_struct(Hq=18, topk_clusters=3)     # G = 9 > 8
    assert e.value.status == 2
    with pytest.raises(wb.WaveError):
        wb.wave_index_plan(torch.float16, 1, 1, 128, 100, 0, 0, 10, 2)


def test_entry_points_refuse_bad_arguments_on_the_host():
    """All of these must return before anything is launched (no GPU here)."""
    L = wb.lib()
    c, sizes, bws, dws = _plan_struct(Hq=8, topk_clusters=4)
    fake = ctypes.c_void_p(0x1000)    # never dereferenced: checks fail first
    # null K
    assert L.wave_index_build(None, fake, ctypes.byref(c), 10, 0, fake, bws, None) == 1
    # iters < 1
    assert L.wave_index_build(fake, fake, ctypes.byref(c), 0, 0, fake, bws, None) == 1
    # index buffers missing
    assert L.wave_index_build(fake, fake, ctypes.byref(c), 10, 0, fake, bws, None) == 1
    for name in wb.BUFFER_NAMES:
        setattr(c, name, 0x1000)
    # workspace too small / misaligned / null
    assert L.wave_index_build(fake, fake, ctypes.byref(c), 10, 0, fake, bws - 1, None) == 4
    assert L.wave_index_build(fake, fake, ctypes.byref(c), 10, 0, ctypes.c_void_p(0x1010), bws, None) == 4
    assert L.wave_index_build(fake, fake, ctypes.byref(c), 10, 0, None, bws, None) == 4
    # planned fields tampered with
    c.m += 1
    assert L.wave_index_build(fake, fake, ctypes.byref(c), 10, 0, fake, bws, None) == 2
    c.m -= 1
    # decode: steady mismatch, bad Hq, small workspace, negative topk
    dec = lambda Hq, topk, ns, nl, wsb: L.wave_attention_decode(fake, ctypes.byref(c), Hq, topk, ns, nl,
                                                                fake, fake, None, fake, wsb, None)
    assert dec(8, 4, 4, 65, dws) == 5
    assert dec(8, 4, 5, 64, dws) == 5
    assert dec(7, 4, 4, 64, dws) == 2
    assert dec(8, -1, 4, 64, dws) == 1
    assert dec(8, 4, 4, 64, dws - 1) == 4
    # a larger topk needs a larger workspace than the one planned for topk = 4
    assert dec(8, 60, 4, 64, dws) == 4
    # the entry point with the static scratch array: same checks, and a step that does not fit
    sdec = lambda Hq, topk, ns, nl: L.wave_attention_decode_static(fake, ctypes.byref(c), Hq, topk, ns, nl,
                                                                   fake, fake, None, None)
    assert sdec(8, 4, 4, 65) == 5 and sdec(7, 4, 4, 64) == 2 and sdec(8, -1, 4, 64) == 1
    assert L.wave_attention_decode_static(None, ctypes.byref(c), 8, 4, 4, 64, fake, fake, None, None) == 1
    assert L.wave_attention_decode_static_capacity() == 64 << 20
    cb, _, _, dwb = wb.wave_index_plan(torch.bfloat16, 64, 8, 128, 8192 * 32 + 1028, 4, 1024, 8192, 512,
                                       Hq=32, topk_clusters=100)
    assert dwb > 64 << 20
    for name in wb.BUFFER_NAMES:
        setattr(cb, name, 0x1000)
    assert L.wave_attention_decode_static(fake, ctypes.byref(cb), 32, 100, 4, 1024, fake, fake, None,
                                          None) == 4
    # full attention: workspace size formula, bad shapes, small workspace
    need = L.wave_full_attention_workspace(2, 8, 5000, 128)
    assert need >= 4 * 2 * 8 * 5 * 130 and need % 256 == 0
    assert L.wave_full_attention_workspace(2, 8, 5000, 96) == 0
    full = lambda dt, Hq, Hkv, d, wsb: L.wave_full_attention_decode(fake, fake, fake, dt, 2, Hq, Hkv,
                                                                    5000, d, fake, fake, fake, wsb, None)
    assert full(9, 8, 2, 128, need) == 3
    assert full(1, 8, 3, 128, need) == 2
    assert full(1, 8, 2, 96, need) == 2
    assert full(1, 8, 2, 128, need - 1) == 4
    assert L.wave_full_attention_decode(None, fake, fake, 1, 2, 8, 2, 5000, 128, fake, fake, fake, need,
                                        None) == 1
    # assign-step hook
    assert L.wave_kmeans_assign_step(fake, fake, 1, 100, 200, 128, fake, fake, 1 << 20, None) == 2
    assert L.wave_kmeans_assign_step(fake, fake, 7, 100, 10, 128, fake, fake, 1 << 20, None) == 3
    assert L.wave_kmeans_assign_step(fake, fake, 1, 100, 10, 128, fake, fake, 100, None) == 4


def test_init_indices_match_the_oracle():
    grid = [(0, 0, 0, 0, 2048, 128), (0, 0, 0, 1, 1980, 128), (7, 3, 5, 11, 8192, 512),
            (2 ** 63 + 5, 15, 7, 14, 7164, 512), (1, 0, 0, 0, 40, 40), (9, 2, 1, 0, 1, 1),
            (123456789, 63, 3, 7, 300, 299), (5, 0, 1, 2, 8192, 1)]
    for seed, b, h, s, L_s, k_s in grid:
        got = wb.wave_init_indices(seed, b, h, s, L_s, k_s)
        want = wo.init_indices(seed, b, h, s, L_s, k_s).tolist()
        assert got == want, (seed, b, h, s, L_s, k_s)
    with pytest.raises(wb.WaveError):
        wb.wave_init_indices(0, 0, 0, 0, 10, 11)


def test_product_path_does_not_touch_the_oracle():
    """The package (binding, build script, input generators) neither imports nor names the
    oracle: only tests, the smoke check and the benchmark's baseline leg may."""
    pkg = os.path.join(ROOT, "paper_2505_02922_amd")
    for base, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(base, f)).read()
                assert "wave_oracle" not in text and "import oracle" not in text and "from oracle" not in text, f


def test_bench_touches_the_oracle_only_in_its_cpu_baseline_leg():
    """bench.py may import the oracle (or the test helpers that import it) only inside
    cpu_baseline(): everything timed or reported for the GPU path runs without it."""
    import ast
    tree = ast.parse(open(os.path.join(ROOT, "bench.py")).read())

    def names_oracle(node):
        if isinstance(node, ast.Import):
            return any(a.name.split(".")[0] in ("oracle", "tests") for a in node.names)
        if isinstance(node, ast.ImportFrom):
            return (node.module or "").split(".")[0] in ("oracle", "tests")
        return False

    inside = set()
    for fn in ast.walk(tree):
        if isinstance(fn, ast.FunctionDef) and fn.name == "cpu_baseline":
            inside = {id(n) for n in ast.walk(fn)}
    assert inside, "bench.py has no cpu_baseline()"
    hits = [n for n in ast.walk(tree) if names_oracle(n)]
    assert hits and all(id(n) in inside for n in hits), [n.lineno for n in hits if id(n) not in inside]
    text = open(os.path.join(ROOT, "bench.py")).read()
    assert text.count("wave_oracle") == 1


def test_workload_retrieve_count_matches_the_oracle():
    from oracle import wave_oracle as wo
    from paper_2505_02922_amd import synth
    for wl in synth.WORKLOADS.values():
        for m in (1, 37, 256, 2048, 4096, 7680, 8192, 65536):
            want = wl.retrieve_abs if wl.retrieve_abs is not None else wo.retrieve_count(wl.retrieve_frac, m)
            assert wl.retrieve_count(m) == want


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_append_refuses_bad_arguments_on_the_host():
    """Returns before anything is launched (no GPU here)."""
    L_ = wb.lib()
    c0, _, _, _ = wb.wave_index_plan(torch.bfloat16, 1, 2, 128, 5000, 4, 64, 1024, 64)
    cn = wb.wave_index()
    sizes = (ctypes.c_size_t * 9)()
    wsb = ctypes.c_size_t(0)
    plan = lambda n, nl, U, ku: L_.wave_index_append_plan(ctypes.byref(c0), n, nl, U, ku, ctypes.byref(cn),
                                                          sizes, ctypes.byref(wsb))
    assert plan(-1, 64, 256, 16) == 1 and plan(10, -1, 256, 16) == 1
    assert plan(10, 64, 0, 16) == 1 and plan(10, 64, 256, 0) == 1
    assert plan(10, 64, 256, 8193) == 2
    assert plan(300, 64, 256, 16) == 0 and cn.appended_segments == 1 and wsb.value > 0
    fake = ctypes.c_void_p(0x1000)
    for name in wb.BUFFER_NAMES:
        setattr(c0, name, 0x1000)
        setattr(cn, name, 0x2000)
    app = lambda new, ws, wsbytes, iters=3: L_.wave_index_append(
        ctypes.byref(c0), fake, fake, 300, 64, 256, 16, iters, 0, ctypes.byref(new), ws, wsbytes, None)
    assert app(cn, fake, wsb.value - 1) == 4            # workspace too small
    assert app(cn, None, wsb.value) == 4                # no workspace
    assert app(cn, fake, wsb.value, iters=0) == 1
    cn.m += 1                                           # not the plan of this update
    assert app(cn, fake, wsb.value) == 2
    cn.m -= 1
    cn.k_perm = c0.k_perm                               # rows in place without room for them
    assert app(cn, fake, wsb.value) == 1
    cn.k_perm = 0x2000
    cn.centroids = c0.centroids                         # clusters in place without room for them
    assert app(cn, fake, wsb.value) == 1
    cn.centroids = 0x2000
    # an update that flushes nothing may share the clustered arrays, but not at other strides
    cs = wb.wave_index()
    assert L_.wave_index_append_plan(ctypes.byref(c0), 10, 64, 256, 16, ctypes.byref(cs), sizes, None) == 0
    assert cs.appended_segments == 0
    for name in wb.BUFFER_NAMES:
        setattr(cs, name, 0x2000 if name in ("k_steady", "v_steady") else 0x1000)
    small = lambda new: L_.wave_index_append(ctypes.byref(c0), fake, fake, 10, 64, 256, 16, 3, 0,
                                             ctypes.byref(new), None, 0, ctypes.c_void_p(1))
    cs.cluster_capacity = cs.m + 8
    assert small(cs) == 1
    cs.cluster_capacity = 0
    cs.row_capacity = cs.N_idx + 8
    assert small(cs) == 1
    c0.appended_segments = 0
    # an index that holds update segments cannot be rebuilt by the plain build
    cn2 = wb.wave_index()
    ctypes.memmove(ctypes.byref(cn2), ctypes.byref(cn), ctypes.sizeof(wb.wave_index))
    assert L_.wave_index_build(fake, fake, ctypes.byref(cn2), 3, 0, fake, 1 << 30, None) == 2
