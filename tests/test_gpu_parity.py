"""GPU parity: the HIP path through the C ABI against the CPU oracle, element
by element on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

from oracle import wave_oracle as wo
from paper_2505_02922_amd import binding as wb
from paper_2505_02922_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

WL = synth.WORKLOADS


def _small(base, **kw):
    return synth.scaled(WL[base], **kw)


CASES = {
    # the tiny single-head f32 workload as defined
    "tiny_f32": WL["tiny_f32"],
    # bf16, GQA 4:1, d = 128, two full segments and a ragged tail, several score/gather tiles
    "bf16_g4": _small("llama8b_32k", name="bf16_g4", N=5000, Hq=8, Hkv=2, segment_len=2048,
                      clusters_per_segment=128, n_local=200, n_components=256, iters=4,
                      retrieve_frac=0.05),
    # GQA 7:1 with heavy-tailed channels, two sequences
    "bf16_g7": _small("qwen7b_64k_b64", name="bf16_g7", B=2, N=3000, Hq=7, Hkv=1, segment_len=1024,
                      clusters_per_segment=64, n_local=100, n_components=128, iters=3,
                      retrieve_frac=0.08),
    # d = 64 in bf16 (8 lanes per row) and G = 2
    "bf16_d64": _small("llama8b_32k", name="bf16_d64", d=64, N=2500, Hq=4, Hkv=2, segment_len=1024,
                       clusters_per_segment=100, n_local=50, n_components=128, iters=3,
                       retrieve_frac=0.1),
    # 384 query heads: selection and retrieval run fused in one workgroup per head
    "bf16_many_heads": _small("llama8b_32k", name="bf16_many_heads", B=48, N=1300, Hq=8, Hkv=2,
                              segment_len=512, clusters_per_segment=32, n_local=40, n_components=64,
                              iters=3, retrieve_frac=0.1),
    # 392 query heads, 7 per KV head: the fused selection + retrieval kernel at GQA 7:1
    "bf16_many_heads_g7": _small("qwen7b_64k_b64", name="bf16_many_heads_g7", B=28, N=900, Hq=14,
                                 Hkv=2, segment_len=400, clusters_per_segment=24, n_local=300,
                                 n_components=64, iters=2, retrieve_frac=0.1),
    # 800 query heads: selection in a launch of its own beside the estimation ranges, retrieval
    # from one work list of token ranges over all heads (uneven heads: outlier tokens make
    # large clusters)
    "bf16_listed_heads": _small("llama8b_32k", name="bf16_listed_heads", B=100, N=1100, Hq=8, Hkv=2,
                                segment_len=512, clusters_per_segment=32, n_local=40, n_components=48,
                                iters=2, retrieve_frac=0.1, outlier_token_frac=0.05,
                                outlier_token_scale=3.0),
    # the same path at 7 query heads per KV head (840 heads)
    "bf16_listed_heads_g7": _small("qwen7b_64k_b64", name="bf16_listed_heads_g7", B=60, N=700, Hq=14,
                                   Hkv=2, segment_len=300, clusters_per_segment=20, n_local=200,
                                   n_components=40, iters=2, retrieve_frac=0.15),
    # 600 clusters per segment: more centroid rows than fit in LDS at once, so the assign step
    # stages them tile by tile instead of keeping them resident
    "bf16_big_k": _small("llama8b_32k", name="bf16_big_k", N=2900, Hq=4, Hkv=1, segment_len=1400,
                         clusters_per_segment=600, n_local=60, n_components=512, iters=3,
                         retrieve_frac=0.05),
    # 4096 clusters per segment at 4 tokens per cluster,
    # with a ragged tail segment: the staged assign step and the two-wave counting sort
    "bf16_max_k": _small("llama8b_32k", name="bf16_max_k", N=19500, Hq=2, Hkv=1, segment_len=16384,
                         clusters_per_segment=4096, n_local=60, n_components=2048, iters=2,
                         retrieve_frac=0.02),
    # 8192 clusters in one segment (the library's limit; the segment-size study's global k-means
    # baseline clusters a whole 128K-token sequence this way), d = 64, a ragged second segment
    "bf16_k8192": _small("llama8b_32k", name="bf16_k8192", d=64, N=13000, Hq=2, Hkv=1, segment_len=12288,
                         clusters_per_segment=8192, n_local=40, n_components=4096, iters=2,
                         retrieve_frac=0.01),
    # d = 128 in f32 (32 lanes per row)
    "f32_d128": _small("tiny_f32", name="f32_d128", d=128, N=1500, Hq=2, Hkv=1, segment_len=512,
                       clusters_per_segment=32, n_local=30, iters=3, retrieve_abs=9),
}


def _inputs(wl, query_set=0):
    K, V = synth.make_kv(wl)
    q = synth.make_queries(wl, query_set)
    return K, V, q


def _decode_and_check(wl, ix_gpu, index_ref, q, r, what):
    out, lse, sel = wb.wave_attention_decode(q.cuda(), ix_gpu, r, want_selected=True)
    torch.cuda.synchronize()
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    sel = sel.cpu().numpy() if sel is not None else None
    qn = q.double().numpy()
    swaps = 0
    for b in range(wl.B):
        for hq in range(wl.Hq):
            parts = {}
            o, l, s = wo.decode_unit(qn[b, hq], index_ref[(b, hq // wl.G)], r, parts)
            tag = f"{what} b={b} hq={hq} r={r}"
            pu.check_outputs(out[b, hq], lse[b, hq:hq + 1], o, np.array([l]), wl.dtype, tag)
            if r > 0:
                swaps += pu.check_selected(sel[b, hq], s, parts["z"], tag)
    return swaps


@pytest.mark.parametrize("case", list(CASES))
def test_decode_on_oracle_index(case):
    """Decode kernels alone: the index is the oracle's, copied to the device, into arrays with
    room behind every unit's clusters, rows and steady rows (odd amounts: the kernels must take
    the units' strides from the capacities, not from m, N_idx and p)."""
    wl = CASES[case]
    K, V, q = _inputs(wl)
    index_ref = pu.oracle_build(wl, K, V)
    arrays = pu.oracle_index_arrays(wl, index_ref)
    plan = index_ref[(0, 0)].plan
    ix = wb.index_from_arrays(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                              wl.segment_len, wl.clusters_per_segment, arrays,
                              row_capacity=plan.N_idx + 3, steady_capacity=index_ref[(0, 0)].k_steady.shape[0] + 1,
                              cluster_capacity=plan.m + 5)
    assert ix.cluster_capacity == plan.m + 5
    m = ix.m
    for r in sorted({0, 1, pu.retrieve_count(wl), m // 2, m, m + 3}):
        _decode_and_check(wl, ix, index_ref, q, r, case)


@pytest.mark.parametrize("case", list(CASES))
def test_assign_step_teacher_forced(case):
    """One assign step on the oracle's normalised keys and centroids of every
    k-means round of the first segment."""
    wl = CASES[case]
    K, V, _ = _inputs(wl)
    plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
    for s in (0, plan.S - 1):
        lo, Ls, ks = plan.seg_start[s], plan.seg_len[s], plan.seg_k[s]
        trace = []
        wo.kmeans_segment(K[0, 0, lo:lo + Ls].double().numpy(), wo.init_indices(0, 0, 0, s, Ls, ks),
                          wl.iters, wl.dtype, trace)
        for t, (xhat, chat, a_ref) in enumerate(trace):
            xg = torch.from_numpy(xhat).to(wl.torch_dtype()).cuda()
            cg = torch.from_numpy(chat).to(wl.torch_dtype()).cuda()
            a = wb.wave_kmeans_assign_step(xg, cg)
            torch.cuda.synchronize()
            pu.check_assign(a.cpu().numpy(), xhat, chat, f"{case} seg {s} round {t}")


def _compare_index(wl, ix, index_ref, what):
    torch.cuda.synchronize()
    got = {n: ix.t[n].float().cpu().numpy() if ix.t[n].is_floating_point() else ix.t[n].cpu().numpy()
           for n in wb.BUFFER_NAMES}
    ties = 0
    for b in range(wl.B):
        for h in range(wl.Hkv):
            ref = index_ref[(b, h)]
            tag = f"{what} b={b} h={h}"
            # the partition: cluster of every indexed token, recovered from perm + offsets
            a_gpu = np.empty(ref.plan.N_idx, dtype=np.int64)
            sizes = got["sizes"][b, h]
            offs = got["offsets"][b, h]
            assert offs[0] == 0 and offs[-1] == ref.plan.N_idx, tag
            assert np.array_equal(np.diff(offs), sizes), tag
            perm = got["perm"][b, h]
            assert sorted(perm.tolist()) == list(range(ref.plan.n_sink, ref.plan.local_start)), tag
            a_gpu[perm - ref.plan.n_sink] = np.repeat(np.arange(ref.plan.m), sizes)
            if not np.array_equal(a_gpu, ref.assign):
                ties += int((a_gpu != ref.assign).sum())
                continue    # a legal tie flipped: later rounds may differ; counted below
            assert np.array_equal(sizes, ref.sizes), tag
            assert np.array_equal(perm, ref.perm), tag
            assert np.array_equal(got["k_perm"][b, h], ref.k_perm.astype(np.float32)), tag
            assert np.array_equal(got["v_perm"][b, h], ref.v_perm.astype(np.float32)), tag
            assert np.array_equal(got["centroids"][b, h], ref.centroids.astype(np.float32)), tag
            assert np.array_equal(got["vsum"][b, h], ref.vsum.astype(np.float32)), tag
            assert np.array_equal(got["k_steady"][b, h], ref.k_steady.astype(np.float32)), tag
            assert np.array_equal(got["v_steady"][b, h], ref.v_steady.astype(np.float32)), tag
    return ties


@pytest.mark.parametrize("case", list(CASES))
def test_build_matches_oracle_then_decode(case):
    """Whole path: GPU build, every index array against the oracle's, then GPU
    decode on the GPU-built index against the oracle's decode on its own."""
    wl = CASES[case]
    K, V, q = _inputs(wl)
    index_ref = pu.oracle_build(wl, K, V)
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, wl.iters, 0)
    ties = _compare_index(wl, ix, index_ref, case)
    assert ties == 0, f"{case}: {ties} points assigned differently from the oracle"
    _decode_and_check(wl, ix, index_ref, q, pu.retrieve_count(wl), case)


@pytest.mark.parametrize("case", ["bf16_g4", "bf16_g7", "bf16_d64", "bf16_many_heads_g7"])
def test_short_segments_build_the_same_index_launch_by_launch(case, monkeypatch):
    """Short segments are clustered by one workgroup per segment that runs all iterations (the
    default, which the other build tests cover); WAVE_NO_SMALL_KMEANS=1 keeps them on the kernels
    of the long segments, one launch per step.  Both against the oracle."""
    wl = CASES[case]
    K, V, _ = _inputs(wl)
    index_ref = pu.oracle_build(wl, K, V)
    monkeypatch.setenv("WAVE_NO_SMALL_KMEANS", "1")
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, wl.iters, 0)
    torch.cuda.synchronize()
    monkeypatch.delenv("WAVE_NO_SMALL_KMEANS")
    assert _compare_index(wl, ix, index_ref, case) == 0


def test_all_retrieved_is_full_attention():
    wl = CASES["bf16_g4"]
    K, V, q = _inputs(wl, 1)
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, 2, 5)
    out, lse, _ = wb.wave_attention_decode(q.cuda(), ix, ix.m)
    torch.cuda.synchronize()
    for hq in range(wl.Hq):
        o, l = wo.full_attention(q[0, hq].double().numpy(), K[0, hq // wl.G].double().numpy(),
                                 V[0, hq // wl.G].double().numpy())
        pu.check_outputs(out[0, hq].cpu().numpy(), lse[0, hq:hq + 1].cpu().numpy(), o, np.array([l]),
                         wl.dtype, f"full hq={hq}")


@pytest.mark.parametrize("N,n_sink,n_local,L,k", [
    (60, 4, 64, 256, 16),      # N <= p: no index at all, exact attention over everything
    (68, 4, 64, 256, 16),      # N == p
    (69, 4, 64, 256, 16),      # one indexed token
    (100, 4, 64, 256, 64),     # one short segment, k capped by its length (singleton clusters)
    (600, 0, 0, 256, 8),       # no steady zone
    (513, 1, 0, 256, 16),      # last segment of a single token
])
def test_degenerate_shapes(N, n_sink, n_local, L, k):
    wl = _small("llama8b_32k", name="deg", N=N, Hq=4, Hkv=2, n_sink=n_sink, n_local=n_local,
                segment_len=L, clusters_per_segment=k, n_components=16, iters=3)
    K, V, q = _inputs(wl)
    index_ref = pu.oracle_build(wl, K, V)
    ix = wb.wave_index_build(K.cuda(), V.cuda(), n_sink, n_local, L, k, wl.iters, 0)
    assert _compare_index(wl, ix, index_ref, "deg") == 0
    for r in (0, 2, 1000):
        _decode_and_check(wl, ix, index_ref, q, r, f"deg N={N}")


def test_duplicate_keys_and_empty_clusters():
    """Every key of a component identical: many exact ties in assign (lowest
    centroid wins, the others stay empty) and in the centroid scores."""
    wl = _small("llama8b_32k", name="dups", N=1200, Hq=4, Hkv=1, n_sink=2, n_local=10,
                segment_len=512, clusters_per_segment=48, n_components=20, iters=4, sigma=0.0,
                rope_base=None)
    K, V, q = _inputs(wl)
    index_ref = pu.oracle_build(wl, K, V)
    assert (index_ref[(0, 0)].sizes == 0).any()
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, wl.iters, 0)
    assert _compare_index(wl, ix, index_ref, "dups") == 0
    for r in (0, 3, 10, 40):
        _decode_and_check(wl, ix, index_ref, q, r, "dups")


@pytest.mark.parametrize("tiny_exp", [None, -40])
def test_large_clusters_are_summed_by_the_whole_workgroup(tiny_exp):
    """Clusters of several hundred tokens (a 4096-token segment into 8 clusters): their update
    is split over the groups of a workgroup, which equals the reference's one-by-one sum bit for
    bit when no addition can round.  Second case: one channel keeps a zero segment mean (values in
    +/- pairs) and holds values of 2^-40 beside values of order one, so that a cluster's sum over
    that channel spans more exponents than fp64 can add without rounding: the kernel notices and
    sums such a cluster one by one.  Every index array against the oracle's in both cases."""
    wl = _small("llama8b_32k", name="bf16_large_clusters", N=4 + 60 + 4096, Hq=2, Hkv=1, segment_len=4096,
                clusters_per_segment=8, n_local=60, n_components=8, iters=4, retrieve_abs=2)
    K, V, q = _inputs(wl)
    if tiny_exp is not None:
        g = torch.Generator().manual_seed(3)
        v = torch.randn(2048, generator=g)
        v[::3] *= 2.0 ** tiny_exp                      # a third of the pairs are tiny
        ch = torch.stack([v, -v], dim=1).reshape(-1)   # (+v, -v) side by side: every partial sum cancels
        K = K.clone()
        K[0, 0, wl.n_sink:wl.n_sink + 4096, 0] = ch.to(K.dtype)
    index_ref = pu.oracle_build(wl, K, V)
    assert index_ref[(0, 0)].sizes.max() > 128
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, wl.iters, 0)
    assert _compare_index(wl, ix, index_ref, wl.name) == 0
    _decode_and_check(wl, ix, index_ref, q, 2, wl.name)


def test_errors_surface_as_status_codes():
    wl = CASES["bf16_d64"]
    K, V, q = _inputs(wl)
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, 1, 0)
    with pytest.raises(wb.WaveError) as e:
        wb.wave_attention_decode(q.cuda(), ix, 4, n_sink=wl.n_sink + 1)
    assert e.value.status == 5
    with pytest.raises(wb.WaveError) as e:
        wb.wave_attention_decode(q.cuda(), ix, 4, ws=wb.workspace(256))
    assert e.value.status == 4
    torch.cuda.synchronize()


def _hand_index(m, d, dtype, n_steady, seed, dup_scores=False):
    """A random index that no k-means produced: sizes 0..3, centroids and value
    sums consistent with the member rows.  Decode only reads the arrays."""
    g = np.random.default_rng(seed)
    sizes = g.integers(0, 4, m)
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    n = int(offsets[-1])
    Kp = wo.quant(g.standard_normal((n, d)), dtype)
    Vp = wo.quant(g.standard_normal((n, d)), dtype)
    C = np.zeros((m, d))
    VS = np.zeros((m, d))
    for c in np.nonzero(sizes)[0]:
        C[c] = Kp[offsets[c]:offsets[c + 1]].mean(0)
        VS[c] = Vp[offsets[c]:offsets[c + 1]].sum(0)
    if dup_scores:   # many clusters with the very same centroid: exact score ties
        C[::7] = wo.quant(C[7], dtype)
        for c in range(0, m, 7):   # their rows are that centroid, so it still is their mean
            if c != 7:
                Kp[offsets[c]:offsets[c + 1]] = C[c]
    Ks = wo.quant(g.standard_normal((n_steady, d)), dtype)
    Vs = wo.quant(g.standard_normal((n_steady, d)), dtype)
    return dict(centroids=wo.quant(C, dtype), vsum=wo.quant(VS, dtype), sizes=sizes, offsets=offsets,
                perm=np.arange(n), k_perm=Kp, v_perm=Vp, k_steady=Ks, v_steady=Vs), n


@pytest.mark.parametrize("m,dup,Hq,dtype,d", [(3000, True, 2, "bf16", 128), (20000, False, 2, "bf16", 128),
                                              (40000, True, 2, "bf16", 128), (70000, False, 2, "bf16", 128),
                                              (20000, True, 7, "bf16", 128), (20000, True, 3, "f32", 128),
                                              (20000, False, 4, "bf16", 64), (70000, True, 2, "f32", 64)])
def test_decode_many_clusters_hand_index(m, dup, Hq, dtype, d):
    """Every size class of the selection (32-bit keys in LDS, slices + union, 16-bit keys
    in LDS, and the streaming fallback), with and without exact score ties; once with 7
    query heads on the KV head (the estimation and steady work beside the slices at G = 7)
    and once in f32 through the slices (scores and tile maxima without MFMA)."""
    p, Hkv = 8, 1
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    arrs, n = _hand_index(m, d, dtype, p, seed=m, dup_scores=dup)
    # Dimensions whose plan has exactly m clusters: segments of 4 tokens with one
    # cluster each.  The hand index then fills sizes/offsets as it likes (0..3 rows
    # per cluster); rows beyond its n are padding that no offset points at.
    L = 4
    c, sizes_b, bws, dws = wb.wave_index_plan(tdt, 1, Hkv, d, 4 * m + p, 4, p - 4, L, 1)
    assert c.m == m
    # rows of k_perm/v_perm are allocated for N_idx = 4 m >= n; pad the hand rows
    pad = c.N_idx - n
    arrs["k_perm"] = np.concatenate([arrs["k_perm"], np.zeros((pad, d))])
    arrs["v_perm"] = np.concatenate([arrs["v_perm"], np.zeros((pad, d))])
    arrs["perm"] = np.arange(c.N_idx)
    tens = {k: torch.from_numpy(np.asarray(v)[None, None].astype(
        np.int32 if k in ("sizes", "offsets", "perm") else np.float32)) for k, v in arrs.items()}
    ix = wb.index_from_arrays(tdt, 1, Hkv, d, 4 * m + p, 4, p - 4, L, 1, tens)
    plan = wo.make_plan(4 * m + p, 4, p - 4, L, 1)
    ref = wo.UnitIndex(plan, dtype, arrs["centroids"], arrs["vsum"], arrs["sizes"], arrs["offsets"],
                       arrs["perm"], arrs["k_perm"], arrs["v_perm"], arrs["k_steady"],
                       arrs["v_steady"], np.zeros(0, dtype=np.int64))
    g = np.random.default_rng(5)
    q = torch.from_numpy(wo.quant(g.standard_normal((1, Hq, d)) * 2.0, dtype).astype(np.float32)
                         ).to(tdt)
    if dup:   # head 0 looks straight at the shared centroid: the tied scores are the largest
        q[0, 0] = torch.from_numpy(wo.quant(arrs["centroids"][7] * 3.0, dtype).astype(np.float32)
                                   ).to(tdt)
    wl = _small("llama8b_32k", name="hand", B=1, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype)
    # r = 2000 at m = 20000: more clusters asked for than there are 16-cluster tiles, so
    # the slices' cheap first stage has no bound to offer and every slice is ranked exactly;
    # with the tied scores on top a slice holds more than r candidates, same fallback
    for r in (0, 5, 300, m) + ((2000,) if m == 20000 else ()):
        _decode_and_check(wl, ix, {(0, 0): ref}, q, r, f"hand m={m}")
    # the estimation budget through every selection size class as well
    qn = q.double().numpy()
    for r, e in ((300, 2000), (5, 5000)):
        out, lse, sel = wb.wave_attention_decode_budget(q.cuda(), ix, r, e, want_selected=True)
        torch.cuda.synchronize()
        for hq in range(Hq):
            parts = {}
            o, l, s_ref = wo.decode_unit(qn[0, hq], ref, r, parts, est_clusters=e)
            tag = f"hand m={m} budget r={r} e={e} hq={hq}"
            pu.check_outputs(out[0, hq].cpu().numpy(), lse[0, hq:hq + 1].cpu().numpy(), o, np.array([l]),
                             dtype, tag)
            pu.check_selected(sel[0, hq].cpu().numpy(), s_ref, parts["z"], tag)


def _decode_hand(arrs, n, m, d, dtype, q, r, Hq=2):
    """Decode on a hand-filled index of m clusters (one KV head) and the oracle on the same arrays."""
    p, Hkv = 8, 1
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    c, _, _, _ = wb.wave_index_plan(tdt, 1, Hkv, d, 4 * m + p, 4, p - 4, 4, 1)
    pad = c.N_idx - n
    arrs = dict(arrs)
    arrs["k_perm"] = np.concatenate([arrs["k_perm"], np.zeros((pad, d))])
    arrs["v_perm"] = np.concatenate([arrs["v_perm"], np.zeros((pad, d))])
    arrs["perm"] = np.arange(c.N_idx)
    tens = {k: torch.from_numpy(np.asarray(v)[None, None].astype(
        np.int32 if k in ("sizes", "offsets", "perm") else np.float32)) for k, v in arrs.items()}
    ix = wb.index_from_arrays(tdt, 1, Hkv, d, 4 * m + p, 4, p - 4, 4, 1, tens)
    plan = wo.make_plan(4 * m + p, 4, p - 4, 4, 1)
    ref = wo.UnitIndex(plan, dtype, arrs["centroids"], arrs["vsum"], arrs["sizes"], arrs["offsets"],
                       arrs["perm"], arrs["k_perm"], arrs["v_perm"], arrs["k_steady"],
                       arrs["v_steady"], np.zeros(0, dtype=np.int64))
    out, lse, sel = wb.wave_attention_decode(q.cuda(), ix, r, want_selected=True)
    torch.cuda.synchronize()
    qn = q.double().numpy()
    res = []
    for hq in range(Hq):
        parts = {}
        o, l, s_ref = wo.decode_unit(qn[0, hq], ref, r, parts)
        res.append((out[0, hq].cpu().numpy(), float(lse[0, hq]), sel[0, hq].cpu().numpy(), o, l, s_ref,
                    parts["z"]))
    return res


@pytest.mark.parametrize("m", [3000, 40000])
def test_decode_on_an_index_whose_centroids_are_not_the_member_means(m):
    """The decode step takes the selected clusters' estimation terms out of a sum over ALL
    clusters, which is exact only up to cancellation; the header states what the index must
    satisfy.  (a) Centroids a little off the mean (5 % noise: far more than storage rounding)
    still match the oracle, which never subtracts, on the same arrays.  (b) A centroid grossly
    off the mean, selected and dominating everything, is outside that contract; it must still
    not come back as a silent zero."""
    d, dtype = 128, "bf16"
    arrs, n = _hand_index(m, d, dtype, 8, seed=m + 1)
    g = np.random.default_rng(11)
    q = torch.from_numpy(wo.quant(g.standard_normal((1, 2, d)) * 1.5, dtype).astype(np.float32)
                         ).to(torch.bfloat16)
    off = g.random(m) < 0.3
    C = np.array(arrs["centroids"], dtype=np.float64)
    C[off] += 0.05 * g.standard_normal((int(off.sum()), d)) * np.abs(C[off]).mean()
    mild = dict(arrs, centroids=wo.quant(C, dtype))
    for r in (50, 300):
        for hq, (o_g, l_g, s_g, o, l, s_ref, z) in enumerate(_decode_hand(mild, n, m, d, dtype, q, r)):
            tag = f"mild m={m} r={r} hq={hq}"
            pu.check_outputs(o_g, np.array([l_g]), o, np.array([l]), dtype, tag)
            pu.check_selected(s_g, s_ref, z, tag)
    # (b) one non-empty cluster whose centroid points along q with a huge norm: its estimation
    # term is ~e^40 times everything else, it is selected, and its rows do not back it
    C2 = np.array(arrs["centroids"], dtype=np.float64)
    big = int(np.nonzero(arrs["sizes"])[0][5])
    C2[big] = q[0, 0].double().numpy() * 4.0
    gross = dict(arrs, centroids=wo.quant(C2, dtype))
    o_g, l_g, s_g, o, l, s_ref, z = _decode_hand(gross, n, m, d, dtype, q, 50)[0]
    assert big in set(int(x) for x in s_g)
    # outside the contract the header states: what is left after the cancellation is rounding
    # residue of the dominating term, positive or negative.  The one promise left is that a
    # normaliser that cancels to zero or below is reported as NaN, never as an output of zeros
    # with lse = -inf.
    assert not np.all(o_g == 0.0) and l_g != float("-inf")
    assert (np.isnan(o_g).all() and np.isnan(l_g)) or (np.isfinite(o_g).all() and np.isfinite(l_g))


@pytest.mark.parametrize("m,r", [(3000, 700), (3000, 1), (40000, 900)])
def test_more_near_equal_scores_than_the_candidate_list_holds(m, r):
    """1500 clusters whose centroids differ from one vector only in the last bf16 bit of three
    small-weight coordinates: 1500 scores, hundreds of them distinct, inside the fp32 error band around the
    selection threshold (fp32 accumulation orders them differently from fp64), more than the
    1024 the exact ranking keeps in LDS.  The selected set must still be the fp64 ranking's,
    ties to the lower id: here it is compared for equality, not up to a tie band."""
    d, dtype = 128, "bf16"
    g = np.random.default_rng(m + r)
    arrs, n = _hand_index(m, d, dtype, 8, seed=m + 7)
    # q: weight 1 on the first 64 coordinates, distinct small weights 2^-8 (1 + t / 128) on the others
    qv = np.ones(d)
    qv[64:] = 2.0 ** -8 * (1.0 + np.arange(64) / 128.0)
    c0 = np.ones(d)
    nb = 1500
    band_ids = np.sort(g.choice(np.nonzero(arrs["sizes"])[0], nb, replace=False))
    C = np.array(arrs["centroids"], dtype=np.float64) * 0.05      # every other cluster scores far lower
    Kp = np.array(arrs["k_perm"], dtype=np.float64)
    off = arrs["offsets"]
    for c in band_ids:
        row = c0.copy()
        for a in g.choice(64, 3, replace=False) + 64:
            row[a] += g.integers(-1, 2) * 2.0 ** -7               # one bf16 ulp of 1.0 up or down
        C[c] = row
        Kp[off[c]:off[c + 1]] = row                               # the rows are the centroid: still their mean
    arrs = dict(arrs, centroids=wo.quant(C, dtype), k_perm=wo.quant(Kp, dtype))
    assert np.array_equal(arrs["centroids"][band_ids], C[band_ids])   # exactly representable
    q = torch.from_numpy(np.stack([qv, wo.quant(g.standard_normal(d), dtype)])[None].astype(np.float32)
                         ).to(torch.bfloat16)
    zb = C[band_ids] @ qv
    assert np.unique(zb).size > 400                               # many distinct fp64 scores (and exact ties) ...
    assert zb.max() - zb.min() < 2 * 48 * 2.0 ** -24 * np.linalg.norm(qv) * np.linalg.norm(c0)   # ... inside the band
    res = _decode_hand(arrs, n, m, d, dtype, q, r)
    for hq, (o_g, l_g, s_g, o, l, s_ref, z) in enumerate(res):
        tag = f"band m={m} r={r} hq={hq}"
        assert np.array_equal(s_g[s_g >= 0], np.asarray(s_ref)), tag
        pu.check_outputs(o_g, np.array([l_g]), o, np.array([l]), dtype, tag)


def _used(ix, nm, b, h):
    """The entries in use of one unit's array (capacities leave room behind them)."""
    n = {"sizes": ix.m, "centroids": ix.m, "vsum": ix.m, "offsets": ix.m + 1, "perm": ix.N_idx,
         "k_perm": ix.N_idx, "v_perm": ix.N_idx, "k_steady": ix.p, "v_steady": ix.p}[nm]
    return ix.t[nm][b, h][:n]


@pytest.mark.parametrize("name,units", [("llama8b_120k_b16", [(0, 0), (15, 7)]),
                                        ("llama8b_32k", [(0, 0), (0, 3), (0, 7)]),
                                        ("llama8b_1m", [(0, 5)]),
                                        ("qwen7b_64k_b64", [(0, 0), (63, 3)])])
def test_full_size_workload_sampled_units(name, units):
    """The benchmark's own workloads at full size, in the launch configuration
    bench.py times: whole-batch GPU build and decode; the oracle builds and
    decodes the sampled (sequence, KV head) units from the same keys and values
    and every array of those units, their selected sets and outputs must agree.
    The 120K x 16 index is built with room for new rows and clusters, as the benchmark's
    index update has it: the update below then writes in place."""
    wl = WL[name]
    dev = torch.device("cuda")
    K, V = synth.make_kv(wl, device=dev)
    q = synth.make_queries(wl, 3, device=dev)
    plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
    U, ku = 1024, 64
    caps = {}
    if name == "llama8b_120k_b16":
        caps = dict(row_capacity=plan.N_idx + 2 * U, cluster_capacity=plan.m + 2 * ku)
    ix = wb.wave_index_build(K, V, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment,
                             wl.iters, 0, **caps)
    r = pu.retrieve_count(wl)
    out, lse, sel = wb.wave_attention_decode(q, ix, r, want_selected=True)
    torch.cuda.synchronize()
    qn = q.double().cpu().numpy()
    refs = {}
    for (b, h) in units:
        ref = wo.build_unit(K[b, h].double().cpu().numpy(), V[b, h].double().cpu().numpy(), plan,
                            wl.iters, 0, b, h, wl.dtype)
        refs[(b, h)] = ref
        tag = f"{name} b={b} h={h}"
        for nm in ("sizes", "offsets", "perm"):
            assert np.array_equal(_used(ix, nm, b, h).cpu().numpy(), getattr(ref, nm)), (tag, nm)
        for nm in ("centroids", "vsum", "k_perm", "v_perm", "k_steady", "v_steady"):
            assert np.array_equal(_used(ix, nm, b, h).float().cpu().numpy(),
                                  getattr(ref, nm).astype(np.float32)), (tag, nm)
        for g in range(wl.G):
            hq = h * wl.G + g
            parts = {}
            o, l, s = wo.decode_unit(qn[b, hq], ref, r, parts)
            pu.check_outputs(out[b, hq].cpu().numpy(), lse[b, hq:hq + 1].cpu().numpy(), o,
                             np.array([l]), wl.dtype, f"{tag} hq={hq}")
            pu.check_selected(sel[b, hq].cpu().numpy(), s, parts["z"], f"{tag} hq={hq}")
    if name != "llama8b_120k_b16":
        return
    # the index update at full size: one update segment of 1024 new tokens per sequence
    # (the paper's update segment size), 64 clusters, on the whole batch; sampled units
    # against the oracle's update of its own index, then decode on the grown index
    del out, lse, sel
    gen = torch.Generator(device=dev)
    gen.manual_seed(17)
    Kn = (K[:, :, -U:] + 0.05 * torch.randn(wl.B, wl.Hkv, U, wl.d, generator=gen, device=dev).to(K.dtype)).contiguous()
    Vn = torch.randn(wl.B, wl.Hkv, U, wl.d, generator=gen, device=dev).to(V.dtype)
    ix2 = wb.wave_index_append(ix, Kn, Vn, wl.n_local, U, ku, wl.iters, 0)
    torch.cuda.synchronize()
    assert (ix2.N, ix2.m, ix2.N_idx, ix2.n_local) == (wl.N + U, ix.m + ku, ix.N_idx + U, wl.n_local)
    # in place: the new rows and clusters went behind the old ones in the same buffers
    assert ix2.k_perm.data_ptr() == ix.k_perm.data_ptr() and ix2.centroids.data_ptr() == ix.centroids.data_ptr()
    assert ix2.row_capacity == ix.row_capacity and ix2.cluster_capacity == ix.cluster_capacity
    out, lse, sel = wb.wave_attention_decode(q, ix2, r, want_selected=True)
    torch.cuda.synchronize()
    for (b, h) in units:
        ref = wo.append_unit(refs[(b, h)], Kn[b, h].double().cpu().numpy(), Vn[b, h].double().cpu().numpy(),
                             wl.n_local, U, ku, wl.iters, 0, b, h)
        tag = f"{name} grown b={b} h={h}"
        for nm in ("sizes", "offsets", "perm"):
            assert np.array_equal(_used(ix2, nm, b, h).cpu().numpy(), getattr(ref, nm)), (tag, nm)
        for nm in ("centroids", "vsum", "k_perm", "v_perm", "k_steady", "v_steady"):
            assert np.array_equal(_used(ix2, nm, b, h).float().cpu().numpy(),
                                  getattr(ref, nm).astype(np.float32)), (tag, nm)
        for g in range(wl.G):
            hq = h * wl.G + g
            parts = {}
            o, l, s = wo.decode_unit(qn[b, hq], ref, r, parts)
            pu.check_outputs(out[b, hq].cpu().numpy(), lse[b, hq:hq + 1].cpu().numpy(), o,
                             np.array([l]), wl.dtype, f"{tag} hq={hq}")
            pu.check_selected(sel[b, hq].cpu().numpy(), s, parts["z"], f"{tag} hq={hq}")


@pytest.mark.parametrize("case", ["tiny_f32", "bf16_g4", "bf16_g7", "bf16_d64", "f32_d128"])
def test_full_attention_matches_oracle(case):
    """The brute-force decode kernel (the attention equation over all N tokens)
    against the oracle's full attention, every head."""
    wl = CASES[case]
    K, V = synth.make_kv(wl)
    q = synth.make_queries(wl, 1)
    out, lse = wb.wave_full_attention_decode(q.cuda(), K.cuda(), V.cuda())
    torch.cuda.synchronize()
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    Kn, Vn, qn = K.double().numpy(), V.double().numpy(), q.double().numpy()
    for b in range(wl.B):
        for hq in range(wl.Hq):
            o, l = wo.full_attention(qn[b, hq], Kn[b, hq // wl.G], Vn[b, hq // wl.G])
            pu.check_outputs(out[b, hq], lse[b, hq:hq + 1], o, np.array([l]), wl.dtype,
                             f"{case} full b={b} hq={hq}")


def test_full_attention_is_the_limit_of_the_wave_decode():
    """Retrieving every cluster reproduces what the brute-force kernel computes."""
    wl = CASES["bf16_g4"]
    K, V = synth.make_kv(wl)
    q = synth.make_queries(wl, 2).cuda()
    Kc, Vc = K.cuda(), V.cuda()
    ix = wb.wave_index_build(Kc, Vc, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment,
                             wl.iters, 0)
    o1, l1, _ = wb.wave_attention_decode(q, ix, ix.m)
    o2, l2 = wb.wave_full_attention_decode(q, Kc, Vc)
    torch.cuda.synchronize()
    assert float((o1 - o2).abs().max()) < 2e-5
    assert float((l1 - l2).abs().max()) < 2e-5


@pytest.mark.parametrize("case", ["tiny_f32", "bf16_g4", "bf16_g7", "bf16_d64", "f32_d128",
                                  "bf16_many_heads_g7", "bf16_listed_heads"])
def test_decode_with_estimation_budget(case):
    """The estimation-zone budget (the e best-ranked clusters after the retrieved ones are
    estimated, the rest ignored) against the oracle, including e = 0 and budgets that
    reach every cluster (then it is the plain decode).  392 heads: both selections of every
    head in one resident round on 16-bit keys; 800 heads: on 32-bit keys in several rounds."""
    wl = CASES[case]
    K, V, q = _inputs(wl, 1)
    index_ref = pu.oracle_build(wl, K, V)
    arrays = pu.oracle_index_arrays(wl, index_ref)
    ix = wb.index_from_arrays(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink, wl.n_local,
                              wl.segment_len, wl.clusters_per_segment, arrays,
                              cluster_capacity=index_ref[(0, 0)].plan.m + 7)   # (strides other than m)
    m = ix.m
    qn = q.double().numpy()
    r0 = pu.retrieve_count(wl)
    for r, e in [(r0, 0), (r0, 1), (r0, max(1, round(0.232 * m))), (0, 5), (0, 0), (1, m // 2),
                 (r0, m - r0 - 1), (r0, m), (r0, -1)]:
        out, lse, sel = wb.wave_attention_decode_budget(q.cuda(), ix, r, e, want_selected=True)
        torch.cuda.synchronize()
        out, lse = out.cpu().numpy(), lse.cpu().numpy()
        sel = sel.cpu().numpy() if sel is not None else None
        for b in range(wl.B):
            for hq in range(wl.Hq):
                parts = {}
                o, l, s = wo.decode_unit(qn[b, hq], index_ref[(b, hq // wl.G)], r, parts,
                                         est_clusters=None if e < 0 else e)
                tag = f"{case} budget b={b} hq={hq} r={r} e={e}"
                pu.check_outputs(out[b, hq], lse[b, hq:hq + 1], o, np.array([l]), wl.dtype, tag)
                if r > 0:
                    pu.check_selected(sel[b, hq], s, parts["z"], tag)


def test_recall_measurement_matches_oracle():
    """The recall@100 figure the segment-size study reports, computed from the device
    index, against the oracle's on the oracle-built index (the two indexes are equal)."""
    wl = CASES["bf16_g4"]
    K, V, q = _inputs(wl, 2)
    index_ref = pu.oracle_build(wl, K, V)
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, wl.iters, 0)
    r = pu.retrieve_count(wl)
    _, _, sel = wb.wave_attention_decode(q.cuda(), ix, r, want_selected=True)
    torch.cuda.synchronize()
    import bench
    rec = bench.recall_at_gpu(q.cuda(), ix, sel, wl.Hq, top=100).cpu().numpy()
    qn = q.double().numpy()
    for b in range(wl.B):
        for hq in range(wl.Hq):
            ref = index_ref[(b, hq // wl.G)]
            s_ref, _ = wo.select_clusters(qn[b, hq], ref.centroids, ref.sizes, r)
            want = wo.recall_at(qn[b, hq], ref, s_ref, top=100)
            assert abs(rec[b, hq] - want) <= 0.011, (b, hq, rec[b, hq], want)   # one token of 100: score ties


# a context shorter than its steady zone: nothing is indexed before the first update
_SHORT = _small("tiny_f32", name="f32_short", N=50, n_sink=4, n_local=64, segment_len=2048,
                clusters_per_segment=128, iters=3, retrieve_abs=2)


@pytest.mark.parametrize("case,n_news,U,ku,cap,scap,ccap", [
    ("bf16_g4", (300, 37, 1000), 256, 16, 0, 0, 0),
    ("bf16_g4", (300, 37, 1, 1000), 256, 16, 5400, 480, 0),
    ("bf16_g4", (300, 37, 1, 1000), 256, 16, 8192, 480, 470),   # room for every new row and cluster
    ("bf16_g4", (300, 37, 1, 1000), 256, 16, 8192, 0, 420),     # the room for clusters runs out
    ("tiny_f32", (5, 200), 64, 8, 0, 0, 0),
    ("tiny_f32", (5, 1, 200, 3), 64, 8, 8192, 140, 0),
    ("tiny_f32", (5, 1, 200, 3), 64, 8, 8192, 140, 4096),
    ("bf16_d64", (130,), 128, 200, 0, 0, 0),
    (_SHORT, (10, 100), 32, 4, 0, 0, 0),
    (_SHORT, (10, 100), 32, 4, 8192, 0, 64)])   # nothing indexed yet, with room: the first clusters in place
def test_index_append_matches_oracle_then_decode(case, n_news, U, ku, cap, scap, ccap):
    """Incremental index update through the C ABI, several times in a row (without and with
    flushed update segments, more clusters asked for than an update segment has tokens, an
    index with no clusters yet; once with room for the new rows and the new steady rows,
    which are then added in place, and once with room that runs out on the way): every array
    of the grown index against the oracle's, then decode on it."""
    wl = CASES[case] if isinstance(case, str) else case
    total_new = sum(n_news)
    big = synth.scaled(wl, N=wl.N + total_new)
    Kall, Vall, _ = _inputs(big, 1)
    K0, V0 = Kall[:, :, :wl.N].contiguous(), Vall[:, :, :wl.N].contiguous()
    ref = pu.oracle_build(wl, K0, V0)
    ix = wb.wave_index_build(K0.cuda(), V0.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, wl.iters, 0, row_capacity=cap, steady_capacity=scap,
                             cluster_capacity=ccap)
    first, shared_rows, shared_steady, shared_meta = ix, 0, 0, 0
    pos = wl.N
    for n_new in n_news:
        Kn, Vn = Kall[:, :, pos:pos + n_new].contiguous(), Vall[:, :, pos:pos + n_new].contiguous()
        before = ix
        ix = wb.wave_index_append(ix, Kn.cuda(), Vn.cuda(), wl.n_local, U, ku, wl.iters, 0)
        torch.cuda.synchronize()
        shared_rows += int(ix.k_perm.data_ptr() == before.k_perm.data_ptr() and ix.m > before.m)
        shared_steady += int(ix.k_steady.data_ptr() == before.k_steady.data_ptr())
        shared_meta += int(ix.centroids.data_ptr() == before.centroids.data_ptr() and ix.m > before.m)
        for (b, h), u in ref.items():
            ref[(b, h)] = wo.append_unit(u, Kn[b, h].double().numpy(), Vn[b, h].double().numpy(),
                                         wl.n_local, U, ku, wl.iters, 0, b, h)
        pos += n_new
        u0 = ref[(0, 0)]
        assert (ix.N, ix.S, ix.m, ix.N_idx, ix.p) == (u0.plan.N, u0.plan.S, u0.plan.m, u0.plan.N_idx,
                                                      u0.k_steady.shape[0])
        for (b, h), u in ref.items():
            for name in ("sizes", "offsets", "perm"):
                got = getattr(ix, name)[b, h].cpu().numpy()
                got = got[:ix.N_idx] if name == "perm" else got[:ix.m + (name == "offsets")]   # entries in use
                assert np.array_equal(got, getattr(u, name)), (n_new, b, h, name)
            for name in ("centroids", "vsum", "k_perm", "v_perm", "k_steady", "v_steady"):
                t = getattr(ix, name)[b, h]
                t = t[:ix.N_idx] if name in ("k_perm", "v_perm") else t    # rows in use
                t = t[:ix.p] if name in ("k_steady", "v_steady") else t
                t = t[:ix.m] if name in ("centroids", "vsum") else t
                got = t.float().cpu().numpy().astype(np.float64)
                assert np.array_equal(got, getattr(u, name)), (n_new, b, h, name)
    assert ix.appended_segments > 0
    if scap:
        assert shared_steady >= 1     # an update without a flush wrote its rows behind the old window
    if cap == 8192:
        assert shared_rows >= 1 and ix.row_capacity == cap      # the rows were added in place
    if cap == 5400:
        assert ix.row_capacity == 0                              # the room ran out: dense again
    if ccap == 64:
        assert shared_meta >= 1 and ix.cluster_capacity == ccap
    if ccap == 470 or ccap == 4096:
        assert shared_meta >= 1 and ix.cluster_capacity == ccap   # the clusters were added in place
        assert ix.centroids.data_ptr() == first.centroids.data_ptr()
    if ccap == 420:
        assert shared_meta >= 1 and ix.cluster_capacity == 0      # the room ran out: dense again
    if cap:   # the index before the updates is untouched by rows and clusters written behind its own
        u = pu.oracle_build(wl, K0, V0)[(0, 0)]
        assert np.array_equal(first.k_perm[0, 0, :first.N_idx].float().cpu().numpy().astype(np.float64), u.k_perm)
        assert np.array_equal(first.centroids[0, 0, :first.m].float().cpu().numpy().astype(np.float64), u.centroids)
        assert np.array_equal(first.sizes[0, 0, :first.m].cpu().numpy(), u.sizes)
        assert np.array_equal(first.offsets[0, 0, :first.m + 1].cpu().numpy(), u.offsets)
    q = synth.make_queries(big, 2)
    wl_now = synth.scaled(big, n_local=ix.n_local)
    r = pu.retrieve_count(wl)
    _decode_and_check(wl_now, ix, ref, q, r, f"append {wl.name}")
    _decode_and_check(wl_now, ix, ref, q, ix.m, f"append {wl.name} all")
