"""Pins of the CPU oracle against what the paper and the mathematics fix.
None of these tests touches the GPU library."""
import dataclasses
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import wave_oracle as wo
from paper_2505_02922_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _tiny_unit(seed=0, N=600, d=16, n_sink=4, n_local=20, L=256, k=16, T=5, dtype="f32",
               ncomp=12, sigma=0.3):
    g = _rng(seed)
    means = g.standard_normal((ncomp, d))
    K = means[g.integers(0, ncomp, N)] + sigma * g.standard_normal((N, d))
    V = g.standard_normal((N, d))
    K, V = wo.quant(K, dtype), wo.quant(V, dtype)
    plan = wo.make_plan(N, n_sink, n_local, L, k)
    ix, C, VS = wo.build_unit(K, V, plan, T, seed=7, b=0, h=0, dtype=dtype, keep_exact=True)
    q = wo.quant(means[3] + 0.5 * g.standard_normal(d), dtype)
    return K, V, q, plan, ix, C, VS


# ---------------------------------------------------------------- rounding
def test_bf16_rne_matches_enumeration():
    # Brute force: nearest of all finite bf16 values, ties to the even pattern.
    pats = np.arange(0, 1 << 16, dtype=np.uint32)
    vals = (pats << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    finite = np.isfinite(vals)
    pats, vals = pats[finite], vals[finite]
    order = np.argsort(vals, kind="stable")
    vals_sorted, pats_sorted = vals[order], pats[order]
    g = _rng(1)
    xs = np.concatenate([g.standard_normal(300) * 10.0 ** g.integers(-6, 6, 300),
                         [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e-39, 1e-41,
                          1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40]])
    got = wo.bf16_rne(xs)
    for x, y in zip(xs, got):
        i = np.searchsorted(vals_sorted, x)
        cands = [j for j in (i - 1, i, i + 1) if 0 <= j < vals_sorted.size]
        best = min(cands, key=lambda j: (abs(vals_sorted[j] - x), pats_sorted[j] & 1))
        assert y == vals_sorted[best], (x, y, vals_sorted[best])


def test_bf16_rne_matches_library_on_fp32_inputs():
    g = _rng(2)
    x32 = (g.standard_normal(5000) * 10.0 ** g.integers(-20, 20, 5000)).astype(np.float32)
    lib = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(wo.bf16_rne(x32.astype(np.float64)), lib)


def test_bf16_rne_single_rounding():
    # 1 + 2^-8 + 2^-40 lies just above a bf16 tie; rounding through fp32 first
    # would land on the tie and go to even (1.0); one rounding gives 1 + 2^-7.
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert wo.bf16_rne(x) == 1.0 + 2.0 ** -7


# ---------------------------------------------------------------- init
def test_splitmix64_published_outputs():
    want = [int(l) for l in open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt"))
            if l.strip() and not l.startswith("#")]
    st, got = 1234567, []
    for _ in want:
        st, out = wo.splitmix64(st)
        got.append(out)
    assert got == want


def test_init_indices_distinct_in_range_and_keyed():
    a = wo.init_indices(0, 0, 0, 0, 2048, 128)
    assert a.shape == (128,) and len(set(a.tolist())) == 128
    assert a.min() >= 0 and a.max() < 2048
    assert np.array_equal(a, wo.init_indices(0, 0, 0, 0, 2048, 128))
    for other in [(1, 0, 0, 0), (0, 1, 0, 0), (0, 0, 1, 0), (0, 0, 0, 1)]:
        assert not np.array_equal(a, wo.init_indices(*other, 2048, 128))
    full = wo.init_indices(3, 1, 2, 0, 37, 37)
    assert sorted(full.tolist()) == list(range(37))


def test_init_indices_roughly_uniform():
    counts = np.zeros(16)
    for s in range(4000):
        counts[wo.init_indices(11, 0, 0, s, 16, 1)[0]] += 1
    assert counts.min() > 170 and counts.max() < 340   # 250 expected each


# ---------------------------------------------------------------- layout
def test_plan_paper_parameters():
    kv = dict(l.split() for l in open(os.path.join(GOLDEN, "paper_parameters.txt"))
              if l.strip() and not l.startswith("#"))
    L = int(kv["segment_len"])
    k = L // int(kv["tokens_per_centroid"])
    plan = wo.make_plan(int(kv["tokens"]), 0, 0, L, k)
    assert plan.m == int(kv["clusters"]) and plan.S == 16
    assert round(100.0 * int(kv["retrieved"]) / plan.m, 1) == float(kv["budget_percent"])


def test_plan_ragged_and_degenerate():
    p = wo.make_plan(4096, 4, 64, 2048, 128)
    assert (p.N_idx, p.seg_len, p.seg_k, p.m) == (4028, [2048, 1980], [128, 128], 256)
    p = wo.make_plan(122880, 4, 1024, 8192, 512)
    assert (p.S, p.seg_len[-1], p.m) == (15, 7164, 7680)
    assert wo.retrieve_count(0.018, p.m) == 138
    # nearest, not floor: 2 % of 4096 clusters is 81.92 -> 82; the paper's own 150 of 8192 is
    # 1.83 % and 1.8 % of 8192 is 147.456 -> 147; halves go up (0.5 -> 1)
    assert wo.retrieve_count(0.02, 4096) == 82
    assert wo.retrieve_count(0.018, 8192) == 147
    assert wo.retrieve_count(0.01, 65536) == 655 and wo.retrieve_count(0.5, 1) == 1
    assert wo.retrieve_count(0.0, 100) == 0 and wo.retrieve_count(1.0, 100) == 100
    p = wo.make_plan(50, 4, 64, 2048, 128)       # N <= p: nothing to index
    assert p.m == 0 and p.N_idx == 0 and p.steady_positions.tolist() == list(range(50))
    p = wo.make_plan(100, 4, 64, 2048, 128)      # one short segment, k capped by its length
    assert p.seg_len == [32] and p.seg_k == [32]
    assert p.steady_positions.tolist() == list(range(4)) + list(range(36, 100))


# ---------------------------------------------------------------- brute force
def test_full_attention_matches_library_softmax():
    g = _rng(3)
    K, V, q = g.standard_normal((50, 8)), g.standard_normal((50, 8)), g.standard_normal(8)
    o, lse = wo.full_attention(q, K, V)
    tq, tK, tV = (torch.from_numpy(a) for a in (q, K, V))
    logits = (tK @ tq) / math.sqrt(8)
    assert np.allclose(o, (torch.softmax(logits, 0) @ tV).numpy(), rtol=0, atol=1e-13)
    assert abs(lse - torch.logsumexp(logits, 0).item()) < 1e-12


def test_full_attention_by_hand():
    # Two tokens, d = 4, logits 1 and 0 after the 1/sqrt(d) scale.
    q = np.array([2.0, 0.0, 0.0, 0.0])
    K = np.array([[1.0, 0, 0, 0], [0.0, 1, 0, 0]])
    V = np.array([[1.0, 0, 0, 0], [0.0, 1, 0, 0]])
    o, lse = wo.full_attention(q, K, V)
    w0 = math.e / (math.e + 1.0)
    assert np.allclose(o, [w0, 1 - w0, 0, 0], atol=1e-15)
    assert abs(lse - math.log(math.e + 1.0)) < 1e-15


# ---------------------------------------------------------------- decode pins
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_all_clusters_retrieved_equals_full_attention(dtype):
    K, V, q, plan, ix, _, _ = _tiny_unit(seed=4, dtype=dtype)
    o, lse, sel = wo.decode_unit(q, ix, r=plan.m + 5)
    of, lsef = wo.full_attention(q, K, V)
    assert sel.size == int((ix.sizes > 0).sum())
    assert np.allclose(o, of, rtol=0, atol=1e-12) and abs(lse - lsef) < 1e-12


def test_singleton_clusters_make_estimation_exact():
    # k = L_s: every token its own cluster, so C_i = K_i, VS_i = V_i, s_i = 1.
    K, V, q, plan, ix, _, _ = _tiny_unit(seed=5, N=300, L=128, k=128, n_local=16, T=3)
    assert ix.sizes.max() == 1 and ix.sizes.sum() == plan.N_idx
    of, lsef = wo.full_attention(q, K, V)
    for r in (0, 1, 17, plan.m):
        o, lse, _ = wo.decode_unit(q, ix, r)
        assert np.allclose(o, of, rtol=0, atol=1e-12) and abs(lse - lsef) < 1e-12


def _hand_index(K, V, groups, plan, dtype="f32"):
    """An index built by hand from a given partition of the indexed tokens."""
    d = K.shape[1]
    m = len(groups)
    sizes = np.array([len(gp) for gp in groups])
    C = np.array([K[gp].mean(axis=0) if len(gp) else np.zeros(d) for gp in groups])
    VS = np.array([V[gp].sum(axis=0) if len(gp) else np.zeros(d) for gp in groups])
    perm = np.concatenate([np.sort(gp) for gp in groups]).astype(np.int64)
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    sp = plan.steady_positions
    return wo.UnitIndex(plan, dtype, C, VS, sizes, offsets, perm, K[perm], V[perm], K[sp], V[sp],
                        np.zeros(0, dtype=np.int64))


def test_identical_keys_per_cluster_make_estimation_exact():
    g = _rng(6)
    N, d, ncl = 200, 8, 9
    protos = g.standard_normal((ncl, d))
    lab = g.integers(0, ncl, N)
    K, V, q = protos[lab], g.standard_normal((N, d)), g.standard_normal(d)
    plan = wo.make_plan(N, 3, 5, 64, 4)
    idxed = np.arange(plan.n_sink, plan.local_start)
    groups = [idxed[lab[idxed] == c] for c in range(ncl)] + [np.zeros(0, dtype=np.int64)]
    ix = _hand_index(K, V, groups, plan)
    of, lsef = wo.full_attention(q, K, V)
    for r in (0, 2, 5, 20):
        o, lse, sel = wo.decode_unit(q, ix, r)
        assert ncl not in sel.tolist()                   # the empty cluster is never retrieved
        assert np.allclose(o, of, rtol=0, atol=1e-12) and abs(lse - lsef) < 1e-12


def test_estimation_by_hand():
    # One steady token and two clusters, nothing retrieved: the estimation
    # equations evaluated by hand.  d = 4 so the scale is 1/2.
    q = np.array([2.0, 0, 0, 0])
    Ks = np.array([[0.0, 0, 0, 0]])
    Vs = np.array([[1.0, 1, 1, 1]])
    C = np.array([[2.0, 0, 0, 0], [-2.0, 0, 0, 0]])     # centroid logits 2 and -2
    VS = np.array([[3.0, 0, 0, 0], [0.0, 5, 0, 0]])
    sizes = np.array([3, 5])
    plan = wo.make_plan(9, 1, 0, 8, 2)
    ix = wo.UnitIndex(plan, "f32", C, VS, sizes, np.array([0, 3, 8]), np.arange(8),
                      np.zeros((8, 4)), np.zeros((8, 4)), Ks, Vs, np.zeros(0, dtype=np.int64))
    o, lse, sel = wo.decode_unit(q, ix, 0)
    Z = 1.0 + 3 * math.exp(2.0) + 5 * math.exp(-2.0)
    want = (np.array([1.0, 1, 1, 1]) + math.exp(2.0) * VS[0] + math.exp(-2.0) * VS[1]) / Z
    assert sel.size == 0 and np.allclose(o, want, atol=1e-15) and abs(lse - math.log(Z)) < 1e-14


@pytest.mark.parametrize("r", [0, 3, 11])
def test_zone_weights_sum_to_one(r):
    _, _, q, _, ix, _, _ = _tiny_unit(seed=8)
    parts = {}
    wo.decode_unit(q, ix, r, parts)
    total = parts["w_steady"].sum() + parts["w_retr"].sum() + parts["w_est"].sum()
    assert abs(total - 1.0) < 1e-13
    assert parts["w_retr"].size == int(ix.sizes[wo.select_clusters(q, ix.centroids, ix.sizes, r)[0]].sum())


def test_jensen_bound_and_monotone_in_r():
    K, V, q, plan, ix, C, VS = _tiny_unit(seed=9)
    exact = dataclasses_replace(ix, centroids=C, vsum=VS)      # unrounded means
    _, lse_full = wo.full_attention(q, K, V)
    scale = 1.0 / math.sqrt(q.size)
    for c in range(plan.m):                                     # per-cluster bound
        rows = np.arange(ix.offsets[c], ix.offsets[c + 1])
        if rows.size:
            lhs = rows.size * math.exp(C[c] @ q * scale)
            rhs = np.exp(ix.k_perm[rows] @ q * scale).sum()
            assert lhs <= rhs * (1 + 1e-12)
    prev = -np.inf
    for r in range(0, plan.m + 1, 3):
        _, lse, _ = wo.decode_unit(q, exact, r)
        assert lse <= lse_full + 1e-12 and lse >= prev - 1e-12
        prev = lse


def test_estimation_budget_by_hand():
    # One steady token, three clusters with centroid logits 2, 0, -2 (d = 4, scale 1/2),
    # nothing retrieved, budget of one estimated cluster: only the best-ranked one counts.
    q = np.array([2.0, 0, 0, 0])
    Ks, Vs = np.array([[0.0, 0, 0, 0]]), np.array([[1.0, 1, 1, 1]])
    C = np.array([[-2.0, 0, 0, 0], [2.0, 0, 0, 0], [0.0, 0, 0, 0]])
    VS = np.array([[0.0, 5, 0, 0], [3.0, 0, 0, 0], [0.0, 0, 7, 0]])
    sizes = np.array([5, 3, 2])
    plan = wo.make_plan(11, 1, 0, 10, 3)
    ix = wo.UnitIndex(plan, "f32", C, VS, sizes, np.array([0, 5, 8, 10]), np.arange(10),
                      np.zeros((10, 4)), np.zeros((10, 4)), Ks, Vs, np.zeros(0, dtype=np.int64))
    o, lse, _ = wo.decode_unit(q, ix, 0, est_clusters=1)
    Z = 1.0 + 3 * math.exp(2.0)
    want = (np.array([1.0, 1, 1, 1]) + math.exp(2.0) * VS[1]) / Z
    assert np.allclose(o, want, atol=1e-15) and abs(lse - math.log(Z)) < 1e-14
    o, lse, _ = wo.decode_unit(q, ix, 0, est_clusters=2)    # clusters 1 and 2, not 0
    Z = 1.0 + 3 * math.exp(2.0) + 2 * math.exp(0.0)
    want = (np.array([1.0, 1, 1, 1]) + math.exp(2.0) * VS[1] + VS[2]) / Z
    assert np.allclose(o, want, atol=1e-15) and abs(lse - math.log(Z)) < 1e-14
    o, lse, sel = wo.decode_unit(q, ix, 1, est_clusters=1)  # cluster 1 retrieved, 2 estimated
    assert sel.tolist() == [1]


def test_estimation_budget_limits():
    K, V, q, plan, ix, _, _ = _tiny_unit(seed=21)
    nonempty = int((ix.sizes > 0).sum())
    for r in (0, 4, 9):
        o_all, l_all, s_all = wo.decode_unit(q, ix, r)
        # a budget that covers every other cluster is the method as stated
        for e in (nonempty - r, nonempty, 10 ** 6):
            o, l, s = wo.decode_unit(q, ix, r, est_clusters=e)
            assert np.array_equal(o, o_all) and l == l_all and np.array_equal(s, s_all)
        # no estimation: exact softmax attention over the steady and retrieved tokens alone
        o0, l0, s0 = wo.decode_unit(q, ix, r, est_clusters=0)
        rows = (np.concatenate([np.arange(ix.offsets[c], ix.offsets[c + 1]) for c in s0])
                if s0.size else np.zeros(0, dtype=np.int64))
        Ksub = np.concatenate([ix.k_steady, ix.k_perm[rows]])
        Vsub = np.concatenate([ix.v_steady, ix.v_perm[rows]])
        o_ref, l_ref = wo.full_attention(q, Ksub, Vsub)
        assert np.allclose(o0, o_ref, atol=1e-13) and abs(l0 - l_ref) < 1e-12
        # every estimated cluster adds positive mass: lse grows with the budget, up to the full one
        prev = l0
        for e in range(1, nonempty - r + 1, 3):
            parts = {}
            _, l, _ = wo.decode_unit(q, ix, r, parts, est_clusters=e)
            assert l >= prev - 1e-13 and l <= l_all + 1e-13
            assert parts["est"].size == e
            total = parts["w_steady"].sum() + parts["w_retr"].sum() + parts["w_est"].sum()
            assert abs(total - 1.0) < 1e-13
            # the estimated clusters are the best-ranked ones after the retrieved
            order, z = wo.rank_clusters(q, ix.centroids, ix.sizes)
            assert set(parts["est"].tolist()) == set(order[min(r, nonempty):min(r, nonempty) + e].tolist())
            prev = l


def test_recall_by_hand():
    # Six indexed tokens in three clusters of two; scores 6, 5, 1, 4, 3, 2 in row order.
    q = np.array([1.0, 0.0])
    Kp = np.array([[6.0, 0], [5.0, 0], [1.0, 0], [4.0, 0], [3.0, 0], [2.0, 0]])
    plan = wo.make_plan(6, 0, 0, 6, 3)
    ix = wo.UnitIndex(plan, "f32", np.zeros((3, 2)), np.zeros((3, 2)), np.array([2, 2, 2]),
                      np.array([0, 2, 4, 6]), np.arange(6), Kp, np.zeros((6, 2)), np.zeros((0, 2)),
                      np.zeros((0, 2)), np.zeros(0, dtype=np.int64))
    assert wo.recall_at(q, ix, np.array([0]), top=2) == 1.0          # rows 0, 1
    assert wo.recall_at(q, ix, np.array([0]), top=3) == 2 / 3         # row 3 is in cluster 1
    assert wo.recall_at(q, ix, np.array([1, 2]), top=4) == 0.5        # rows 3, 4 of 0, 1, 3, 4
    assert wo.recall_at(q, ix, np.array([0, 1, 2]), top=6) == 1.0
    assert wo.recall_at(q, ix, np.zeros(0, dtype=np.int64), top=3) == 0.0


def dataclasses_replace(ix, **kw):
    return dataclasses.replace(ix, **kw)


# ---------------------------------------------------------------- incremental update pins
def _grown_context(seed, dtype, N0, n_new, d=16, ncomp=10):
    g = _rng(seed)
    means = g.standard_normal((ncomp, d))
    K = wo.quant(means[g.integers(0, ncomp, N0 + n_new)] + 0.3 * g.standard_normal((N0 + n_new, d)), dtype)
    V = wo.quant(g.standard_normal((N0 + n_new, d)), dtype)
    q = wo.quant(means[2] + 0.5 * g.standard_normal(d), dtype)
    return K, V, q


def _same_index(a, b):
    for name in ("centroids", "vsum", "sizes", "offsets", "perm", "k_perm", "v_perm", "k_steady",
                 "v_steady", "assign"):
        assert np.array_equal(getattr(a, name), getattr(b, name)), name
    assert (a.plan.N, a.plan.local_start, a.plan.seg_start, a.plan.seg_len, a.plan.seg_k) == \
           (b.plan.N, b.plan.local_start, b.plan.seg_start, b.plan.seg_len, b.plan.seg_k)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_append_equals_a_fresh_build_when_the_segments_line_up(dtype):
    """Update segments as long as the build's, an indexed range that is a whole number of
    them: the grown index must be, array by array, the index built from scratch over the
    grown context with the local window the update leaves (Wave Index, "Lightweight Index
    Construction": new clusters are appended, nothing is re-clustered)."""
    ns, nl, L, k, T = 2, 5, 32, 4, 4
    N0, n_new = ns + 2 * L + nl, 75          # window 5 + 75 = 80 = 2 segments + 16 local
    K, V, _ = _grown_context(11, dtype, N0, n_new)
    base = wo.build_unit(K[:N0], V[:N0], wo.make_plan(N0, ns, nl, L, k), T, 9, 1, 2, dtype)
    grown = wo.append_unit(base, K[N0:], V[N0:], nl, L, k, T, 9, 1, 2)
    fresh = wo.build_unit(K, V, wo.make_plan(N0 + n_new, ns, 16, L, k), T, 9, 1, 2, dtype)
    assert grown.plan.S == 4 and grown.k_steady.shape[0] == ns + 16
    _same_index(grown, fresh)


def test_append_in_one_step_or_in_two_is_the_same():
    ns, nl, L, k, U, ku, T = 3, 7, 40, 5, 16, 3, 3
    N0, n_new = 130, 61
    K, V, _ = _grown_context(12, "f32", N0, n_new)
    base = wo.build_unit(K[:N0], V[:N0], wo.make_plan(N0, ns, nl, L, k), T, 5, 0, 0, "f32")
    once = wo.append_unit(base, K[N0:], V[N0:], nl, U, ku, T, 5, 0, 0)
    half = wo.append_unit(base, K[N0:N0 + 22], V[N0:N0 + 22], nl, U, ku, T, 5, 0, 0)
    twice = wo.append_unit(half, K[N0 + 22:], V[N0 + 22:], nl, U, ku, T, 5, 0, 0)
    _same_index(once, twice)
    assert once.plan.S == base.plan.S + (nl + n_new - nl) // U
    # the index before the update is a prefix of the index after it
    for name in ("centroids", "vsum", "sizes", "perm", "k_perm", "v_perm"):
        assert np.array_equal(getattr(once, name)[:getattr(base, name).shape[0]], getattr(base, name))


@pytest.mark.parametrize("n_new", [1, 9, 40])
def test_append_keeps_every_token_once(n_new):
    """Without a full update segment only the window grows; with one, its tokens move into
    the index.  Either way every token of the grown context is in exactly one place, the
    meta index still obeys its conservation laws, and retrieving every cluster gives
    brute-force attention over the grown context."""
    ns, nl, L, k, U, ku, T = 2, 6, 48, 6, 16, 4, 3
    N0 = 120
    K, V, q = _grown_context(13, "f32", N0, n_new)
    base = wo.build_unit(K[:N0], V[:N0], wo.make_plan(N0, ns, nl, L, k), T, 3, 0, 1, "f32")
    ix = wo.append_unit(base, K[N0:], V[N0:], nl, U, ku, T, 3, 0, 1)
    F = n_new // U
    assert ix.plan.S == base.plan.S + F and ix.plan.m == base.plan.m + F * ku
    assert ix.k_steady.shape[0] == ns + nl + n_new - F * U
    where = np.concatenate([np.arange(ns), ix.perm, np.arange(ix.plan.local_start, N0 + n_new)])
    assert np.array_equal(np.sort(where), np.arange(N0 + n_new))
    assert np.array_equal(ix.k_perm, K[ix.perm]) and np.array_equal(ix.k_steady[ns:], K[ix.plan.local_start:])
    assert ix.sizes.sum() == ix.perm.size == ix.offsets[-1]
    for c in range(base.plan.m, ix.plan.m):
        rows = slice(ix.offsets[c], ix.offsets[c + 1])
        if ix.sizes[c]:
            assert np.allclose(ix.centroids[c], ix.k_perm[rows].mean(axis=0), atol=1e-6)
            assert np.allclose(ix.vsum[c], ix.v_perm[rows].sum(axis=0), atol=1e-6)
    o, lse, _ = wo.decode_unit(q, ix, r=ix.plan.m)
    of, lsef = wo.full_attention(q, K, V)
    assert np.allclose(o, of, rtol=0, atol=1e-12) and abs(lse - lsef) < 1e-12


def test_selection_order_and_ties():
    q = np.array([1.0, 0.0])
    C = np.array([[3.0, 0], [5.0, 0], [5.0, 1], [9.0, 0], [1.0, 0]])
    sizes = np.array([1, 1, 1, 0, 1])                    # cluster 3 is empty
    sel, z = wo.select_clusters(q, C, sizes, 2)
    assert sel.tolist() == [1, 2] and z[3] == -np.inf
    assert wo.select_clusters(q, C, sizes, 1)[0].tolist() == [1]   # tie 1 vs 2 -> lower id
    assert wo.select_clusters(q, C, sizes, 3)[0].tolist() == [0, 1, 2]
    assert wo.select_clusters(q, C, sizes, 99)[0].tolist() == [0, 1, 2, 4]


def test_shift_invariance():
    # Adding one vector to every key changes no softmax weight: the output is
    # unchanged and the log-sum-exp moves by q.shift/sqrt(d).  Per-segment
    # centring makes the clustering see the same centred keys.
    K, V, q, plan, ix, _, _ = _tiny_unit(seed=10, dtype="f32")
    shift = _rng(11).standard_normal(K.shape[1])
    ix2 = wo.build_unit(K + shift, V, plan, 5, 7, 0, 0, "f32")     # fp64 keys, not re-rounded
    assert np.array_equal(ix2.assign, ix.assign)
    assert np.allclose(ix2.centroids, ix.centroids + shift, atol=1e-5)
    for r in (0, 4, plan.m):
        o1, l1, s1 = wo.decode_unit(q, ix, r)
        o2, l2, s2 = wo.decode_unit(q, ix2, r)
        assert np.array_equal(s1, s2)
        assert np.allclose(o1, o2, atol=2e-6)
        assert abs((l2 - l1) - q @ shift / math.sqrt(q.size)) < 2e-6


# ---------------------------------------------------------------- meta index pins
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_meta_index_conservation(dtype):
    K, V, q, plan, ix, C, VS = _tiny_unit(seed=12, dtype=dtype, N=900, L=300, k=20)
    assert ix.sizes.sum() == plan.N_idx and ix.offsets[-1] == plan.N_idx
    assert sorted(ix.perm.tolist()) == list(range(plan.n_sink, plan.local_start))
    for s in range(plan.S):
        lo, Ls, ks, base = plan.seg_start[s], plan.seg_len[s], plan.seg_k[s], plan.seg_cluster_base[s]
        cl = slice(base, base + ks)
        assert ix.sizes[cl].sum() == Ls
        assert np.allclose((ix.sizes[cl, None] * C[cl]).sum(0), K[lo:lo + Ls].sum(0), atol=1e-9)
        assert np.allclose(VS[cl].sum(0), V[lo:lo + Ls].sum(0), atol=1e-9)
        rows = ix.perm[ix.offsets[base]:ix.offsets[base + ks]]
        assert rows.min() >= lo and rows.max() < lo + Ls       # segments do not mix
    for c in range(plan.m):
        rows = ix.perm[ix.offsets[c]:ix.offsets[c + 1]]
        assert np.all(np.diff(rows) > 0)                        # by position inside a cluster
        assert np.all(ix.assign[rows - plan.n_sink] == c)
    assert np.array_equal(ix.k_perm, K[ix.perm]) and np.array_equal(ix.v_perm, V[ix.perm])
    assert np.array_equal(ix.centroids, wo.quant(C, dtype))
    sp = plan.steady_positions
    assert np.array_equal(ix.k_steady, K[sp]) and sp.size == plan.n_sink + plan.N - plan.local_start


# ---------------------------------------------------------------- k-means pins
def _objective(xhat, a, k):
    """Spherical k-means objective at its optimal centroids: sum_i |sum of members|."""
    return sum(np.linalg.norm(xhat[a == i].sum(0)) for i in range(k))


def test_kmeans_objective_non_decreasing():
    g = _rng(13)
    K = g.standard_normal((24, 6))[g.integers(0, 24, 700)] + 0.3 * g.standard_normal((700, 6))
    trace = []
    wo.kmeans_segment(K, wo.init_indices(1, 0, 0, 0, 700, 24), 12, "f32", trace)
    xhat = trace[0][0]
    # objective with the centroids the assign step used, then after its update
    vals = []
    for (_, chat, a) in trace:
        vals.append((xhat * chat[a]).sum())
    assert all(b >= a - 1e-5 for a, b in zip(vals, vals[1:])), vals
    assert vals[-1] > vals[0]


def test_kmeans_small_vs_brute_force_optimum():
    g = _rng(14)
    for trial in range(6):
        n, k = 9, 3
        K = g.standard_normal((n, 4)) + 3.0 * np.eye(4)[g.integers(0, 3, n)]
        xhat = wo.normalise_segment(K, "f32")
        best = max(_objective(xhat, np.array(lab), k)
                   for lab in itertools.product(range(k), repeat=n))
        a = wo.kmeans_segment(K, wo.init_indices(trial, 0, 0, 0, n, k), 10, "f32")
        assert _objective(xhat, a, k) <= best + 1e-9


def test_kmeans_recovers_planted_clusters():
    g = _rng(15)
    dirs = np.eye(8)[:4] * 10.0 - 10.0 * np.eye(8)[4:8]       # four far-apart directions
    lab = np.repeat(np.arange(4), 25)
    K = dirs[lab] + 0.05 * g.standard_normal((100, 8))
    init = np.array([0, 25, 50, 75])                            # one seed point per planted cluster
    a = wo.kmeans_segment(K, init, 5, "bf16")
    assert np.array_equal(a, lab)
    xhat = wo.normalise_segment(K, "bf16")
    best_possible = _objective(xhat, lab, 4)
    assert abs(_objective(xhat, a, 4) - best_possible) < 1e-12


def test_kmeans_k_equals_len_is_identity_partition():
    g = _rng(16)
    K = g.standard_normal((40, 8))
    idx = wo.init_indices(5, 0, 0, 0, 40, 40)
    a = wo.kmeans_segment(K, idx, 4, "f32")
    assert np.array_equal(idx[a], np.arange(40))               # each point sits in its own seed's cluster


def test_assign_ties_go_to_lowest_index_and_empty_keeps_centroid():
    xhat = np.array([[1.0, 0], [0, 1.0], [1.0, 0]])
    chat = np.array([[1.0, 0], [1.0, 0], [0, 1.0]])            # centroids 0 and 1 identical
    a = wo.assign_step(xhat, chat)
    assert a.tolist() == [0, 2, 0]
    new = wo.update_step(xhat, a, chat, "f32")
    assert np.array_equal(new[1], chat[1])                      # no members: unchanged
    assert np.allclose(new[0], [1, 0]) and np.allclose(new[2], [0, 1])


def test_normalise_segment_is_centred_unit_and_quantised():
    g = _rng(17)
    K = g.standard_normal((64, 16)) + 5.0
    x = wo.normalise_segment(K, "bf16")
    assert np.array_equal(x, wo.bf16_rne(x))
    assert np.allclose(np.linalg.norm(x, axis=1), 1.0, atol=2e-2)
    ref = K - K.mean(0)
    ref /= np.linalg.norm(ref, axis=1, keepdims=True)
    assert np.abs(x - ref).max() < 2.0 ** -8
    Z = np.zeros((4, 3))                                        # a zero vector stays zero
    assert np.array_equal(wo.normalise_segment(Z, "f32"), Z)


# ---------------------------------------------------------------- whole-batch wrapper
def test_gqa_mapping_and_workload_tiny():
    wl = synth.scaled(synth.WORKLOADS["tiny_f32"], N=700, segment_len=256, clusters_per_segment=16,
                      Hq=4, Hkv=2, n_components=16)
    K, V = synth.make_kv(wl)
    q = synth.make_queries(wl)
    Kn, Vn, qn = K.double().numpy(), V.double().numpy(), q.double().numpy()
    index = wo.build_index(Kn, Vn, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment,
                           3, 0, wl.dtype)
    out, lse, sel = wo.decode(qn, index, 5)
    for hq in range(4):
        o, l, s = wo.decode_unit(qn[0, hq], index[0][hq // 2], 5)
        assert np.array_equal(out[0, hq], o) and lse[0, hq] == l and np.array_equal(sel[0][hq], s)
    # with everything retrieved the batch result is full attention per head
    out, lse, _ = wo.decode(qn, index, 10 ** 6)
    for hq in range(4):
        of, lf = wo.full_attention(qn[0, hq], Kn[0, hq // 2], Vn[0, hq // 2])
        assert np.allclose(out[0, hq], of, atol=1e-12) and abs(lse[0, hq] - lf) < 1e-12


def test_storage_rounding_of_a_centroid_stays_within_the_stated_logit_bound():
    """The GPU path subtracts a selected cluster's estimation term from a sum over all clusters,
    which is harmless while the term does not exceed the cluster's exact terms (the estimation
    bound, which needs the centroid to be the mean).  A stored centroid is the mean rounded to
    bf16: its logit moves by at most 2^-8 |q| |C| / sqrt(d), so the bound is broken by at most
    that much.  Checked on an oracle-built index."""
    from paper_2505_02922_amd import synth
    wl = synth.scaled(synth.WORKLOADS["llama8b_32k"], N=3000, Hq=4, Hkv=1, segment_len=1024,
                      clusters_per_segment=64, n_local=100, n_components=64, iters=3)
    K, V = synth.make_kv(wl)
    q = synth.make_queries(wl).double().numpy()[0]
    plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
    ix = wo.build_unit(K[0, 0].double().numpy(), V[0, 0].double().numpy(), plan, wl.iters, 0, 0, 0, "bf16")
    C = np.asarray(ix.centroids, dtype=np.float64)
    Kp = np.asarray(ix.k_perm, dtype=np.float64)
    off = np.asarray(ix.offsets)
    worst = 0.0
    for hq in range(wl.Hq):
        for c in np.nonzero(np.asarray(ix.sizes))[0]:
            rows = Kp[off[c]:off[c + 1]] @ q[hq] / math.sqrt(wl.d)
            lme = rows.max() + math.log(np.exp(rows - rows.max()).mean())     # log of the mean exponential
            lc = C[c] @ q[hq] / math.sqrt(wl.d)
            bound = 2.0 ** -8 * np.linalg.norm(q[hq]) * np.linalg.norm(C[c]) / math.sqrt(wl.d)
            assert lc <= lme + bound
            worst = max(worst, lc - lme)
    assert worst < 0.1     # e^0.1: a tenth of a bit of the fp32 result


def test_a_cluster_nobody_entered_or_left_keeps_its_centroid():
    """Spherical k-means update: the centroid is a function of the member set alone, so a
    cluster whose members are the same after two consecutive assign steps has the same
    centroid, bit for bit, after both updates; and on clustered keys most clusters are in that
    state after a few rounds (which is what lets an implementation sum only the others again).
    An empty cluster keeps its centroid by the rule for empty clusters."""
    wl = synth.scaled(synth.WORKLOADS["llama8b_32k"], B=1, Hkv=1, Hq=4, N=4 + 64 + 2048, n_local=64,
                      segment_len=2048, clusters_per_segment=128, iters=8)
    K, _ = synth.make_kv(wl)
    plan = wo.make_plan(wl.N, wl.n_sink, wl.n_local, wl.segment_len, wl.clusters_per_segment)
    lo, Ls, ks = plan.seg_start[0], plan.seg_len[0], plan.seg_k[0]
    trace = []
    wo.kmeans_segment(K[0, 0, lo:lo + Ls].double().numpy(), wo.init_indices(0, 0, 0, 0, Ls, ks), wl.iters,
                      wl.dtype, trace)
    same_total, checked = [], 0
    for t in range(1, len(trace) - 1):
        a_prev, a_now = trace[t - 1][2], trace[t][2]
        c_after_prev, c_after_now = trace[t][1], trace[t + 1][1]   # centroids after update t-1 and t
        moved = a_prev != a_now
        touched = np.zeros(ks, dtype=bool)
        touched[a_prev[moved]] = True
        touched[a_now[moved]] = True
        same = ~touched
        assert np.array_equal(c_after_now[same], c_after_prev[same]), t
        same_total.append(same.mean())
        checked += int(same.sum())
    assert checked > 0
    assert same_total[-1] > same_total[0]          # fewer and fewer clusters change
    assert same_total[-1] > 0.5
