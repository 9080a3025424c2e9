"""CPU oracle for the wave index: segmented spherical k-means build and
tripartite decode attention, in fp64 with numpy.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
GPU library must compute.  It is imported by the tests, by the smoke check and
by the benchmark's CPU-baseline leg, never by the product path, and it shares
no code with the HIP kernels.

Every function takes the steps of the method in the paper's order and
notation (d head dim, N tokens, p steady tokens, m clusters, r retrieved
clusters, C centroids, s sizes, VS value sums, L segment length, k clusters
per segment, T iterations).  Where the paper leaves a choice open the reading
taken is stated at the function.

Arithmetic: inputs are up-converted exactly to fp64; every floating-point step
is fp64; the only rounding points are the explicit `quant` calls, which are
part of the method's definition (normalised keys, iteration centroids, stored
centroids and value sums are held in the KV storage type).

Pins (see tests): brute-force attention against a library softmax; decode with
every cluster retrieved equals brute force; singleton clusters and
identical-key clusters make estimation exact; zone weights sum to one; the
Jensen bound of the estimation section; shift invariance; meta-index
conservation laws; k-means objective monotonicity and brute-force optimum on
tiny inputs; splitmix64 published outputs; bf16 rounding against enumeration;
the incremental update against a fresh build of the grown context when the
segments line up, against itself in one step or two, and against brute force.
Parity unpinned: the size of the approximation error against full attention at
the paper's budgets (the paper gives task accuracies on datasets only).
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

_MASK64 = (1 << 64) - 1


# --------------------------------------------------------------------------
# Storage-type rounding (definition points of the method)
# --------------------------------------------------------------------------
def bf16_rne(x) -> np.ndarray:
    """Round fp64 values to the nearest bfloat16 (8 significant bits, fp32
    exponent range), ties to even, returned as fp64.  Written from the format
    definition: scale so that one bf16 ulp is 1, round to nearest-even integer,
    scale back.  Subnormal spacing is 2**-133; overflow goes to infinity."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                       # x = f * 2**e with 0.5 <= |f| < 1
    q = np.maximum(e - 8, -133)              # exponent of one ulp at x
    y = np.ldexp(np.rint(np.ldexp(x, -q)), q)
    big = np.abs(y) > 3.3895313892515355e38  # largest finite bf16 = (2 - 2**-7) * 2**127
    y = np.where(big, np.copysign(np.inf, x), y)
    return np.where(np.isfinite(x), y, x)


def quant(x, dtype: str) -> np.ndarray:
    """Round fp64 to the KV storage type ("bf16" or "f32"), result as fp64."""
    if dtype == "bf16":
        return bf16_rne(x)
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# Seeded initial centroids
# --------------------------------------------------------------------------
def splitmix64(state: int) -> Tuple[int, int]:
    """One step of the splitmix64 generator: returns (new state, output)."""
    state = (state + 0x9E3779B97F4A7C15) & _MASK64
    z = state
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return state, z ^ (z >> 31)


def init_indices(seed: int, b: int, h: int, s: int, L_s: int, k_s: int) -> np.ndarray:
    """The k_s distinct seed tokens of segment s of unit (b, h): the first k_s
    entries of a Fisher-Yates shuffle of 0..L_s-1.  The paper does not say how
    spherical k-means is initialised; this reading (random distinct points of
    the segment) is the common one.  The generator state is keyed by folding
    seed, b, h, s in that order: xor the integer in, take one splitmix64
    output, continue from that output.  Draw i picks j = i + out mod (L_s-i)."""
    st = 0
    for v in (seed, b, h, s):
        st ^= int(v) & _MASK64
        _, st = splitmix64(st)
    a = list(range(L_s))
    for i in range(k_s):
        st, out = splitmix64(st)
        j = i + out % (L_s - i)
        a[i], a[j] = a[j], a[i]
    return np.array(a[:k_s], dtype=np.int64)


# --------------------------------------------------------------------------
# Segment layout
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Plan:
    """Token ranges of one sequence.  Steady tokens (first n_sink and last
    n_local positions) are attended by position and are not clustered
    ("Steady, Retrieval, and Estimation Zones"); the tokens in between are
    tiled by segments of L tokens, the last one ragged, each clustered on its
    own into min(k, L_s) clusters ("segmented clustering")."""
    N: int
    n_sink: int
    local_start: int
    seg_start: List[int]
    seg_len: List[int]
    seg_k: List[int]
    seg_cluster_base: List[int]

    @property
    def N_idx(self) -> int:
        return self.local_start - self.n_sink

    @property
    def m(self) -> int:
        return sum(self.seg_k)

    @property
    def S(self) -> int:
        return len(self.seg_len)

    @property
    def steady_positions(self) -> np.ndarray:
        return np.concatenate([np.arange(0, self.n_sink), np.arange(self.local_start, self.N)])


def make_plan(N: int, n_sink: int, n_local: int, L: int, k: int) -> Plan:
    ns = min(n_sink, N)
    ls = max(ns, N - n_local)
    starts, lens, ks, bases = [], [], [], []
    pos, base = ns, 0
    while pos < ls:
        Ls = min(L, ls - pos)
        starts.append(pos)
        lens.append(Ls)
        ks.append(min(k, Ls))
        bases.append(base)
        base += ks[-1]
        pos += Ls
    return Plan(N, ns, ls, starts, lens, ks, bases)


def retrieve_count(frac: float, m: int) -> int:
    """r from a retrieval budget given as a fraction of all clusters (the
    paper's 150 of 8192 clusters is quoted as 1.8 %)."""
    return int(math.floor(frac * m + 0.5))


# --------------------------------------------------------------------------
# Spherical k-means on one segment
# --------------------------------------------------------------------------
def normalise_segment(K_seg: np.ndarray, dtype: str) -> np.ndarray:
    """Centre the segment's keys on their mean (the centering step named in
    "Lightweight Index Construction"; the mean is per segment because segments
    are clustered independently), scale each to unit length (spherical k-means
    works on directions) and hold the result in the storage type."""
    K_seg = np.asarray(K_seg, dtype=np.float64)
    mu = K_seg.sum(axis=0) / K_seg.shape[0]
    x = K_seg - mu
    nrm = np.sqrt((x * x).sum(axis=1))
    safe = np.where(nrm > 0.0, nrm, 1.0)
    return quant(x / safe[:, None], dtype)


def assign_step(xhat: np.ndarray, chat: np.ndarray) -> np.ndarray:
    """a_j = argmax_i xhat_j . chat_i, exact ties to the lowest i."""
    return np.argmax(xhat @ chat.T, axis=1)


def update_step(xhat: np.ndarray, a: np.ndarray, chat: np.ndarray, dtype: str) -> np.ndarray:
    """chat_i <- quant(u_i / |u_i|), u_i the sum of the members of cluster i.
    A cluster without members, or whose members cancel, keeps its centroid."""
    k, d = chat.shape
    u = np.zeros((k, d), dtype=np.float64)
    np.add.at(u, a, xhat)
    nrm = np.sqrt((u * u).sum(axis=1))
    count = np.bincount(a, minlength=k)
    ok = (count > 0) & (nrm > 0.0)
    new = chat.copy()
    new[ok] = quant(u[ok] / nrm[ok, None], dtype)
    return new


def kmeans_segment(K_seg: np.ndarray, init_idx: np.ndarray, T: int, dtype: str,
                   trace: Optional[list] = None) -> np.ndarray:
    """T rounds of (assign, update) from the seeded initial centroids.  The
    partition returned is the one of the T-th assign; no assign follows the
    last update.  `trace`, if given, receives (xhat, chat_before, a) per round."""
    xhat = normalise_segment(K_seg, dtype)
    chat = xhat[np.asarray(init_idx)].copy()
    a = np.zeros(xhat.shape[0], dtype=np.int64)
    for _ in range(T):
        a = assign_step(xhat, chat)
        if trace is not None:
            trace.append((xhat, chat.copy(), a.copy()))
        chat = update_step(xhat, a, chat, dtype)
    return a


# --------------------------------------------------------------------------
# Index build for one (sequence, KV head) unit
# --------------------------------------------------------------------------
@dataclasses.dataclass
class UnitIndex:
    """Meta index and cluster-contiguous KV of one (sequence, KV head) unit.
    Floating arrays hold storage-type values as fp64."""
    plan: Plan
    dtype: str
    centroids: np.ndarray   # [m, d]  mean of the raw member keys
    vsum: np.ndarray        # [m, d]  sum of the member values
    sizes: np.ndarray       # [m]
    offsets: np.ndarray     # [m + 1] row ranges into k_perm / v_perm
    perm: np.ndarray        # [N_idx] original position of each permuted row
    k_perm: np.ndarray      # [N_idx, d]
    v_perm: np.ndarray      # [N_idx, d]
    k_steady: np.ndarray    # [p, d] sink rows then local rows
    v_steady: np.ndarray    # [p, d]
    assign: np.ndarray      # [N_idx] cluster (global id) of each indexed token, by position


def build_unit(K: np.ndarray, V: np.ndarray, plan: Plan, T: int, seed: int, b: int, h: int,
               dtype: str, keep_exact: bool = False):
    """Build the wave index of one unit ("Index Organization"; value sums and
    sizes from "Accuracy-Bounded Attention Estimation").  K, V: [N, d].

    Per cluster: size, centroid = arithmetic mean of its raw (uncentred) keys
    as the Jensen bound of the estimation section requires, value sum; all
    rounded once to the storage type.  Rows are laid out by (segment, cluster,
    original position).  With keep_exact the unrounded centroids and value
    sums are returned too (for the pins that need exact means)."""
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    d = K.shape[1]
    m = plan.m
    C = np.zeros((m, d))
    VS = np.zeros((m, d))
    sizes = np.zeros(m, dtype=np.int64)
    assign_global = np.zeros(plan.N_idx, dtype=np.int64)
    perm_parts = []
    for s in range(plan.S):
        lo, Ls, ks, base = plan.seg_start[s], plan.seg_len[s], plan.seg_k[s], plan.seg_cluster_base[s]
        idx = init_indices(seed, b, h, s, Ls, ks)
        a = kmeans_segment(K[lo:lo + Ls], idx, T, dtype)
        assign_global[lo - plan.n_sink: lo - plan.n_sink + Ls] = a + base
        for i in range(ks):
            members = np.nonzero(a == i)[0] + lo          # ascending positions
            sizes[base + i] = members.size
            if members.size:
                C[base + i] = K[members].sum(axis=0) / members.size
                VS[base + i] = V[members].sum(axis=0)
            perm_parts.append(members)
    perm = np.concatenate(perm_parts) if perm_parts else np.zeros(0, dtype=np.int64)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    sp = plan.steady_positions
    ix = UnitIndex(plan, dtype, quant(C, dtype), quant(VS, dtype), sizes, offsets, perm,
                   K[perm], V[perm], K[sp], V[sp], assign_global)
    if keep_exact:
        return ix, C, VS
    return ix


# --------------------------------------------------------------------------
# Incremental update of one unit's index
# --------------------------------------------------------------------------
def append_unit(ix: UnitIndex, K_new: np.ndarray, V_new: np.ndarray, n_local_min: int, U: int,
                k_u: int, T: int, seed: int, b: int, h: int) -> UnitIndex:
    """Index update during decoding ("Lightweight Index Construction", last
    paragraph).  New tokens join the local window of the steady zone.  Whenever
    the window holds a whole update segment of U tokens beyond its n_local_min
    most recent ones, its U oldest tokens are clustered on their own, exactly as
    a segment of the initial build (same seeding rule with the segment's number,
    same iterations), into min(k_u, U) clusters that are appended to the index;
    nothing indexed before is touched.  Reading taken: the window is flushed in
    whole segments, oldest first, as many as fit; the remainder (between
    n_local_min and n_local_min + U - 1 tokens) stays local.  Returns the new
    index; `ix` is not modified."""
    K_new = np.asarray(K_new, dtype=np.float64)
    V_new = np.asarray(V_new, dtype=np.float64)
    plan, dtype = ix.plan, ix.dtype
    ns = plan.n_sink
    d = ix.k_steady.shape[1]
    WK = np.concatenate([ix.k_steady[ns:], K_new.reshape(-1, d)])   # positions local_start ...
    WV = np.concatenate([ix.v_steady[ns:], V_new.reshape(-1, d)])
    F = max(0, (WK.shape[0] - int(n_local_min)) // int(U))
    ks = min(int(k_u), int(U))
    new_plan = Plan(plan.N + K_new.reshape(-1, d).shape[0], ns, plan.local_start + F * U,
                    list(plan.seg_start), list(plan.seg_len), list(plan.seg_k),
                    list(plan.seg_cluster_base))
    C, VS, sizes = [ix.centroids], [ix.vsum], [np.asarray(ix.sizes, dtype=np.int64)]
    perm, kp, vp, asg = [ix.perm], [ix.k_perm], [ix.v_perm], [ix.assign]
    for f in range(F):
        s, lo, base = plan.S + f, plan.local_start + f * U, plan.m + f * ks
        new_plan.seg_start.append(lo)
        new_plan.seg_len.append(U)
        new_plan.seg_k.append(ks)
        new_plan.seg_cluster_base.append(base)
        Kseg, Vseg = WK[f * U:(f + 1) * U], WV[f * U:(f + 1) * U]
        a = kmeans_segment(Kseg, init_indices(seed, b, h, s, U, ks), T, dtype)
        Cs, VSs, ss = np.zeros((ks, d)), np.zeros((ks, d)), np.zeros(ks, dtype=np.int64)
        order = []
        for i in range(ks):
            members = np.nonzero(a == i)[0]                    # ascending positions
            ss[i] = members.size
            if members.size:
                Cs[i] = Kseg[members].sum(axis=0) / members.size
                VSs[i] = Vseg[members].sum(axis=0)
            order.append(members)
        order = np.concatenate(order)
        C.append(quant(Cs, dtype)); VS.append(quant(VSs, dtype)); sizes.append(ss)
        perm.append(order + lo); kp.append(Kseg[order]); vp.append(Vseg[order]); asg.append(a + base)
    sizes = np.concatenate(sizes)
    return UnitIndex(new_plan, dtype, np.concatenate(C), np.concatenate(VS), sizes,
                     np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64), np.concatenate(perm),
                     np.concatenate(kp), np.concatenate(vp),
                     np.concatenate([ix.k_steady[:ns], WK[F * U:]]),
                     np.concatenate([ix.v_steady[:ns], WV[F * U:]]), np.concatenate(asg))


# --------------------------------------------------------------------------
# Decode
# --------------------------------------------------------------------------
def full_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> Tuple[np.ndarray, float]:
    """Softmax(q K^T / sqrt(d)) V over all tokens (the attention equation of
    the background section).  Returns (o, log-sum-exp of the scaled logits)."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    logit = (K @ q) / math.sqrt(q.shape[0])
    M = logit.max()
    w = np.exp(logit - M)
    Z = w.sum()
    return (w @ V) / Z, M + math.log(Z)


def rank_clusters(q: np.ndarray, centroids: np.ndarray, sizes: np.ndarray
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """The non-empty clusters ordered by q . C_i, best first; exact ties go to
    the lower cluster id.  Returns (ids in rank order, scores z of all clusters;
    empty ones -inf)."""
    q = np.asarray(q, dtype=np.float64)
    z = np.asarray(centroids, dtype=np.float64) @ q
    z = np.where(np.asarray(sizes) > 0, z, -np.inf)
    ids = np.nonzero(np.asarray(sizes) > 0)[0]
    return ids[np.lexsort((ids, -z[ids]))], z   # by score descending, then id ascending


def select_clusters(q: np.ndarray, centroids: np.ndarray, sizes: np.ndarray, r: int
                    ) -> Tuple[np.ndarray, np.ndarray]:
    """Rank the non-empty clusters by q . C_i and take the r best (step 1 of
    the decode procedure).  Returns (selected ids ascending, scores z)."""
    order, z = rank_clusters(q, centroids, sizes)
    return np.sort(order[: max(0, min(int(r), order.size))]), z


def decode_unit(q: np.ndarray, ix: UnitIndex, r: int, parts: Optional[dict] = None,
                est_clusters: Optional[int] = None) -> Tuple[np.ndarray, float, np.ndarray]:
    """Tripartite attention of one query head over one unit's index.

    Steady tokens and every token of the r retrieved clusters enter with their
    exact logits q.K_j/sqrt(d); each other non-empty cluster enters once with
    the logit of its centroid, multiplicity s_i in the denominator and its
    value sum in the numerator (estimation equations).  The zones share one
    softmax normalisation: the paper's implementation section merges the exact
    partial output with the estimate, so retrieved clusters contribute their
    exact exponentials and only the others the centroid term.
    est_clusters: None estimates every non-retrieved cluster (the method as
    stated); a number e restricts the estimation zone to the e best-ranked
    clusters after the retrieved ones and ignores the rest (the evaluation's
    zone budgets: an estimation zone of 23.2 % of the clusters; e = 0 is the
    ablation without estimation).
    Returns (o [d], lse, selected ids ascending)."""
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[0]
    scale = 1.0 / math.sqrt(d)
    order, z = rank_clusters(q, ix.centroids, ix.sizes)
    nr = max(0, min(int(r), order.size))
    sel = np.sort(order[:nr])
    rows = (np.concatenate([np.arange(ix.offsets[c], ix.offsets[c + 1]) for c in sel])
            if sel.size else np.zeros(0, dtype=np.int64))
    ne = order.size - nr if est_clusters is None else max(0, min(int(est_clusters), order.size - nr))
    est = np.sort(order[nr:nr + ne])

    l_steady = (np.asarray(ix.k_steady, dtype=np.float64) @ q) * scale
    l_retr = (np.asarray(ix.k_perm, dtype=np.float64)[rows] @ q) * scale
    l_est = z[est] * scale
    M = max([x.max() for x in (l_steady, l_retr, l_est) if x.size] or [0.0])
    w_steady, w_retr, w_est = np.exp(l_steady - M), np.exp(l_retr - M), np.exp(l_est - M)
    s_est = np.asarray(ix.sizes, dtype=np.float64)[est]
    Z = w_steady.sum() + w_retr.sum() + (s_est * w_est).sum()
    A = (w_steady @ np.asarray(ix.v_steady, dtype=np.float64)
         + w_retr @ np.asarray(ix.v_perm, dtype=np.float64)[rows]
         + w_est @ np.asarray(ix.vsum, dtype=np.float64)[est])
    if parts is not None:
        parts.update(M=M, Z=Z, w_steady=w_steady / Z, w_retr=w_retr / Z,
                     w_est=s_est * w_est / Z, est=est, rows=rows, z=z)
    return A / Z, M + math.log(Z), sel


def recall_at(q: np.ndarray, ix: UnitIndex, sel: np.ndarray, top: int = 100) -> float:
    """Clustering accuracy as the evaluation's segment-size study measures it
    (recall@100): of the `top` indexed tokens with the largest q . K_j, the
    share that lies in the retrieved clusters `sel`.  Ties go to the earlier
    row of the cluster-contiguous order."""
    q = np.asarray(q, dtype=np.float64)
    scores = np.asarray(ix.k_perm, dtype=np.float64) @ q
    n = scores.size
    top = min(int(top), n)
    if top == 0:
        return 1.0
    best = np.lexsort((np.arange(n), -scores))[:top]
    hit = np.zeros(n, dtype=bool)
    for c in np.asarray(sel, dtype=np.int64):
        hit[ix.offsets[c]:ix.offsets[c + 1]] = True
    return float(hit[best].mean())


# --------------------------------------------------------------------------
# Whole-batch wrappers (loops over independent units; no arithmetic of their own)
# --------------------------------------------------------------------------
def build_index(K: np.ndarray, V: np.ndarray, n_sink: int, n_local: int, L: int, k: int,
                T: int, seed: int, dtype: str) -> List[List[UnitIndex]]:
    """K, V: [B, Hkv, N, d] -> index[b][h]."""
    B, Hkv, N, _ = K.shape
    plan = make_plan(N, n_sink, n_local, L, k)
    return [[build_unit(K[b, h], V[b, h], plan, T, seed, b, h, dtype) for h in range(Hkv)]
            for b in range(B)]


def decode(q: np.ndarray, index: List[List[UnitIndex]], r: int
           ) -> Tuple[np.ndarray, np.ndarray, List[List[np.ndarray]]]:
    """q: [B, Hq, d].  Query head hq reads the index of KV head hq // G and
    ranks and selects clusters on its own."""
    B, Hq, d = q.shape
    Hkv = len(index[0])
    G = Hq // Hkv
    out = np.zeros((B, Hq, d))
    lse = np.zeros((B, Hq))
    sel = [[None] * Hq for _ in range(B)]
    for b in range(B):
        for hq in range(Hq):
            out[b, hq], lse[b, hq], sel[b][hq] = decode_unit(q[b, hq], index[b][hq // G], r)
    return out, lse, sel
