"""ctypes binding of libwave.so (include/wave.h): argument marshalling only.

Every function here has the name of the C entry point it calls.  torch
supplies device memory and the current HIP stream; no arithmetic of the method
happens in Python.  There is no CPU fallback: if the library has not been
built, loading raises."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# WAVE_LIB names another build of the library (tuning variants); the default is the in-tree one
LIB_PATH = os.environ.get("WAVE_LIB") or os.path.join(_HERE, "libwave.so")

WAVE_F32, WAVE_BF16 = 0, 1
WAVE_INDEX_BUFFERS = 9
BUFFER_NAMES = ("centroids", "vsum", "sizes", "offsets", "perm", "k_perm", "v_perm", "k_steady",
                "v_steady")
STATUS_NAMES = {0: "WAVE_OK", 1: "WAVE_ERR_ARG", 2: "WAVE_ERR_SHAPE", 3: "WAVE_ERR_DTYPE",
                4: "WAVE_ERR_WORKSPACE", 5: "WAVE_ERR_STEADY_MISMATCH", 6: "WAVE_ERR_HIP"}
EXPORTS = ("wave_index_plan", "wave_index_build", "wave_index_append_plan", "wave_index_append",
           "wave_attention_decode", "wave_attention_decode_static_capacity",
           "wave_attention_decode_static",
           "wave_attention_decode_budget_workspace", "wave_attention_decode_budget",
           "wave_full_attention_workspace", "wave_full_attention_decode", "wave_init_indices",
           "wave_kmeans_assign_step", "wave_calibration_copy", "wave_calibration_read",
           "wave_profile_enable", "wave_profile_read", "wave_status_string")


class wave_index(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("N", ctypes.c_int32), ("n_sink", ctypes.c_int32),
                ("n_local", ctypes.c_int32), ("segment_len", ctypes.c_int32),
                ("clusters_per_segment", ctypes.c_int32), ("S", ctypes.c_int32),
                ("m", ctypes.c_int32), ("N_idx", ctypes.c_int32), ("p", ctypes.c_int32),
                ("steady_capacity", ctypes.c_int32),
                ("centroids", ctypes.c_void_p), ("vsum", ctypes.c_void_p),
                ("sizes", ctypes.c_void_p), ("offsets", ctypes.c_void_p),
                ("perm", ctypes.c_void_p), ("k_perm", ctypes.c_void_p),
                ("v_perm", ctypes.c_void_p), ("k_steady", ctypes.c_void_p),
                ("v_steady", ctypes.c_void_p),
                ("appended_segments", ctypes.c_int32), ("update_segment_len", ctypes.c_int32),
                ("update_clusters", ctypes.c_int32), ("row_capacity", ctypes.c_int32),
                ("cluster_capacity", ctypes.c_int32)]


class WaveError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().wave_status_string(status).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({msg})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2505_02922_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, u64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_size_t
        L.wave_index_plan.argtypes = [ctypes.POINTER(wave_index), ctypes.POINTER(sz),
                                      ctypes.POINTER(sz), i32, i32, ctypes.POINTER(sz)]
        L.wave_index_build.argtypes = [vp, vp, ctypes.POINTER(wave_index), i32, u64, vp, sz, vp]
        L.wave_index_append_plan.argtypes = [ctypes.POINTER(wave_index), i32, i32, i32, i32,
                                             ctypes.POINTER(wave_index), ctypes.POINTER(sz),
                                             ctypes.POINTER(sz)]
        L.wave_index_append.argtypes = [ctypes.POINTER(wave_index), vp, vp, i32, i32, i32, i32, i32,
                                        u64, ctypes.POINTER(wave_index), vp, sz, vp]
        L.wave_attention_decode.argtypes = [vp, ctypes.POINTER(wave_index), i32, i32, i32, i32, vp,
                                            vp, vp, vp, sz, vp]
        L.wave_attention_decode_static_capacity.argtypes = []
        L.wave_attention_decode_static.argtypes = [vp, ctypes.POINTER(wave_index), i32, i32, i32, i32,
                                                   vp, vp, vp, vp]
        L.wave_attention_decode_budget_workspace.argtypes = [ctypes.POINTER(wave_index), i32, i32, i32]
        L.wave_attention_decode_budget.argtypes = [vp, ctypes.POINTER(wave_index), i32, i32, i32, i32,
                                                   i32, vp, vp, vp, vp, sz, vp]
        L.wave_full_attention_workspace.argtypes = [i32, i32, i32, i32]
        L.wave_full_attention_decode.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp,
                                                 sz, vp]
        L.wave_init_indices.argtypes = [u64, i32, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_int32)]
        L.wave_kmeans_assign_step.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
        L.wave_calibration_copy.argtypes = [vp, vp, sz, i32, vp]
        L.wave_calibration_read.argtypes = [vp, sz, vp, i32, vp]
        L.wave_profile_enable.argtypes = [i32]
        L.wave_profile_read.argtypes = [ctypes.POINTER(ctypes.c_char_p),
                                        ctypes.POINTER(ctypes.c_float),
                                        ctypes.POINTER(ctypes.c_int), i32]
        L.wave_status_string.argtypes = [i32]
        L.wave_status_string.restype = ctypes.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = i32
        L.wave_full_attention_workspace.restype = sz
        L.wave_attention_decode_static_capacity.restype = sz
        L.wave_attention_decode_budget_workspace.restype = sz
        _lib = L
    return _lib


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return WAVE_F32
    if dt == torch.bfloat16:
        return WAVE_BF16
    raise WaveError(3, "dtype")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None or t.numel() == 0:
        return None
    assert t.is_contiguous()
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Index:
    """A wave_index struct plus the torch tensors that own its buffers."""

    def __init__(self, c: wave_index, tensors: Dict[str, torch.Tensor], dtype: torch.dtype,
                 build_ws_bytes: int):
        self.c = c
        self.t = tensors
        self.dtype = dtype
        self.build_ws_bytes = build_ws_bytes

    def __getattr__(self, name):
        if name in ("B", "Hkv", "d", "N", "n_sink", "n_local", "segment_len",
                    "clusters_per_segment", "S", "m", "N_idx", "p", "appended_segments",
                    "update_segment_len", "update_clusters", "row_capacity", "steady_capacity",
                    "cluster_capacity"):
            return getattr(self.c, name)
        if name in BUFFER_NAMES:
            return self.t[name]
        raise AttributeError(name)


def _shapes(c: wave_index) -> Dict[str, Tuple[int, ...]]:
    u = (c.B, c.Hkv)
    rows = c.row_capacity if c.row_capacity > 0 else c.N_idx   # the first N_idx rows are in use
    prow = c.steady_capacity if c.steady_capacity > 0 else c.p  # the first p rows are in use
    mc = c.cluster_capacity if c.cluster_capacity > 0 else c.m   # the first m clusters are in use
    return {"centroids": u + (mc, c.d), "vsum": u + (mc, c.d), "sizes": u + (mc,),
            "offsets": u + (mc + 1,), "perm": u + (rows,), "k_perm": u + (rows, c.d),
            "v_perm": u + (rows, c.d), "k_steady": u + (prow, c.d), "v_steady": u + (prow, c.d)}


def wave_index_plan(dtype: torch.dtype, B: int, Hkv: int, d: int, N: int, n_sink: int, n_local: int,
                    segment_len: int, clusters_per_segment: int, Hq: Optional[int] = None,
                    topk_clusters: int = 0, row_capacity: int = 0, steady_capacity: int = 0,
                    cluster_capacity: int = 0) -> Tuple[wave_index, List[int], int, Optional[int]]:
    """Returns (struct with derived fields, byte sizes of the nine buffers,
    build workspace bytes, decode workspace bytes or None)."""
    c = wave_index()
    c.dtype, c.B, c.Hkv, c.d, c.N = _dtype_code(dtype), B, Hkv, d, N
    c.n_sink, c.n_local, c.segment_len, c.clusters_per_segment = n_sink, n_local, segment_len, clusters_per_segment
    c.row_capacity, c.steady_capacity = row_capacity, steady_capacity
    c.cluster_capacity = cluster_capacity
    sizes = (ctypes.c_size_t * WAVE_INDEX_BUFFERS)()
    bws, dws = ctypes.c_size_t(0), ctypes.c_size_t(0)
    st = lib().wave_index_plan(ctypes.byref(c), sizes, ctypes.byref(bws), Hq or 0, topk_clusters,
                               ctypes.byref(dws) if Hq else None)
    if st != 0:
        raise WaveError(st, "wave_index_plan")
    return c, list(sizes), bws.value, (dws.value if Hq else None)


def alloc_index(dtype: torch.dtype, B: int, Hkv: int, d: int, N: int, n_sink: int, n_local: int,
                segment_len: int, clusters_per_segment: int, device="cuda",
                row_capacity: int = 0, steady_capacity: int = 0, cluster_capacity: int = 0) -> Index:
    """Plans and allocates an empty index on the device (row_capacity > 0: room for that many
    permuted rows per unit, cluster_capacity > 0: for that many clusters per unit, so that
    index updates can add rows and clusters in place)."""
    c, sizes, bws, _ = wave_index_plan(dtype, B, Hkv, d, N, n_sink, n_local, segment_len,
                                       clusters_per_segment, row_capacity=row_capacity,
                                       steady_capacity=steady_capacity, cluster_capacity=cluster_capacity)
    tensors = {}
    for name, nbytes in zip(BUFFER_NAMES, sizes):
        dt = torch.int32 if name in ("sizes", "offsets", "perm") else dtype
        t = torch.empty(_shapes(c)[name], dtype=dt, device=device)
        assert t.numel() * t.element_size() == nbytes, (name, t.shape, nbytes)
        tensors[name] = t
        setattr(c, name, _ptr(t))
    return Index(c, tensors, dtype, bws)


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def wave_index_build(K: torch.Tensor, V: torch.Tensor, n_sink: int, n_local: int, segment_len: int,
                     clusters_per_segment: int, iters: int, seed: int,
                     ws: Optional[torch.Tensor] = None, index: Optional[Index] = None,
                     row_capacity: int = 0, steady_capacity: int = 0, cluster_capacity: int = 0) -> Index:
    """K, V: [B, Hkv, N, d] device tensors (f32 or bf16).  Enqueues the build on
    the current stream and returns the index (valid after a stream sync)."""
    assert K.is_cuda and V.is_cuda and K.shape == V.shape and K.dtype == V.dtype
    K, V = K.contiguous(), V.contiguous()
    B, Hkv, N, d = K.shape
    ix = index or alloc_index(K.dtype, B, Hkv, d, N, n_sink, n_local, segment_len,
                              clusters_per_segment, K.device, row_capacity=row_capacity,
                              steady_capacity=steady_capacity, cluster_capacity=cluster_capacity)
    if ws is None:
        ws = workspace(ix.build_ws_bytes, K.device)
    st = lib().wave_index_build(K.data_ptr(), V.data_ptr(), ctypes.byref(ix.c), iters, seed,
                                ws.data_ptr(), ws.numel(), _stream())
    if st != 0:
        raise WaveError(st, "wave_index_build")
    ix._keepalive = (K, V, ws)
    return ix


def wave_index_append(ix: Index, K_new: Optional[torch.Tensor], V_new: Optional[torch.Tensor],
                      n_local_min: int, update_segment_len: int, update_clusters: int, iters: int,
                      seed: int) -> Index:
    """K_new, V_new: [B, Hkv, n_new, d] device tensors of the index's dtype (None for no new
    tokens).  Plans and allocates the grown index, enqueues the update on the current stream
    and returns the new index (valid after a stream sync); `ix` is left as it is.  When no
    update segment is flushed the new index shares the arrays of the clustered part with `ix`
    and only its steady rows are new."""
    n_new = 0 if K_new is None else K_new.shape[2]
    if n_new:
        assert K_new.is_cuda and V_new.is_cuda and K_new.shape == V_new.shape and K_new.dtype == ix.dtype
        assert K_new.shape[:2] == (ix.B, ix.Hkv) and K_new.shape[3] == ix.d
        K_new, V_new = K_new.contiguous(), V_new.contiguous()
    c = wave_index()
    sizes = (ctypes.c_size_t * WAVE_INDEX_BUFFERS)()
    wsb = ctypes.c_size_t(0)
    st = lib().wave_index_append_plan(ctypes.byref(ix.c), n_new, n_local_min, update_segment_len,
                                      update_clusters, ctypes.byref(c), sizes, ctypes.byref(wsb))
    if st != 0:
        raise WaveError(st, "wave_index_append_plan")
    device = ix.t["k_steady"].device if ix.t["k_steady"].numel() else ix.t["k_perm"].device
    tensors = {}
    keep = c.appended_segments == ix.c.appended_segments   # nothing flushed: the clustered part is shared
    in_place = c.row_capacity > 0 and c.row_capacity == ix.c.row_capacity   # rows added behind the old ones
    meta_in_place = c.cluster_capacity > 0 and c.cluster_capacity == ix.c.cluster_capacity   # clusters likewise
    for name, nbytes in zip(BUFFER_NAMES, sizes):
        dt = torch.int32 if name in ("sizes", "offsets", "perm") else ix.dtype
        steady_in_place = (keep and c.steady_capacity > 0 and c.steady_capacity == ix.c.steady_capacity
                           and name in ("k_steady", "v_steady"))   # the new tokens' rows behind the window
        if ((keep and name not in ("k_steady", "v_steady")) or steady_in_place
                or (in_place and name in ("perm", "k_perm", "v_perm"))
                or (meta_in_place and name in ("centroids", "vsum", "sizes", "offsets"))):
            t = ix.t[name]
        else:
            t = torch.empty(_shapes(c)[name], dtype=dt, device=device)
        assert t.numel() * t.element_size() == nbytes, (name, t.shape, nbytes)
        tensors[name] = t
        setattr(c, name, _ptr(t))
    ws = workspace(wsb.value, device)
    st = lib().wave_index_append(ctypes.byref(ix.c), _ptr(K_new) if n_new else None,
                                 _ptr(V_new) if n_new else None, n_new, n_local_min,
                                 update_segment_len, update_clusters, iters, seed, ctypes.byref(c),
                                 ws.data_ptr(), ws.numel(), _stream())
    if st != 0:
        raise WaveError(st, "wave_index_append")
    out = Index(c, tensors, ix.dtype, 0)
    out._keepalive = (K_new, V_new, ws, ix)
    return out


def decode_workspace_bytes(ix: Index, Hq: int, topk_clusters: int) -> int:
    c = wave_index()
    ctypes.memmove(ctypes.byref(c), ctypes.byref(ix.c), ctypes.sizeof(wave_index))
    sizes = (ctypes.c_size_t * WAVE_INDEX_BUFFERS)()
    dws = ctypes.c_size_t(0)
    st = lib().wave_index_plan(ctypes.byref(c), sizes, None, Hq, topk_clusters, ctypes.byref(dws))
    if st != 0:
        raise WaveError(st, "wave_index_plan")
    return dws.value


def wave_attention_decode(q: torch.Tensor, ix: Index, topk_clusters: int, n_sink: Optional[int] = None,
                          n_local: Optional[int] = None, out: Optional[torch.Tensor] = None,
                          lse: Optional[torch.Tensor] = None, selected: Optional[torch.Tensor] = None,
                          ws: Optional[torch.Tensor] = None, want_selected: bool = False):
    """q: [B, Hq, d] device tensor of the index's dtype.  Returns (out [B,Hq,d]
    f32, lse [B,Hq] f32, selected [B,Hq,topk] i32 or None)."""
    assert q.is_cuda and q.dtype == ix.dtype
    q = q.contiguous()
    B, Hq, d = q.shape
    n_sink = ix.n_sink if n_sink is None else n_sink
    n_local = ix.n_local if n_local is None else n_local
    if out is None:
        out = torch.empty(B, Hq, d, dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    if selected is None and want_selected:
        selected = torch.empty(B, Hq, max(topk_clusters, 1), dtype=torch.int32, device=q.device)
    if ws is None:
        ws = workspace(decode_workspace_bytes(ix, Hq, topk_clusters), q.device)
    st = lib().wave_attention_decode(q.data_ptr(), ctypes.byref(ix.c), Hq, topk_clusters, n_sink,
                                     n_local, out.data_ptr(), lse.data_ptr(),
                                     selected.data_ptr() if selected is not None and topk_clusters > 0 else None,
                                     ws.data_ptr(), ws.numel(), _stream())
    if st != 0:
        raise WaveError(st, "wave_attention_decode")
    return out, lse, selected


def wave_attention_decode_static_capacity() -> int:
    return int(lib().wave_attention_decode_static_capacity())


def wave_attention_decode_static(q: torch.Tensor, ix: Index, topk_clusters: int, out: torch.Tensor,
                                 lse: torch.Tensor, selected: Optional[torch.Tensor] = None):
    """wave_attention_decode without a workspace (the library's static scratch array): the
    caller passes every buffer, nothing is allocated here or in the library."""
    assert q.is_cuda and q.dtype == ix.dtype and q.is_contiguous()
    B, Hq, d = q.shape
    assert out.shape == (B, Hq, d) and out.dtype == torch.float32 and out.is_contiguous()
    assert lse.shape == (B, Hq) and lse.dtype == torch.float32 and lse.is_contiguous()
    st = lib().wave_attention_decode_static(
        q.data_ptr(), ctypes.byref(ix.c), Hq, topk_clusters, ix.n_sink, ix.n_local, out.data_ptr(),
        lse.data_ptr(), selected.data_ptr() if selected is not None and topk_clusters > 0 else None,
        _stream())
    if st != 0:
        raise WaveError(st, "wave_attention_decode_static")
    return out, lse, selected


def wave_attention_decode_budget_workspace(ix: Index, Hq: int, topk_clusters: int, est_clusters: int) -> int:
    return int(lib().wave_attention_decode_budget_workspace(ctypes.byref(ix.c), Hq, topk_clusters,
                                                            est_clusters))


def wave_attention_decode_budget(q: torch.Tensor, ix: Index, topk_clusters: int, est_clusters: int,
                                 out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                                 selected: Optional[torch.Tensor] = None,
                                 ws: Optional[torch.Tensor] = None, want_selected: bool = False):
    """As wave_attention_decode, with only the est_clusters best-ranked clusters after the
    retrieved ones estimated (negative: all of them; 0: none)."""
    assert q.is_cuda and q.dtype == ix.dtype
    q = q.contiguous()
    B, Hq, d = q.shape
    if out is None:
        out = torch.empty(B, Hq, d, dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    if selected is None and want_selected:
        selected = torch.empty(B, Hq, max(topk_clusters, 1), dtype=torch.int32, device=q.device)
    if ws is None:
        ws = workspace(wave_attention_decode_budget_workspace(ix, Hq, topk_clusters, est_clusters), q.device)
    st = lib().wave_attention_decode_budget(
        q.data_ptr(), ctypes.byref(ix.c), Hq, topk_clusters, est_clusters, ix.n_sink, ix.n_local,
        out.data_ptr(), lse.data_ptr(),
        selected.data_ptr() if selected is not None and topk_clusters > 0 else None,
        ws.data_ptr(), ws.numel(), _stream())
    if st != 0:
        raise WaveError(st, "wave_attention_decode_budget")
    return out, lse, selected


def wave_full_attention_workspace(B: int, Hq: int, N: int, d: int) -> int:
    return int(lib().wave_full_attention_workspace(B, Hq, N, d))


def wave_full_attention_decode(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                               out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                               ws: Optional[torch.Tensor] = None):
    """q [B, Hq, d], K and V [B, Hkv, N, d], device tensors of one dtype.  Returns
    (out [B,Hq,d] f32, lse [B,Hq] f32) of full attention over all N tokens."""
    assert q.is_cuda and K.is_cuda and V.is_cuda and q.dtype == K.dtype == V.dtype and K.shape == V.shape
    q, K, V = q.contiguous(), K.contiguous(), V.contiguous()
    B, Hq, d = q.shape
    _, Hkv, N, _ = K.shape
    if out is None:
        out = torch.empty(B, Hq, d, dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    if ws is None:
        ws = workspace(wave_full_attention_workspace(B, Hq, N, d), q.device)
    st = lib().wave_full_attention_decode(q.data_ptr(), K.data_ptr(), V.data_ptr(), _dtype_code(q.dtype),
                                          B, Hq, Hkv, N, d, out.data_ptr(), lse.data_ptr(),
                                          ws.data_ptr(), ws.numel(), _stream())
    if st != 0:
        raise WaveError(st, "wave_full_attention_decode")
    return out, lse


def wave_init_indices(seed: int, b: int, h: int, s: int, L_s: int, k_s: int) -> List[int]:
    out = (ctypes.c_int32 * max(k_s, 1))()
    st = lib().wave_init_indices(seed, b, h, s, L_s, k_s, out)
    if st != 0:
        raise WaveError(st, "wave_init_indices")
    return list(out[:k_s])


def wave_kmeans_assign_step(xhat: torch.Tensor, chat: torch.Tensor) -> torch.Tensor:
    """xhat [L_s, d], chat [k_s, d] device tensors of one dtype -> assign [L_s] i32."""
    assert xhat.is_cuda and chat.is_cuda and xhat.dtype == chat.dtype
    xhat, chat = xhat.contiguous(), chat.contiguous()
    L_s, d = xhat.shape
    k_s = chat.shape[0]
    assign = torch.empty(L_s, dtype=torch.int32, device=xhat.device)
    ws = workspace(4 * L_s + 1024, xhat.device)
    st = lib().wave_kmeans_assign_step(xhat.data_ptr(), chat.data_ptr(), _dtype_code(xhat.dtype), L_s,
                                       k_s, d, assign.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    if st != 0:
        raise WaveError(st, "wave_kmeans_assign_step")
    return assign


def wave_calibration_copy(dst: torch.Tensor, src: torch.Tensor, workgroups: int = 8192) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    st = lib().wave_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, workgroups, _stream())
    if st != 0:
        raise WaveError(st, "wave_calibration_copy")


def wave_calibration_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int = 8192) -> None:
    nbytes = src.numel() * src.element_size()
    st = lib().wave_calibration_read(src.data_ptr(), nbytes, sink.data_ptr(), workgroups, _stream())
    if st != 0:
        raise WaveError(st, "wave_calibration_read")


def wave_profile_enable(on: bool) -> None:
    st = lib().wave_profile_enable(1 if on else 0)
    if st != 0:
        raise WaveError(st, "wave_profile_enable")


def wave_profile_read() -> Dict[str, Tuple[float, int]]:
    """{kernel name: (total ms, launches)} since the last read."""
    cap = 64
    names = (ctypes.c_char_p * cap)()
    ms = (ctypes.c_float * cap)()
    cnt = (ctypes.c_int * cap)()
    n = lib().wave_profile_read(names, ms, cnt, cap)
    if n < 0:
        raise WaveError(6, "wave_profile_read")
    return {names[i].decode(): (ms[i], cnt[i]) for i in range(min(n, cap))}


def index_from_arrays(dtype: torch.dtype, B: int, Hkv: int, d: int, N: int, n_sink: int, n_local: int,
                      segment_len: int, clusters_per_segment: int, arrays: Dict[str, torch.Tensor],
                      device="cuda", row_capacity: int = 0, steady_capacity: int = 0,
                      cluster_capacity: int = 0) -> Index:
    """Imports an index from host arrays (the index is plain data: importing it
    is copying its nine arrays).  The arrays are dense; with capacities the device arrays have
    room behind each unit's entries."""
    ix = alloc_index(dtype, B, Hkv, d, N, n_sink, n_local, segment_len, clusters_per_segment, device,
                     row_capacity=row_capacity, steady_capacity=steady_capacity,
                     cluster_capacity=cluster_capacity)
    used = {"centroids": ix.m, "vsum": ix.m, "sizes": ix.m, "offsets": ix.m + 1, "perm": ix.N_idx,
            "k_perm": ix.N_idx, "v_perm": ix.N_idx, "k_steady": ix.p, "v_steady": ix.p}
    for name in BUFFER_NAMES:
        t = ix.t[name]
        if t.numel():
            n = used[name]
            t[:, :, :n].copy_(arrays[name].reshape((B, Hkv, n) + tuple(t.shape[3:])).to(t.dtype))
    return ix
