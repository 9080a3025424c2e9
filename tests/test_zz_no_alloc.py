"""The decode entry point that allocates nothing (its scratch is a static device
array inside the library) against wave_attention_decode on the same inputs: two
calls in a row through the C ABI, the second on a smaller index."""
import numpy as np
import pytest
import torch

from paper_2505_02922_amd import binding as wb
from paper_2505_02922_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

WL = synth.WORKLOADS
FIRST = synth.scaled(WL["llama8b_32k"], name="static_first", B=3, N=9000, Hq=8, Hkv=2, segment_len=2048,
                     clusters_per_segment=128, n_local=200, n_components=256, iters=3,
                     retrieve_frac=0.05)
SECOND = synth.scaled(WL["llama8b_32k"], name="static_second", B=1, N=2100, Hq=4, Hkv=2, segment_len=1024,
                      clusters_per_segment=64, n_local=70, n_components=64, iters=2, retrieve_frac=0.1)
# 384 query heads: the path that selects and retrieves in one workgroup per head
THIRD = synth.scaled(WL["llama8b_32k"], name="static_many_heads", B=48, N=1300, Hq=8, Hkv=2,
                     segment_len=512, clusters_per_segment=32, n_local=40, n_components=64, iters=2,
                     retrieve_frac=0.1)


def _both(wl):
    K, V = synth.make_kv(wl)
    q = synth.make_queries(wl).cuda()
    ix = wb.wave_index_build(K.cuda(), V.cuda(), wl.n_sink, wl.n_local, wl.segment_len,
                             wl.clusters_per_segment, wl.iters, 0)
    r = wl.retrieve_count(ix.m)
    ref_out, ref_lse, ref_sel = wb.wave_attention_decode(q, ix, r, want_selected=True)
    torch.cuda.synchronize()
    out = torch.full((wl.B, wl.Hq, wl.d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((wl.B, wl.Hq), float("nan"), dtype=torch.float32, device="cuda")
    sel = torch.full((wl.B, wl.Hq, r), -7, dtype=torch.int32, device="cuda")
    before = torch.cuda.memory_allocated()
    wb.wave_attention_decode_static(q, ix, r, out, lse, sel)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing allocated through torch
    assert np.array_equal(sel.cpu().numpy(), ref_sel.cpu().numpy()), wl.name
    bar = pu.OUT_MAX_ABS if wl.dtype == "bf16" else pu.OUT_MAX_ABS_F32
    assert float((out - ref_out).abs().max()) <= bar, wl.name
    assert float((lse - ref_lse).abs().max()) <= bar, wl.name
    assert float((out - ref_out).norm() / ref_out.norm()) <= pu.OUT_REL, wl.name
    return float((out - ref_out).abs().max())


def test_static_scratch_decode_matches_the_workspace_decode():
    assert wb.wave_attention_decode_static_capacity() == 64 << 20
    worst = [_both(FIRST), _both(SECOND), _both(THIRD), _both(SECOND)]
    print("max |static - workspace| per call:", worst)


def test_static_scratch_decode_refuses_a_step_that_does_not_fit():
    # 64 sequences x 32 heads x 16384 clusters: 134 MB of scores alone
    wl = synth.scaled(WL["llama8b_32k"], name="static_too_big", B=64, N=8192 * 32 + 1028)
    c, sizes, _, dws = wb.wave_index_plan(wl.torch_dtype(), wl.B, wl.Hkv, wl.d, wl.N, wl.n_sink,
                                          wl.n_local, wl.segment_len, wl.clusters_per_segment,
                                          Hq=wl.Hq, topk_clusters=100)
    assert dws > wb.wave_attention_decode_static_capacity()
    for name in wb.BUFFER_NAMES:      # never dereferenced: the size check comes first
        setattr(c, name, 0x1000)
    import ctypes
    fake = ctypes.c_void_p(0x1000)
    st = wb.lib().wave_attention_decode_static(fake, ctypes.byref(c), wl.Hq, 100, wl.n_sink, wl.n_local,
                                               fake, fake, None, None)
    assert st == 4
