"""The entry point that allocates nothing (plc_predict_residual_noalloc, whose workspace is a static
buffer inside libplc.so) against plc_predict_residual, through the C ABI: same symbols, escape lists and
counts, bit for bit, on two calls in a row, the second with a smaller input, so that whatever the first
call left in the shared buffer is there when the second runs."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_15356_amd import plc
from paper_2604_15356_amd.workloads import make_workload

pytestmark = pytest.mark.gpu


def _both_ways(w, dev):
    L = plc.lib()
    dims = plc.make_dims(w.S, w.L, w.H, w.n, w.k, w.d, w.delta, w.qmax,
                         cand_stride=w.cand_k.stride()[:5], act_stride=w.act_k.stride()[:4])
    n_streams, N = w.S * w.L * w.H, 2 * w.n * w.d
    ws_bytes = plc.plc_workspace_bytes(dims)
    assert 0 < ws_bytes <= plc.STATIC_SCRATCH_BYTES
    cap = n_streams * N
    out = []
    for static in (False, True):
        sym = torch.full((n_streams, N), 3, dtype=torch.uint8, device=dev)
        esc_vals = torch.zeros(cap, dtype=torch.int16, device=dev)
        esc_cnt = torch.full((n_streams,), -1, dtype=torch.int32, device=dev)
        esc_off = torch.full((n_streams,), -1, dtype=torch.int64, device=dev)
        pred = torch.zeros((n_streams, N), dtype=torch.float32, device=dev)
        status = torch.zeros(1, dtype=torch.int32, device=dev)
        ptr = lambda t: C.c_void_p(t.data_ptr())
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        common = (C.byref(dims), ptr(w.cand_k), ptr(w.cand_v), ptr(w.probs), ptr(w.act_k), ptr(w.act_v), ptr(sym),
                  ptr(esc_vals), cap, ptr(esc_cnt), ptr(esc_off), ptr(pred))
        if static:
            rc = L.plc_predict_residual_noalloc(*common, ptr(status), stream)
        else:
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
            rc = L.plc_predict_residual(*common, ptr(ws), ws_bytes, ptr(status), stream)
        assert rc == plc.PLC_OK
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        total = int(esc_cnt.sum())
        out.append((sym.cpu().numpy(), esc_cnt.cpu().numpy(), esc_off.cpu().numpy(), esc_vals[:total].cpu().numpy(),
                    pred.cpu().numpy()))
    return out


def test_noalloc_entry_point_matches_the_one_with_a_workspace():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    dev = torch.device("cuda:0")
    plc.lib()
    # first a shape whose tiles overflow their staging rows here and there (noise wide enough to escape
    # often), then a smaller one with few escapes: its tiles find the first call's rows and counts in place
    shapes = [dict(S=2, L=2, H=3, n=700, k=5, d=64, sigma=1.2, seed=71),
              dict(S=1, L=1, H=2, n=37, k=3, d=24, sigma=0.05, seed=72)]
    for i, ov in enumerate(shapes):
        w = make_workload("tiny", device=dev, overrides=ov, random_rows=True)
        print(f"call {i}: S{w.S} L{w.L} H{w.H} n{w.n} k{w.k} d{w.d}", flush=True)
        with_ws, static = _both_ways(w, dev)
        assert int(with_ws[1].sum()) > 0
        for a, b in zip(with_ws, static):
            assert np.array_equal(a, b)


def test_noalloc_entry_point_refuses_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    dims = plc.make_dims(1, 32, 8, 32768, 4, 128, 0.02)          # workspace of 276 MB
    assert plc.plc_workspace_bytes(dims) > plc.STATIC_SCRATCH_BYTES
    p = C.c_void_p(4096)
    rc = plc.lib().plc_predict_residual_noalloc(C.byref(dims), p, p, p, p, p, p, p, 0, p, p, None, p, None)
    assert rc == plc.PLC_ERR_SCRATCH
