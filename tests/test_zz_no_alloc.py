"""The entry point that allocates nothing (fatnn_ternary_gemm_noalloc, scratch in a fixed device array inside
the library) against the existing workspace entry point fatnn_ternary_gemm_ws, through the raw C ABI:
bit-identical int32 and fp32 outputs on two calls in a row, the second with a smaller input, plus the
oracle for the first, the size limit, and a captured graph replayed between eager calls."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from test_gpu_parity import dev, DEV

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")


def raw_calls(Wp, Ap, M, N, K, mode, scale, bias, ws):
    """(C, Cf) from the no-allocation entry point and from the workspace entry point, both via ctypes."""
    L = fatnn.lib()
    vp = ctypes.c_void_p
    st = vp(torch.cuda.current_stream().cuda_stream)
    out = []
    for which in ("noalloc", "ws"):
        C = torch.full((M, N), -7, dtype=torch.int32, device=DEV)
        Cf = torch.full((M, N), -7.0, dtype=torch.float32, device=DEV)
        common = (vp(Wp.data_ptr()), vp(Ap.data_ptr()), M, N, K, mode, vp(C.data_ptr()), N, vp(scale.data_ptr()),
                  vp(bias.data_ptr()), vp(Cf.data_ptr()), N)
        if which == "noalloc":
            rc = L.fatnn_ternary_gemm_noalloc(*common, st)
        else:
            rc = L.fatnn_ternary_gemm_ws(*common, vp(ws.data_ptr()), ws.numel(), st)
        assert rc == 0, fatnn.status_str(rc)
        out.append((C, Cf))
    torch.cuda.synchronize()
    return out


def test_noalloc_matches_workspace_entry_point_on_two_calls_in_a_row():
    rnd = np.random.default_rng(77)
    ws = fatnn.gemm_workspace(DEV)
    first = None
    for (M, N, K, mode) in [(512, 1000, 4609, 0), (200, 130, 1500, 1)]:      # the second call is smaller
        Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
        La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
        scale = dev(rnd.uniform(0.5, 1.5, M).astype(np.float32))
        bias = dev(rnd.standard_normal(M).astype(np.float32))
        Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
        Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
        (C0, F0), (C1, F1) = raw_calls(Wp, Ap, M, N, K, mode, scale, bias, ws)
        assert torch.equal(C0, C1) and torch.equal(F0, F1)
        assert np.array_equal(C0.cpu().numpy(), oracle.ternary_gemm(Lw, La, mode))
        if first is None:
            first = (Wp, Ap, M, N, K, mode, scale, bias, C1.clone(), F1.clone())
    # and the first, larger problem once more after the smaller one
    Wp, Ap, M, N, K, mode, scale, bias, Cw, Fw = first
    (C0, F0), _ = raw_calls(Wp, Ap, M, N, K, mode, scale, bias, ws)
    assert torch.equal(C0, Cw) and torch.equal(F0, Fw)


def test_noalloc_limits_and_tiny_problems():
    L = fatnn.lib()
    assert L.fatnn_noalloc_scratch_bytes() == 65536 + 512 * 2 * 16384
    FAKE = ctypes.c_void_p(0x10000)
    # more than 16384 tiles of 64 x 64: refused before any launch
    assert L.fatnn_ternary_gemm_noalloc(FAKE, FAKE, 64 * 200, 64 * 100, 64, 0, FAKE, 64 * 100, None, None, None, 0,
                                        None) == -5
    rnd = np.random.default_rng(3)
    for (M, N, K) in [(1, 1, 1), (3, 70, 33), (64, 64, 256)]:
        Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
        La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
        C = torch.empty((M, N), dtype=torch.int32, device=DEV)
        fatnn.ternary_gemm_noalloc(fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT), fatnn.pack_ternary(dev(La), fatnn.ACT),
                                   M, N, K, 0, C)
        assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))


def test_noalloc_in_a_captured_graph_replayed_between_eager_calls():
    rnd = np.random.default_rng(5)
    M, N, K = 300, 500, 2000
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    La_d = torch.zeros((N, K), dtype=torch.int8, device=DEV)
    Ap = fatnn.pack_ternary(La_d, fatnn.ACT)
    Wp_small = fatnn.pack_ternary(dev(Lw[:64]), fatnn.WEIGHT)   # its row constants sit behind 64 rows
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    fatnn.ternary_gemm_noalloc(Wp, Ap, M, N, K, 0, C)          # first call on the device: outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fatnn.pack_ternary(La_d, fatnn.ACT, out=Ap)
        fatnn.ternary_gemm_noalloc(Wp, Ap, M, N, K, 0, C)
    for rep in range(4):
        La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
        La_d.copy_(dev(La))
        want = oracle.ternary_gemm(Lw, La, 0)
        C.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), want), rep
        # an eager call of another size between the replays shares the same scratch array
        C2 = torch.empty((64, 96), dtype=torch.int32, device=DEV)
        fatnn.ternary_gemm_noalloc(Wp_small, Ap, 64, 96, K, 0, C2)
        torch.cuda.synchronize()
        assert np.array_equal(C2.cpu().numpy(), want[:64, :96])
