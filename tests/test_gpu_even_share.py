"""The even-share ("stream-K") schedule of the tiled GEMM, and its variant that splits only the remainder
of the tile count over the compute units, against the CPU oracle, bit-exact: every
workgroups-per-compute-unit setting, shapes whose tiles are cut between two workgroups and shapes whose
tiles are shared by many, ragged M / N / K, all operators, the fp32 epilogue, small workspaces, and
repeated calls on one workspace (the tile counters must come back to zero)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from test_gpu_parity import dev, DEV

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")

CODE = np.array([0, 1, 3], dtype=np.int8)


def counters_are_zero(ws):
    return not bool(ws[:65536].view(torch.int32).any().item())


@pytest.mark.parametrize("per_cu", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("M,N,K", [(512, 3136, 4609), (4096, 32, 4608), (200, 130, 2500), (70, 1000, 777)])
def test_even_share_every_split_count(tuning, per_cu, M, N, K):
    tuning(gemm_even_share=per_cu)
    rnd = np.random.default_rng(M + N + K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    ws = fatnn.gemm_workspace(DEV)
    want = oracle.ternary_gemm(Lw, La, 0)
    for _ in range(2):                       # the second call finds the counters as the first left them
        C, _ = fatnn.ternary_gemm(Wp, Ap, M, N, K, 0, workspace=ws)
        assert np.array_equal(C.cpu().numpy(), want)
        assert counters_are_zero(ws)


@pytest.mark.parametrize("M,N,K,mode", [(4096, 17, 4608, 0), (4096, 64, 4608, 1), (4096, 128, 4608, 0),
                                        (1000, 100, 9216, 1), (1536, 1536, 4096, 0), (64, 64, 65536, 0),
                                        (65, 65, 8192, 1), (333, 77, 3000, 0)])
def test_even_share_automatic_choice_matches_oracle(M, N, K, mode):
    rnd = np.random.default_rng(M * 3 + N + K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    scale = rnd.uniform(0.5, 1.5, M).astype(np.float32)
    bias = rnd.standard_normal(M).astype(np.float32)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    C, Cf = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode, scale=dev(scale), bias=dev(bias))
    want = oracle.ternary_gemm(Lw, La, mode)
    assert np.array_equal(C.cpu().numpy(), want)
    assert np.array_equal(Cf.cpu().numpy(), oracle.scale_epilogue(want, scale, bias, channel_is_row=True))
    # and the plain call (no workspace) gives the same
    C0, _ = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode, workspace=None)
    assert torch.equal(C, C0)


@pytest.mark.parametrize("nbytes", [65536, 65536 + 8 * 2 * 16384, 65536 + 100 * 2 * 16384, 1 << 20])
def test_even_share_small_workspaces(tuning, nbytes):
    tuning(gemm_even_share=4)
    case = si.cfg5_ragged()
    Lw, La = case.make()
    Lw, La = Lw[:256], La[:700]
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    ws = fatnn.gemm_workspace(DEV, nbytes)
    C, _ = fatnn.ternary_gemm(Wp, Ap, 256, 700, case.K, 0, workspace=ws)
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))
    assert counters_are_zero(ws)


@pytest.mark.parametrize("basis", [0, 1, 2])
def test_even_share_twobit_and_binary_operators(tuning, basis):
    tuning(gemm_even_share=3)
    rnd = np.random.default_rng(70 + basis)
    M, N, K = 300, 200, 3000
    if basis == 2:                                   # the xnor-only ablation runs on ternary codecs
        Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
        La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
        from oracle import alg1
        want = alg1.gemm_xnor_only(Lw[:8], La[:6])
        C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(CODE[Lw])), fatnn.pack_twobit(dev(CODE[La])), M, N, K, basis)
        assert np.array_equal(C.cpu().numpy()[:8, :6], want)
        C0 = fatnn.twobit_gemm(fatnn.pack_twobit(dev(CODE[Lw])), fatnn.pack_twobit(dev(CODE[La])), M, N, K, basis,
                               workspace=None)
        assert torch.equal(C, C0)
    else:
        Qw = rnd.integers(0, 4, size=(M, K), dtype=np.int8)
        Qa = rnd.integers(0, 4, size=(N, K), dtype=np.int8)
        C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(Qw)), fatnn.pack_twobit(dev(Qa)), M, N, K, basis)
        assert np.array_equal(C.cpu().numpy(), oracle.twobit_gemm(Qw, Qa, basis))
    Bw = rnd.integers(0, 2, size=(M, K + 37), dtype=np.int8)
    Ba = rnd.integers(0, 2, size=(N, K + 37), dtype=np.int8)
    Cb = fatnn.binary_gemm(fatnn.pack_binary(dev(Bw)), fatnn.pack_binary(dev(Ba)), M, N, K + 37)
    assert np.array_equal(Cb.cpu().numpy(), oracle.binary_gemm(Bw, Ba))
    assert counters_are_zero(fatnn.gemm_workspace(DEV))


# ----------------------------------------------------------------------------- whole tiles + split remainder
@pytest.mark.parametrize("M,N,K,mode", [(512, 3136, 4609, 0),      # 1568 tiles = 6 per compute unit + 32 (automatic choice)
                                        (416, 3200, 2304, 1),      # 1300 = 5 x 256 + 20
                                        (320, 1000, 2500, 0),      # 320 = 256 + 64, pieces of 2.5 stages
                                        (290, 900, 300, 1),        # two stages per tile: 32 pieces only
                                        (32, 8224, 4096, 0),       # 257 tiles: one tile split eight ways
                                        (200, 1337, 2000, 1),      # ragged M and N
                                        (1024, 2080, 1024, 0)])    # 2080 = 8 x 256 + 32: nine workgroups per unit
def test_split_remainder_matches_oracle(tuning, M, N, K, mode):
    rnd = np.random.default_rng(M + 5 * N + K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    scale = rnd.uniform(0.5, 1.5, M).astype(np.float32)
    bias = rnd.standard_normal(M).astype(np.float32)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    ws = fatnn.gemm_workspace(DEV)
    want = oracle.ternary_gemm(Lw, La, mode)
    wantf = oracle.scale_epilogue(want, scale, bias, channel_is_row=True)
    for setting in (10, 0):                  # forced wherever there is a remainder, then the automatic choice
        tuning(gemm_even_share=setting, gemm_deepk=2)
        for _ in range(2):                   # the second call finds the counters as the first left them
            C, Cf = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode, scale=dev(scale), bias=dev(bias), workspace=ws)
            assert np.array_equal(C.cpu().numpy(), want)
            assert np.array_equal(Cf.cpu().numpy(), wantf)
            assert counters_are_zero(ws)


@pytest.mark.parametrize("nbytes", [65536 + 8 * 2 * 4096, 65536 + 50 * 2 * 4096, 65536 + 2 * 4096])
def test_split_remainder_small_workspaces(tuning, nbytes):
    """A workspace with room for 8 or 48 pieces limits the split; one too small for 8 sends the call to the
    plain launch."""
    tuning(gemm_even_share=10, gemm_deepk=2)
    rnd = np.random.default_rng(nbytes)
    M, N, K = 320, 1000, 2500
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    ws = fatnn.gemm_workspace(DEV, nbytes)
    C, _ = fatnn.ternary_gemm(fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT), fatnn.pack_ternary(dev(La), fatnn.ACT),
                              M, N, K, 0, workspace=ws)
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))
    assert counters_are_zero(ws)


def test_split_remainder_twobit_and_binary_operators(tuning):
    tuning(gemm_even_share=10, gemm_deepk=2)
    rnd = np.random.default_rng(1010)
    M, N, K = 320, 1000, 1500
    Qw = rnd.integers(0, 4, size=(M, K), dtype=np.int8)
    Qa = rnd.integers(0, 4, size=(N, K), dtype=np.int8)
    for basis in (0, 1):
        C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(Qw)), fatnn.pack_twobit(dev(Qa)), M, N, K, basis)
        assert np.array_equal(C.cpu().numpy(), oracle.twobit_gemm(Qw, Qa, basis))
    Bw = rnd.integers(0, 2, size=(M, 2 * K + 5), dtype=np.int8)
    Ba = rnd.integers(0, 2, size=(N, 2 * K + 5), dtype=np.int8)
    Cb = fatnn.binary_gemm(fatnn.pack_binary(dev(Bw)), fatnn.pack_binary(dev(Ba)), M, N, 2 * K + 5)
    assert np.array_equal(Cb.cpu().numpy(), oracle.binary_gemm(Bw, Ba))
    assert counters_are_zero(fatnn.gemm_workspace(DEV))


# ----------------------------------------------------------------------------- even shares of 32 x 32 tiles
@pytest.mark.parametrize("M,N,K,mode", [(128, 512, 8192, 0),       # the automatic choice: 64 tiles, long K
                                        (256, 1024, 16384, 1),     # one tile per compute unit
                                        (100, 300, 9000, 0),       # ragged M, N and K
                                        (512, 3136, 4609, 1),      # forced only: 1568 tiles, four shares per unit
                                        (32, 32, 65536, 0),        # one tile shared by many
                                        (640, 640, 300, 1)])       # two stages per tile
def test_small_tile_even_shares_match_oracle(tuning, M, N, K, mode):
    rnd = np.random.default_rng(3 * M + N + K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    scale = rnd.uniform(0.5, 1.5, M).astype(np.float32)
    bias = rnd.standard_normal(M).astype(np.float32)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    ws = fatnn.gemm_workspace(DEV)
    want = oracle.ternary_gemm(Lw, La, mode)
    wantf = oracle.scale_epilogue(want, scale, bias, channel_is_row=True)
    for setting in (11, 0):
        tuning(gemm_even_share=setting, gemm_deepk=2)
        for _ in range(2):
            C, Cf = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode, scale=dev(scale), bias=dev(bias), workspace=ws)
            assert np.array_equal(C.cpu().numpy(), want)
            assert np.array_equal(Cf.cpu().numpy(), wantf)
            assert counters_are_zero(ws)


def test_small_tile_even_shares_twobit_and_binary_operators(tuning):
    tuning(gemm_even_share=11, gemm_deepk=2)
    rnd = np.random.default_rng(1111)
    M, N, K = 200, 330, 5000
    Qw = rnd.integers(0, 4, size=(M, K), dtype=np.int8)
    Qa = rnd.integers(0, 4, size=(N, K), dtype=np.int8)
    for basis in (0, 1):
        C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(Qw)), fatnn.pack_twobit(dev(Qa)), M, N, K, basis)
        assert np.array_equal(C.cpu().numpy(), oracle.twobit_gemm(Qw, Qa, basis))
    Bw = rnd.integers(0, 2, size=(M, 2 * K + 5), dtype=np.int8)
    Ba = rnd.integers(0, 2, size=(N, 2 * K + 5), dtype=np.int8)
    Cb = fatnn.binary_gemm(fatnn.pack_binary(dev(Bw)), fatnn.pack_binary(dev(Ba)), M, N, 2 * K + 5)
    assert np.array_equal(Cb.cpu().numpy(), oracle.binary_gemm(Bw, Ba))
    assert counters_are_zero(fatnn.gemm_workspace(DEV))


@pytest.mark.parametrize("setting,M,N,K", [(0, 512, 3136, 4609),     # whole tiles plus a split remainder
                                           (0, 128, 512, 8192),      # even shares of 32 x 32 tiles
                                           (4, 300, 500, 2000)])     # even shares of 64 x 64 tiles
def test_workspace_schedules_in_a_captured_graph(tuning, setting, M, N, K):
    """pack + GEMM with a workspace captured into a HIP graph: every replay (new activations each time, eager
    calls on the same workspace in between) equals the oracle; the schedules clear their own counters, no
    memset node is recorded."""
    tuning(gemm_even_share=setting, gemm_deepk=2)
    rnd = np.random.default_rng(M + K + setting)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    La_d = torch.zeros((N, K), dtype=torch.int8, device=DEV)
    Ap = fatnn.pack_ternary(La_d, fatnn.ACT)
    ws = fatnn.gemm_workspace(DEV)
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    fatnn.ternary_gemm(Wp, Ap, M, N, K, 0, out=C, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fatnn.pack_ternary(La_d, fatnn.ACT, out=Ap)
        fatnn.ternary_gemm(Wp, Ap, M, N, K, 0, out=C, workspace=ws)
    for rep in range(4):
        La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
        La_d.copy_(dev(La))
        want = oracle.ternary_gemm(Lw, La, 0)
        C.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(C.cpu().numpy(), want), rep
        C2, _ = fatnn.ternary_gemm(Wp, Ap, M, N, K, 1, workspace=ws)       # eager, other mode, same workspace
        assert np.array_equal(C2.cpu().numpy(), oracle.ternary_gemm(Lw, La, 1))
        assert counters_are_zero(ws)


# ----------------------------------------------------------------------------- few columns, long K
@pytest.mark.parametrize("M,N,K,mode", [(4096, 17, 4608, 0), (4096, 32, 4608, 1), (4096, 64, 4608, 0),
                                        (4096, 128, 4608, 1), (1000, 100, 9216, 0), (70, 33, 2048, 1),
                                        (4096, 127, 4609, 0), (33, 128, 2049, 0), (512, 20, 65536, 1)])
def test_deepk_kernel_matches_oracle(tuning, M, N, K, mode):
    """Fully connected layers at batch 17-128 (Supplementary S1: a convolution whose filter covers the map)."""
    tuning(gemm_deepk=1)          # the kernel itself, also where the automatic choice would take another
    rnd = np.random.default_rng(M + 7 * N + K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    scale = rnd.uniform(0.5, 1.5, M).astype(np.float32)
    bias = rnd.standard_normal(M).astype(np.float32)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    C, Cf = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode, scale=dev(scale), bias=dev(bias))
    want = oracle.ternary_gemm(Lw, La, mode)
    assert np.array_equal(C.cpu().numpy(), want)
    assert np.array_equal(Cf.cpu().numpy(), oracle.scale_epilogue(want, scale, bias, channel_is_row=True))
    # odd output pitch (no paired stores) and the tiled kernel on the same operands
    Cbig = torch.full((M, N + 3), -5, dtype=torch.int32, device=DEV)
    fatnn.ternary_gemm(Wp, Ap, M, N, K, mode, out=Cbig[:, :N])
    assert np.array_equal(Cbig.cpu().numpy()[:, :N], want) and bool((Cbig[:, N:] == -5).all())
    tuning(gemm_deepk=2)
    C2, _ = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode)
    assert torch.equal(C, C2)


def test_deepk_kernel_twobit_and_binary_operators(tuning):
    tuning(gemm_deepk=1)
    rnd = np.random.default_rng(123)
    M, N, K = 700, 50, 4000
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    want = oracle.ternary_gemm(Lw, La, 0)
    C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(CODE[Lw])), fatnn.pack_twobit(dev(CODE[La])), M, N, K, 0)
    assert np.array_equal(C.cpu().numpy(), want)          # Eq. 2 on Table 1's codecs = the ternary product
    Qw = rnd.integers(0, 4, size=(M, K), dtype=np.int8)
    Qa = rnd.integers(0, 4, size=(N, K), dtype=np.int8)
    for basis in (0, 1):
        C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(Qw)), fatnn.pack_twobit(dev(Qa)), M, N, K, basis)
        assert np.array_equal(C.cpu().numpy(), oracle.twobit_gemm(Qw, Qa, basis))
    Bw = rnd.integers(0, 2, size=(M, 2 * K + 5), dtype=np.int8)
    Ba = rnd.integers(0, 2, size=(N, 2 * K + 5), dtype=np.int8)
    Cb = fatnn.binary_gemm(fatnn.pack_binary(dev(Bw)), fatnn.pack_binary(dev(Ba)), M, N, 2 * K + 5)
    assert np.array_equal(Cb.cpu().numpy(), oracle.binary_gemm(Bw, Ba))


@pytest.mark.parametrize("per_cu,M,N,K", [(8, 4096, 32, 4608), (4, 512, 3136, 4609), (3, 640, 640, 16384),
                                          (10, 512, 3136, 4609), (10, 32, 8224, 8192), (11, 128, 512, 16384),
                                          (11, 32, 64, 65536)])
def test_even_share_hand_over_is_stable_over_many_calls(tuning, per_cu, M, N, K):
    """The hand-over between workgroups (write-through stores, counter, device-scope loads) has no ordering
    slack: 300 calls in a row, many pieces per tile, every result equal to the oracle's."""
    tuning(gemm_even_share=per_cu, gemm_deepk=2)
    rnd = np.random.default_rng(per_cu + M)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    want = dev(oracle.ternary_gemm(Lw, La, 0))
    ws = fatnn.gemm_workspace(DEV)
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    for _ in range(300):
        C.fill_(-1)
        fatnn.ternary_gemm(Wp, Ap, M, N, K, 0, out=C, workspace=ws)
        bad += (C != want).sum()
    assert int(bad.item()) == 0
    assert counters_are_zero(ws)


@pytest.mark.parametrize("N,deepk", [(5, 0), (20, 1), (33, 2)])
def test_gemm_at_the_k_limit(tuning, N, deepk):
    """K = 2^24, the largest supported: |C| reaches 2K = 2^25 in ReLU mode and stays exact in int32.  The three
    column counts go to the matrix-vector kernel, the K-splitting kernel and the tiled kernel (even shares)."""
    tuning(gemm_deepk=deepk)
    K, M = 1 << 24, 3
    rnd = np.random.default_rng(N)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    Lw[0] = 2                                             # all +1: closed forms below
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    La[0] = 2
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    for mode in (0, 1):
        C, _ = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode)
        C = C.cpu().numpy()
        assert C[0, 0] == (K if mode == 0 else 2 * K)
        assert np.array_equal(C, oracle.ternary_gemm(Lw, La, mode))
