"""tlt_gemm (the projection / LM-head kernel) against a float64 matrix product."""
import numpy as np
import pytest
import torch

from paper_2511_16665_amd import binding as tlt

pytestmark = pytest.mark.gpu


def _case(M, N, K, dtype, out_mode, seed):
    g = torch.Generator().manual_seed(seed)
    A = torch.randn((M, K), generator=g)
    W = torch.randn((N, K), generator=g) * 0.05
    C0 = torch.randn((M, N), generator=g)
    if dtype == tlt.TLT_BF16:
        A, W = A.bfloat16(), W.bfloat16()
    want = A.double().numpy() @ W.double().numpy().T
    if out_mode == 0:
        out = torch.zeros((M, N), dtype=A.dtype, device="cuda")
    else:
        out = C0.clone().cuda() if out_mode == 2 else torch.zeros((M, N), dtype=torch.float32, device="cuda")
    if out_mode == 2:
        want = want + C0.double().numpy()
    print(f"gemm M={M} N={N} K={K} dtype={dtype} out_mode={out_mode}", flush=True)
    tlt.gemm(dtype, out_mode, A.cuda(), W.cuda(), out)
    torch.cuda.synchronize()
    got = out.double().cpu().numpy()
    scale = np.abs(want).max()
    tol = 1e-5 if dtype == tlt.TLT_F32 else (1e-2 if out_mode == 0 else 2e-3)   # bf16 store rounds to 2^-9
    assert np.abs(got - want).max() <= tol * scale


@pytest.mark.parametrize("out_mode", [0, 1, 2])
@pytest.mark.parametrize("M,N,K", [(1, 7, 5), (70, 130, 33), (257, 64, 256)])
def test_gemm_fp32_generic(M, N, K, out_mode):
    _case(M, N, K, tlt.TLT_F32, out_mode, 1)


@pytest.mark.parametrize("out_mode", [0, 1, 2])
@pytest.mark.parametrize("M,N,K", [
    (300, 512, 256),      # 128x128 tiles, ragged M tail, 4 K steps
    (8, 384, 64),         # one K step, tiny M
    (129, 128, 640),      # single N tile
    (1000, 16384, 128),   # 256x256 tiles (>= 256 of them), ragged M tail
    (50, 200, 96),        # shape the MFMA path cannot take -> generic kernel on bf16
    (1100, 3584, 2048),   # few 256x256 tiles, long K: split-K with atomic accumulation in mode 2, ragged M tail
    (1000, 16768, 128),   # 256x256 tiles for the whole rounds of the chip + 128x128 tiles for the remaining columns
    (1000, 16896, 128),   # 256x256 tiles for the whole rounds of the chip + 256x128 tiles for the remaining columns
    (200, 512, 1600),     # 25 K tiles split unevenly over 3 workgroups per tile... when the chip is under-filled
    (1500, 3584, 256),    # 192x128 tiles (more than one round of 128-row tiles, one of 192-row tiles), ragged M tail
    (1530, 4608, 256),    # 256x128 tiles (432 tiles of 128 rows would oversubscribe the chip, 216 of 256 rows fill it once), ragged M tail
    (48, 3584, 2048),     # a handful of rows: 128x128 tiles, K cut four ways when accumulating (mode 2)
    (100, 25600, 192),    # one row of 128x256 tiles (at most 128 rows, a hundred column tiles or more), ragged M
    (200, 66048, 128),    # one row of 256x256 tiles, more than a round of them: whole rounds + a rest of 256x128 tiles
    (100, 66304, 128),    # one row of 128x256 tiles, more than a round: whole rounds + a rest of 128x128 tiles
])
def test_gemm_bf16(M, N, K, out_mode):
    _case(M, N, K, tlt.TLT_BF16, out_mode, 2)


def test_gemm_bf16_split_k_with_uneven_cut_sampled_rows():
    """Down-projection shape class (few 256x256 tiles, K long enough for three splits whose lengths differ
    on purpose), accumulating into fp32 with a ragged M tail: sampled rows against float64."""
    M, N, K = 1100, 3584, 9216
    g = torch.Generator().manual_seed(5)
    A = torch.randn((M, K), generator=g).bfloat16()
    W = (torch.randn((N, K), generator=g) * 0.02).bfloat16()
    C0 = torch.randn((M, N), generator=g)
    out = C0.clone().cuda()
    print(f"gemm split-K M={M} N={N} K={K}", flush=True)
    tlt.gemm(tlt.TLT_BF16, 2, A.cuda(), W.cuda(), out)
    torch.cuda.synchronize()
    rows = [0, 1, 255, 256, 511, 512, 1023, 1024, 1099]
    want = A[rows].double().numpy() @ W.double().numpy().T + C0[rows].double().numpy()
    got = out[rows].double().cpu().numpy()
    assert np.abs(got - want).max() <= 2e-3 * np.abs(want).max()


def test_gemm_bf16_7b_layer_shape_sampled_rows():
    """qkv projection shape of the 7B workload (M = 1536): check a sample of output rows."""
    M, N, K = 1536, 4608, 3584
    g = torch.Generator().manual_seed(3)
    A = torch.randn((M, K), generator=g).bfloat16()
    W = (torch.randn((N, K), generator=g) * 0.02).bfloat16()
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    tlt.gemm(tlt.TLT_BF16, 1, A.cuda(), W.cuda(), out)
    torch.cuda.synchronize()
    rows = [0, 1, 127, 128, 255, 256, 777, 1535]
    want = A[rows].double().numpy() @ W.double().numpy().T
    got = out[rows].double().cpu().numpy()
    assert np.abs(got - want).max() <= 2e-3 * np.abs(want).max()


@pytest.mark.parametrize("M", [40, 100, 256])
def test_lm_head_shape_with_few_rows_sampled_entries(M):
    """The LM head of the 7B workload at the row counts of the drafter's levels and of the long-tail verification
    (40: 128x128 tiles; 100: two rounds of 128x256 tiles and a rest of 128x128 tiles; 256: two rounds of 256x256 tiles
    and a rest of 256x128 tiles): sampled rows against float64, every column."""
    N, K = 152064, 3584
    g = torch.Generator().manual_seed(40 + M)
    A = torch.randn((M, K), generator=g).bfloat16()
    W = torch.empty((N, K), dtype=torch.bfloat16)
    for c0 in range(0, N, 19008):                                  # (drawn in pieces: the fp32 draws of the whole matrix are 2.2 GB)
        W[c0:c0 + 19008] = (torch.randn((19008, K), generator=g) * 0.02).bfloat16()
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    print(f"LM-head shape M={M}", flush=True)
    tlt.gemm(tlt.TLT_BF16, 1, A.cuda(), W.cuda(), out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all().item()
    rows = sorted({0, 1, 31, M // 2, M - 1})
    a = A[rows].double().numpy()
    got = out[rows].double().cpu().numpy()
    scale = 0.0
    worst = 0.0
    for c0 in range(0, N, 19008):
        want = a @ W[c0:c0 + 19008].double().numpy().T
        scale = max(scale, np.abs(want).max())
        worst = max(worst, np.abs(got[:, c0:c0 + 19008] - want).max())
    assert worst <= 2e-3 * scale


@pytest.mark.parametrize("M,N,K,ties", [(1536, 8192, 256, False), (300, 1024, 192, False), (1000, 4096, 320, True),
                                        (129, 512, 3584, False), (1536, 152064, 256, False)])
def test_fused_row_argmax_equals_argmax_of_the_stored_product(M, N, K, ties):
    """tlt_gemm_argmax (the LM head when only the most likely token is wanted) against the argmax of
    the product the plain kernel stores: same accumulation, so the result must be identical, ragged M
    tail and exact ties (small-integer operands: many equal maxima, lowest column must win) included.
    The product itself is checked against float64 on sampled rows: the oracle's argmax wherever its
    top-two gap is above the bf16 bar."""
    g = torch.Generator().manual_seed(M + N)
    if ties:
        A = torch.randint(-2, 3, (M, K), generator=g).float().bfloat16()
        W = torch.randint(-1, 2, (N, K), generator=g).float().bfloat16()
    else:
        A = torch.randn((M, K), generator=g).bfloat16()
        W = (torch.randn((N, K), generator=g) * 0.02).bfloat16()
    Ad, Wd = A.cuda(), W.cuda()
    C = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    tlt.gemm(tlt.TLT_BF16, 1, Ad, Wd, C)
    ws = torch.zeros((M * (N // 128) * 2,), dtype=torch.float32, device="cuda")
    out = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    print(f"fused argmax M={M} N={N} K={K}", flush=True)
    assert tlt.gemm_argmax(Ad, Wd, ws, out) == 0
    torch.cuda.synchronize()
    Cn = C.cpu().numpy()
    np.testing.assert_array_equal(out.cpu().numpy(), Cn.argmax(axis=1))     # numpy: first maximum = lowest column
    rows = [0, 1, M // 2, M - 1]
    want = A[rows].double().numpy() @ W.double().numpy().T
    for r, w in zip(rows, want):
        srt = np.sort(w)
        if ties:
            assert Cn[r].argmax() == w.argmax()                                # small integers: the product is exact
        elif srt[-1] - srt[-2] > 2 * 2e-2 * np.abs(w).max():
            assert out[r].item() == w.argmax()


def test_fused_row_argmax_refuses_shapes_it_does_not_cover():
    A = torch.zeros((32, 256), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((512, 256), dtype=torch.bfloat16, device="cuda")
    ws = torch.zeros((4096,), dtype=torch.float32, device="cuda")
    out = torch.zeros((32,), dtype=torch.int32, device="cuda")
    assert tlt.gemm_argmax(A, W, ws, out) == -5                                # M <= 64
    A = torch.zeros((128, 256), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((128,), dtype=torch.int32, device="cuda")
    assert tlt.gemm_argmax(A, W[:384], ws, out) == -5                          # N % 256
    assert tlt.gemm_argmax(A, W, ws[:16], out) == -2                           # scratch too small


@pytest.mark.parametrize("M,N,K", [(300, 512, 256), (1536, 18944, 256), (1000, 16512, 192), (129, 128, 640),
                                   (100, 25600, 256), (200, 33024, 128), (256, 18944, 512), (200, 12928, 256),
                                   (160, 18432, 128), (130, 24576, 64), (256, 18944, 3584)])
def test_fused_gate_up_projection_matches_float64(M, N, K):
    """tlt_gemm_glu: silu(A Wg^T) * (A Wu^T) in one kernel (256-row weight tiles for the whole rounds of
    the chip, 128-row tiles for the rest, ragged M tail; one row of 128x256 or 256x256 tiles when M is small, or
    of tiles 96 output columns wide, the last of them partial: 18944 = 197 x 96 + 32, 12928 = 134 x 96 + 64),
    against float64 on sampled rows."""
    g = torch.Generator().manual_seed(M + K)
    A = torch.randn((M, K), generator=g).bfloat16()
    Wg = (torch.randn((N, K), generator=g) * 0.1).bfloat16()
    Wu = (torch.randn((N, K), generator=g) * 0.1).bfloat16()
    act = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    print(f"fused gate/up M={M} N={N} K={K}", flush=True)
    assert tlt.gemm_glu(A.cuda(), Wg.cuda(), Wu.cuda(), act) == 0
    torch.cuda.synchronize()
    rows = sorted({r for r in (0, 1, 127, 128, 255, 256, M // 2, M - 1) if r < M})
    a = A[rows].double().numpy()
    gate, up = a @ Wg.double().numpy().T, a @ Wu.double().numpy().T
    want = gate / (1.0 + np.exp(-gate)) * up
    got = act[rows].double().cpu().numpy()
    assert np.abs(got - want).max() <= 2e-2 * np.abs(want).max()
