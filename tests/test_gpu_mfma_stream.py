"""tlt_mfma_stream (the measurement aid that loops a wave tile's matrix instructions on register operands):
its result against the product it stands for, written out with numpy."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def expected_lane_sums(frags_f64, iters):
    """frags_f64 [4 slices][8 fragments][64 lanes][8]: fragment f < 4 is activation block f, f >= 4 weight block f - 4;
    lane l holds row l % 32, k = 8 * (l // 32) .. + 7 of the slice.  Returns the 64 lane sums: lane l holds, of each
    of the 16 blocks C_ij = sum_s A_si B_sj^T (32 x 32), column l % 32 of rows 8 * (v // 4) + 4 * (l // 32) + v % 4."""
    A = np.zeros((4, 4, 32, 16))   # [slice][block][row][k]
    B = np.zeros((4, 4, 32, 16))
    for lane in range(64):
        r, k0 = lane % 32, 8 * (lane // 32)
        A[:, :, r, k0:k0 + 8] = frags_f64[:, :4, lane, :]
        B[:, :, r, k0:k0 + 8] = frags_f64[:, 4:, lane, :]
    out = np.zeros(64)
    for i in range(4):
        for j in range(4):
            Cij = sum(A[s, i] @ B[s, j].T for s in range(4)) * iters
            for lane in range(64):
                rows = [8 * (v // 4) + 4 * (lane // 32) + v % 4 for v in range(16)]
                out[lane] += Cij[rows, lane % 32].sum()
    return out


@pytest.mark.parametrize("iters", [1, 3])
def test_mfma_stream_computes_the_wave_tile_product(iters):
    from paper_2511_16665_amd import binding as tlt
    g = torch.Generator().manual_seed(5 + iters)
    frags = torch.randn(4, 8, 64, 8, generator=g).bfloat16()
    out = torch.full((65536,), float("nan"), dtype=torch.float32, device="cuda")
    assert tlt.mfma_stream(frags.cuda().reshape(-1), out, iters) == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().reshape(1024, 64)   # every wave computes the same product
    want = expected_lane_sums(frags.double().numpy(), iters)
    assert np.array_equal(got, np.broadcast_to(got[0], got.shape))
    # 256 products of 64 terms each per lane, fp32 accumulation of bf16 x bf16 products (exact in fp32)
    assert np.max(np.abs(got[0] - want)) <= 1e-4 * np.sqrt(256 * 64 * iters) * 4


def test_mfma_stream_rejects_bad_arguments():
    from paper_2511_16665_amd import binding as tlt
    frags = torch.zeros(16384, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(65536, dtype=torch.float32, device="cuda")
    lib = tlt.load()
    assert lib.tlt_mfma_stream(None, None, out.data_ptr(), 1) != 0
    assert lib.tlt_mfma_stream(None, frags.data_ptr(), None, 1) != 0
    assert lib.tlt_mfma_stream(None, frags.data_ptr(), out.data_ptr(), 0) != 0
    assert lib.tlt_mfma_stream(None, frags.data_ptr() + 2, out.data_ptr(), 1) != 0
