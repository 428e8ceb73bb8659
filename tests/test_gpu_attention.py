"""tlt_attention (the tree-attention kernels on their own) against the oracle's attention, element by
element, on random trees over random paged caches: both kernels, several key chunks, ragged tails,
a one-row tree, empty contexts, 5 and 7 query heads per kv head."""
import numpy as np
import pytest
import torch

from oracle import decoder as dec
from paper_2511_16665_amd import binding as tlt
from synth import fill_kv_pool, random_block_table

from gpu_util import dense_cache, rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Hq,Hkv,n,ctxs,impl", [
    (8, 2, 13, [0, 37, 150], 1),
    (8, 2, 13, [0, 37, 150], 0),
    (28, 4, 48, [700, 90, 4099], 1),        # 336 query rows per kv head: three row tiles per wave
    (40, 8, 32, [1500, 64, 63, 65], 1),     # 160 rows: waves with one and with two row tiles
    (28, 4, 64, [2100, 5], 1),              # 448 rows: two row groups
    (4, 4, 1, [1, 16, 1000], 1),            # one row, one query head per kv head
    (14, 2, 8, [9000], 1),                  # one long sequence cut into many chunks
])
def test_attention_matches_oracle(Hq, Hkv, n, ctxs, impl):
    d, page = 128, 16
    B = len(ctxs)
    ctxs = np.array(ctxs, dtype=np.int32)
    rng = np.random.default_rng(Hq * 100 + n)
    table, n_pages = random_block_table(ctxs + n + 8, page, seed=3, extra_pages=3)
    k, v = fill_kv_pool(1, n_pages, Hkv, page, d, seed=9, dtype=torch.bfloat16)
    qkv_dim = (Hq + 2 * Hkv) * d
    qkv = (torch.randn((B, n, qkv_dim), generator=torch.Generator().manual_seed(1)) * 1.5).bfloat16()
    parent = np.full((B, n), -1, dtype=np.int64)
    mask = np.zeros((B, n), dtype=np.uint64)
    for b in range(B):
        for i in range(n):
            if i > 0:
                parent[b, i] = rng.integers(max(0, i - 4), i)
            mask[b, i] = (mask[b, parent[b, i]] if i > 0 else np.uint64(0)) | np.uint64(1 << i)
    kv = tlt.KV(k[0].cuda(), v[0].cuda(), torch.from_numpy(table.astype(np.int32)).cuda(), torch.from_numpy(ctxs).cuda(),
                int(ctxs.max()))
    out = torch.full((B, n, Hq * d), 7.0, dtype=torch.bfloat16, device="cuda")
    ws = tlt.attention_workspace(B, n, Hq, Hkv, d, int(ctxs.max()) + n + 8)
    print(f"attention Hq={Hq} Hkv={Hkv} n={n} ctx={list(ctxs)} impl={impl}", flush=True)
    rc = tlt.attention(tlt.TLT_BF16, Hq, page, qkv.cuda(), torch.from_numpy(mask.view(np.int64)).cuda(), kv, out, ws, impl)
    assert rc == 0, tlt.ERRORS.get(rc, rc)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().reshape(B, n, Hq, d)
    q = qkv[:, :, : Hq * d].double().numpy().reshape(B, n, Hq, d)
    for b in range(B):
        c = int(ctxs[b])
        K = dense_cache(k, table, b, c + n, page)[0]
        V = dense_cache(v, table, b, c + n, page)[0]
        visible = np.zeros((n, c + n), dtype=bool)
        visible[:, :c] = True
        for i in range(n):
            for j in range(n):
                visible[i, c + j] = bool((int(mask[b, i]) >> j) & 1)
        want = dec.attention(q[b], K, V, visible)
        assert rel_err(got[b], want) <= 2e-2, (b, rel_err(got[b], want))
