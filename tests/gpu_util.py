"""Helpers shared by the GPU parity tests (host-side plumbing only)."""
import numpy as np
import torch

from oracle import decoder as dec
from paper_2511_16665_amd import binding as tlt
from paper_2511_16665_amd import engine as eng
from synth import make_decoder_weights, make_drafter_weights, random_block_table


def dtype_code(name):
    return tlt.TLT_F32 if name == "fp32" else tlt.TLT_BF16


def make_models(cfg, seed, dtype_name, std=0.02, qkv_bias=False):
    """Weights drawn on the CPU in the storage dtype; returns (device dicts, float64 oracle dicts)."""
    dt = torch.float32 if dtype_name == "fp32" else torch.bfloat16
    tw = make_decoder_weights(cfg, seed, device="cpu", dtype=dt, std=std, qkv_bias=qkv_bias)
    dw = make_drafter_weights(cfg, seed, device="cpu", dtype=dt, std=std)
    to_dev = lambda w: {k: ([{kk: vv.cuda() for kk, vv in l.items()} for l in v] if isinstance(v, list)
                            else ({kk: vv.cuda() for kk, vv in v.items()} if isinstance(v, dict) else v.cuda()))
                        for k, v in w.items()}
    return to_dev(tw), to_dev(dw), dec.weights_to_f64(tw), dec.weights_to_f64(dw)


def make_engine(cfg, dtype_name, tw_dev, dw_dev, B, max_n, max_depth, max_topk, capacity, seed=0, seq_len=None):
    """Engine with empty caches able to hold `capacity` tokens per sequence, pages scattered."""
    code = dtype_code(dtype_name)
    caps = np.full(B, capacity)
    table, n_pages = random_block_table(caps, cfg.page_size, seed, extra_pages=3)
    dtable, dn_pages = random_block_table(caps, cfg.page_size, seed + 1, extra_pages=2)
    sl = np.zeros(B, np.int32) if seq_len is None else seq_len
    kv = eng.alloc_kv(cfg, code, cfg.n_layers, table, n_pages, sl)
    dkv = eng.alloc_kv(cfg, code, 1, dtable, dn_pages, sl)
    e = eng.Engine(cfg, code, tw_dev, dw_dev, B, max_n, max_depth, max_topk, capacity, kv, dkv)
    return e, table, dtable


def dense_cache(pool: torch.Tensor, table: np.ndarray, b: int, length: int, page_size: int):
    """Gather sequence b's first `length` cache rows of every layer: [L, length, Hkv, d] float64."""
    slots = np.arange(length)
    pg = torch.from_numpy(table[b, slots // page_size].astype(np.int64))
    off = torch.from_numpy((slots % page_size).astype(np.int64))
    rows = pool.cpu()[:, pg, :, off, :]                     # advanced indices split by a slice: [length, L, Hkv, d]
    return rows.permute(1, 0, 2, 3).double().numpy()


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    return float(np.max(np.abs(got - want)) / max(np.max(np.abs(want)), 1e-30))


class LazyLayers:
    """Widens one decoder layer at a time to float64 on the host (all layers of a 7B shape at once
    would be tens of GB); prints the layer index so a long oracle run shows progress."""

    def __init__(self, layers):
        self.layers = layers

    def __len__(self):
        return len(self.layers)

    def __iter__(self):
        for l, lw in enumerate(self.layers):
            print(f"  oracle layer {l}", flush=True)
            yield dec.weights_to_f64(lw)


class EmbedRows:
    """Embedding table kept on the device; rows are widened to float64 when the oracle indexes it."""

    def __init__(self, w):
        self.w = w

    def __getitem__(self, idx):
        return self.w[torch.as_tensor(np.asarray(idx), device=self.w.device).long()].double().cpu().numpy()
