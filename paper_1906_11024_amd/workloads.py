"""Seeded synthetic workloads: model shapes, weight tensors and source batches.

This module only *draws inputs*.  It contains none of the method's arithmetic
(no attention, no normalisation, no positional table, no search): both the CPU
oracle's tests and the HIP path's tests/benchmarks take their inputs from here,
so neither side ever sees a value produced by the other.

The model shapes follow the paper's experimental setup (Sec. 4.1: 6+6 layers,
512 hidden units, 8 heads, 2048 FFN units, 32K shared vocabulary, beam 4,
sentences of at most 80 words).  No dataset or trained weight is used: weights
are N(0, 0.02^2) draws and source ids are uniform, which is enough because the
cost and the data flow of the decoder step depend only on shapes.

Random numbers come from numpy's counter-based Philox generator keyed by the
seed; every tensor is drawn in the fixed order of `tensor_specs`.
"""
from __future__ import annotations

import numpy as np

PAD_ID, BOS_ID, EOS_ID = 0, 1, 2

# name -> shape parameters, decode workload and sharing policy (block sizes,
# bottom-up, as in Sec. 3.3 of the paper).
CONFIGS = {
    "tiny": dict(n_enc=2, n_dec=2, d=64, H=4, F=256, V=1000, dtype="f32",
                 batch=2, beam=1, src_len=(16, 16), steps=16,
                 self_pi=[2], encdec_pi=[2], self_kind="dot"),
    "base": dict(n_enc=6, n_dec=6, d=512, H=8, F=2048, V=32000, dtype="f32",
                 batch=64, beam=4, src_len=(20, 60), steps=64,
                 self_pi=[2, 2, 2], encdec_pi=[3, 3], self_kind="dot"),
    "big": dict(n_enc=6, n_dec=6, d=1024, H=16, F=4096, V=32000, dtype="bf16",
                batch=128, beam=4, src_len=(20, 80), steps=96,
                self_pi=[2, 2, 2], encdec_pi=[3, 3], self_kind="dot"),
    "long": dict(n_enc=6, n_dec=12, d=512, H=8, F=2048, V=32000, dtype="f32",
                 batch=32, beam=4, src_len=(128, 128), steps=256,
                 self_pi=[2] * 6, encdec_pi=[4, 4, 4], self_kind="dot"),
    "aan": dict(n_enc=6, n_dec=6, d=512, H=8, F=2048, V=32000, dtype="bf16",
                batch=256, beam=4, src_len=(20, 60), steps=64,
                self_pi=[1] * 6, encdec_pi=[3, 3], self_kind="aan"),
}


def get_config(name: str, **overrides) -> dict:
    cfg = dict(CONFIGS[name])
    cfg["name"] = name
    cfg.update(overrides)
    return cfg


def singleton(n_layers: int) -> list:
    """The policy in which every block has one layer (the unshared model)."""
    return [1] * n_layers


# --------------------------------------------------------------------------
# Weight tensors.  All linear maps are stored [out_features, in_features]
# (y = x W^T + b).  This list *is* the order of the flat weight blob that the
# library's init call takes.
# --------------------------------------------------------------------------
def _attn_specs(prefix, d):
    out = []
    for p in ("q", "k", "v", "o"):
        out.append((f"{prefix}.w{p}", (d, d), "mat"))
        out.append((f"{prefix}.b{p}", (d,), "vec"))
    return out


def _ln_specs(prefix, d):
    return [(f"{prefix}.g", (d,), "gain"), (f"{prefix}.b", (d,), "vec")]


def _ffn_specs(prefix, d, F):
    return [(f"{prefix}.w1", (F, d), "mat"), (f"{prefix}.b1", (F,), "vec"),
            (f"{prefix}.w2", (d, F), "mat"), (f"{prefix}.b2", (d,), "vec")]


def tensor_specs(cfg: dict) -> list:
    """[(name, shape, kind)] in blob order; kind in {mat, vec, gain}."""
    d, F, V = cfg["d"], cfg["F"], cfg["V"]
    specs = [("src_emb", (V, d), "mat"), ("tgt_emb", (V, d), "mat")]
    for i in range(cfg["n_enc"]):
        specs += _attn_specs(f"enc{i}.attn", d) + _ln_specs(f"enc{i}.ln1", d)
        specs += _ffn_specs(f"enc{i}.ffn", d, F) + _ln_specs(f"enc{i}.ln2", d)
    for i in range(cfg["n_dec"]):
        if cfg["self_kind"] == "aan":
            specs += _ffn_specs(f"dec{i}.aan", d, F)
            specs += [(f"dec{i}.aan.wg", (2 * d, 2 * d), "mat"),
                      (f"dec{i}.aan.bg", (2 * d,), "vec")]
        else:
            specs += _attn_specs(f"dec{i}.self", d)
        specs += _ln_specs(f"dec{i}.ln1", d)
        specs += _attn_specs(f"dec{i}.ctx", d) + _ln_specs(f"dec{i}.ln2", d)
        specs += _ffn_specs(f"dec{i}.ffn", d, F) + _ln_specs(f"dec{i}.ln3", d)
    specs.append(("w_out", (V, d), "mat"))
    return specs


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to
    even) and return them as fp32.  Storage-format conversion only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    u2 = (u + r) & np.uint32(0xFFFF0000)
    return u2.view(np.float32).reshape(a.shape)


def make_weights(cfg: dict, seed: int = 0, std: float = 0.02, sharp: float = 1.0) -> dict:
    """name -> fp32 ndarray.  Matrices, embeddings and biases ~ N(0, std^2);
    LayerNorm gains ~ 1 + N(0, std^2).  With dtype 'bf16' the values are
    rounded once to bf16-representable numbers.  `sharp` multiplies every
    attention W_Q and W_K (a test variant with peaked attention weights)."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    w = {}
    for name, shape, kind in tensor_specs(cfg):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if kind == "gain":
            a = a + np.float32(1.0)
        if sharp != 1.0 and (name.endswith(".wq") or name.endswith(".wk")):
            a = a * np.float32(sharp)
        if cfg["dtype"] == "bf16":
            a = round_to_bf16(a)
        w[name] = a
    return w


def pack_weights(cfg: dict, weights: dict) -> np.ndarray:
    """Flat blob in `tensor_specs` order: fp32 words for dtype 'f32', the upper
    16 bits of each (already bf16-representable) fp32 word for 'bf16'."""
    parts = []
    for name, shape, _ in tensor_specs(cfg):
        a = np.ascontiguousarray(weights[name], dtype=np.float32)
        assert a.shape == tuple(shape), (name, a.shape, shape)
        if cfg["dtype"] == "bf16":
            u = a.view(np.uint32)
            assert not np.any(u & np.uint32(0xFFFF)), f"{name} is not bf16-representable"
            parts.append((u >> np.uint32(16)).astype(np.uint16).ravel().view(np.uint8))
        else:
            parts.append(a.ravel().view(np.uint8))
    return np.concatenate(parts)


def make_source(cfg: dict, seed: int = 0):
    """(src_ids [batch, max_src] int32 padded with PAD_ID, src_len [batch] int32).
    Lengths uniform in cfg['src_len'] (inclusive); ids uniform in [3, V)."""
    rng = np.random.Generator(np.random.Philox(key=seed + 7919))
    lo, hi = cfg["src_len"]
    batch = cfg["batch"]
    lens = rng.integers(lo, hi + 1, size=batch).astype(np.int32)
    max_src = int(hi)
    ids = rng.integers(3, cfg["V"], size=(batch, max_src)).astype(np.int32)
    ids[np.arange(max_src)[None, :] >= lens[:, None]] = PAD_ID
    return ids, lens
