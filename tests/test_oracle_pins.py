"""Pins for the CPU oracle: each test ties oracle/san_oracle.py to something
other than itself -- a library routine (torch.nn.Transformer*), a closed form, an
invariant the paper states, or a scalar brute-force restatement on tiny inputs.
None of these tests needs a GPU and none touches the HIP library.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import san_oracle as so
from paper_1906_11024_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(**kw):
    cfg = wl.get_config("tiny", **kw)
    return cfg, wl.make_weights(cfg, seed=3, sharp=4.0)


def make_oracle(cfg, w, self_pi=None, encdec_pi=None, share="A", **kw):
    return so.SanOracle(cfg, w, self_pi or cfg["self_pi"], encdec_pi or cfg["encdec_pi"],
                        encdec_share=share, **kw)


def ragged_source(cfg, seed=0):
    src, lens = wl.make_source(cfg, seed)
    lens = lens.copy()
    lens[0] = 9                       # ragged batch: one short sentence
    src[0, 9:] = wl.PAD_ID
    return src, lens


# ---------------------------------------------------------------- primitives
def test_positional_table_closed_forms():
    pe = so.positional_table(50, 64)
    assert np.allclose(pe[0, 0::2], 0.0) and np.allclose(pe[0, 1::2], 1.0)
    assert pe[1, 0] == pytest.approx(math.sin(1.0), abs=1e-15)
    assert pe[1, 1] == pytest.approx(math.cos(1.0), abs=1e-15)
    # independent formulation: angle = pos * exp(-(2i) ln(10000) / d)
    for pos, i in [(7, 3), (49, 31), (13, 0), (20, 16)]:
        ang = pos * math.exp(-(2 * i) * math.log(10000.0) / 64)
        assert pe[pos, 2 * i] == pytest.approx(math.sin(ang), abs=1e-12)
        assert pe[pos, 2 * i + 1] == pytest.approx(math.cos(ang), abs=1e-12)
    # last channel pair of d=64 has wavelength 10000^(62/64) * 2 pi
    assert pe[10, 62] == pytest.approx(math.sin(10 / 10000 ** (62 / 64)), abs=1e-15)


def test_softmax_rows_sum_to_one_and_mask():
    rng = np.random.default_rng(0)
    Q, K = rng.standard_normal((3, 5, 8)), rng.standard_normal((3, 7, 8))
    S = so.attention_weights(Q, K, 8)
    assert S.shape == (3, 5, 7)
    assert np.allclose(S.sum(-1), 1.0, atol=1e-14) and (S > 0).all()
    mask = np.arange(7)[None, None, :] < 4
    Sm = so.attention_weights(Q, K, 8, mask)
    assert np.allclose(Sm.sum(-1), 1.0, atol=1e-14) and (Sm[..., 4:] == 0).all()
    # masked softmax over 4 keys == unmasked softmax over those 4 keys
    assert np.allclose(Sm[..., :4], so.attention_weights(Q, K[:, :4], 8), atol=1e-15)
    # no key at all -> all-zero weights (degenerate source of length 0)
    S0 = so.attention_weights(Q, K, 8, np.zeros((1, 1, 7), dtype=bool))
    assert (S0 == 0).all()


def test_attention_matches_scalar_loops_and_torch_sdpa():
    rng = np.random.default_rng(1)
    lq, lk, dk, dv = 4, 6, 8, 5
    Q, K, V = rng.standard_normal((lq, dk)), rng.standard_normal((lk, dk)), rng.standard_normal((lk, dv))
    A = so.attention_output(so.attention_weights(Q, K, dk), V)
    # scalar loops straight from Eq. 1-2
    ref = np.zeros((lq, dv))
    for i in range(lq):
        z = [sum(Q[i, c] * K[j, c] for c in range(dk)) / math.sqrt(dk) for j in range(lk)]
        den = sum(math.exp(v) for v in z)
        for j in range(lk):
            for c in range(dv):
                ref[i, c] += math.exp(z[j]) / den * V[j, c]
    assert np.allclose(A, ref, atol=1e-13)
    # library routine
    sd = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])
    assert np.allclose(A, sd[0].numpy(), atol=1e-12)


def test_closed_forms_one_key_and_uniform_and_onehot():
    rng = np.random.default_rng(2)
    Q, K, V = rng.standard_normal((1, 8)), rng.standard_normal((5, 8)), rng.standard_normal((5, 3))
    # one key: S = [1], A = v_0
    S = so.attention_weights(Q, K[:1], 8)
    assert np.array_equal(S, [[1.0]]) and np.array_equal(so.attention_output(S, V[:1]), V[:1])
    # q = 0: uniform weights, A = mean of V
    S = so.attention_weights(np.zeros((1, 8)), K, 8)
    assert np.allclose(S, 0.2) and np.allclose(so.attention_output(S, V), V.mean(0))
    # one dominant score: A -> V_j
    Kd = K.copy()
    Kd[3] = 200.0 * Q[0]
    assert np.allclose(so.attention_output(so.attention_weights(Q, Kd, 8), V), V[3], atol=1e-9)


def test_layer_norm_and_log_softmax_against_torch():
    rng = np.random.default_rng(3)
    x, g, b = rng.standard_normal((4, 16)), rng.standard_normal(16), rng.standard_normal(16)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), torch.from_numpy(b), 1e-5)
    assert np.allclose(so.layer_norm(x, g, b, 1e-5), ref.numpy(), atol=1e-13)
    z = rng.standard_normal((3, 11)) * 5
    assert np.allclose(so.log_softmax(z), torch.log_softmax(torch.from_numpy(z), -1).numpy(), atol=1e-13)
    assert np.allclose(np.exp(so.log_softmax(z)).sum(-1), 1.0)


def test_policy_examples_from_the_paper():
    """Sec. 3.2 / 3.3 / 4.2 name these policies for a 6-layer decoder."""
    rows = [l.split("|") for l in open(os.path.join(GOLDEN, "policies.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 5
    for pol, heads in rows:
        pi = [int(v) for v in pol.split()]
        want = [int(v) - 1 for v in heads.split()]        # file is 1-based like the paper
        assert so.block_heads(pi, 6) == want
    for bad in ([2, 2], [3, 4], [0, 6], [], [6, 1], [-1, 7]):
        with pytest.raises(ValueError):
            so.block_heads(bad, 6)


# ---------------------------------- singleton policy == the standard Transformer
def _pe_independent(n, d):
    pe = torch.zeros(n, d, dtype=torch.float64)
    for pos in range(n):
        for i in range(d // 2):
            ang = pos * math.exp(-(2 * i) * math.log(10000.0) / d)
            pe[pos, 2 * i], pe[pos, 2 * i + 1] = math.sin(ang), math.cos(ang)
    return pe


def _load_mha(mha, w, p):
    t = lambda k: torch.from_numpy(np.asarray(w[k], dtype=np.float64))
    with torch.no_grad():
        mha.in_proj_weight.copy_(torch.cat([t(f"{p}.wq"), t(f"{p}.wk"), t(f"{p}.wv")]))
        mha.in_proj_bias.copy_(torch.cat([t(f"{p}.bq"), t(f"{p}.bk"), t(f"{p}.bv")]))
        mha.out_proj.weight.copy_(t(f"{p}.wo"))
        mha.out_proj.bias.copy_(t(f"{p}.bo"))


def _load_common(layer, w, p, lns):
    t = lambda k: torch.from_numpy(np.asarray(w[k], dtype=np.float64))
    with torch.no_grad():
        layer.linear1.weight.copy_(t(f"{p}.ffn.w1")); layer.linear1.bias.copy_(t(f"{p}.ffn.b1"))
        layer.linear2.weight.copy_(t(f"{p}.ffn.w2")); layer.linear2.bias.copy_(t(f"{p}.ffn.b2"))
        for norm, name in lns:
            norm.weight.copy_(t(f"{p}.{name}.g")); norm.bias.copy_(t(f"{p}.{name}.b"))


def _torch_transformer(cfg, w):
    d, H, F = cfg["d"], cfg["H"], cfg["F"]
    kw = dict(dropout=0.0, activation="relu", batch_first=True, norm_first=False, dtype=torch.float64)
    enc_layers, dec_layers = [], []
    for i in range(cfg["n_enc"]):
        l = torch.nn.TransformerEncoderLayer(d, H, F, layer_norm_eps=1e-5, **kw)
        _load_mha(l.self_attn, w, f"enc{i}.attn")
        _load_common(l, w, f"enc{i}", [(l.norm1, "ln1"), (l.norm2, "ln2")])
        enc_layers.append(l)
    for i in range(cfg["n_dec"]):
        l = torch.nn.TransformerDecoderLayer(d, H, F, layer_norm_eps=1e-5, **kw)
        _load_mha(l.self_attn, w, f"dec{i}.self")
        _load_mha(l.multihead_attn, w, f"dec{i}.ctx")
        _load_common(l, w, f"dec{i}", [(l.norm1, "ln1"), (l.norm2, "ln2"), (l.norm3, "ln3")])
        dec_layers.append(l)
    return enc_layers, dec_layers


def test_singleton_policy_is_the_standard_transformer():
    """Fig. 3(a): with every block of size 1 SAN is the standard model.  The
    standard model here is torch.nn.TransformerEncoder/DecoderLayer (post-norm,
    ReLU) fed the same weights; it is compared with the oracle's encoder, its
    full causal re-forward and (through the next test) its cached decoding."""
    cfg, w = tiny()
    src, lens = ragged_source(cfg)
    orc = make_oracle(cfg, w, [1, 1], [1, 1])
    enc_o = orc.encode(src, lens)
    enc_layers, dec_layers = _torch_transformer(cfg, w)
    d = cfg["d"]
    pe = _pe_independent(32, d)
    pad = torch.from_numpy(np.arange(src.shape[1])[None, :] >= lens[:, None])
    with torch.no_grad():
        x = torch.from_numpy(w["src_emb"].astype(np.float64))[torch.from_numpy(src).long()] * math.sqrt(d) + pe[: src.shape[1]]
        for l in enc_layers:
            l.train()                       # train mode (dropout 0) keeps the plain math path
            x = l(x, src_key_padding_mask=pad)
        for b in range(src.shape[0]):
            assert np.allclose(enc_o[b, : lens[b]], x[b, : lens[b]].numpy(), atol=1e-11)
        rng = np.random.default_rng(5)
        hist = rng.integers(3, cfg["V"], size=(src.shape[0], 9))
        y = torch.from_numpy(w["tgt_emb"].astype(np.float64))[torch.from_numpy(hist).long()] * math.sqrt(d) + pe[:9]
        causal = torch.triu(torch.ones(9, 9, dtype=torch.bool), diagonal=1)
        for l in dec_layers:
            l.train()
            y = l(y, x, tgt_mask=causal, memory_key_padding_mask=pad)
        ref_logits = (y @ torch.from_numpy(w["w_out"].astype(np.float64)).T).numpy()
    got = orc.decode_full(hist, return_all=True)
    assert np.abs(got - ref_logits).max() < 1e-10
    assert np.abs(ref_logits).max() > 0.1


# -------------------------------------------- cached == full causal re-forward
POLICY_CASES = [
    ("dot", [1, 1], [1, 1], "A"),
    ("dot", [2], [2], "A"),
    ("dot", [2], [2], "S"),
    ("dot", [1, 1], [2], "S"),
    ("dot", [2], [1, 1], "A"),
    ("aan", [1, 1], [2], "A"),
    ("aan", [1, 1], [1, 1], "A"),
]


@pytest.mark.parametrize("kind,spi,cpi,share", POLICY_CASES)
def test_cached_decoding_equals_full_reforward(kind, spi, cpi, share):
    """Sec. 4.1: the cache only removes double counting.  Brute force: at every
    step, the cached step's logits must equal a re-forward of the whole prefix
    under a causal mask, for SAN blocks as well (row t of the head's S depends
    only on positions <= t)."""
    cfg = wl.get_config("tiny", self_kind=kind, batch=3, beam=2)
    w = wl.make_weights(cfg, seed=11, sharp=4.0)
    src, lens = wl.make_source(cfg, 1)
    lens[1] = 5
    orc = make_oracle(cfg, w, spi, cpi, share)
    orc.encode(src, lens)
    B = cfg["batch"] * cfg["beam"]
    rng = np.random.default_rng(9)
    hist = np.full((B, 1), wl.BOS_ID)
    for t in range(7):
        logits_c = orc.decode_step(hist[:, -1])
        logits_f = orc.decode_full(hist)
        assert np.abs(logits_c - logits_f).max() < 1e-11, t
        # a beam step with a non-trivial permutation inside each sentence
        parent = (np.arange(B) // 2) * 2 + rng.integers(0, 2, size=B)
        orc.beam_reorder(parent)
        hist = np.concatenate([hist[parent], rng.integers(3, cfg["V"], size=(B, 1))], axis=1)


def test_search_cached_equals_uncached_tokens():
    cfg = wl.get_config("tiny", batch=2, beam=3)
    w = wl.make_weights(cfg, seed=4, sharp=4.0)
    src, lens = wl.make_source(cfg, 2)
    a = make_oracle(cfg, w).search(src, lens, 8, 3, use_cache=True)
    b = make_oracle(cfg, w).search(src, lens, 8, 3, use_cache=False)
    for t in range(8):
        assert np.array_equal(a["tokens"][t], b["tokens"][t])
        assert np.array_equal(a["parents"][t], b["parents"][t])
        assert np.allclose(a["scores"][t], b["scores"][t], atol=1e-10)


# --------------------------------------------------------- SAN block invariants
def _run_steps(orc, cfg, src, lens, steps=5, beam=1):
    orc.encode(src, lens)
    B = cfg["batch"] * beam
    rng = np.random.default_rng(21)
    tok = np.full(B, wl.BOS_ID)
    outs = []
    for _ in range(steps):
        outs.append(orc.decode_step(tok))
        tok = rng.integers(3, cfg["V"], size=B)
    return outs


def test_shared_weights_identical_in_block_and_step0_closed_form():
    cfg, w = tiny()
    src, lens = ragged_source(cfg)
    orc = make_oracle(cfg, w, [2], [2], "S")
    orc.encode(src, lens)
    logits = orc.decode_step(np.full(2, wl.BOS_ID))
    dmp = orc.dump
    # step 0: one key -> S = [1] and A = v_0 = W_V x + b of that layer's own V
    assert np.array_equal(dmp["S_self"][0], np.ones((2, cfg["H"], 1)))
    x0 = w["tgt_emb"][[1, 1]].astype(np.float64) * math.sqrt(cfg["d"]) + _pe_independent(1, cfg["d"]).numpy()
    v0 = x0 @ w["dec0.self.wv"].astype(np.float64).T + w["dec0.self.bv"]
    assert np.allclose(dmp["A_self"][0], v0, atol=1e-13)
    orc.decode_step(np.array([5, 6]))
    orc.decode_step(np.array([7, 8]))
    dmp = orc.dump
    assert np.array_equal(dmp["S_self"][0], dmp["S_self"][1])          # Eq. 4
    assert np.array_equal(dmp["S_ctx"][0], dmp["S_ctx"][1])
    assert np.allclose(dmp["S_self"][0].sum(-1), 1.0) and np.allclose(dmp["S_ctx"][0].sum(-1), 1.0)
    assert (dmp["S_ctx"][0][0, :, 9:] == 0).all()                       # masked source padding
    assert not np.allclose(dmp["A_self"][0], dmp["A_self"][1])          # own V per layer (Fig. 3(b))
    assert not np.allclose(dmp["A_ctx"][0], dmp["A_ctx"][1])            # mode S: own V
    orcA = make_oracle(cfg, w, [2], [2], "A")
    _run_steps(orcA, cfg, src, lens, 3)
    assert np.array_equal(orcA.dump["A_ctx"][0], orcA.dump["A_ctx"][1])  # Eq. 5
    assert np.isfinite(logits).all()


def test_follower_output_is_head_weights_times_own_values():
    """Eq. 4 + Fig. 3(b) restated with scalar loops: A^{m+1} = S^m V^{m+1}."""
    cfg, w = tiny()
    src, lens = ragged_source(cfg)
    orc = make_oracle(cfg, w, [2], [2], "A")
    _run_steps(orc, cfg, src, lens, 4)
    S = orc.dump["S_self"][0]                       # [B,H,n]
    Vc = orc.cache_V[1]                             # [B,H,n,dh]
    B, H, n = S.shape
    dh = cfg["d"] // H
    for r in range(B):
        for h in range(H):
            for c in range(dh):
                want = sum(S[r, h, j] * Vc[r, h, j, c] for j in range(n))
                assert orc.dump["A_self"][1][r, h * dh + c] == pytest.approx(want, abs=1e-14)
    assert 1 not in orc.cache_K                     # followers keep no key cache (Sec. 3.2)


def test_discarded_projections_do_not_matter():
    """Sec. 3.2: Q/K transformations of non-head layers can be discarded; in the
    enc-dec block (Eq. 5) a follower has no Q, K or V of its own."""
    cfg, w = tiny()
    src, lens = ragged_source(cfg)
    ref = _run_steps(make_oracle(cfg, w, [2], [2], "A"), cfg, src, lens)
    w2 = dict(w)
    rng = np.random.default_rng(0)
    for k in ("dec1.self.wq", "dec1.self.bq", "dec1.self.wk", "dec1.self.bk",
              "dec1.ctx.wq", "dec1.ctx.bq", "dec1.ctx.wk", "dec1.ctx.bk", "dec1.ctx.wv", "dec1.ctx.bv"):
        w2[k] = rng.standard_normal(w[k].shape)
    got = _run_steps(make_oracle(cfg, w2, [2], [2], "A"), cfg, src, lens)
    assert all(np.array_equal(a, b) for a, b in zip(ref, got))
    # ...while the tensors a follower keeps do matter
    for k in ("dec1.self.wv", "dec1.self.wo", "dec1.ctx.wo"):
        w3 = dict(w); w3[k] = w[k] * 1.5
        got = _run_steps(make_oracle(cfg, w3, [2], [2], "A"), cfg, src, lens)
        assert not np.allclose(ref[-1], got[-1])
    # in mode S the follower's own V projection matters, its Q/K still do not
    refS = _run_steps(make_oracle(cfg, w, [2], [2], "S"), cfg, src, lens)
    w4 = dict(w); w4["dec1.ctx.wq"] = w2["dec1.ctx.wq"]; w4["dec1.ctx.wk"] = w2["dec1.ctx.wk"]
    assert all(np.array_equal(a, b) for a, b in zip(refS, _run_steps(make_oracle(cfg, w4, [2], [2], "S"), cfg, src, lens)))
    w5 = dict(w); w5["dec1.ctx.wv"] = w["dec1.ctx.wv"] * 1.5
    assert not np.allclose(refS[-1], _run_steps(make_oracle(cfg, w5, [2], [2], "S"), cfg, src, lens)[-1])


def test_zero_queries_make_sharing_a_no_op():
    """With W_Q = 0 and b_Q = 0 every layer's weights are uniform, so a shared
    block must give exactly the unshared model's output (the follower still uses
    its own V, W_O, LayerNorm and FFN)."""
    cfg, w = tiny()
    w = dict(w)
    for n in range(2):
        for p in ("self", "ctx"):
            w[f"dec{n}.{p}.wq"] = np.zeros_like(w[f"dec{n}.{p}.wq"])
            w[f"dec{n}.{p}.bq"] = np.zeros_like(w[f"dec{n}.{p}.bq"])
    src, lens = ragged_source(cfg)
    un = _run_steps(make_oracle(cfg, w, [1, 1], [1, 1], "A"), cfg, src, lens)
    sh = _run_steps(make_oracle(cfg, w, [2], [1, 1], "A"), cfg, src, lens)
    shS = _run_steps(make_oracle(cfg, w, [2], [2], "S"), cfg, src, lens)
    for a, b, c in zip(un, sh, shS):
        assert np.allclose(a, b, atol=1e-12) and np.allclose(a, c, atol=1e-12)
    # with live queries the shared model is a different model
    cfg2, wq = tiny()
    un = _run_steps(make_oracle(cfg2, wq, [1, 1], [1, 1]), cfg2, src, lens)
    sh = _run_steps(make_oracle(cfg2, wq, [2], [2]), cfg2, src, lens)
    assert not np.allclose(un[-1], sh[-1])


def test_share_s_with_aliased_values_equals_share_a():
    """Tab. 4 reports one BLEU for both enc-dec rows: sharing S with the same V
    in every layer of the block is the same function as sharing A = S V."""
    cfg, w = tiny()
    w = dict(w)
    w["dec1.ctx.wv"], w["dec1.ctx.bv"] = w["dec0.ctx.wv"], w["dec0.ctx.bv"]
    src, lens = ragged_source(cfg)
    a = _run_steps(make_oracle(cfg, w, [2], [2], "A"), cfg, src, lens)
    s = _run_steps(make_oracle(cfg, w, [2], [2], "S"), cfg, src, lens)
    assert all(np.allclose(x, y, atol=1e-12) for x, y in zip(a, s))


def test_policy_blocks_are_independent():
    """{2,2} on 4 layers: the second block's weights come from layer 3, not 1."""
    cfg = wl.get_config("tiny", n_dec=4)
    w = wl.make_weights(cfg, seed=8, sharp=4.0)
    src, lens = wl.make_source(cfg, 0)
    orc = make_oracle(cfg, w, [2, 2], [1, 3])
    _run_steps(orc, cfg, src, lens, 4)
    d = orc.dump
    assert np.array_equal(d["S_self"][2], d["S_self"][3]) and not np.allclose(d["S_self"][0], d["S_self"][2])
    assert np.array_equal(d["A_ctx"][1], d["A_ctx"][3]) and not np.allclose(d["A_ctx"][0], d["A_ctx"][1])
    assert sorted(orc.cache_K) == [0, 2] and sorted(orc.cache_V) == [0, 1, 2, 3]
    assert sorted(orc.mem_K) == [0, 1] and sorted(orc.mem_V) == [0, 1]


# ------------------------------------------------------------------------ AAN
def test_aan_step0_mean_is_input_and_matches_averaging_matrix():
    cfg = wl.get_config("tiny", self_kind="aan")
    w = wl.make_weights(cfg, seed=2)
    src, lens = wl.make_source(cfg, 0)
    orc = make_oracle(cfg, w, [1, 1], [2])
    orc.encode(src, lens)
    hist = np.array([[1, 9, 30, 7], [1, 12, 5, 99]])
    for t in range(4):
        orc.decode_step(hist[:, t])
        if t == 0:
            x0 = w["tgt_emb"][hist[:, 0]].astype(np.float64) * math.sqrt(cfg["d"]) + _pe_independent(1, cfg["d"]).numpy()
            assert np.allclose(orc.aan_sum[0], x0, atol=1e-13)
    # re-forward with an explicit lower-triangular averaging matrix
    n, d = 4, cfg["d"]
    M = np.tril(np.ones((n, n))) / np.arange(1, n + 1)[:, None]
    x = w["tgt_emb"][hist].astype(np.float64) * math.sqrt(d) + _pe_independent(n, d).numpy()[None]
    avg = np.einsum("ij,bjd->bid", M, x)
    assert np.allclose(orc.aan_sum[0] / 4.0, avg[:, -1], atol=1e-13)


# ---- the AAN gate (Tab. 6 rows "+AAN"): pins that do not repeat the oracle's formula
def _ln_torch(v, g, b, eps=1e-5):
    return torch.nn.functional.layer_norm(torch.from_numpy(v), (v.shape[-1],), torch.from_numpy(g),
                                          torch.from_numpy(b), eps).numpy()


def _gate_fixture(d=8, rows=3, seed=11):
    """An oracle whose only meaningful tensors are the gate and LayerNorm of decoder layer 0."""
    cfg = wl.get_config("tiny", self_kind="aan", d=d, H=2, F=16)
    w = {k: v.astype(np.float64) for k, v in wl.make_weights(cfg, seed=seed).items()}
    rng = np.random.default_rng(seed)
    w["dec0.ln1.g"] = 1.0 + 0.3 * rng.standard_normal(d)
    w["dec0.ln1.b"] = 0.2 * rng.standard_normal(d)
    # magnitudes of at least 1/2, so that a gate fed 100 * value is saturated to rounding
    x = rng.standard_normal((rows, d))
    g = rng.standard_normal((rows, d))
    x, g = x + 0.5 * np.sign(x), g + 0.5 * np.sign(g)
    return cfg, w, x, g


def _gate_pins(oracle_cls):
    """Every closed form the written-down AAN gate must satisfy; returns the names of those that fail.
    Block structure of W_g [2d out, 2d in]: out rows 0..d-1 = input gate i, d..2d-1 = forget gate f;
    in columns 0..d-1 multiply the layer input x, d..2d-1 the averaged-and-transformed state g."""
    failed = []
    cfg, w, x, g = _gate_fixture()
    d = cfg["d"]
    lng, lnb = w["dec0.ln1.g"], w["dec0.ln1.b"]

    def run(wg, bg):
        w2 = dict(w)
        w2["dec0.aan.wg"], w2["dec0.aan.bg"] = wg, bg
        return oracle_cls(cfg, w2, [1, 1], [2])._aan_gate(0, x, g)

    def check(name, got, want, tol=1e-12):
        if not np.allclose(got, want, atol=tol, rtol=0):
            failed.append(name)

    Z, I, z1 = np.zeros((2 * d, 2 * d)), np.eye(d), np.zeros(2 * d)
    # no gate weights, no bias: both gates are 1/2
    check("half_gates", run(Z, z1), _ln_torch(1.5 * x + 0.5 * g, lng, lnb))
    # saturating biases: i = 1, f = 0  ->  LN(2 x);  mirrored: i = 0, f = 1  ->  LN(x + g)
    b_if = np.concatenate([np.full(d, 40.0), np.full(d, -40.0)])
    check("i_open_f_closed", run(Z, b_if), _ln_torch(2.0 * x, lng, lnb), 1e-14)
    check("i_closed_f_open", run(Z, -b_if), _ln_torch(x + g, lng, lnb), 1e-14)
    # one block of W_g at a time, 100 * identity: that gate becomes a step function of x or of g
    def blocks(P=0, Q=0, R=0, S=0):
        wg = Z.copy()
        wg[:d, :d], wg[:d, d:], wg[d:, :d], wg[d:, d:] = P * I, Q * I, R * I, S * I
        return wg
    sx, sg = (x > 0).astype(np.float64), (g > 0).astype(np.float64)
    check("i_from_x", run(blocks(P=100.0), z1), _ln_torch(x + sx * x + 0.5 * g, lng, lnb))
    check("i_from_g", run(blocks(Q=100.0), z1), _ln_torch(x + sg * x + 0.5 * g, lng, lnb))
    check("f_from_x", run(blocks(R=100.0), z1), _ln_torch(1.5 * x + sx * g, lng, lnb))
    check("f_from_g", run(blocks(S=100.0), z1), _ln_torch(1.5 * x + sg * g, lng, lnb))
    # a full asymmetric W_g, recomputed with scalar loops and math.exp on a 2 x 4 problem
    cfg4, w4, x4, g4 = _gate_fixture(d=4, rows=2, seed=12)
    rng = np.random.default_rng(5)
    wg, bg = rng.standard_normal((8, 8)), rng.standard_normal(8)
    w4["dec0.aan.wg"], w4["dec0.aan.bg"] = wg, bg
    got = oracle_cls(cfg4, w4, [1, 1], [2])._aan_gate(0, x4, g4)
    pre = np.zeros((2, 4))
    for r in range(2):
        for c in range(4):
            zi, zf = bg[c], bg[4 + c]
            for k in range(4):
                zi += wg[c, k] * x4[r, k] + wg[c, 4 + k] * g4[r, k]
                zf += wg[4 + c, k] * x4[r, k] + wg[4 + c, 4 + k] * g4[r, k]
            pre[r, c] = x4[r, c] + x4[r, c] / (1.0 + math.exp(-zi)) + g4[r, c] / (1.0 + math.exp(-zf))
    check("scalar_loops", got, _ln_torch(pre, w4["dec0.ln1.g"], w4["dec0.ln1.b"]))
    return failed


def test_sigmoid_against_math_exp():
    for z in (0.0, 1.0, -1.0, 30.0, -30.0, 0.25):
        assert so.sigmoid(np.float64(z)) == pytest.approx(1.0 / (1.0 + math.exp(-z)), rel=1e-15)
    assert so.sigmoid(np.float64(0.0)) == 0.5
    assert so.sigmoid(np.float64(30.0)) > 1 - 1e-12 and so.sigmoid(np.float64(-30.0)) < 1e-12
    v = so.sigmoid(np.array([-2.0, 2.0]))
    assert v[0] + v[1] == pytest.approx(1.0, abs=1e-15) and v[1] > v[0]


def test_aan_gate_closed_forms():
    assert _gate_pins(so.SanOracle) == []


def test_aan_gate_pins_catch_planted_mistakes():
    """The pins above must turn red for each plausible mistake in the gate (planted here, in
    copies of the oracle on the CPU): gate halves swapped, [x; g] order swapped, sigmoid of +z
    in place of -z, W_g applied transposed."""
    class SwapHalves(so.SanOracle):
        def _aan_gate(self, n, x, g):
            z = so.linear(np.concatenate([x, g], -1), self.w[f"dec{n}.aan.wg"], self.w[f"dec{n}.aan.bg"])
            f_gate, i_gate = so.sigmoid(z[..., : self.d]), so.sigmoid(z[..., self.d:])
            return self._ln(f"dec{n}.ln1", x + i_gate * x + f_gate * g)

    class SwapConcat(so.SanOracle):
        def _aan_gate(self, n, x, g):
            z = so.linear(np.concatenate([g, x], -1), self.w[f"dec{n}.aan.wg"], self.w[f"dec{n}.aan.bg"])
            i_gate, f_gate = so.sigmoid(z[..., : self.d]), so.sigmoid(z[..., self.d:])
            return self._ln(f"dec{n}.ln1", x + i_gate * x + f_gate * g)

    class WrongSigmoid(so.SanOracle):
        def _aan_gate(self, n, x, g):
            z = so.linear(np.concatenate([x, g], -1), self.w[f"dec{n}.aan.wg"], self.w[f"dec{n}.aan.bg"])
            i_gate, f_gate = 1 / (1 + np.exp(z[..., : self.d])), 1 / (1 + np.exp(z[..., self.d:]))
            return self._ln(f"dec{n}.ln1", x + i_gate * x + f_gate * g)

    class Transposed(so.SanOracle):
        def _aan_gate(self, n, x, g):
            z = np.concatenate([x, g], -1) @ self.w[f"dec{n}.aan.wg"] + self.w[f"dec{n}.aan.bg"]
            i_gate, f_gate = so.sigmoid(z[..., : self.d]), so.sigmoid(z[..., self.d:])
            return self._ln(f"dec{n}.ln1", x + i_gate * x + f_gate * g)

    class NoResidual(so.SanOracle):
        def _aan_gate(self, n, x, g):
            z = so.linear(np.concatenate([x, g], -1), self.w[f"dec{n}.aan.wg"], self.w[f"dec{n}.aan.bg"])
            i_gate, f_gate = so.sigmoid(z[..., : self.d]), so.sigmoid(z[..., self.d:])
            return self._ln(f"dec{n}.ln1", i_gate * x + f_gate * g)

    for cls in (SwapHalves, SwapConcat, WrongSigmoid, Transposed, NoResidual):
        assert _gate_pins(cls) != [], cls.__name__


def test_aan_layer_through_decode_step_closed_form():
    """The whole AAN self layer as decode_step runs it, at steps 0 and 1, with the layer's FFN
    output made a known constant (w2 = 0, so g = b2) and the gates saturated: the layer output
    (the oracle's A_self dump) is LN(2 x) resp. LN(x + b2), x = the scaled embedding + position."""
    cfg = wl.get_config("tiny", self_kind="aan")
    w = {k: v.copy() for k, v in wl.make_weights(cfg, seed=2).items()}
    d = cfg["d"]
    w["dec0.aan.w2"][:] = 0.0
    w["dec0.aan.wg"][:] = 0.0
    src, lens = wl.make_source(cfg, 0)
    toks = np.array([[1, 9], [1, 12]])
    pe = _pe_independent(2, d).numpy()
    lng, lnb = w["dec0.ln1.g"].astype(np.float64), w["dec0.ln1.b"].astype(np.float64)
    b2 = w["dec0.aan.b2"].astype(np.float64)
    for sign, want in ((+1.0, lambda x: 2.0 * x), (-1.0, lambda x: x + b2)):
        w["dec0.aan.bg"] = np.concatenate([np.full(d, 40.0 * sign), np.full(d, -40.0 * sign)]).astype(np.float32)
        orc = make_oracle(cfg, w, [1, 1], [2])
        orc.encode(src, lens)
        for t in range(2):
            orc.decode_step(toks[:, t])
            x = w["tgt_emb"][toks[:, t]].astype(np.float64) * math.sqrt(d) + pe[t]
            assert np.allclose(orc.dump["A_self"][0], _ln_torch(want(x), lng, lnb), atol=1e-12)


# --------------------------------------------------------------------- search
def test_topk_brute_force_and_tie_break():
    cfg = wl.get_config("tiny", V=7, batch=2, beam=3)
    orc = so.SanOracle.__new__(so.SanOracle)
    orc.batch, orc.dt, orc.eos_id, orc.last_tokens = 2, np.float64, -1, None
    rng = np.random.default_rng(0)
    logits = rng.integers(-2, 3, size=(6, 7)).astype(np.float64)       # many exact ties
    cum = np.array([0.0, -0.5, -0.5, 0.0, 0.0, -np.inf])
    tok, par, sc, margin = orc.topk(logits, cum, 4)
    lp = logits - np.log(np.exp(logits).sum(-1, keepdims=True))
    for b in range(2):
        cands = []
        for k in range(3):
            for v in range(7):
                cands.append((-(cum[b * 3 + k] + lp[b * 3 + k, v]), k * 7 + v))
        cands.sort()
        for i in range(4):
            assert tok[b, i] == cands[i][1] % 7 and par[b, i] == b * 3 + cands[i][1] // 7
            assert sc[b, i] == pytest.approx(-cands[i][0], abs=1e-12)
        assert margin[b] == pytest.approx(cands[4][0] - cands[3][0], abs=1e-12)
    assert (par[1] != 5).all()                   # a dead (-inf) beam is never a parent


def test_topk_eos_rule():
    orc = so.SanOracle.__new__(so.SanOracle)
    orc.batch, orc.dt, orc.eos_id = 1, np.float64, 2
    logits = np.zeros((2, 5))
    tok, par, sc, _ = orc.topk(logits, np.array([-1.0, -3.0]), 2, last_tokens=np.array([2, 4]))
    # finished row 0 extends only with EOS at no cost: score stays -1.0
    assert tok[0, 0] == 2 and par[0, 0] == 0 and sc[0, 0] == pytest.approx(-1.0)
    assert par[0, 1] == 1 and sc[0, 1] == pytest.approx(-3.0 - math.log(5))


def test_greedy_equals_argmax_and_beam1():
    cfg, w = tiny()
    src, lens = ragged_source(cfg)
    out = make_oracle(cfg, w).search(src, lens, 6, 1)
    for t in range(6):
        assert np.array_equal(out["tokens"][t], out["logits"][t].argmax(-1))
        assert np.array_equal(out["parents"][t], np.arange(2))


# ----------------------------------------------------------- precision guard
def test_fp32_oracle_agrees_with_fp64():
    cfg, w = tiny()
    src, lens = ragged_source(cfg)
    a = _run_steps(make_oracle(cfg, w), cfg, src, lens)
    b = _run_steps(make_oracle(cfg, w, dtype=np.float32), cfg, src, lens)
    assert b[0].dtype == np.float32
    for x, y in zip(a, b):
        assert np.abs(x - y).max() < 1e-4 * np.abs(x).max()


def test_workload_generator_is_seeded_and_shaped():
    cfg = wl.get_config("tiny")
    w1, w2 = wl.make_weights(cfg, 5), wl.make_weights(cfg, 5)
    assert all(np.array_equal(w1[k], w2[k]) for k in w1)
    assert not np.array_equal(w1["w_out"], wl.make_weights(cfg, 6)["w_out"])
    assert abs(w1["w_out"].std() - 0.02) < 2e-3 and abs(w1["dec0.ln1.g"].mean() - 1) < 0.02
    blob = wl.pack_weights(cfg, w1)
    assert blob.nbytes == 4 * sum(int(np.prod(s)) for _, s, _ in wl.tensor_specs(cfg))
    cb = wl.get_config("tiny", dtype="bf16")
    wb = wl.make_weights(cb, 5)
    assert wl.pack_weights(cb, wb).nbytes * 2 == blob.nbytes
    assert np.abs(wb["w_out"] - w1["w_out"]).max() <= np.abs(w1["w_out"]).max() * 2 ** -8
    src, lens = wl.make_source(wl.get_config("base"), 0)
    assert src.shape == (64, 60) and lens.min() >= 20 and lens.max() <= 60
    assert (src[np.arange(60)[None] >= lens[:, None]] == wl.PAD_ID).all() and (src[:, :20] >= 3).all()


# ------------------------------------------------- encoder-side sharing (Tab. 5)
def test_encoder_side_sharing():
    cfg = wl.get_config("tiny", n_enc=3)
    w = wl.make_weights(cfg, seed=14, sharp=4.0)
    src, lens = ragged_source(cfg)
    a = so.SanOracle(cfg, w, [2], [2])
    b = so.SanOracle(cfg, w, [2], [2], enc_pi=[1, 2])
    ea, eb = a.encode(src, lens), b.encode(src, lens)
    assert np.array_equal(b.enc_S[1], b.enc_S[2]) and not np.allclose(b.enc_S[0], b.enc_S[1])
    assert np.array_equal(a.enc_S[1], b.enc_S[1])           # layers up to the first follower are untouched
    assert not np.allclose(ea, eb)
    assert np.allclose(b.enc_S[1].sum(-1), 1.0) and (b.enc_S[2][0, :, :, 9:] == 0).all()
    # the follower's Q/K projections are discarded, its V projection is not
    w2 = dict(w)
    w2["enc2.attn.wq"] = w["enc2.attn.wq"] * 3 + 1
    w2["enc2.attn.bk"] = w["enc2.attn.bk"] + 1
    assert np.array_equal(so.SanOracle(cfg, w2, [2], [2], enc_pi=[1, 2]).encode(src, lens), eb)
    w3 = dict(w)
    w3["enc2.attn.wv"] = w["enc2.attn.wv"] * 1.5
    assert not np.allclose(so.SanOracle(cfg, w3, [2], [2], enc_pi=[1, 2]).encode(src, lens), eb)
    # zero queries: all weights uniform over the source, sharing is a no-op
    w0 = dict(w)
    for i in range(3):
        w0[f"enc{i}.attn.wq"] = np.zeros_like(w[f"enc{i}.attn.wq"])
        w0[f"enc{i}.attn.bq"] = np.zeros_like(w[f"enc{i}.attn.bq"])
    e0 = so.SanOracle(cfg, w0, [2], [2]).encode(src, lens)
    e1 = so.SanOracle(cfg, w0, [2], [2], enc_pi=[3]).encode(src, lens)
    assert np.allclose(e0, e1, atol=1e-12)
    with pytest.raises(ValueError):
        so.SanOracle(cfg, w, [2], [2], enc_pi=[2, 2])


def test_finished_count_definition():
    """a sentence is finished when every kept hypothesis ends in EOS; none is with EOS handling off"""
    cfg = wl.get_config("tiny")
    w = wl.make_weights(cfg, seed=0)
    orc = so.SanOracle(cfg, w, cfg["self_pi"], cfg["encdec_pi"], eos_id=2)
    toks = np.array([2, 2, 2,   2, 5, 2,   7, 7, 7,   2, 2, 2])
    assert orc.finished(toks, 3) == 2
    assert orc.finished(toks, 1) == 8
    assert so.SanOracle(cfg, w, cfg["self_pi"], cfg["encdec_pi"], eos_id=-1).finished(toks, 3) == 0
