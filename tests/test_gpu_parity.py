"""Parity of the HIP library (through its C ABI) against the CPU oracle, element
by element on the same seeded inputs.

Bars (stated by the task's north star; U13 reading for "relative"):
  fp32: per row max|g-o| / max|o| <= 1e-4 on logits, token ids bit-exact under
        greedy / beam search (on seeds whose smallest top-k margin exceeds 1e-3, so
        that fp32 rounding cannot flip a decision);
  bf16: logits within 2e-2, top-1 agreement wherever the oracle's top-1 margin
        exceeds twice that tolerance.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1906_11024_amd import binding as sb
from paper_1906_11024_amd import workloads as wl
from tests import harness as hz

F32_TOL = 1e-4
BF16_TOL = 2e-2


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run them with -m gpu on an MI355X)")


@pytest.fixture(autouse=True)
def _gpu():
    _need_gpu()
    yield
    torch.cuda.synchronize()


# a shape that spans several GEMM tiles with ragged edges in M (20 rows), N (vocab
# 2004) and in the attention streams (70 cached positions, source lengths 1..37)
MID = dict(n_enc=2, n_dec=4, d=256, H=4, F=512, V=2004, dtype="f32", batch=5, beam=4,
           src_len=(1, 37), steps=70, self_pi=[1, 3], encdec_pi=[2, 2], self_kind="dot", name="mid")


def mid_cfg(**kw):
    c = dict(MID)
    c.update(kw)
    return c


def ragged(cfg, seed):
    src, lens = wl.make_source(cfg, seed)
    lens[0] = cfg["src_len"][0]
    lens[-1] = cfg["src_len"][1]
    src[np.arange(src.shape[1])[None, :] >= lens[:, None]] = wl.PAD_ID
    return src, lens


# ------------------------------------------------------------------ Tiny, fp32
@pytest.mark.parametrize("spi,cpi,share", [([2], [2], "A"), ([1, 1], [1, 1], "A"), ([2], [2], "S"),
                                           ([1, 1], [2], "S"), ([2], [1, 1], "A")])
def test_tiny_greedy_tokens_bit_exact_and_debug_tensors(spi, cpi, share):
    cfg = wl.get_config("tiny")
    steps = cfg["steps"]
    seed, w, src, lens, ref = hz.pick_seed_with_margin(cfg, spi, cpi, share, steps, 1, 1e-3, sharp=4.0)
    gpu = hz.make_gpu(cfg, w, spi, cpi, share, debug=1)
    out = hz.gpu_free_run(gpu, src, lens, 1, steps, keep_logits=True)
    for t in range(steps):
        assert np.array_equal(out["tokens"][t], ref["tokens"][t]), (seed, t)
        assert hz.rel_err_rows(out["logits"][t], ref["logits"][t]).max() <= F32_TOL, (seed, t)
        assert np.abs(out["scores"][t] - ref["scores"][t]).max() <= 1e-3
    # per-layer tensors of the last step against the oracle's dump of the same step
    orc = hz.make_oracle(cfg, w, spi, cpi, share)
    orc.encode(src, lens)
    tok = np.full(2, wl.BOS_ID)
    for t in range(steps):
        orc.decode_step(tok)
        tok = ref["tokens"][t]
    for n in range(cfg["n_dec"]):
        S = gpu.debug_get(sb.SAN_DBG_S_SELF, n).cpu().numpy()
        assert S.shape == (2, cfg["H"], steps)
        assert np.abs(S.sum(-1) - 1).max() < 1e-5                     # rows of S sum to 1 (Eq. 1)
        assert np.abs(S - orc.dump["S_self"][n]).max() < 2e-6
        Sc = gpu.debug_get(sb.SAN_DBG_S_CTX, n).cpu().numpy()
        assert np.abs(Sc - orc.dump["S_ctx"][n]).max() < 2e-6
        for what, key in ((sb.SAN_DBG_A_SELF, "A_self"), (sb.SAN_DBG_A_CTX, "A_ctx"), (sb.SAN_DBG_HIDDEN, "hidden")):
            g = gpu.debug_get(what, n).cpu().numpy()
            assert hz.rel_err_rows(g, orc.dump[key][n]).max() < 2e-5, (n, key)
    # shared tensors are the same memory inside a block (Eq. 4, Eq. 5)
    if spi == [2]:
        a, b = gpu.debug_get(sb.SAN_DBG_S_SELF, 0), gpu.debug_get(sb.SAN_DBG_S_SELF, 1)
        assert torch.equal(a, b)
    if cpi == [2] and share == "A":
        assert torch.equal(gpu.debug_get(sb.SAN_DBG_A_CTX, 0), gpu.debug_get(sb.SAN_DBG_A_CTX, 1))
    gpu.close()


def test_tiny_beam_search_bit_exact():
    cfg = wl.get_config("tiny", batch=3, beam=3)
    steps = 16
    seed, w, src, lens, ref = hz.pick_seed_with_margin(cfg, [2], [2], "A", steps, 3, 1e-3, sharp=4.0)
    gpu = hz.make_gpu(cfg, w, [2], [2], "A")
    out = hz.gpu_free_run(gpu, src, lens, 3, steps)
    for t in range(steps):
        assert np.array_equal(out["tokens"][t], ref["tokens"][t]), (seed, t)
        assert np.array_equal(out["parents"][t], ref["parents"][t]), (seed, t)
    assert any((p != np.arange(9)).any() for p in ref["parents"][1:])    # the beams did reorder
    gpu.close()


# ----------------------------------------------- Mid: several tiles, ragged edges
@pytest.mark.parametrize("share,sharp", [("A", 1.0), ("S", 4.0)])
def test_mid_fp32_lockstep(share, sharp):
    cfg = mid_cfg()
    w = wl.make_weights(cfg, seed=1, sharp=sharp)
    src, lens = ragged(cfg, 1)
    gpu = hz.make_gpu(cfg, w, share=share)
    orc = hz.make_oracle(cfg, w, share=share)
    ls = hz.Lockstep(gpu, orc, src, lens, cfg["beam"])
    for t in range(cfg["steps"]):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    assert sum(ls.log["exact"]) >= 0.9 * cfg["steps"]
    assert any((p.reshape(-1) != np.arange(20)).any() for p in ls.log["parents"][1:])
    gpu.close()


@pytest.mark.parametrize("spi,cpi,share", [([4], [4], "A"), ([4], [2, 2], "S"), ([2, 2], [1, 3], "A"),
                                           ([3, 1], [4], "S"), ([1, 1, 2], [3, 1], "A")])
def test_mid_fp32_policies(spi, cpi, share):
    """Other policies than the default one, among them one block over the whole
    stack (the uniform self-attention policy of Sec. 4.2) and blocks of unequal
    sizes in either attention (Sec. 3.3's learned policies)."""
    cfg = mid_cfg(steps=20)
    w = wl.make_weights(cfg, seed=21, sharp=4.0)
    src, lens = ragged(cfg, 21)
    gpu = hz.make_gpu(cfg, w, spi, cpi, share)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w, spi, cpi, share), src, lens, cfg["beam"])
    for t in range(cfg["steps"]):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    assert sum(ls.log["exact"]) >= 0.8 * cfg["steps"]
    gpu.close()


@pytest.mark.parametrize("beam", [8, 20])
def test_mid_fp32_large_beams(beam):
    """Beam sizes of the paper's speed-vs-beam study (Fig. 5: 4..20)."""
    cfg = mid_cfg(batch=3, beam=beam, steps=24)
    w = wl.make_weights(cfg, seed=12, sharp=4.0)
    src, lens = ragged(cfg, 12)
    gpu = hz.make_gpu(cfg, w, share="S")
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w, share="S"), src, lens, beam)
    for t in range(cfg["steps"]):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    assert sum(ls.log["exact"]) >= 0.8 * cfg["steps"]
    gpu.close()


def test_mid_fp32_empty_source_and_single_row():
    """Degenerate inputs: a sentence of length 0 (zero context vector), batch 1,
    beam 1, and a batch smaller than max_batch."""
    cfg = mid_cfg(batch=3, beam=2)
    w = wl.make_weights(cfg, seed=2)
    src, lens = ragged(cfg, 2)
    lens[1] = 0
    src[1, :] = wl.PAD_ID
    gpu = hz.make_gpu(cfg, w, max_batch=7)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w), src, lens, 2)
    for t in range(6):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    gpu.close()
    cfg1 = mid_cfg(batch=1, beam=1)
    gpu = hz.make_gpu(cfg1, w)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg1, w), src[:1], lens[:1], 1)
    for t in range(6):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    gpu.close()


def test_mid_uncached_mode_matches_oracle_and_cached():
    cfg = mid_cfg(steps=12)
    w = wl.make_weights(cfg, seed=3, sharp=4.0)
    src, lens = ragged(cfg, 3)
    for share in ("A", "S"):
        gpu = hz.make_gpu(cfg, w, share=share, use_cache=0)
        ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w, share=share), src, lens, cfg["beam"])
        for t in range(cfg["steps"]):
            ls.step(logit_tol=F32_TOL)
        assert max(ls.log["logit_err"]) <= F32_TOL
        gpu.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mid_uncached_aan_matches_oracle(dtype):
    """Tab. 6 puts "-Cache" and "+AAN" in one table: the average-attention layer with nothing
    cached (prefix means over all re-computed positions) against the oracle, with beam reordering."""
    cfg = mid_cfg(steps=12, self_kind="aan", self_pi=[1, 1, 1, 1], dtype=dtype)
    w = wl.make_weights(cfg, seed=23, sharp=2.0)
    src, lens = ragged(cfg, 23)
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    gpu = hz.make_gpu(cfg, w, use_cache=0)
    orc = hz.make_oracle(cfg, w)
    ls = hz.Lockstep(gpu, orc, src, lens, cfg["beam"])
    hist = [ls.tokens.cpu().numpy()]
    for t in range(cfg["steps"]):
        lg, lo = ls.step(logit_tol=tol)
        if t in (0, 5):          # the oracle's own full re-forward of the same prefix (its un-cached mode)
            full = orc.decode_full(np.stack(hist, axis=1))
            assert hz.rel_err_rows(lg, full).max() <= tol
        par = ls.log["parents"][-1].reshape(-1)
        hist = [h[par] for h in hist] + [ls.tokens.cpu().numpy()]
    assert max(ls.log["logit_err"]) <= tol
    assert any((p.reshape(-1) != np.arange(20)).any() for p in ls.log["parents"][1:])
    gpu.close()


def test_mid_eos_handling():
    cfg = mid_cfg(steps=10, V=8, batch=4, beam=3)          # tiny vocabulary: EOS gets picked often
    w = wl.make_weights(cfg, seed=4)
    src, lens = wl.make_source(mid_cfg(batch=4), 4)
    src = np.minimum(src, 7)
    gpu = hz.make_gpu(cfg, w, eos_id=wl.EOS_ID)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w, eos_id=wl.EOS_ID), src, lens, 3)
    for t in range(10):
        ls.step(logit_tol=F32_TOL)
    toks = np.stack(ls.log["tokens"])
    assert (toks == wl.EOS_ID).any()
    gpu.close()


# ------------------------------------------------------------------------ bf16
@pytest.mark.parametrize("base,kind", [("tiny", "dot"), ("mid", "dot"), ("mid", "aan")])
def test_bf16_lockstep(base, kind):
    cfg = wl.get_config("tiny", dtype="bf16", batch=3, beam=2) if base == "tiny" else mid_cfg(dtype="bf16", steps=40)
    cfg["self_kind"] = kind
    if kind == "aan":
        cfg["self_pi"] = [1] * cfg["n_dec"]
    w = wl.make_weights(cfg, seed=5, sharp=2.0)
    src, lens = ragged(cfg, 5)
    gpu = hz.make_gpu(cfg, w)
    orc = hz.make_oracle(cfg, w)
    ls = hz.Lockstep(gpu, orc, src, lens, cfg["beam"])
    agree = total = 0
    for t in range(cfg["steps"]):
        lg, lo = ls.step(logit_tol=BF16_TOL)
        scale = np.abs(lo).max(-1)
        top2 = np.sort(lo, axis=-1)[:, -2:]
        safe = (top2[:, 1] - top2[:, 0]) > 2 * BF16_TOL * scale
        assert np.array_equal(lg.argmax(-1)[safe], lo.argmax(-1)[safe])
        agree += int((lg.argmax(-1) == lo.argmax(-1)).sum())
        total += lg.shape[0]
    assert max(ls.log["logit_err"]) <= BF16_TOL
    assert agree >= 0.9 * total
    gpu.close()


@pytest.mark.parametrize("beam,src_len,share,zero_len", [(4, (1, 37), "A", True), (1, (5, 64), "A", False),
                                                         (8, (1, 100), "S", True), (20, (30, 33), "A", False),
                                                         (32, (1, 140), "A", False)])
def test_bf16_memory_attention_on_matrix_cores(beam, src_len, share, zero_len):
    """bf16 models with 64-wide heads run the block head's attention over the encoder memory on
    the matrix cores (memories of 1, 2, 3, 4 and more than 4 blocks of 32 positions take different
    variants; 1 to 32 hypotheses per sentence).  Checked three ways: the logits against the oracle
    (Lockstep), the weights and the context vectors of every layer against the oracle's within what
    bf16 inputs allow, and -- where both get bit-identical inputs, the first block head -- against the
    general-purpose kernel of a second context (cfg.debug bit 2): the same weights to fp32 rounding,
    the same context vectors to one bf16 rounding step."""
    cfg = mid_cfg(dtype="bf16", batch=4, beam=beam, src_len=src_len, steps=5, encdec_pi=[2, 2])
    w = wl.make_weights(cfg, seed=19, sharp=3.0)
    src, lens = ragged(cfg, 19)
    if zero_len:
        lens[1] = 0
        src[1, :] = wl.PAD_ID
    gpu = hz.make_gpu(cfg, w, share=share, debug=1)
    ref = hz.make_gpu(cfg, w, share=share, debug=3)
    orc = hz.make_oracle(cfg, w, share=share)
    ls = hz.Lockstep(gpu, orc, src, lens, beam)
    ref.encode(ls.src_d, ls.len_d)
    ref_logits = torch.empty_like(ls.logits)
    for t in range(cfg["steps"]):
        tokens = ls.tokens.clone()
        ls.step(logit_tol=BF16_TOL)
        ref.decode_step(tokens, ref_logits)
        for n in range(cfg["n_dec"]):
            S = gpu.debug_get(sb.SAN_DBG_S_CTX, n).cpu().numpy()
            A = gpu.debug_get(sb.SAN_DBG_A_CTX, n).cpu().numpy()
            So, Ao = orc.dump["S_ctx"][n], orc.dump["A_ctx"][n]
            live = np.repeat(lens > 0, beam)
            assert np.abs(S[live].sum(-1) - 1).max() < 1e-5 and np.all(S[~live] == 0)
            assert np.abs(S - So[..., :S.shape[-1]]).max() < 3e-2, (t, n)
            assert np.abs(A - Ao).max() <= 3e-2 * max(1.0, np.abs(Ao).max()), (t, n)
            if n == 0:
                Sr = ref.debug_get(sb.SAN_DBG_S_CTX, n).cpu().numpy()
                Ar = ref.debug_get(sb.SAN_DBG_A_CTX, n).cpu().numpy()
                assert np.abs(S - Sr).max() < 2e-6, (t, np.abs(S - Sr).max())
                assert np.all(np.abs(A - Ar) <= 2.0 ** -7 * np.abs(Ar) + 1e-6), (t, np.abs(A - Ar).max())
        assert hz.rel_err_rows(ref_logits.cpu().numpy(), ls.logits.cpu().numpy()).max() < 2e-2
        ref.beam_reorder(ls.o_par.reshape(-1))
    assert max(ls.log["logit_err"]) <= BF16_TOL
    gpu.close()
    ref.close()


@pytest.mark.parametrize("beam", [4, 6, 12, 20])   # each beam range has its own state-reorder kernel
def test_aan_fp32_lockstep(beam):
    cfg = mid_cfg(self_kind="aan", self_pi=[1, 1, 1, 1], steps=30 if beam == 4 else 12, beam=beam)
    w = wl.make_weights(cfg, seed=6)
    src, lens = ragged(cfg, 6)
    gpu = hz.make_gpu(cfg, w)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w), src, lens, cfg["beam"])
    for t in range(cfg["steps"]):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    gpu.close()


def test_aan_gate_closed_forms_on_gpu():
    """The AAN self layer (Tab. 6 rows "+AAN") against closed forms that do not go through the
    oracle's gate: the layer's FFN made a constant (w2 = 0, so g = b2) and the gate weights 0,
    a bias of +-40 saturates the gates (i = 1, f = 0: LN(2 x); i = 0, f = 1: LN(x + b2)), a
    zero bias halves them (LN(1.5 x + 0.5 b2)); x = scaled embedding + position.  These fail
    if the kernel swaps the gate halves or the [x; g] halves of its input."""
    import math
    cfg = mid_cfg(self_kind="aan", self_pi=[1, 1, 1, 1], steps=4)
    d = cfg["d"]
    w = {k: v.copy() for k, v in wl.make_weights(cfg, seed=6).items()}
    w["dec0.aan.w2"][:] = 0.0
    w["dec0.aan.wg"][:] = 0.0
    src, lens = ragged(cfg, 6)
    B = cfg["batch"] * cfg["beam"]
    rng = np.random.default_rng(3)
    toks = rng.integers(3, cfg["V"], size=(2, B)).astype(np.int32)
    pos = np.arange(2, dtype=np.float64)[:, None]
    ang = pos * np.exp(-np.arange(0, d, 2, dtype=np.float64)[None, :] * math.log(10000.0) / d)
    pe = np.zeros((2, d))
    pe[:, 0::2], pe[:, 1::2] = np.sin(ang), np.cos(ang)
    lng, lnb = w["dec0.ln1.g"].astype(np.float64), w["dec0.ln1.b"].astype(np.float64)
    b2 = w["dec0.aan.b2"].astype(np.float64)

    def ln(v):
        return torch.nn.functional.layer_norm(torch.from_numpy(v), (d,), torch.from_numpy(lng), torch.from_numpy(lnb),
                                              1e-5).numpy()

    cases = ((40.0, lambda x: 2.0 * x), (-40.0, lambda x: x + b2), (0.0, lambda x: 1.5 * x + 0.5 * b2))
    for bias, want in cases:
        w["dec0.aan.bg"] = np.concatenate([np.full(d, bias), np.full(d, -bias)]).astype(np.float32)
        gpu = hz.make_gpu(cfg, w, debug=1)
        orc = hz.make_oracle(cfg, w)
        gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
        orc.encode(src, lens)
        logits = torch.empty((B, cfg["V"]), dtype=torch.float32, device="cuda")
        for t in range(2):
            gpu.decode_step(torch.from_numpy(toks[t]).cuda(), logits)
            lo = orc.decode_step(toks[t])
            x = w["tgt_emb"][toks[t]].astype(np.float64) * math.sqrt(d) + pe[t]
            got = gpu.debug_get(sb.SAN_DBG_A_SELF, 0).cpu().numpy()
            assert hz.rel_err_rows(got, ln(want(x))).max() < 2e-5, (bias, t)
            assert hz.rel_err_rows(got, orc.dump["A_self"][0]).max() < 2e-5, (bias, t)
            assert hz.rel_err_rows(logits.cpu().numpy(), lo).max() <= F32_TOL
        gpu.close()


# ------------------------------------------------------- stand-alone beam step
@pytest.mark.parametrize("V,beam,k", [(1000, 1, 1), (2004, 4, 4), (32000, 4, 4), (32000, 5, 20), (40000, 2, 3)])
def test_topk_kernel_against_oracle_same_inputs(V, beam, k):
    cfg = mid_cfg(V=V, batch=3, beam=beam, steps=2)
    w = wl.make_weights(cfg, seed=7)
    src, lens = wl.make_source(cfg, 7)
    gpu = hz.make_gpu(cfg, w)
    gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
    rng = np.random.default_rng(V + beam)
    B = 3 * beam
    # half the rows carry many exact ties (small integers), the rest are continuous
    logits = rng.standard_normal((B, V)).astype(np.float32) * 3
    logits[::2] = rng.integers(-3, 4, size=logits[::2].shape).astype(np.float32)
    cum = (rng.standard_normal(B) * 0.01).astype(np.float32)
    cum[0::beam] = 0.0
    lg, cm = torch.from_numpy(logits).cuda(), torch.from_numpy(cum).cuda()
    o_tok = torch.empty((3, k), dtype=torch.int32, device="cuda")
    o_par = torch.empty((3, k), dtype=torch.int32, device="cuda")
    o_sc = torch.empty((3, k), dtype=torch.float32, device="cuda")
    gpu.topk(lg, cm, k, o_tok, o_par, o_sc)
    orc = hz.make_oracle(cfg, w)
    orc.batch, orc.last_tokens = 3, None
    tok, par, sc, _ = orc.topk(logits, cum, k)
    lp = logits.astype(np.float64) - np.log(np.exp(logits.astype(np.float64)).sum(-1, keepdims=True))
    tg, pg, sg = o_tok.cpu().numpy(), o_par.cpu().numpy(), o_sc.cpu().numpy()
    for b in range(3):
        s_true = cum[pg[b]] + lp[pg[b], tg[b]]
        assert np.abs(s_true - sc[b]).max() < 2e-5 and np.abs(sg[b] - sc[b]).max() < 2e-5
        assert len({(p, t) for p, t in zip(pg[b], tg[b])}) == k
        # exact ties must come out in index order: the integer rows tie exactly
        gaps = np.abs(np.diff(sc[b]))
        if (gaps > 1e-4).all() or beam == 1:
            assert np.array_equal(tg[b], tok[b]) and np.array_equal(pg[b], par[b])
    gpu.close()


# --------------------------------------------------- determinism and footprint
def test_determinism_and_memory_saving():
    cfg = mid_cfg(steps=8)
    w = wl.make_weights(cfg, seed=8)
    src, lens = ragged(cfg, 8)
    runs = []
    for _ in range(2):
        gpu = hz.make_gpu(cfg, w)
        runs.append(hz.gpu_free_run(gpu, src, lens, cfg["beam"], 8, keep_logits=True))
        shared_bytes = (gpu.device_bytes(0), gpu.device_bytes(1))
        gpu.close()
    for a, b in zip(runs[0]["logits"], runs[1]["logits"]):
        assert np.array_equal(a, b)
    gpu = hz.make_gpu(cfg, w, [1, 1, 1, 1], [1, 1, 1, 1])
    single_bytes = (gpu.device_bytes(0), gpu.device_bytes(1))
    gpu.close()
    # Sec. 3.2: fewer parameters and a smaller footprint under sharing
    assert shared_bytes[0] < single_bytes[0] and shared_bytes[1] < single_bytes[1]


def test_rewind_and_reencode_reproduce():
    cfg = mid_cfg(steps=6)
    w = wl.make_weights(cfg, seed=9)
    src, lens = ragged(cfg, 9)
    gpu = hz.make_gpu(cfg, w)
    a = hz.gpu_free_run(gpu, src, lens, cfg["beam"], 6, keep_logits=True)
    gpu.rewind()
    assert gpu.step == 0
    b = hz.gpu_free_run(gpu, src, lens, cfg["beam"], 6, keep_logits=True)
    assert all(np.array_equal(x, y) for x, y in zip(a["logits"], b["logits"]))
    gpu.close()


def test_state_and_capacity_errors():
    cfg = mid_cfg(steps=2)
    w = wl.make_weights(cfg, seed=1)
    gpu = hz.make_gpu(cfg, w)
    tok = torch.ones(20, dtype=torch.int32, device="cuda")
    logits = torch.empty((20, cfg["V"]), dtype=torch.float32, device="cuda")
    gpu.rows = 20
    with pytest.raises(sb.SanError) as e:
        gpu.decode_step(tok, logits)
    assert e.value.code == sb.SAN_ESTATE
    with pytest.raises(sb.SanError) as e:
        gpu.beam_reorder(tok)
    assert e.value.code == sb.SAN_ESTATE
    src, lens = wl.make_source(cfg, 0)
    big = torch.zeros((6, 37), dtype=torch.int32, device="cuda")
    with pytest.raises(sb.SanError) as e:
        gpu.encode(big, torch.ones(6, dtype=torch.int32, device="cuda"))
    assert e.value.code == sb.SAN_ECAPACITY
    gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
    gpu.decode_step(tok, logits)
    gpu.decode_step(tok, logits)
    with pytest.raises(sb.SanError) as e:
        gpu.decode_step(tok, logits)
    assert e.value.code == sb.SAN_ECAPACITY
    # the beam step reads the logits with 16-byte loads and refuses a misaligned buffer
    shifted = torch.zeros(20 * cfg["V"] + 4, dtype=torch.float32, device="cuda")[1:1 + 20 * cfg["V"]]
    cum = torch.zeros(20, dtype=torch.float32, device="cuda")
    o_i = torch.zeros((5, 4), dtype=torch.int32, device="cuda")
    o_f = torch.zeros((5, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(sb.SanError) as e:
        gpu.topk(shifted, cum, 4, o_i, o_i.clone(), o_f)
    assert e.value.code == sb.SAN_EINVAL
    gpu.close()


def test_stream_read_leaves_memory_untouched():
    """the measurement aid only reads: odd sizes and a tail below 16 bytes included"""
    cfg = wl.get_config("tiny")
    gpu = hz.make_gpu(cfg, wl.make_weights(cfg, seed=0))
    for nbytes in (16, 4096 + 16, (1 << 22) + 48, 1000):
        buf = torch.arange(nbytes, dtype=torch.int64, device="cuda").to(torch.uint8)
        ref = buf.clone()
        gpu.stream_read(buf)
        torch.cuda.synchronize()
        assert torch.equal(buf, ref)
    gpu.close()


# ---------------------------------------------------- policy statistics (Sec. 3.3)
def test_js_divergence_between_layers_matches_oracle():
    from oracle import policy_oracle as po
    cfg = mid_cfg(steps=20, self_pi=[1, 1, 1, 1], encdec_pi=[1, 1, 1, 1])
    w = wl.make_weights(cfg, seed=13, sharp=6.0)           # peaked weights: divergences well above 0
    src, lens = ragged(cfg, 13)
    gpu = hz.make_gpu(cfg, w, debug=1)
    orc = hz.make_oracle(cfg, w)
    ls = hz.Lockstep(gpu, orc, src, lens, cfg["beam"])
    L = cfg["n_dec"]
    want_self, want_ctx, count = np.zeros((L, L)), np.zeros((L, L)), 0
    for t in range(cfg["steps"]):
        # the oracle's weights of this step, before the beam step reorders anything
        gpu.decode_step(ls.tokens, ls.logits)
        gpu.policy_accumulate()
        orc.decode_step(ls.tokens.cpu().numpy())
        S_self = [orc.dump["S_self"][n] for n in range(L)]
        S_ctx = [orc.dump["S_ctx"][n] for n in range(L)]
        B, H = S_self[0].shape[:2]
        want_self += po.layer_js_matrix(S_self) * B * H
        want_ctx += po.layer_js_matrix(S_ctx) * B * H
        count += B * H
        # free-running greedy-like continuation on both sides with the oracle's choice
        tok = torch.from_numpy(np.argsort(-orc.dump["hidden"][L - 1][:, :7], axis=-1)[:, 0].astype(np.int32) + 3).cuda()
        ls.tokens = tok
    js_self, n_self = gpu.policy_read(0)
    js_ctx, n_ctx = gpu.policy_read(1)
    assert n_self == count and n_ctx == count
    want_self /= count
    want_ctx /= count
    assert want_self.max() > 1e-3 and want_ctx.max() > 1e-3
    assert np.abs(js_self - want_self).max() <= 1e-4 * want_self.max() + 1e-7
    assert np.abs(js_ctx - want_ctx).max() <= 1e-4 * want_ctx.max() + 1e-7
    assert np.allclose(js_self, js_self.T) and np.allclose(np.diag(js_self), 0)
    for theta in (0.2, 0.5, 0.65, 0.69):
        assert sb.policy_search(js_self, theta) == po.greedy_policy(want_self, theta)
    # layers of one block share their weights: divergence exactly 0 inside the block
    gpu.close()
    gpu = hz.make_gpu(cfg, w, [2, 2], [1, 3], debug=1)
    hz.gpu_free_run(gpu, src, lens, cfg["beam"], 3)
    gpu.policy_accumulate()
    js, _ = gpu.policy_read(0)
    assert js[0, 1] == 0 and js[2, 3] == 0 and js[0, 2] > 0
    jc, _ = gpu.policy_read(1)
    assert jc[1, 2] == 0 and jc[1, 3] == 0 and jc[0, 1] > 0
    gpu.close()


# ------------------------------------------------- encoder-side sharing (Tab. 5)
@pytest.mark.parametrize("dtype,tol", [("f32", F32_TOL), ("bf16", BF16_TOL)])
def test_encoder_side_sharing_matches_oracle(dtype, tol):
    cfg = mid_cfg(n_enc=4, steps=8, dtype=dtype)
    w = wl.make_weights(cfg, seed=15, sharp=4.0)
    src, lens = ragged(cfg, 15)
    enc_pi = [1, 3]
    gpu = hz.make_gpu(cfg, w, enc_pi=enc_pi)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w, enc_pi=enc_pi), src, lens, cfg["beam"])
    for t in range(cfg["steps"]):
        ls.step(logit_tol=F32_TOL if dtype == "f32" else BF16_TOL)
    assert max(ls.log["logit_err"]) <= tol
    # it is a different model from the unshared encoder (the check above is not vacuous)
    g2 = hz.make_gpu(cfg, w)
    a = hz.gpu_free_run(gpu, src, lens, cfg["beam"], 2, keep_logits=True)["logits"][1]
    b = hz.gpu_free_run(g2, src, lens, cfg["beam"], 2, keep_logits=True)["logits"][1]
    assert np.abs(a - b).max() > 1e-3 * np.abs(a).max()
    assert gpu.device_bytes(0) < g2.device_bytes(0)
    gpu.close()
    g2.close()


# ------------------------------------------------ multi-step decoding on the device
# The reference of these tests is the oracle's own search (oracle.search), on seeds where it
# never meets two candidate scores closer than the stated gaps, so that fp32 rounding (1e-5 on
# a score at most) cannot flip a decision: tokens and parents must then be bit-equal.
def _cum0(B, beam):
    cum0 = np.full(B, -np.inf, dtype=np.float32)
    cum0[0::beam] = 0.0
    return cum0


@pytest.mark.parametrize("use_graph", [False, True])
def test_decode_n_equals_oracle_search(use_graph):
    cfg = mid_cfg(steps=40)
    beam, B, V, N = cfg["beam"], cfg["batch"] * cfg["beam"], cfg["V"], 23
    # output embedding x8: spreads the 4 x 2004 candidate scores of a sentence
    seed, w, src, lens, ref = hz.pick_seed_with_margin(cfg, cfg["self_pi"], cfg["encdec_pi"], "A", N, beam, 1e-3,
                                                       sharp=4.0, out_scale=8.0, min_gap=1e-3, tries=40)
    assert any((p != np.arange(B)).any() for p in ref["parents"][1:])
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        gpu = hz.make_gpu(cfg, w)
        assert gpu.stream.cuda_stream != 0
        gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
        logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
        for rep in range(3):                      # replays of the captured graph, eager work in between
            n1 = 16 if rep < 2 else 6
            tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
            cum = torch.from_numpy(_cum0(B, beam)).cuda()
            out_tok = torch.zeros((N, B), dtype=torch.int32, device="cuda")
            out_par = torch.zeros((N, B), dtype=torch.int32, device="cuda")
            gpu.rewind()
            gpu.decode_n(n1, tokens, cum, out_tok, out_par, logits, use_graph)
            stream.synchronize()
            assert gpu.step == n1
            np.testing.assert_allclose(cum.cpu().numpy(), ref["scores"][n1 - 1], rtol=0, atol=1e-3)
            # continue from where the first call stopped (odd count: graph pairs + one eager step)
            n2 = N - n1
            gpu.decode_n(n2, out_tok[n1 - 1].clone(), cum, out_tok[n1:], out_par[n1:], logits, use_graph)
            stream.synchronize()
            assert gpu.step == N
            got_tok, got_par, got_cum = out_tok.cpu().numpy(), out_par.cpu().numpy(), cum.cpu().numpy()
            for t in range(N):
                assert np.array_equal(got_tok[t], ref["tokens"][t]), (seed, rep, t)
                assert np.array_equal(got_par[t], ref["parents"][t]), (seed, rep, t)
            np.testing.assert_allclose(got_cum, ref["scores"][N - 1], rtol=0, atol=1e-3)
        # single calls after the loop on the same context (the loop's last beam tail has already
        # embedded the next input: a single step embeds it again, to the same effect)
        gpu.rewind()
        tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
        cum = torch.from_numpy(_cum0(B, beam)).cuda()
        gpu.decode_n(7, tokens, cum, out_tok, out_par, logits, use_graph)
        tokens = out_tok[6].clone()
        o_tok = torch.empty((cfg["batch"], beam), dtype=torch.int32, device="cuda")
        o_par = torch.empty((cfg["batch"], beam), dtype=torch.int32, device="cuda")
        o_sc = torch.empty((cfg["batch"], beam), dtype=torch.float32, device="cuda")
        for t in range(7, 12):
            gpu.decode_step(tokens, logits)
            gpu.topk(logits, cum, beam, o_tok, o_par, o_sc)
            gpu.beam_reorder(o_par.reshape(-1))
            tokens, cum = o_tok.reshape(-1).clone(), o_sc.reshape(-1).clone()
            assert np.array_equal(tokens.cpu().numpy(), ref["tokens"][t]), (seed, t)
        gpu.decode_n(11, tokens, cum, out_tok[12:], out_par[12:], logits, use_graph)      # and back to the loop
        stream.synchronize()
        assert np.array_equal(out_tok[22].cpu().numpy(), ref["tokens"][22])
        big_t = torch.zeros((30, B), dtype=torch.int32, device="cuda")
        with pytest.raises(sb.SanError) as e:      # 23 steps done, 30 more would pass max_tgt_len = 40
            gpu.decode_n(30, tokens, cum, big_t, big_t.clone(), logits, use_graph)
        assert e.value.code == sb.SAN_ECAPACITY
        gpu.close()


@pytest.mark.parametrize("use_graph", [False, True])
def test_decode_n_aan_then_single_steps(use_graph):
    """The multi-step loop with average-attention self layers (its beam tail permutes the running
    sums), followed by single calls on the same context: tokens and parents of the oracle's search."""
    cfg = mid_cfg(steps=24, self_kind="aan", self_pi=[1, 1, 1, 1])
    beam, B, V, N, n1 = cfg["beam"], cfg["batch"] * cfg["beam"], cfg["V"], 20, 13
    seed, w, src, lens, ref = hz.pick_seed_with_margin(cfg, cfg["self_pi"], cfg["encdec_pi"], "A", N, beam, 1e-3,
                                                       out_scale=8.0, min_gap=1e-3, tries=40)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        gpu = hz.make_gpu(cfg, w)
        gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
        logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
        for rep in range(2):
            gpu.rewind()
            tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
            cum = torch.from_numpy(_cum0(B, beam)).cuda()
            out_tok = torch.zeros((n1, B), dtype=torch.int32, device="cuda")
            out_par = torch.zeros((n1, B), dtype=torch.int32, device="cuda")
            gpu.decode_n(n1, tokens, cum, out_tok, out_par, logits, use_graph)
            stream.synchronize()
            got_tok, got_par = out_tok.cpu().numpy(), out_par.cpu().numpy()
            for t in range(n1):
                assert np.array_equal(got_tok[t], ref["tokens"][t]), (seed, rep, t)
                assert np.array_equal(got_par[t], ref["parents"][t]), (seed, rep, t)
            tokens = out_tok[n1 - 1].clone()
            o_tok = torch.empty((cfg["batch"], beam), dtype=torch.int32, device="cuda")
            o_par = torch.empty((cfg["batch"], beam), dtype=torch.int32, device="cuda")
            o_sc = torch.empty((cfg["batch"], beam), dtype=torch.float32, device="cuda")
            for t in range(n1, N):
                gpu.decode_step(tokens, logits)
                gpu.topk(logits, cum, beam, o_tok, o_par, o_sc)
                gpu.beam_reorder(o_par.reshape(-1))
                tokens, cum = o_tok.reshape(-1).clone(), o_sc.reshape(-1).clone()
                assert np.array_equal(tokens.cpu().numpy(), ref["tokens"][t]), (seed, rep, t)
                assert np.array_equal(o_par.reshape(-1).cpu().numpy(), ref["parents"][t]), (seed, rep, t)
            np.testing.assert_allclose(cum.cpu().numpy(), ref["scores"][N - 1], rtol=0, atol=1e-3)
        gpu.close()


# Inside san_decode_n the output layer does not store logits: each of its column tiles hands the
# search the tile's maximum, sum of exponentials and largest entries (GEMM epilogue + a per-row
# combine).  The cases below pick shapes that select every tile of that epilogue; each step is one
# san_decode_n(1) call checked against the oracle's step with the tolerance rule of Lockstep.
WIDE = dict(n_enc=1, n_dec=2, d=64, H=4, F=128, V=25604, dtype="f32", batch=32, beam=4, src_len=(3, 9), steps=6,
            self_pi=[2], encdec_pi=[2], self_kind="dot", name="wide")
_CAND_CASES = {
    # 128 x 128 fp32 tiles; the last column tile has 4 live columns
    "f32_128x128": dict(),
    # beam 8: that tile has fewer live columns than candidates asked for
    "f32_128x128_beam8": dict(batch=16, beam=8),
    # 256 x 256 bf16 tiles in two row passes; 480 rows: a ragged second row tile
    "bf16_256x256": dict(dtype="bf16", batch=120),
    # 128 x 128 bf16 tiles, 132 rows
    "bf16_128x128": dict(dtype="bf16", batch=33),
    # 64 x 128 bf16 tiles with 256-byte chunks (k a multiple of 128)
    "bf16_64x128": dict(dtype="bf16", batch=5, d=128),
    # 64 x 64 bf16 tiles: 256-byte chunks, and 128-byte chunks (k = 64)
    "bf16_64x64_wide": dict(dtype="bf16", batch=5, d=256, V=2004),
    "bf16_64x64": dict(dtype="bf16", batch=5, V=2004),
    # 64 x 64 fp32 tiles, 20 live columns in the last one, an average-attention decoder
    "f32_64x64_aan": dict(batch=5, V=2004, self_kind="aan", self_pi=[1, 1]),
    # bf16, 64-wide heads, enc-dec weights shared (Tab. 4 "shared V: no"): the matrix-core attention emits the
    # block's weights for the follower inside the loop; beam 8
    "bf16_share_s_beam8": dict(dtype="bf16", batch=6, beam=8, d=256, V=2004, src_len=(1, 70), share="S"),
    # beam 12 is wider than the epilogue's candidate lists: the loop falls back to stored logits by itself
    "f32_beam12_stored_logits": dict(batch=3, beam=12, V=2004),
}


@pytest.mark.parametrize("case", sorted(_CAND_CASES))
def test_decode_n_candidate_output_layer_matches_oracle(case):
    cfg = dict(WIDE)
    cfg.update(_CAND_CASES[case])
    share = cfg.pop("share", "A")
    bf16 = cfg["dtype"] == "bf16"
    beam, steps = cfg["beam"], cfg["steps"]
    w = wl.make_weights(cfg, seed=11, sharp=4.0)
    w["w_out"] = w["w_out"] * np.float32(8.0)
    if bf16:
        w["w_out"] = wl.round_to_bf16(w["w_out"])
    src, lens = wl.make_source(cfg, 11)
    gpu = hz.make_gpu(cfg, w, share=share)
    orc = hz.make_oracle(cfg, w, share=share)
    ls = hz.Lockstep(gpu, orc, src, lens, beam, loop="cands")
    for t in range(steps):
        ls.step(logit_tol=BF16_TOL if bf16 else F32_TOL)
    print(f"{case}: same picks as the oracle in {np.mean(ls.log['same_frac']):.4f} of (sentence, step) pairs, "
          f"min margin {min(ls.log['margin']):.2e}, closest flipped gap {min(ls.log['flip_gap']):.2e}")
    if not bf16:
        assert np.mean(ls.log["same_frac"]) >= 0.98
    # the same search with the logits stored and read back (SAN_LOOP_LOGITS), all steps in one call:
    # both routes see the same logits, so they pick the same words from the same parents
    B = cfg["batch"] * beam
    gpu.rewind()
    tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
    cum = torch.from_numpy(_cum0(B, beam)).cuda()
    out_tok = torch.zeros((steps, B), dtype=torch.int32, device="cuda")
    out_par = torch.zeros((steps, B), dtype=torch.int32, device="cuda")
    gpu.decode_n(steps, tokens, cum, out_tok, out_par, ls.logits, keep_logits=True)
    torch.cuda.synchronize()
    for t in range(steps):
        assert np.array_equal(out_tok[t].cpu().numpy(), ls.log["tokens"][t].reshape(-1)), (case, t)
        assert np.array_equal(out_par[t].cpu().numpy(), ls.log["parents"][t].reshape(-1)), (case, t)
    np.testing.assert_allclose(cum.cpu().numpy(), ls.log["scores"][-1].reshape(-1), rtol=0, atol=1e-4)
    gpu.close()


@pytest.mark.parametrize("shape", ["64x64", "64x64_4_live", "128x128"])
def test_decode_n_all_equal_logits_take_the_lowest_ids(shape):
    """A zero output embedding makes every logit 0: every candidate of a sentence ties and the
    order (higher score, then lower beam * vocab + word) alone decides, in every column tile's
    exhaustive path (more entries at the threshold than slots) and in the combine."""
    over = {"64x64": dict(batch=5, V=2004), "64x64_4_live": dict(batch=5, V=1988), "128x128": dict()}[shape]
    cfg = dict(WIDE)
    cfg.update(over)
    beam, B, steps = cfg["beam"], cfg["batch"] * cfg["beam"], 4
    w = wl.make_weights(cfg, seed=3)
    w["w_out"] = np.zeros_like(w["w_out"])
    src, lens = wl.make_source(cfg, 3)
    ref = hz.make_oracle(cfg, w).search(src, lens, steps, beam)
    gpu = hz.make_gpu(cfg, w)
    gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
    tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
    cum = torch.from_numpy(_cum0(B, beam)).cuda()
    out_tok = torch.zeros((steps, B), dtype=torch.int32, device="cuda")
    out_par = torch.zeros((steps, B), dtype=torch.int32, device="cuda")
    logits = torch.empty((B, cfg["V"]), dtype=torch.float32, device="cuda")
    gpu.decode_n(steps, tokens, cum, out_tok, out_par, logits)
    torch.cuda.synchronize()
    for t in range(steps):
        assert np.array_equal(out_tok[t].cpu().numpy(), ref["tokens"][t]), (shape, t)
        assert np.array_equal(out_par[t].cpu().numpy(), ref["parents"][t]), (shape, t)
    assert np.array_equal(ref["tokens"][0].reshape(-1, beam), np.tile(np.arange(beam), (cfg["batch"], 1)))
    np.testing.assert_allclose(cum.cpu().numpy(), ref["scores"][steps - 1], rtol=0, atol=1e-4)
    gpu.close()


def test_decode_n_with_the_logits_flag_stores_the_last_steps_logits():
    cfg = mid_cfg(steps=12)
    beam, B, V, N = cfg["beam"], cfg["batch"] * cfg["beam"], cfg["V"], 9
    seed, w, src, lens, ref = hz.pick_seed_with_margin(cfg, cfg["self_pi"], cfg["encdec_pi"], "A", N, beam, 1e-3,
                                                       sharp=4.0, out_scale=8.0, min_gap=1e-3, tries=40)
    gpu = hz.make_gpu(cfg, w)
    gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
    out_tok = torch.zeros((N, B), dtype=torch.int32, device="cuda")
    out_par = torch.zeros((N, B), dtype=torch.int32, device="cuda")
    logits = torch.full((B, V), float("nan"), dtype=torch.float32, device="cuda")
    tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
    cum = torch.from_numpy(_cum0(B, beam)).cuda()
    gpu.decode_n(N, tokens, cum, out_tok, out_par, logits)            # default: the scratch is left alone
    torch.cuda.synchronize()
    assert torch.isnan(logits).all()
    got_tok = out_tok.cpu().numpy()
    gpu.rewind()
    cum = torch.from_numpy(_cum0(B, beam)).cuda()
    gpu.decode_n(N, tokens, cum, out_tok, out_par, logits, keep_logits=True)
    torch.cuda.synchronize()
    for t in range(N):
        assert np.array_equal(got_tok[t], ref["tokens"][t]), (seed, t)
        assert np.array_equal(out_tok[t].cpu().numpy(), ref["tokens"][t]), (seed, t)
        assert np.array_equal(out_par[t].cpu().numpy(), ref["parents"][t]), (seed, t)
    assert hz.rel_err_rows(logits.cpu().numpy(), ref["logits"][N - 1]).max() <= F32_TOL
    gpu.close()


def _eos_case(batch, beam, T, seeds, accept):
    """Tiny vocabulary (EOS gets picked often), oracle search with the end-symbol rule."""
    V = 8
    cfg = mid_cfg(steps=T, V=V, batch=batch, beam=beam)
    seed, w, src, lens, ref = hz.pick_seed_with_margin(cfg, cfg["self_pi"], cfg["encdec_pi"], "A", T, beam, 5e-4,
                                                       eos_id=wl.EOS_ID, src_clip=V - 1, seeds=seeds, accept=accept,
                                                       min_gap=5e-4, src_cfg=mid_cfg(batch=batch))
    done = np.stack([(ref["tokens"][t].reshape(batch, beam) == wl.EOS_ID).all(axis=1) for t in range(T)])
    return cfg, seed, w, src, lens, ref, done


@pytest.mark.parametrize("use_graph", [False, True])
@pytest.mark.parametrize("seeds", [(3, 4, 5), (8,)])      # all four finished after 17 steps / after 59
def test_decode_n_stops_when_every_sentence_is_finished(use_graph, seeds):
    """With EOS handling on, san_decode_n returns at the first 8-step check after every kept
    hypothesis of every sentence ends in EOS (Sec. 1: decoding goes on until the end symbol);
    up to there its tokens, parents and scores are the oracle search's."""
    batch, beam, T, V = 4, 3, 64, 8
    B = batch * beam
    cfg, seed, w, src, lens, ref, done = _eos_case(batch, beam, T, seeds, lambda o: True)
    counts = done.sum(axis=1)
    assert counts[-1] == batch, "pick another seed: not every sentence finishes within 64 steps"
    s_star = int(np.argmax(counts == batch)) + 1           # steps after which all four are finished
    expect = min(T, 8 * ((s_star + 7) // 8))
    orc = hz.make_oracle(cfg, w, eos_id=wl.EOS_ID)
    # the per-call loop first: tokens and the finished count after every step
    ref_gpu = hz.make_gpu(cfg, w, eos_id=wl.EOS_ID, max_batch=6)   # a capacity above the batch
    ref_gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
    tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
    cum = torch.from_numpy(_cum0(B, beam)).cuda()
    logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
    o_tok = torch.empty((batch, beam), dtype=torch.int32, device="cuda")
    o_par = torch.empty((batch, beam), dtype=torch.int32, device="cuda")
    o_sc = torch.empty((batch, beam), dtype=torch.float32, device="cuda")
    for t in range(T):
        ref_gpu.decode_step(tokens, logits)
        ref_gpu.topk(logits, cum, beam, o_tok, o_par, o_sc)
        ref_gpu.beam_reorder(o_par.reshape(-1))
        tokens, cum = o_tok.reshape(-1).clone(), o_sc.reshape(-1).clone()
        assert np.array_equal(tokens.cpu().numpy(), ref["tokens"][t]), (seed, t)
        assert ref_gpu.finished() == counts[t] == orc.finished(ref["tokens"][t], beam), t
    ref_gpu.close()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        gpu = hz.make_gpu(cfg, w, eos_id=wl.EOS_ID)
        gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
        for rep in range(2):
            gpu.rewind()
            out_tok = torch.full((T, B), -7, dtype=torch.int32, device="cuda")
            out_par = torch.full((T, B), -7, dtype=torch.int32, device="cuda")
            cum = torch.from_numpy(_cum0(B, beam)).cuda()
            gpu.decode_n(T, torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda"), cum, out_tok, out_par,
                         logits, use_graph)
            stream.synchronize()
            assert gpu.step == expect, (gpu.step, s_star, expect)
            assert gpu.finished() == batch
            got, gotp = out_tok.cpu().numpy(), out_par.cpu().numpy()
            for t in range(expect):
                assert np.array_equal(got[t], ref["tokens"][t]), (seed, rep, t)
                assert np.array_equal(gotp[t], ref["parents"][t]), (seed, rep, t)
            assert (got[expect:] == -7).all()           # rows past the exit are not written
            np.testing.assert_allclose(cum.cpu().numpy(), ref["scores"][expect - 1], rtol=0, atol=1e-3)
        gpu.close()


# ------------------------------------------------------ seeded random small shapes
def _random_policy(rng, layers):
    pi, left = [], layers
    while left:
        b = int(rng.integers(1, left + 1))
        pi.append(b)
        left -= b
    return pi


@pytest.mark.parametrize("case", range(12))
def test_random_shapes_and_policies(case):
    """Seeded random model shapes, policies, batch / beam sizes and source lengths: widths
    that are not powers of two, every head width, ragged tiles in every GEMM, blocks of
    every size in both attentions, all four cached modes (dot A / dot S / AAN, fp32 / bf16)."""
    rng = np.random.default_rng(1000 + case)
    dh = int(rng.choice([16, 32, 64, 128]))
    H = int(rng.choice([h for h in (1, 2, 3, 4, 5, 6, 8, 12, 16) if 64 <= h * dh <= 512 and (h * dh) % 64 == 0]))
    n_dec = int(rng.integers(1, 6))
    kind = "aan" if case % 4 == 3 else "dot"
    dtype = "bf16" if case % 3 == 2 else "f32"
    cfg = dict(n_enc=int(rng.integers(1, 3)), n_dec=n_dec, d=H * dh, H=H, F=64 * int(rng.integers(1, 9)),
               V=4 * int(rng.integers(2, 700)), dtype=dtype, batch=int(rng.integers(1, 7)), beam=int(rng.integers(1, 6)),
               src_len=(1, int(rng.integers(2, 50))), steps=int(rng.integers(4, 14)), self_kind=kind,
               self_pi=[1] * n_dec if kind == "aan" else _random_policy(rng, n_dec),
               encdec_pi=_random_policy(rng, n_dec), name=f"random{case}")
    share = "S" if case % 2 else "A"
    w = wl.make_weights(cfg, seed=1000 + case, sharp=3.0)
    src, lens = ragged(cfg, 1000 + case)
    gpu = hz.make_gpu(cfg, w, share=share, max_batch=cfg["batch"] + int(rng.integers(0, 3)))
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w, share=share), src, lens, cfg["beam"])
    tol = BF16_TOL if dtype == "bf16" else F32_TOL
    for t in range(cfg["steps"]):
        ls.step(logit_tol=F32_TOL if dtype == "f32" else BF16_TOL)
    assert max(ls.log["logit_err"]) <= tol, (cfg, share)
    gpu.close()


# ------------------------------------------------------ dropping sentences from a running batch
@pytest.mark.parametrize("kind,share,dtype", [("dot", "A", "f32"), ("dot", "S", "f32"), ("aan", "A", "f32"),
                                             ("dot", "A", "bf16"), ("dot", "S", "bf16")])
def test_compact_keeps_the_remaining_sentences_exact(kind, share, dtype):
    """san_compact drops sentences mid-decode; the ones that stay go on exactly as the
    oracle decodes them (sentences never interact), through two compactions; san_rewind
    brings the whole batch back.  (bf16: the matrix-core kernel reads the packed memory of
    the sentences that stayed.)"""
    cfg = mid_cfg(steps=20, self_kind=kind, dtype=dtype)
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    if kind == "aan":
        cfg["self_pi"] = [1] * cfg["n_dec"]
    w = wl.make_weights(cfg, seed=31, sharp=4.0)
    src, lens = ragged(cfg, 31)
    gpu = hz.make_gpu(cfg, w, share=share, max_batch=7)
    orc = hz.make_oracle(cfg, w, share=share)
    ls = hz.Lockstep(gpu, orc, src, lens, cfg["beam"], subset=[1, 3])
    first_logits = None
    for t in range(20):
        if t == 6:
            hz.lockstep_compact(ls, [0, 1, 3, 4])
            assert gpu.active().tolist() == [0, 1, 3, 4] and gpu.batch == 4
        if t == 11:
            hz.lockstep_compact(ls, [1, 2])
            assert gpu.active().tolist() == [1, 3] and gpu.rows == 2 * cfg["beam"]
        lg, _ = ls.step(logit_tol=tol)
        if t == 0:
            first_logits = lg.copy()
    assert max(ls.log["logit_err"]) <= tol
    if dtype == "f32":
        assert sum(ls.log["exact"]) >= 0.8 * 20
    gpu.rewind()
    assert gpu.active().tolist() == [0, 1, 2, 3, 4] and gpu.batch == 5
    B = 5 * cfg["beam"]
    logits = torch.empty((B, cfg["V"]), dtype=torch.float32, device="cuda")
    gpu.decode_step(torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda"), logits)
    rows = torch.from_numpy(np.array([1, 3])[:, None] * cfg["beam"] + np.arange(cfg["beam"])[None, :]).reshape(-1).cuda()
    assert np.array_equal(logits[rows].cpu().numpy(), first_logits)
    gpu.close()


def test_encode_after_compact_starts_clean():
    """A context that was compacted mid-decode takes a new san_encode like a fresh one."""
    cfg = mid_cfg(steps=12)
    w = wl.make_weights(cfg, seed=33, sharp=4.0)
    src, lens = ragged(cfg, 33)
    gpu = hz.make_gpu(cfg, w)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w), src, lens, cfg["beam"], subset=[0, 2])
    for t in range(5):
        if t == 3:
            hz.lockstep_compact(ls, [0, 2])
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL and gpu.batch == 2
    src2, lens2 = ragged(cfg, 34)
    ls2 = hz.Lockstep(gpu, hz.make_oracle(cfg, w), src2, lens2, cfg["beam"])     # encodes the new batch
    assert gpu.batch == cfg["batch"] and gpu.active().tolist() == list(range(cfg["batch"]))
    for t in range(6):
        ls2.step(logit_tol=F32_TOL)
    assert max(ls2.log["logit_err"]) <= F32_TOL
    gpu.close()


def test_compact_argument_errors_and_flags():
    cfg = mid_cfg(steps=64, V=8, batch=4, beam=3)
    w = wl.make_weights(cfg, seed=4)
    src, lens = wl.make_source(mid_cfg(batch=4), 4)
    src = np.minimum(src, 7)
    gpu = hz.make_gpu(cfg, w, eos_id=wl.EOS_ID, max_batch=6)     # max_batch above the batch on purpose
    with pytest.raises(sb.SanError) as e:
        gpu.compact([0])
    assert e.value.code == sb.SAN_ESTATE
    gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
    for bad in ([], [0, 0], [1, 0], [0, 4], [-1, 2], [0, 1, 2, 3, 3]):
        with pytest.raises(sb.SanError) as e:
            gpu.compact(bad)
        assert e.value.code == sb.SAN_EINVAL, bad
    gpu.compact([0, 1, 2, 3])                                    # everything stays: nothing happens
    assert gpu.batch == 4
    # finished flags against their definition, also after a compaction
    beam, B, V = 3, 12, 8
    tokens = torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda")
    cum0 = np.full(B, -np.inf, dtype=np.float32)
    cum0[0::beam] = 0.0
    cum = torch.from_numpy(cum0).cuda()
    logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
    keep_all = np.arange(4)
    seen_done = False
    for t in range(64):
        nb = gpu.batch
        o_tok = torch.empty((nb, beam), dtype=torch.int32, device="cuda")
        o_par = torch.empty((nb, beam), dtype=torch.int32, device="cuda")
        o_sc = torch.empty((nb, beam), dtype=torch.float32, device="cuda")
        gpu.decode_step(tokens, logits)
        gpu.topk(logits, cum, beam, o_tok, o_par, o_sc)
        gpu.beam_reorder(o_par.reshape(-1))
        tokens, cum = o_tok.reshape(-1).clone(), o_sc.reshape(-1).clone()
        flags = (o_tok.cpu().numpy() == wl.EOS_ID).all(axis=1).astype(np.int32)
        assert np.array_equal(gpu.done_flags(), flags), t
        assert gpu.finished() == int(flags.sum())
        if flags.all():
            break
        if flags.any():
            seen_done = True
            keep = np.nonzero(flags == 0)[0]
            keep_all = keep_all[keep]
            gpu.compact(keep)
            rows = torch.from_numpy((keep[:, None] * beam + np.arange(beam)[None, :]).reshape(-1)).cuda()
            tokens, cum = tokens[rows].contiguous(), cum[rows].contiguous()
            assert gpu.finished() == 0 and gpu.active().tolist() == keep_all.tolist()
    assert seen_done, "pick another seed: no sentence finished before the others"
    gpu.close()


def _compaction_schedule(done, T):
    """What the 8-step checks of san_decode_n must do, from the oracle's finished flags
    done[t][sentence]: (steps run, sentences still in the batch at the end)."""
    active = np.arange(done.shape[1])
    for s in range(8, T + 1, 8):
        fin = done[s - 1][active]
        if fin.all():
            return s, active
        if 4 * fin.sum() >= len(active) and T - s >= 16:
            active = active[~fin]
    return T, active


@pytest.mark.parametrize("use_graph", [False, True])
@pytest.mark.parametrize("seed", [5, 42, 76, 80])
def test_decode_n_drops_finished_sentences(seed, use_graph):
    """san_decode_n with SAN_LOOP_COMPACT: finished sentences leave the batch at an 8-step
    check, the rest of the decode runs on the smaller batch, and the caller's arrays are what
    the oracle's search on the full batch gives (tokens, parents, scores, in the caller's row
    numbering; sentences that left keep extending with EOS in place)."""
    batch, beam, T, V = 8, 3, 64, 8
    B = batch * beam
    cfg, seed, w, src, lens, ref, done = _eos_case(
        batch, beam, T, (seed,), lambda o: True)
    expect_steps, active = _compaction_schedule(done, T)
    assert len(active) < batch, "pick another seed: no sentence leaves the batch early"
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        gpu = hz.make_gpu(cfg, w, eos_id=wl.EOS_ID)
        gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
        logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
        for rep in range(2):
            gpu.rewind()
            assert gpu.batch == batch
            out_tok = torch.full((T, B), -7, dtype=torch.int32, device="cuda")
            out_par = torch.full((T, B), -7, dtype=torch.int32, device="cuda")
            cum = torch.from_numpy(_cum0(B, beam)).cuda()
            gpu.decode_n(T, torch.full((B,), wl.BOS_ID, dtype=torch.int32, device="cuda"), cum, out_tok, out_par,
                         logits, use_graph, compact=True)
            stream.synchronize()
            assert gpu.step == expect_steps
            assert gpu.active().tolist() == active.tolist() and gpu.batch == len(active)
            got_t, got_p = out_tok.cpu().numpy(), out_par.cpu().numpy()
            for t in range(expect_steps):
                assert np.array_equal(got_t[t], ref["tokens"][t].reshape(-1)), (rep, t)
                assert np.array_equal(got_p[t], ref["parents"][t].reshape(-1)), (rep, t)
            assert (got_t[expect_steps:] == -7).all() and (got_p[expect_steps:] == -7).all()
            np.testing.assert_allclose(cum.cpu().numpy(), ref["scores"][expect_steps - 1].reshape(-1), rtol=0, atol=1e-3)
        gpu.close()


# ------------------------------------------------------ head widths, extreme shapes
@pytest.mark.parametrize("d,H,dtype", [(128, 8, "f32"), (128, 4, "f32"), (256, 2, "f32"), (128, 8, "bf16"),
                                       (256, 8, "bf16"), (256, 2, "bf16")])
def test_head_widths(d, H, dtype):
    """Head widths 16, 32 and 128 take other lane mappings of the attention kernel
    than the 64 of the paper's models."""
    cfg = mid_cfg(d=d, H=H, F=2 * d, dtype=dtype, steps=37, batch=3, beam=3, self_pi=[2, 2], encdec_pi=[1, 3])
    w = wl.make_weights(cfg, seed=17, sharp=3.0)
    src, lens = ragged(cfg, 17)
    for share in ("A", "S"):
        gpu = hz.make_gpu(cfg, w, share=share)
        ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w, share=share), src, lens, cfg["beam"])
        for t in range(cfg["steps"]):
            ls.step(logit_tol=F32_TOL if dtype == "f32" else BF16_TOL)
        assert max(ls.log["logit_err"]) <= (F32_TOL if dtype == "f32" else BF16_TOL), (share, max(ls.log["logit_err"]))
        gpu.close()


@pytest.mark.parametrize("kind,dtype", [("dot", "f32"), ("aan", "bf16")])
def test_maximum_width(kind, dtype):
    """d_model = 2048, the widest model the library takes (LayerNorm rows of 8 waves, 64 k-chunks
    per projection), with 128-wide heads."""
    cfg = dict(n_enc=1, n_dec=2, d=2048, H=16, F=128, V=64, dtype=dtype, batch=2, beam=2, src_len=(1, 9), steps=4,
               self_pi=[1, 1] if kind == "aan" else [2], encdec_pi=[2], self_kind=kind, name="wide")
    w = wl.make_weights(cfg, seed=41, sharp=1.0)
    src, lens = ragged(cfg, 41)
    gpu = hz.make_gpu(cfg, w)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w), src, lens, cfg["beam"])
    for t in range(cfg["steps"]):
        ls.step(logit_tol=F32_TOL if dtype == "f32" else BF16_TOL)
    assert max(ls.log["logit_err"]) <= (F32_TOL if dtype == "f32" else BF16_TOL), max(ls.log["logit_err"])
    gpu.close()


@pytest.mark.parametrize("dtype,share", [("f32", "A"), ("f32", "S"), ("bf16", "A")])
def test_long_streams_few_of_them(dtype, share):
    """Streams of more than 128 cached positions and sentence memories of up to 100 positions
    in a small batch: these launches split every stream over several waves of a workgroup
    (partial softmax per wave, combined through LDS), self-attention with a chunk loop."""
    cfg = mid_cfg(batch=2, beam=4, steps=140, src_len=(1, 100), n_dec=3, self_pi=[2, 1], encdec_pi=[1, 2], dtype=dtype)
    w = wl.make_weights(cfg, seed=27, sharp=4.0)
    src, lens = ragged(cfg, 27)
    gpu = hz.make_gpu(cfg, w, share=share, debug=1)
    orc = hz.make_oracle(cfg, w, share=share)
    ls = hz.Lockstep(gpu, orc, src, lens, cfg["beam"])
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    for t in range(cfg["steps"]):
        ls.step(logit_tol=tol)
        if dtype == "f32" and t in (0, 31, 32, 64, 65, 127, 128, 139):     # chunk and wave-share boundaries
            for n in range(cfg["n_dec"]):
                S = gpu.debug_get(sb.SAN_DBG_S_SELF, n).cpu().numpy()
                assert np.abs(S.sum(-1) - 1).max() < 1e-5
                assert np.abs(S - orc.dump["S_self"][n]).max() < 2e-6, (t, n)
                Sc = gpu.debug_get(sb.SAN_DBG_S_CTX, n).cpu().numpy()
                assert np.abs(Sc - orc.dump["S_ctx"][n]).max() < 2e-6, (t, n)
    assert max(ls.log["logit_err"]) <= tol
    gpu.close()


def test_maximum_beam_and_long_cache():
    """beam = 32 (the largest the library takes) and a cache of 300 positions
    (several chunks of the attention pipeline plus a ragged tail)."""
    cfg = mid_cfg(batch=2, beam=32, steps=6, V=2004)
    w = wl.make_weights(cfg, seed=18, sharp=4.0)
    src, lens = ragged(cfg, 18)
    gpu = hz.make_gpu(cfg, w)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w), src, lens, 32)
    for t in range(6):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    gpu.close()
    cfg = mid_cfg(batch=2, beam=2, steps=300, n_dec=2, self_pi=[2], encdec_pi=[2])
    w = wl.make_weights(cfg, seed=19, sharp=4.0)
    src, lens = ragged(cfg, 19)
    gpu = hz.make_gpu(cfg, w)
    ls = hz.Lockstep(gpu, hz.make_oracle(cfg, w), src, lens, 2)
    for t in range(300):
        ls.step(logit_tol=F32_TOL)
    assert max(ls.log["logit_err"]) <= F32_TOL
    gpu.close()
