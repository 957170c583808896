"""The allocation-free beam step (san_topk_noalloc) against san_topk, through the C ABI:
same picks and scores bit for bit, on two calls in a row of which the second is smaller
(the fixed scratch still holds the first call's candidates), then the capacity error."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1906_11024_amd import binding as sb
from paper_1906_11024_amd import workloads as wl
from tests import harness as hz


def _both(gpu, logits, cum, batch, k):
    outs = []
    for fn in (gpu.topk, gpu.topk_noalloc):
        o_tok = torch.full((batch, k), -5, dtype=torch.int32, device="cuda")
        o_par = torch.full((batch, k), -5, dtype=torch.int32, device="cuda")
        o_sc = torch.full((batch, k), -5.0, dtype=torch.float32, device="cuda")
        fn(logits, cum, k, o_tok, o_par, o_sc)
        torch.cuda.synchronize()
        outs.append((o_tok.cpu().numpy(), o_par.cpu().numpy(), o_sc.cpu().numpy()))
    return outs


def test_topk_noalloc_equals_topk_on_two_calls_the_second_smaller():
    if not torch.cuda.is_available():
        pytest.fail("needs a GPU")
    V, beam = 2004, 4
    cfg = dict(n_enc=1, n_dec=1, d=64, H=1, F=64, V=V, dtype="f32", batch=6, beam=beam, src_len=(1, 9), steps=4,
               self_pi=[1], encdec_pi=[1], self_kind="dot", name="noalloc")
    w = wl.make_weights(cfg, seed=3)
    gpu = hz.make_gpu(cfg, w, eos_id=wl.EOS_ID)
    rng = np.random.default_rng(5)
    for batch, k in ((6, 4), (2, 3)):            # the second call: fewer sentences, fewer picks
        src, lens = wl.make_source(dict(cfg, batch=batch), batch)
        gpu.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
        B = batch * beam
        # a decode step so that the context knows each row's last input word (row 1 ends in EOS)
        toks = rng.integers(3, V, size=B).astype(np.int32)
        toks[1] = wl.EOS_ID
        logits_work = torch.empty((B, V), dtype=torch.float32, device="cuda")
        gpu.decode_step(torch.from_numpy(toks).cuda(), logits_work)
        logits = rng.standard_normal((B, V)).astype(np.float32) * 3
        logits[::3] = rng.integers(-3, 4, size=logits[::3].shape).astype(np.float32)    # rows full of exact ties
        cum = (rng.standard_normal(B) * 0.01).astype(np.float32)
        lg, cm = torch.from_numpy(logits).cuda(), torch.from_numpy(cum).cuda()
        (t0, p0, s0), (t1, p1, s1) = _both(gpu, lg, cm, batch, k)
        assert np.array_equal(t0, t1) and np.array_equal(p0, p1)
        assert np.array_equal(s0, s1)             # the same kernels: the same bits
        assert (t0 >= 0).all() and (t0 < V).all()
        # and both are the oracle's beam step (valid top-k of its scores; exact where it has no ties)
        orc = hz.make_oracle(cfg, w, eos_id=wl.EOS_ID)
        orc.batch = batch
        tok, par, sc, _ = orc.topk(logits, cum, k, last_tokens=toks)
        assert np.abs(s1 - sc).max() < 2e-5
    # beyond the fixed scratch: refused, nothing queued
    big = dict(cfg, batch=1100, beam=1)
    g2 = hz.make_gpu(big, w, beam=1)
    src, lens = wl.make_source(big, 1)
    g2.encode(torch.from_numpy(src).cuda(), torch.from_numpy(lens).cuda())
    lg = torch.zeros((1100, V), dtype=torch.float32, device="cuda")
    cm = torch.zeros(1100, dtype=torch.float32, device="cuda")
    o_i = torch.zeros((1100, 32), dtype=torch.int32, device="cuda")
    o_f = torch.zeros((1100, 32), dtype=torch.float32, device="cuda")
    with pytest.raises(sb.SanError) as e:
        g2.topk_noalloc(lg, cm, 32, o_i, o_i.clone(), o_f)
    assert e.value.code == sb.SAN_ECAPACITY
    g2.topk_noalloc(lg, cm, 29, o_i, o_i.clone(), o_f)     # 1100 * 29 = 31900 candidates fit
    torch.cuda.synchronize()
    g2.close()
    gpu.close()
