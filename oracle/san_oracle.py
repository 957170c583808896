"""CPU oracle for the shared-attention (SAN) Transformer decoder.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, fp64 numpy statement of
what the decoder computes, written from the paper.  It shares no code with the
HIP library and must never be imported by the product path; only the tests, the
smoke check and the benchmark's `cpu_baseline` leg use it.

What follows the paper, and where:
  * attention weights  S = Softmax(Q K^T / sqrt(d_k))            (Eq. 1, Sec. 2)
  * attention output   A = S V                                     (Eq. 2, Sec. 2)
  * SAN self-attention: the first layer m of a block computes S^m = s(Q^m, K^m)
    (Eq. 3); the other pi-1 layers of the block take S^{m+i} = S^m (Eq. 4) and
    multiply it by their own V (Fig. 3(b)); their Q/K projections do not exist
    (Sec. 3.2, last paragraphs).
  * SAN encoder-decoder attention: the block head computes A^m = S^m V with K, V
    from the encoder output; the other layers take A^{m+i} = A^m (Eq. 5,
    Fig. 3(c)).  The variant that shares only S and keeps a per-layer V is the
    "shared V: no" row of Tab. 4 (mode "S" here, "A" is Eq. 5).
  * a sharing policy is the list of block sizes {pi_1..pi_N}, bottom-up, with
    sum pi_i = number of layers (Sec. 3.3).
  * decoding is auto-regressive, one target word per step, with a cache of the
    previous positions' keys/values; the un-cached variant recomputes every
    position at every step (Sec. 1, Sec. 4.1).  Beam search over a batch
    (Sec. 4.1).

Readings taken where the paper is silent (all listed in the design notes):
  softmax is over key positions; d_k in the scale is the per-head width; layers
  are post-norm, x = LN(x + sublayer(x)), biased variance; every layer keeps its
  own output projection, LayerNorm and FFN; head h of a follower reuses head h of
  the block head; embeddings are scaled by sqrt(d) and added to the sinusoidal
  position table; ReLU FFN; linear maps have biases except the output embedding;
  beam score = sum of log-probabilities, ties broken by the lower flat candidate
  index; a source sentence of length 0 yields a zero context vector.
  The average-attention self layer (AAN) is not defined in the paper; it is taken
  as cumulative mean -> FFN -> input/forget gates -> residual LayerNorm.

Parity pins live in tests/test_oracle_pins.py.  Parity unpinned (no external
ground truth exists for them, only internal invariants): the choice among the
readings above, and whether the AAN layer as read here is the one the paper's
"+AAN" systems ran.  The arithmetic of that reading (running mean, gate layout,
sigmoid) is itself pinned by closed forms.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------- primitives
def positional_table(max_len: int, d: int) -> np.ndarray:
    """PE[pos, 2i] = sin(pos / 10000^(2i/d)),  PE[pos, 2i+1] = cos(same)."""
    pe = np.zeros((max_len, d), dtype=np.float64)
    pos = np.arange(max_len, dtype=np.float64)[:, None]
    i2 = np.arange(0, d, 2, dtype=np.float64)[None, :]
    ang = pos / np.power(10000.0, i2 / d)
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)
    return pe


def linear(x, W, b=None):
    """y = x W^T (+ b); W is [out, in]."""
    y = x @ W.T
    return y if b is None else y + b


def layer_norm(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def softmax(z):
    """Softmax along the last axis; entries equal to -inf get weight 0; a row
    that is entirely -inf (no key at all) gets all-zero weights."""
    m = z.max(axis=-1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(z - m)
    s = e.sum(axis=-1, keepdims=True)
    return np.divide(e, s, out=np.zeros_like(e), where=s > 0)


def attention_weights(Q, K, d_k, mask=None):
    """Eq. 1.  Q [..., lq, d_k], K [..., lk, d_k] -> S [..., lq, lk].
    mask (bool, broadcastable to S): False entries are excluded (-inf)."""
    z = Q @ np.swapaxes(K, -1, -2)
    z = z / z.dtype.type(np.sqrt(float(d_k)))
    if mask is not None:
        z = np.where(mask, z, -np.inf)
    return softmax(z)


def attention_output(S, V):
    """Eq. 2.  S [..., lq, lk], V [..., lk, d_v] -> A [..., lq, d_v]."""
    return S @ V


def log_softmax(z):
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def block_heads(pi, n_layers):
    """For a policy {pi_i} return head[n] = index of the first layer of the
    block that holds layer n (0-based)."""
    pi = [int(p) for p in pi]
    if len(pi) == 0 or any(p < 1 for p in pi) or sum(pi) != n_layers:
        raise ValueError(f"policy {pi} does not partition {n_layers} layers")
    head, start = [], 0
    for p in pi:
        head += [start] * p
        start += p
    return head


def split_heads(x, H):
    """[..., l, d] -> [..., H, l, d/H]"""
    *lead, l, d = x.shape
    return np.moveaxis(x.reshape(*lead, l, H, d // H), -2, -3)


def merge_heads(x):
    """[..., H, l, dh] -> [..., l, H*dh]"""
    x = np.moveaxis(x, -3, -2)
    *lead, l, H, dh = x.shape
    return x.reshape(*lead, l, H * dh)


# --------------------------------------------------------------------- oracle
class SanOracle:
    """cfg keys: n_enc, n_dec, d, H, F, V, self_kind ('dot'|'aan').
    weights: name -> array (see the workload module's tensor list).
    self_pi / encdec_pi: sharing policies (block sizes).
    encdec_share: 'A' (Eq. 5: reuse the attended state) or 'S' (reuse weights
    only, per-layer V).  dtype: arithmetic type (float64 unless a pin says so)."""

    def __init__(self, cfg, weights, self_pi, encdec_pi, encdec_share="A",
                 ln_eps=1e-5, eos_id=-1, max_len=None, dtype=np.float64, enc_pi=None):
        self.cfg = cfg
        self.dt = dtype
        self.w = {k: np.asarray(v, dtype=dtype) for k, v in weights.items()}
        self.d, self.H, self.F, self.V = cfg["d"], cfg["H"], cfg["F"], cfg["V"]
        self.dh = self.d // self.H
        self.n_enc, self.n_dec = cfg["n_enc"], cfg["n_dec"]
        self.aan = cfg.get("self_kind", "dot") == "aan"
        self.self_head = block_heads(self_pi, self.n_dec)
        self.ctx_head = block_heads(encdec_pi, self.n_dec)
        # encoder-side sharing (Tab. 5): same rule on the encoder self-attention
        self.enc_head = block_heads(enc_pi if enc_pi else [1] * self.n_enc, self.n_enc)
        assert encdec_share in ("A", "S")
        self.share = encdec_share
        self.eps = ln_eps
        self.eos_id = eos_id
        self.max_len = max_len or 1024
        self.pe = positional_table(self.max_len, self.d).astype(dtype)
        self.emb_scale = dtype(np.sqrt(float(self.d)))
        self.dump = {}

    # ------------------------------------------------------------- sub-layers
    def _mha_proj(self, prefix, which, x):
        return linear(x, self.w[f"{prefix}.w{which}"], self.w[f"{prefix}.b{which}"])

    def _ln(self, name, x):
        return layer_norm(x, self.w[f"{name}.g"], self.w[f"{name}.b"], self.eps)

    def _ffn(self, prefix, x):
        h = np.maximum(linear(x, self.w[f"{prefix}.w1"], self.w[f"{prefix}.b1"]), 0.0)
        return linear(h, self.w[f"{prefix}.w2"], self.w[f"{prefix}.b2"])

    # ---------------------------------------------------------------- encoder
    def encode(self, src, src_len):
        """src [batch, max_src] ids, src_len [batch].  Runs the encoder stack
        (self-attention + FFN per layer, Sec. 2) with keys beyond each sentence's
        length masked out, then prepares the encoder-decoder keys/values of every
        decoder layer that needs them.  Resets the decoder state."""
        src = np.asarray(src)
        self.src_len = np.asarray(src_len).astype(np.int64)
        batch, L = src.shape
        self.batch, self.max_src = batch, L
        x = self.w["src_emb"][src] * self.emb_scale + self.pe[:L][None]
        key_ok = (np.arange(L)[None, :] < self.src_len[:, None])      # [batch, L]
        mask = key_ok[:, None, None, :]                                # over [b,H,lq,lk]
        S_enc = {}
        for i in range(self.n_enc):
            p = f"enc{i}.attn"
            Vv = split_heads(self._mha_proj(p, "v", x), self.H)
            if self.enc_head[i] == i:
                Q = split_heads(self._mha_proj(p, "q", x), self.H)
                K = split_heads(self._mha_proj(p, "k", x), self.H)
                S_enc[i] = attention_weights(Q, K, self.dh, mask)
            else:                                   # weights of the block head, own V
                S_enc[i] = S_enc[self.enc_head[i]]
            S = S_enc[i]
            A = merge_heads(attention_output(S, Vv))
            x = self._ln(f"enc{i}.ln1", x + self._mha_proj(p, "o", A))
            x = self._ln(f"enc{i}.ln2", x + self._ffn(f"enc{i}.ffn", x))
        self.enc_S = S_enc
        self.enc_out = x                                               # [batch, L, d]
        # memory keys / values: K for block heads only; V for block heads, or for
        # every layer in mode 'S' (each follower keeps its own V projection).
        self.mem_K, self.mem_V = {}, {}
        for n in range(self.n_dec):
            p = f"dec{n}.ctx"
            if self.ctx_head[n] == n:
                self.mem_K[n] = split_heads(self._mha_proj(p, "k", x), self.H)
            if self.ctx_head[n] == n or self.share == "S":
                self.mem_V[n] = split_heads(self._mha_proj(p, "v", x), self.H)
        self.key_ok = key_ok
        self.reset_decoder()
        return x

    def reset_decoder(self):
        self.t = 0
        self.rows = None
        self.cache_K, self.cache_V, self.aan_sum = {}, {}, {}
        self.last_tokens = None

    # ------------------------------------------------------- cached decoding
    def decode_step(self, tokens):
        """One auto-regressive step for all rows (row r belongs to sentence
        r // beam).  Appends this position's keys/values to the cache and
        returns logits [rows, V]."""
        tokens = np.asarray(tokens).astype(np.int64)
        B = tokens.shape[0]
        if self.rows is None:
            self.rows = B
            self.beam = B // self.batch
        assert B == self.rows and B == self.batch * self.beam
        t = self.t
        sent = np.arange(B) // self.beam
        H, dh = self.H, self.dh
        x = self.w["tgt_emb"][tokens] * self.emb_scale + self.pe[t][None]    # [B, d]
        dump = {"S_self": {}, "A_self": {}, "S_ctx": {}, "A_ctx": {}, "hidden": {}}
        S_self, S_ctx, A_ctx = {}, {}, {}
        for n in range(self.n_dec):
            # ---- self-attention sub-layer (or AAN)
            if self.aan:
                x = self._aan_step(n, x, t)
                dump["A_self"][n] = x                        # output of the whole AAN sub-layer
            else:
                p = f"dec{n}.self"
                m = self.self_head[n]
                v_new = self._mha_proj(p, "v", x).reshape(B, H, 1, dh)
                self.cache_V[n] = v_new if t == 0 else np.concatenate([self.cache_V[n], v_new], axis=2)
                if m == n:                                   # block head: Eq. 3
                    q = self._mha_proj(p, "q", x).reshape(B, H, 1, dh)
                    k_new = self._mha_proj(p, "k", x).reshape(B, H, 1, dh)
                    self.cache_K[n] = k_new if t == 0 else np.concatenate([self.cache_K[n], k_new], axis=2)
                    S_self[n] = attention_weights(q, self.cache_K[n], dh)     # [B,H,1,t+1]
                else:                                        # Eq. 4: S^{m+i} = S^m
                    S_self[n] = S_self[m]
                A = attention_output(S_self[n], self.cache_V[n])             # [B,H,1,dh]
                A = A.reshape(B, self.d)
                dump["S_self"][n] = S_self[n][:, :, 0, :]
                dump["A_self"][n] = A
                x = self._ln(f"dec{n}.ln1", x + self._mha_proj(p, "o", A))
            # ---- encoder-decoder attention sub-layer
            p = f"dec{n}.ctx"
            m = self.ctx_head[n]
            mask = self.key_ok[sent][:, None, None, :]                       # [B,1,1,L]
            if m == n:
                q = self._mha_proj(p, "q", x).reshape(B, H, 1, dh)
                S_ctx[n] = attention_weights(q, self.mem_K[n][sent], dh, mask)
                A_ctx[n] = attention_output(S_ctx[n], self.mem_V[n][sent]).reshape(B, self.d)
            elif self.share == "A":                          # Eq. 5: A^{m+i} = A^m
                S_ctx[n] = S_ctx[m]
                A_ctx[n] = A_ctx[m]
            else:                                            # weights shared, own V
                S_ctx[n] = S_ctx[m]
                A_ctx[n] = attention_output(S_ctx[n], self.mem_V[n][sent]).reshape(B, self.d)
            dump["S_ctx"][n] = S_ctx[n][:, :, 0, :]
            dump["A_ctx"][n] = A_ctx[n]
            x = self._ln(f"dec{n}.ln2", x + self._mha_proj(p, "o", A_ctx[n]))
            # ---- feed-forward sub-layer
            x = self._ln(f"dec{n}.ln3", x + self._ffn(f"dec{n}.ffn", x))
            dump["hidden"][n] = x
        self.dump = dump
        self.t = t + 1
        self.last_tokens = tokens
        return linear(x, self.w["w_out"])

    def _aan_step(self, n, x, t):
        """Average-attention self layer, incremental form: running sum of the
        layer inputs over positions 0..t."""
        p = f"dec{n}.aan"
        self.aan_sum[n] = x.copy() if t == 0 else self.aan_sum[n] + x
        g = self._ffn(p, self.aan_sum[n] / float(t + 1))
        return self._aan_gate(n, x, g)

    def _aan_gate(self, n, x, g):
        p = f"dec{n}.aan"
        z = linear(np.concatenate([x, g], axis=-1), self.w[f"{p}.wg"], self.w[f"{p}.bg"])
        i_gate, f_gate = sigmoid(z[..., : self.d]), sigmoid(z[..., self.d:])
        return self._ln(f"dec{n}.ln1", x + i_gate * x + f_gate * g)

    def beam_reorder(self, parent):
        """Row r continues the hypothesis that was row parent[r]."""
        parent = np.asarray(parent).astype(np.int64)
        for n in list(self.cache_K):
            self.cache_K[n] = self.cache_K[n][parent]
        for n in list(self.cache_V):
            self.cache_V[n] = self.cache_V[n][parent]
        for n in list(self.aan_sum):
            self.aan_sum[n] = self.aan_sum[n][parent]
        if self.last_tokens is not None:
            pass  # last_tokens are the tokens just chosen; the caller supplies them next step

    # ------------------------------------------ un-cached (full re-forward)
    def decode_full(self, history, return_all=False):
        """history [rows, n]: all target-side inputs so far (position 0 = BOS).
        Runs the decoder over the whole prefix with a causal mask (what an
        implementation without the attention cache does at every step) and
        returns the last position's logits [rows, V]."""
        history = np.asarray(history).astype(np.int64)
        B, n_pos = history.shape
        beam = B // self.batch
        sent = np.arange(B) // beam
        H, dh = self.H, self.dh
        x = self.w["tgt_emb"][history] * self.emb_scale + self.pe[:n_pos][None]  # [B,n,d]
        causal = np.tril(np.ones((n_pos, n_pos), dtype=bool))[None, None]
        S_self, S_ctx, A_ctx = {}, {}, {}
        for n in range(self.n_dec):
            if self.aan:
                avg = np.cumsum(x, axis=1) / np.arange(1, n_pos + 1, dtype=self.dt)[None, :, None]
                x = self._aan_gate(n, x, self._ffn(f"dec{n}.aan", avg))
            else:
                p = f"dec{n}.self"
                m = self.self_head[n]
                Vv = split_heads(self._mha_proj(p, "v", x), H)
                if m == n:
                    Q = split_heads(self._mha_proj(p, "q", x), H)
                    K = split_heads(self._mha_proj(p, "k", x), H)
                    S_self[n] = attention_weights(Q, K, dh, causal)
                else:
                    S_self[n] = S_self[m]
                A = merge_heads(attention_output(S_self[n], Vv))
                x = self._ln(f"dec{n}.ln1", x + self._mha_proj(p, "o", A))
            p = f"dec{n}.ctx"
            m = self.ctx_head[n]
            mask = self.key_ok[sent][:, None, None, :]
            if m == n:
                Q = split_heads(self._mha_proj(p, "q", x), H)
                S_ctx[n] = attention_weights(Q, self.mem_K[n][sent], dh, mask)
                A_ctx[n] = merge_heads(attention_output(S_ctx[n], self.mem_V[n][sent]))
            elif self.share == "A":
                A_ctx[n] = A_ctx[m]
            else:
                S_ctx[n] = S_ctx[m]
                A_ctx[n] = merge_heads(attention_output(S_ctx[m], self.mem_V[n][sent]))
            x = self._ln(f"dec{n}.ln2", x + self._mha_proj(p, "o", A_ctx[n]))
            x = self._ln(f"dec{n}.ln3", x + self._ffn(f"dec{n}.ffn", x))
        self.full_S_self = S_self
        logits = linear(x, self.w["w_out"])
        return logits if return_all else logits[:, -1, :]

    # ------------------------------------------------------------------ search
    def finished(self, tokens, beam):
        """Sentences whose kept hypotheses all end in EOS after a beam step (Sec. 1:
        decoding goes on until the end symbol is reached); tokens [batch*beam]."""
        if self.eos_id < 0:
            return 0
        return int((np.asarray(tokens).reshape(-1, beam) == self.eos_id).all(axis=1).sum())

    def topk(self, logits, cum_score, k, last_tokens=None):
        """Beam step.  logits [rows, V], cum_score [rows]; rows of sentence b are
        b*beam .. b*beam+beam-1.  Candidate (row r, word v) scores
        cum_score[r] + log_softmax(logits[r])[v]; a row whose last input token was
        EOS (when EOS handling is on) can only be extended by EOS at no cost.
        Per sentence the k best candidates are kept, ordered by higher score, then
        lower flat index (beam_index * V + v).
        Returns token [batch,k], parent [batch,k] (global row index),
        score [batch,k], margin [batch] (k-th minus (k+1)-th score)."""
        logits = np.asarray(logits, dtype=self.dt)
        cum = np.asarray(cum_score, dtype=self.dt)
        B, V = logits.shape
        beam = B // self.batch
        lp = log_softmax(logits)
        if last_tokens is None:
            last_tokens = self.last_tokens
        if self.eos_id >= 0 and last_tokens is not None:
            done = np.asarray(last_tokens) == self.eos_id
            lp[done, :] = -np.inf
            lp[done, self.eos_id] = 0.0
        cand = (cum[:, None] + lp).reshape(self.batch, beam * V)
        tok = np.zeros((self.batch, k), dtype=np.int32)
        par = np.zeros((self.batch, k), dtype=np.int32)
        sc = np.zeros((self.batch, k), dtype=self.dt)
        margin = np.zeros(self.batch, dtype=self.dt)
        for b in range(self.batch):
            # stable sort on the negated score: score descending, equal scores
            # stay in ascending flat-index order
            order = np.argsort(-cand[b], kind="stable")
            top = order[:k]
            tok[b] = top % V
            par[b] = b * beam + top // V
            sc[b] = cand[b, top]
            if order.size > k:
                margin[b] = cand[b, order[k - 1]] - cand[b, order[k]]
            else:
                margin[b] = np.inf
        return tok, par, sc, margin

    def search(self, src, src_len, steps, beam, bos_id=1, use_cache=True):
        """Greedy (beam 1) or beam search for a fixed number of steps.
        Returns per-step lists of tokens [rows], parents [rows], scores [rows],
        the logits of every step and the smallest top-k margin seen."""
        self.encode(src, src_len)
        B = self.batch * beam
        tokens = np.full(B, bos_id, dtype=np.int64)
        cum = np.full(B, -np.inf)
        cum[0::beam] = 0.0                       # only beam 0 of a sentence is live at step 0
        history = tokens[:, None]
        out = {"tokens": [], "parents": [], "scores": [], "logits": [], "margin": np.inf}
        for _ in range(steps):
            if use_cache:
                logits = self.decode_step(tokens)
            else:
                self.rows, self.beam = B, beam
                logits = self.decode_full(history)
                self.last_tokens = tokens
            tok, par, sc, margin = self.topk(logits, cum, beam, last_tokens=tokens)
            out["margin"] = min(out["margin"], float(margin.min()))
            tokens = tok.reshape(B).astype(np.int64)
            parent = par.reshape(B)
            cum = sc.reshape(B)
            if use_cache:
                self.beam_reorder(parent)
            history = np.concatenate([history[parent], tokens[:, None]], axis=1)
            out["tokens"].append(tokens.copy())
            out["parents"].append(parent.copy())
            out["scores"].append(cum.copy())
            out["logits"].append(logits)
        return out
