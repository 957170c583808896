"""ctypes binding of libsan.so: argument marshalling only.

Every step of the decoder runs in the library's HIP kernels; torch is used here
for device buffers and for the stream handle.  There is no CPU fallback: if the
library is not built, importing `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsan.so")

SAN_OK, SAN_EINVAL, SAN_EPOLICY, SAN_ESTATE, SAN_ECAPACITY, SAN_EHIP, SAN_ENOMEM = range(7)
SAN_F32, SAN_BF16 = 0, 1
SAN_SELF_DOT, SAN_SELF_AAN = 0, 1
SAN_SHARE_A, SAN_SHARE_S = 0, 1
SAN_DBG_S_SELF, SAN_DBG_A_SELF, SAN_DBG_S_CTX, SAN_DBG_A_CTX, SAN_DBG_HIDDEN, SAN_DBG_ENC_OUT, SAN_DBG_MEM = range(7)

EXPORTS = ["san_weight_bytes", "san_init", "san_encode", "san_rewind", "san_decode_step", "san_topk",
           "san_beam_reorder", "san_debug_get", "san_step", "san_device_bytes", "san_last_launch_count",
           "san_last_error", "san_free", "san_profile", "san_profile_read",
           "san_policy_accumulate", "san_policy_read", "san_policy_search", "san_decode_n", "san_stream_read", "san_finished",
           "san_done_flags", "san_compact", "san_active", "san_topk_noalloc"]

SAN_LOOP_GRAPH, SAN_LOOP_COMPACT, SAN_LOOP_LOGITS = 1, 2, 4

KINDS = ["misc", "proj", "attn_self", "attn_apply", "out", "ln", "attn_ctx", "attn_ctx_apply", "ffn", "logits",
         "topk", "reorder", "aan"]


class SanConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_enc_layers", "n_dec_layers", "d_model", "n_heads", "d_ff", "vocab", "max_batch", "beam",
        "max_src_len", "max_tgt_len", "dtype", "self_kind", "encdec_share", "use_cache",
        "pad_id", "bos_id", "eos_id", "debug")] + [("ln_eps", C.c_float)]


class SanPolicy(C.Structure):
    _fields_ = [("n_self", C.c_int32), ("self_pi", C.POINTER(C.c_int32)),
                ("n_encdec", C.c_int32), ("encdec_pi", C.POINTER(C.c_int32)),
                ("n_enc", C.c_int32), ("enc_pi", C.POINTER(C.c_int32))]


class SanError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libsan error {code}: {msg}")
        self.code = code


_lib = None


def lib_state() -> dict:
    """Which sources the loaded library was built from: the hash recorded by build.py next to
    libsan.so, the hash of the sources in the tree now, and whether they differ (a library
    older than csrc/ -- built binaries are not part of the history, so nothing else records it)."""
    from . import build
    now, then = build.source_hash(), build.built_from()
    return {"source_hash": now, "built_from": then, "stale": now != then}


def lib():
    """Load libsan.so (built in-tree by build.py).  Fails loudly if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_1906_11024_amd.build`")
        l = C.CDLL(LIB_PATH)
        st = lib_state()
        if st["stale"]:
            import warnings
            warnings.warn(f"libsan.so was built from sources {st['built_from'] or '(no record)'} but the tree holds "
                          f"{st['source_hash']}: run `python -m paper_1906_11024_amd.build`", RuntimeWarning)
        vp, i32, f32p, i32p = C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p
        l.san_weight_bytes.restype = C.c_size_t
        l.san_weight_bytes.argtypes = [C.POINTER(SanConfig)]
        l.san_init.restype = C.c_int
        l.san_init.argtypes = [C.POINTER(SanConfig), vp, C.c_size_t, C.POINTER(SanPolicy), vp, C.POINTER(vp)]
        l.san_encode.restype = C.c_int
        l.san_encode.argtypes = [vp, i32p, i32p, i32, i32]
        l.san_rewind.restype = C.c_int
        l.san_rewind.argtypes = [vp]
        l.san_decode_step.restype = C.c_int
        l.san_decode_step.argtypes = [vp, i32p, f32p]
        l.san_topk.restype = C.c_int
        l.san_topk.argtypes = [vp, f32p, f32p, i32, i32p, i32p, f32p]
        l.san_topk_noalloc.restype = C.c_int
        l.san_topk_noalloc.argtypes = [vp, f32p, f32p, i32, i32p, i32p, f32p]
        l.san_beam_reorder.restype = C.c_int
        l.san_beam_reorder.argtypes = [vp, i32p]
        l.san_debug_get.restype = C.c_int
        l.san_debug_get.argtypes = [vp, i32, i32, vp, C.c_size_t]
        l.san_step.restype = i32
        l.san_step.argtypes = [vp]
        l.san_device_bytes.restype = C.c_size_t
        l.san_device_bytes.argtypes = [vp, i32]
        l.san_stream_read.restype = C.c_int
        l.san_stream_read.argtypes = [vp, vp, C.c_size_t]
        l.san_finished.restype = C.c_int
        l.san_finished.argtypes = [vp, C.POINTER(C.c_int32)]
        l.san_done_flags.restype = C.c_int
        l.san_done_flags.argtypes = [vp, C.POINTER(C.c_int32)]
        l.san_compact.restype = C.c_int
        l.san_compact.argtypes = [vp, C.POINTER(C.c_int32), i32]
        l.san_active.restype = C.c_int
        l.san_active.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        l.san_last_launch_count.restype = i32
        l.san_last_launch_count.argtypes = [vp]
        l.san_last_error.restype = C.c_char_p
        l.san_last_error.argtypes = [vp]
        l.san_profile.restype = C.c_int
        l.san_profile.argtypes = [vp, i32]
        l.san_profile_read.restype = C.c_int
        l.san_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]
        l.san_decode_n.restype = C.c_int
        l.san_decode_n.argtypes = [vp, i32, i32p, f32p, i32p, i32p, f32p, i32]
        l.san_policy_accumulate.restype = C.c_int
        l.san_policy_accumulate.argtypes = [vp]
        l.san_policy_read.restype = C.c_int
        l.san_policy_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]
        l.san_policy_search.restype = C.c_int
        l.san_policy_search.argtypes = [C.POINTER(C.c_double), i32, C.c_double, C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32)]
        l.san_free.restype = None
        l.san_free.argtypes = [vp]
        _lib = l
    return _lib


def make_config(cfg: dict, *, max_batch=None, beam=None, max_src_len=None, max_tgt_len=None,
                encdec_share=SAN_SHARE_A, use_cache=1, eos_id=-1, debug=0, ln_eps=1e-5) -> SanConfig:
    """Fill a san_config from a workload description (see workloads.CONFIGS)."""
    return SanConfig(
        n_enc_layers=cfg["n_enc"], n_dec_layers=cfg["n_dec"], d_model=cfg["d"], n_heads=cfg["H"],
        d_ff=cfg["F"], vocab=cfg["V"], max_batch=max_batch or cfg["batch"], beam=beam or cfg["beam"],
        max_src_len=max_src_len or cfg["src_len"][1], max_tgt_len=max_tgt_len or cfg["steps"],
        dtype=SAN_BF16 if cfg["dtype"] == "bf16" else SAN_F32,
        self_kind=SAN_SELF_AAN if cfg.get("self_kind") == "aan" else SAN_SELF_DOT,
        encdec_share=encdec_share, use_cache=use_cache, pad_id=0, bos_id=1, eos_id=eos_id,
        debug=debug, ln_eps=ln_eps)


def policy_search(js: np.ndarray, theta: float) -> list:
    """Greedy block search of Sec. 3.3 on a JS matrix (host code of the library)."""
    js = np.ascontiguousarray(js, dtype=np.float64)
    L = js.shape[0]
    pi = (C.c_int32 * L)()
    nb = C.c_int32()
    rc = lib().san_policy_search(js.ctypes.data_as(C.POINTER(C.c_double)), L, float(theta), pi, C.byref(nb))
    if rc != SAN_OK:
        raise SanError(rc, "san_policy_search")
    return list(pi[: nb.value])


def weight_bytes(sc: SanConfig) -> int:
    return int(lib().san_weight_bytes(C.byref(sc)))


class San:
    """Thin handle around a san_ctx.  Tensor arguments are torch CUDA tensors
    (int32 / float32, contiguous); only their data pointers cross the boundary."""

    def __init__(self, sc: SanConfig, blob: np.ndarray, self_pi, encdec_pi, stream=None, enc_pi=None):
        import torch
        self._torch = torch
        self._l = lib()
        self.cfg = sc
        blob = np.ascontiguousarray(blob).view(np.uint8)
        sp = (C.c_int32 * max(1, len(self_pi)))(*self_pi)
        ep = (C.c_int32 * max(1, len(encdec_pi)))(*encdec_pi)
        enc_pi = list(enc_pi) if enc_pi else []
        np_ = (C.c_int32 * max(1, len(enc_pi)))(*enc_pi)
        pol = SanPolicy(len(self_pi), C.cast(sp, C.POINTER(C.c_int32)), len(encdec_pi), C.cast(ep, C.POINTER(C.c_int32)),
                        len(enc_pi), C.cast(np_, C.POINTER(C.c_int32)) if enc_pi else None)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        rc = self._l.san_init(C.byref(sc), blob.ctypes.data_as(C.c_void_p), blob.nbytes, C.byref(pol),
                              C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if rc != SAN_OK:
            raise SanError(rc, self._l.san_last_error(None).decode())
        self._h = h
        self.rows = 0

    # -- helpers
    def _check(self, rc):
        if rc != SAN_OK:
            raise SanError(rc, self._l.san_last_error(self._h).decode())

    @staticmethod
    def _p(t):
        return C.c_void_p(t.data_ptr())

    def _want(self, t, dtype, numel=None):
        torch = self._torch
        if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
            raise TypeError(f"expected a contiguous CUDA tensor of {dtype}")
        if numel is not None and t.numel() < numel:
            raise ValueError(f"tensor has {t.numel()} elements, need {numel}")

    # -- the five calls (+ utilities)
    def encode(self, src_ids, src_len):
        torch = self._torch
        self._want(src_ids, torch.int32)
        self._want(src_len, torch.int32)
        batch, max_src = src_ids.shape
        self._check(self._l.san_encode(self._h, self._p(src_ids), self._p(src_len), batch, max_src))
        self.batch = batch
        self.batch_encoded = batch
        self.max_src_of_batch = max_src
        self.rows = batch * self.cfg.beam

    def rewind(self):
        self._check(self._l.san_rewind(self._h))
        self._sync_batch()

    def _sync_batch(self):
        n = C.c_int32(0)
        self._check(self._l.san_active(self._h, None, C.byref(n)))
        self.batch = int(n.value)
        self.rows = self.batch * self.cfg.beam

    def done_flags(self):
        """per-sentence finished flags of the current batch (numpy int32; synchronises the stream)"""
        out = np.zeros(max(1, self.batch), dtype=np.int32)
        self._check(self._l.san_done_flags(self._h, out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out[:self.batch]

    def compact(self, keep):
        """keep: increasing indices (into the current batch) of the sentences that stay"""
        keep = np.ascontiguousarray(np.asarray(keep, dtype=np.int32))
        self._check(self._l.san_compact(self._h, keep.ctypes.data_as(C.POINTER(C.c_int32)), len(keep)))
        self._sync_batch()

    def active(self):
        """indices, into the encoded batch, of the sentences of the current batch"""
        out = np.zeros(max(1, self.cfg.max_batch), dtype=np.int32)
        n = C.c_int32(0)
        self._check(self._l.san_active(self._h, out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n)))
        return out[:int(n.value)].copy()

    def decode_step(self, tokens, logits):
        torch = self._torch
        self._want(tokens, torch.int32, self.rows)
        self._want(logits, torch.float32, self.rows * self.cfg.vocab)
        self._check(self._l.san_decode_step(self._h, self._p(tokens), self._p(logits)))

    def topk(self, logits, cum_score, k, out_token, out_parent, out_score):
        torch = self._torch
        self._want(logits, torch.float32, self.rows * self.cfg.vocab)
        self._want(cum_score, torch.float32, self.rows)
        for t, dt in ((out_token, torch.int32), (out_parent, torch.int32), (out_score, torch.float32)):
            self._want(t, dt, self.batch * k)
        self._check(self._l.san_topk(self._h, self._p(logits), self._p(cum_score), k, self._p(out_token),
                                     self._p(out_parent), self._p(out_score)))

    def topk_noalloc(self, logits, cum_score, k, out_token, out_parent, out_score):
        torch = self._torch
        self._want(logits, torch.float32, self.rows * self.cfg.vocab)
        self._want(cum_score, torch.float32, self.rows)
        for t, dt in ((out_token, torch.int32), (out_parent, torch.int32), (out_score, torch.float32)):
            self._want(t, dt, self.batch * k)
        self._check(self._l.san_topk_noalloc(self._h, self._p(logits), self._p(cum_score), k, self._p(out_token),
                                             self._p(out_parent), self._p(out_score)))

    def beam_reorder(self, parent):
        self._want(parent, self._torch.int32, self.rows)
        self._check(self._l.san_beam_reorder(self._h, self._p(parent)))

    def debug_get(self, what, layer, follower=False):
        torch = self._torch
        n = self.step
        H, d = self.cfg.n_heads, self.cfg.d_model
        if what == SAN_DBG_S_SELF:
            shape = (self.rows, H, n)
        elif what == SAN_DBG_S_CTX:
            shape = (self.rows, H, self.max_src_of_batch)
        elif what == SAN_DBG_ENC_OUT:
            shape = (self.batch_encoded, self.max_src_of_batch, d)
        elif what == SAN_DBG_MEM:
            # a block head keeps [K | V]; a follower that shares only the weights keeps its own V
            shape = (self.batch_encoded, self.max_src_of_batch, d if follower else 2 * d)
        else:
            shape = (self.rows, d)
        out = torch.empty(shape, dtype=torch.float32, device="cuda")
        self._check(self._l.san_debug_get(self._h, what, layer, self._p(out), out.numel() * 4))
        return out

    @property
    def step(self):
        return int(self._l.san_step(self._h))

    def device_bytes(self, which):
        return int(self._l.san_device_bytes(self._h, which))

    def finished(self):
        """sentences of the batch whose kept hypotheses all end in EOS (synchronises the stream)"""
        n = C.c_int32(0)
        self._check(self._l.san_finished(self._h, C.byref(n)))
        return int(n.value)

    def stream_read(self, buf):
        """queue one plain streaming read of the whole device tensor `buf` (measurement aid)"""
        self._check(self._l.san_stream_read(self._h, self._p(buf), buf.numel() * buf.element_size()))

    @property
    def last_launch_count(self):
        return int(self._l.san_last_launch_count(self._h))

    def profile(self, enable: bool):
        self._check(self._l.san_profile(self._h, 1 if enable else 0))

    def profile_read(self, reset=True):
        """{class name: (milliseconds, launches)} accumulated since the last reset."""
        ms = (C.c_double * len(KINDS))()
        n = (C.c_int64 * len(KINDS))()
        self._check(self._l.san_profile_read(self._h, ms, n, 1 if reset else 0))
        return {k: (ms[i], int(n[i])) for i, k in enumerate(KINDS)}

    def decode_n(self, n, tokens, cum_io, out_tokens, out_parents, logits_work, use_graph=False, compact=False,
                 keep_logits=False):
        torch = self._torch
        self._want(tokens, torch.int32, self.rows)
        self._want(cum_io, torch.float32, self.rows)
        self._want(out_tokens, torch.int32, n * self.rows)
        self._want(out_parents, torch.int32, n * self.rows)
        self._want(logits_work, torch.float32, self.rows * self.cfg.vocab)
        self._check(self._l.san_decode_n(self._h, n, self._p(tokens), self._p(cum_io), self._p(out_tokens),
                                         self._p(out_parents), self._p(logits_work),
                                         (SAN_LOOP_GRAPH if use_graph else 0) | (SAN_LOOP_COMPACT if compact else 0) |
                                         (SAN_LOOP_LOGITS if keep_logits else 0)))
        if compact:
            self._sync_batch()

    def policy_accumulate(self):
        self._check(self._l.san_policy_accumulate(self._h))

    def policy_read(self, which, reset=False):
        """(mean JS matrix [L, L] as numpy float64, number of samples)"""
        L = self.cfg.n_dec_layers
        js = np.zeros((L, L), dtype=np.float64)
        cnt = C.c_int64()
        self._check(self._l.san_policy_read(self._h, which, js.ctypes.data_as(C.POINTER(C.c_double)),
                                            C.byref(cnt), 1 if reset else 0))
        return js, int(cnt.value)

    def close(self):
        if getattr(self, "_h", None):
            self._l.san_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
