"""ctypes binding to the CPU oracle (oracle/sdlm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg, never by the GPU library or its Python binding.
All arithmetic lives in the C file; this module only marshals arguments.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdlm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11 + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-march=x86-64-v3", "-fopenmp", "-std=c11", "-Wall", "-Wextra",
                               "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn",
                                         "vocab", "mask_token_id", "has_qkv_bias", "wdtype")] + \
               [(n, C.c_double) for n in ("rope_theta", "rms_eps", "logit_scale")] + [("bf16_points", C.c_int32),
                                                                                     ("block_causal", C.c_int32)]


_PP = C.POINTER(C.c_void_p)
_LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "bq", "bk", "bv", "ffn_norm", "w_gate", "w_up", "w_down")


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, _PP) for n in _LAYER_FIELDS]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i32, f32, f64, vp = C.c_int32, C.c_float, C.c_double, C.c_void_p
        L.orc_num_threads.restype = i32
        L.orc_num_threads.argtypes = []
        L.orc_argmax.restype = i32
        L.orc_argmax.argtypes = [vp, i32]
        L.orc_conf_logit.restype = f64
        L.orc_conf_logit.argtypes = [vp, i32]
        L.orc_conf_entropy.restype = f64
        L.orc_conf_entropy.argtypes = [vp, i32]
        L.orc_gamma.restype = i32
        L.orc_gamma.argtypes = [vp, i32, f32, i32]
        L.orc_block_mask.restype = None
        L.orc_block_mask.argtypes = [vp, i32, i32, i32]
        L.orc_forward_masked_logits.restype = C.c_int
        L.orc_forward_masked_logits.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp]
        L.orc_brute_step.restype = C.c_int
        L.orc_brute_step.argtypes = [vp, vp, vp, i32, i32, f32, i32, i32, vp, vp, vp, vp]
        L.orc_ntp_logits.restype = C.c_int
        L.orc_ntp_logits.argtypes = [vp, vp, vp, i32, vp]
        L.orc_seq_new.restype = vp
        L.orc_seq_new.argtypes = [vp, vp, i32]
        L.orc_seq_free.restype = None
        L.orc_seq_free.argtypes = [vp]
        L.orc_seq_len.restype = i32
        L.orc_seq_len.argtypes = [vp]
        L.orc_seq_cached.restype = i32
        L.orc_seq_cached.argtypes = [vp]
        L.orc_seq_tokens.restype = C.POINTER(i32)
        L.orc_seq_tokens.argtypes = [vp]
        L.orc_seq_prefill.restype = C.c_int
        L.orc_seq_prefill.argtypes = [vp, vp, i32]
        L.orc_seq_step.restype = C.c_int
        L.orc_seq_step.argtypes = [vp, i32, f32, i32, i32, vp, vp, vp, vp]
        L.orc_seq_commit.restype = C.c_int
        L.orc_seq_commit.argtypes = [vp, vp, i32]
        L.orc_gamma_verify.restype = i32
        L.orc_gamma_verify.argtypes = [vp, vp, i32, i32]
        L.orc_seq_verify.restype = C.c_int
        L.orc_seq_verify.argtypes = [vp, i32, vp, vp, vp]
        L.orc_seq_read_kv.restype = C.c_int
        L.orc_seq_read_kv.argtypes = [vp, i32, i32, i32, vp, vp]
        L.orc_probe_logit.restype = f64
        L.orc_probe_logit.argtypes = [vp, vp, vp, i32]
        L.orc_probe_logits_row.restype = None
        L.orc_probe_logits_row.argtypes = [vp, vp, vp, vp]
        L.orc_probe_linear.restype = f64
        L.orc_probe_linear.argtypes = [vp, vp, i32, vp, i32, i32]
        L.orc_probe_attend.restype = None
        L.orc_probe_attend.argtypes = [vp, vp, vp, i32, i32, vp]
        L.orc_probe_rmsnorm.restype = None
        L.orc_probe_rmsnorm.argtypes = [vp, vp, i32, i32, f64, vp]
        L.orc_probe_rope.restype = None
        L.orc_probe_rope.argtypes = [vp, i32, i32, f64]
        L.orc_probe_round_bf16.restype = f64
        L.orc_probe_round_bf16.argtypes = [f64]
        L.orc_probe_silu.restype = f64
        L.orc_probe_silu.argtypes = [f64]
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _as_weight_array(t) -> np.ndarray:
    """torch CPU tensor (fp32 / bf16) or numpy array -> contiguous numpy (float32 or uint16 bit patterns)."""
    if isinstance(t, np.ndarray):
        assert t.dtype in (np.float32, np.uint16)
        return np.ascontiguousarray(t)
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    assert t.dtype == torch.float32
    return t.numpy()


class Model:
    """Model configuration + weights held as numpy arrays for the oracle."""

    def __init__(self, *, n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
                 rope_theta, rms_eps, logit_scale, mask_token_id, has_qkv_bias,
                 globals_: Dict[str, object], layers: Sequence[Dict[str, object]], bf16_points: bool = False,
                 block_causal: bool = False):
        self.vocab, self.hidden, self.n_layers = vocab, hidden, n_layers
        self.head_dim, self.n_kv_heads, self.n_q_heads = head_dim, n_kv_heads, n_q_heads
        self._keep: List[np.ndarray] = []
        emb = _as_weight_array(globals_["embed"])
        wdtype = 0 if emb.dtype == np.float32 else 1
        self.wdtype = wdtype
        self.cfg = _Cfg(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, mask_token_id,
                        int(bool(has_qkv_bias)), wdtype, rope_theta, rms_eps, logit_scale, int(bool(bf16_points)),
                        int(bool(block_causal)))
        self.w = _Weights()
        self.arrays: Dict[str, object] = {}
        for name in ("embed", "lm_head", "final_norm"):
            a = _as_weight_array(globals_[name])
            self._keep.append(a)
            self.arrays[name] = a
            setattr(self.w, name, a.ctypes.data)
        self._tables = []
        for name in _LAYER_FIELDS:
            tab = (C.c_void_p * n_layers)()
            per = []
            for l in range(n_layers):
                t = layers[l].get(name)
                if t is None:
                    tab[l] = None
                    per.append(None)
                else:
                    a = _as_weight_array(t)
                    self._keep.append(a)
                    per.append(a)
                    tab[l] = a.ctypes.data
            self.arrays[name] = per
            self._tables.append(tab)
            setattr(self.w, name, C.cast(tab, _PP))

    def set_bf16_points(self, on: bool) -> None:
        self.cfg.bf16_points = int(bool(on))

    @property
    def cfg_p(self):
        return C.addressof(self.cfg)

    @property
    def w_p(self):
        return C.addressof(self.w)


def model_from_inputs(mcfg, globals_, layers, bf16_points: bool = False) -> Model:
    """Build an oracle Model from the synthetic-input module's ModelCfg and tensors.

    bf16_points=True makes the oracle round activations to bf16 at the points where a bf16 pipeline must
    (see round_rows in the C file); the default keeps every intermediate in double."""
    return Model(n_layers=mcfg.n_layers, hidden=mcfg.hidden, n_q_heads=mcfg.n_q_heads, n_kv_heads=mcfg.n_kv_heads,
                 head_dim=mcfg.head_dim, ffn=mcfg.ffn, vocab=mcfg.vocab, rope_theta=mcfg.rope_theta,
                 rms_eps=mcfg.rms_eps, logit_scale=mcfg.logit_scale, mask_token_id=mcfg.mask_token_id,
                 has_qkv_bias=mcfg.has_qkv_bias, globals_=globals_, layers=layers, bf16_points=bf16_points,
                 block_causal=getattr(mcfg, "block_causal", False))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ------------------------------------------------------------------ scalar rules

def argmax(z) -> int:
    z = np.ascontiguousarray(z, dtype=np.float64)
    return int(lib().orc_argmax(_ptr(z), z.size))


def conf_logit(z) -> float:
    z = np.ascontiguousarray(z, dtype=np.float64)
    return float(lib().orc_conf_logit(_ptr(z), z.size))


def conf_entropy(z) -> float:
    z = np.ascontiguousarray(z, dtype=np.float64)
    return float(lib().orc_conf_entropy(_ptr(z), z.size))


def gamma(conf, tau: float, rule: int = 0) -> int:
    c = np.ascontiguousarray(conf, dtype=np.float32)
    return int(lib().orc_gamma(_ptr(c), c.size, float(tau), rule))


def gamma_verify(yhat, ytilde, rule: int = 0) -> int:
    a, b = _i32(yhat), _i32(ytilde)
    assert a.size == b.size
    return int(lib().orc_gamma_verify(_ptr(a), _ptr(b), a.size, rule))


def block_mask(n: int, D: int, causal: bool = False) -> np.ndarray:
    T = n + D - 1
    m = np.zeros((T, T), dtype=np.uint8)
    lib().orc_block_mask(_ptr(m), n, D, int(bool(causal)))
    return m


# ------------------------------------------------------------------ forwards

def forward_masked_logits(model: Model, ids, mask: np.ndarray, r0: int, nr: int) -> np.ndarray:
    ids = _i32(ids)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    assert mask.shape == (ids.size, ids.size)
    out = np.empty((nr, model.vocab), dtype=np.float64)
    rc = lib().orc_forward_masked_logits(model.cfg_p, model.w_p, _ptr(ids), ids.size, _ptr(mask), r0, nr, _ptr(out))
    assert rc == 0
    return out


def brute_step(model: Model, tokens, D: int, tau: float, rule: int = 0, conf_fn: int = 0):
    """Full recomputation of one decode step -> (logits[D,V], ids[D], conf[D] float32, gamma)."""
    tokens = _i32(tokens)
    logits = np.empty((D, model.vocab), dtype=np.float64)
    ids = np.empty(D, dtype=np.int32)
    conf = np.empty(D, dtype=np.float32)
    g = C.c_int32(0)
    rc = lib().orc_brute_step(model.cfg_p, model.w_p, _ptr(tokens), tokens.size, D, float(tau), rule, conf_fn,
                              _ptr(logits), _ptr(ids), _ptr(conf), C.addressof(g))
    assert rc == 0, rc
    return logits, ids, conf, int(g.value)


def ntp_logits(model: Model, tokens) -> np.ndarray:
    tokens = _i32(tokens)
    out = np.empty(model.vocab, dtype=np.float64)
    rc = lib().orc_ntp_logits(model.cfg_p, model.w_p, _ptr(tokens), tokens.size, _ptr(out))
    assert rc == 0
    return out


class Seq:
    """One sequence decoded incrementally with the clean cache."""

    def __init__(self, model: Model, max_len: int):
        self.model = model
        self.h = lib().orc_seq_new(model.cfg_p, model.w_p, max_len)
        assert self.h

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_seq_free(self.h)
            self.h = None

    def prefill(self, ids) -> None:
        ids = _i32(ids)
        rc = lib().orc_seq_prefill(self.h, _ptr(ids), ids.size)
        assert rc == 0, rc

    def step(self, D: int, tau: float, rule: int = 0, conf_fn: int = 0, want_logits: bool = True):
        logits = np.empty((D, self.model.vocab), dtype=np.float64) if want_logits else None
        ids = np.empty(D, dtype=np.int32)
        conf = np.empty(D, dtype=np.float32)
        g = C.c_int32(0)
        rc = lib().orc_seq_step(self.h, D, float(tau), rule, conf_fn, _ptr(logits), _ptr(ids), _ptr(conf),
                                C.addressof(g))
        assert rc == 0, rc
        self._last_D = D
        return logits, ids, conf, int(g.value)

    def commit(self, ids=None, count: int = 0) -> int:
        if ids is None:
            return int(lib().orc_seq_commit(self.h, None, 0))
        ids = _i32(ids)
        return int(lib().orc_seq_commit(self.h, _ptr(ids), int(count)))

    def verify(self, rule: int = 0, want_logits: bool = False):
        """Second pass of a self-speculative step -> (ytilde[D], gamma_verify[, logits[D,V] (row 0 unused)])."""
        D = self._last_D
        logits = np.zeros((D, self.model.vocab), dtype=np.float64) if want_logits else None
        yt = np.empty(D, dtype=np.int32)
        g = C.c_int32(0)
        rc = lib().orc_seq_verify(self.h, rule, _ptr(logits), _ptr(yt), C.addressof(g))
        assert rc == 0, rc
        return (yt, int(g.value), logits) if want_logits else (yt, int(g.value))

    @property
    def n(self) -> int:
        return int(lib().orc_seq_len(self.h))

    @property
    def c(self) -> int:
        return int(lib().orc_seq_cached(self.h))

    @property
    def tokens(self) -> np.ndarray:
        p = lib().orc_seq_tokens(self.h)
        return np.ctypeslib.as_array(p, shape=(self.n,)).copy()

    def read_kv(self, layer: int, pos: int, kv_head: int):
        d = self.model.head_dim
        k = np.empty(d, dtype=np.float64)
        v = np.empty(d, dtype=np.float64)
        rc = lib().orc_seq_read_kv(self.h, layer, pos, kv_head, _ptr(k), _ptr(v))
        assert rc == 0
        return k, v


# ------------------------------------------------------------------ probes

def probe_logit(model: Model, xhat, v: int) -> float:
    x = np.ascontiguousarray(xhat, dtype=np.float64)
    return float(lib().orc_probe_logit(model.cfg_p, model.w_p, _ptr(x), int(v)))


def probe_logits_row(model: Model, xhat) -> np.ndarray:
    x = np.ascontiguousarray(xhat, dtype=np.float64)
    out = np.empty(model.vocab, dtype=np.float64)
    lib().orc_probe_logits_row(model.cfg_p, model.w_p, _ptr(x), _ptr(out))
    return out


def probe_linear(W: np.ndarray, b: Optional[np.ndarray], x, o: int) -> float:
    x = np.ascontiguousarray(x, dtype=np.float64)
    wdtype = 0 if W.dtype == np.float32 else 1
    return float(lib().orc_probe_linear(_ptr(W), _ptr(b), wdtype, _ptr(x), x.size, int(o)))


def probe_attend(q, K, V) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    out = np.empty(q.size, dtype=np.float64)
    lib().orc_probe_attend(_ptr(q), _ptr(K), _ptr(V), K.shape[0], q.size, _ptr(out))
    return out


def probe_rmsnorm(x, g: np.ndarray, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    wdtype = 0 if g.dtype == np.float32 else 1
    y = np.empty_like(x)
    lib().orc_probe_rmsnorm(_ptr(x), _ptr(g), wdtype, x.size, float(eps), _ptr(y))
    return y


def probe_rope(v, pos: int, theta: float) -> np.ndarray:
    v = np.array(v, dtype=np.float64)
    lib().orc_probe_rope(_ptr(v), v.size, int(pos), float(theta))
    return v


def probe_round_bf16(x: float) -> float:
    return float(lib().orc_probe_round_bf16(float(x)))


def probe_silu(x: float) -> float:
    return float(lib().orc_probe_silu(float(x)))
