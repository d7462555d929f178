"""Thin ctypes binding to libsdlm.so (include/sdlm.h).  Argument marshalling only.

torch is used for device memory (the workspace, weights, outputs) and for the stream; every step of the
block-decode path runs in the library's own HIP kernels.  There is no fallback: if the library cannot be
loaded, importing the entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdlm.so")

PHASES = ("rows", "norm", "qkv", "rope", "attn", "oproj", "gateup", "down", "lmhead", "accept", "attn_merge")
OK, EINVAL, ECAPACITY, ESTATE, EHIP = 0, -1, -2, -3, -4

EXPORTS = ("sdlm_workspace_bytes", "sdlm_create", "sdlm_init_weights", "sdlm_prefill", "sdlm_decode_step",
           "sdlm_decode_step_static", "sdlm_graph", "sdlm_verify_step", "sdlm_kv_commit", "sdlm_get_lengths", "sdlm_debug_tap", "sdlm_debug_rows", "sdlm_debug_read_kv",
           "sdlm_debug_gemm_plan", "sdlm_max_rows", "sdlm_profile", "sdlm_profile_every", "sdlm_profile_read", "sdlm_kernel_info", "sdlm_last_error",
           "sdlm_destroy")


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("logit_scale", C.c_float),
                ("dtype", C.c_int32), ("mask_token_id", C.c_int32), ("has_qkv_bias", C.c_int32),
                ("block_causal", C.c_int32)]


class RunCfg(C.Structure):
    _fields_ = [("max_batch", C.c_int32), ("max_seq_len", C.c_int32), ("block_D", C.c_int32), ("kv_layout", C.c_int32),
                ("page_size", C.c_int32), ("n_pages", C.c_int32), ("tau", C.c_float), ("conf_fn", C.c_int32),
                ("accept_rule", C.c_int32), ("prefill_rows", C.c_int32)]


_PP = C.POINTER(C.c_void_p)
_LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "bq", "bk", "bv", "ffn_norm", "w_gate", "w_up", "w_down")


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", _PP), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP),
                ("bq", _PP), ("bk", _PP), ("bv", _PP), ("ffn_norm", _PP), ("w_gate", _PP), ("w_up", _PP), ("w_down", _PP)]


_lib = None


def load():
    """Load libsdlm.so (built by paper_2509_24007_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python paper_2509_24007_amd/build.py` (no fallback exists)")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    L.sdlm_workspace_bytes.restype = sz
    L.sdlm_workspace_bytes.argtypes = [vp, vp]
    L.sdlm_create.restype = C.c_int
    L.sdlm_create.argtypes = [vp, vp, vp, sz, vp, C.POINTER(vp)]
    L.sdlm_init_weights.restype = C.c_int
    L.sdlm_init_weights.argtypes = [vp, vp, i32]
    L.sdlm_prefill.restype = C.c_int
    L.sdlm_prefill.argtypes = [vp, i32, vp, vp]
    L.sdlm_decode_step.restype = C.c_int
    L.sdlm_decode_step.argtypes = [vp, vp, vp, vp, vp]
    L.sdlm_decode_step_static.restype = C.c_int
    L.sdlm_decode_step_static.argtypes = [vp, vp, vp, vp, vp]
    L.sdlm_debug_gemm_plan.restype = C.c_int
    L.sdlm_debug_gemm_plan.argtypes = [C.c_int32] * 5 + [vp, vp, vp]
    L.sdlm_graph.restype = C.c_int
    L.sdlm_graph.argtypes = [vp, C.c_int32]
    L.sdlm_verify_step.restype = C.c_int
    L.sdlm_verify_step.argtypes = [vp, C.c_int32, vp, vp, vp]
    L.sdlm_kv_commit.restype = C.c_int
    L.sdlm_kv_commit.argtypes = [vp, vp, vp]
    L.sdlm_get_lengths.restype = C.c_int
    L.sdlm_get_lengths.argtypes = [vp, vp, vp]
    L.sdlm_debug_tap.restype = C.c_int
    L.sdlm_debug_tap.argtypes = [vp, i32, i32, vp]
    L.sdlm_debug_rows.restype = C.c_int
    L.sdlm_debug_rows.argtypes = [vp, vp, vp, vp, vp, vp]
    L.sdlm_debug_read_kv.restype = C.c_int
    L.sdlm_debug_read_kv.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
    L.sdlm_max_rows.restype = i32
    L.sdlm_max_rows.argtypes = [vp]
    L.sdlm_profile.restype = C.c_int
    L.sdlm_profile.argtypes = [vp, i32]
    L.sdlm_profile_every.restype = C.c_int
    L.sdlm_profile_every.argtypes = [vp, i32]
    L.sdlm_profile_read.restype = C.c_int
    L.sdlm_profile_read.argtypes = [vp, vp, vp]
    L.sdlm_kernel_info.restype = C.c_char_p
    L.sdlm_kernel_info.argtypes = [vp]
    L.sdlm_last_error.restype = C.c_char_p
    L.sdlm_last_error.argtypes = [vp]
    L.sdlm_destroy.restype = None
    L.sdlm_destroy.argtypes = [vp]
    _lib = L
    return L


class SdlmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sdlm error {code}: {msg}")
        self.code = code


def model_cfg(m) -> ModelCfg:
    """From the synthetic-input module's ModelCfg (or any object with the same attributes)."""
    return ModelCfg(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab,
                    m.rope_theta, m.rms_eps, m.logit_scale, 0 if m.dtype == "fp32" else 1, m.mask_token_id,
                    int(bool(m.has_qkv_bias)), int(bool(getattr(m, "block_causal", False))))


def gemm_plan(epilogue: int, rows: int, min_rows: int, n: int, k: int):
    """(tile rows, tile columns, k splits) of the matrix-core GEMM launch for this problem; host logic, no GPU needed."""
    tr, tc, sp = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    rc = load().sdlm_debug_gemm_plan(epilogue, rows, min_rows, n, k, C.byref(tr), C.byref(tc), C.byref(sp))
    if rc != 0:
        raise SdlmError(rc, "bad arguments to sdlm_debug_gemm_plan")
    return tr.value, tc.value, sp.value


def _dp(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


class Context:
    """One sdlm_ctx plus the torch allocations it borrows."""

    def __init__(self, mcfg: ModelCfg, *, max_batch: int, max_seq_len: int, block_D: int, tau: float,
                 paged: bool = False, n_pages: int = 0, conf_fn: int = 0, accept_rule: int = 0,
                 prefill_rows: int = 0, device="cuda:0", poison: bool = False):
        L = load()
        self.L = L
        self.m = mcfg
        self.r = RunCfg(max_batch, max_seq_len, block_D, 1 if paged else 0, 16, n_pages, tau, conf_fn, accept_rule,
                        prefill_rows)
        self.device = torch.device(device)
        self.D, self.max_batch = block_D, max_batch
        need = L.sdlm_workspace_bytes(C.byref(self.m), C.byref(self.r))
        if need == 0:
            h = C.c_void_p()
            rc = L.sdlm_create(C.byref(self.m), C.byref(self.r), None, 0, None, C.byref(h))
            msg = L.sdlm_last_error(h).decode() if h else "invalid configuration"
            L.sdlm_destroy(h)
            raise SdlmError(rc, msg)
        self.workspace_bytes = need
        self.workspace = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        if poison:   # tests: every byte 0xFF (NaN as bf16/fp32, -1 as int) so that reliance on fresh memory shows
            self.workspace.fill_(0xFF)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self.stream = torch.cuda.current_stream(self.device)
        self.h = C.c_void_p()
        rc = L.sdlm_create(C.byref(self.m), C.byref(self.r), C.c_void_p(self._ws_ptr), need,
                           C.c_void_p(self.stream.cuda_stream), C.byref(self.h))
        if rc != 0:
            msg = L.sdlm_last_error(self.h).decode()
            L.sdlm_destroy(self.h)
            self.h = None
            raise SdlmError(rc, msg)
        self.batch = 0
        self._keep: List[object] = []

    # -- helpers
    def _order_inputs(self):
        """The library runs on the stream the context was created on.  When torch's current stream is another one,
        work queued there that produces the tensors being handed over must come first."""
        cur = torch.cuda.current_stream(self.device)
        if cur.cuda_stream != self.stream.cuda_stream:
            self.stream.wait_stream(cur)

    def _check(self, rc: int):
        if rc != 0:
            raise SdlmError(rc, self.L.sdlm_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            torch.cuda.synchronize(self.device)
            self.L.sdlm_destroy(self.h)
            self.h = None
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def kernel_info(self) -> str:
        return self.L.sdlm_kernel_info(self.h).decode()

    @property
    def max_rows(self) -> int:
        return int(self.L.sdlm_max_rows(self.h))

    # -- the four core calls
    def init_weights(self, globals_: Optional[Dict[str, torch.Tensor]] = None,
                     layers: Optional[Dict[int, Dict[str, Optional[torch.Tensor]]]] = None) -> None:
        """globals_: embed / lm_head / final_norm; layers: {layer index: tensors of that layer}.  Either may be
        partial; tensors may live on the device or on the host (all of one call in the same place)."""
        w = Weights()
        nL = self.m.n_layers
        keep = []
        on_dev = None

        def place(t):
            nonlocal on_dev
            assert t.is_contiguous()
            d = t.is_cuda
            assert on_dev is None or on_dev == d, "mixing host and device tensors in one call"
            on_dev = d
            return t.data_ptr()

        for name in ("embed", "lm_head", "final_norm"):
            t = (globals_ or {}).get(name)
            setattr(w, name, place(t) if t is not None else None)
        for name in _LAYER_FIELDS:
            tab = (C.c_void_p * nL)()
            for l in range(nL):
                t = (layers or {}).get(l, {}).get(name)
                tab[l] = place(t) if t is not None else None
            keep.append(tab)
            setattr(w, name, C.cast(tab, _PP))
        self._order_inputs()
        self._check(self.L.sdlm_init_weights(self.h, C.byref(w), 1 if on_dev else 0))

    def prefill(self, prompts: Sequence) -> None:
        ids, offs = [], [0]
        for p in prompts:
            p = [int(v) for v in (p.tolist() if hasattr(p, "tolist") else p)]
            ids.extend(p)
            offs.append(len(ids))
        a = (C.c_int32 * max(1, len(ids)))(*ids)
        o = (C.c_int32 * len(offs))(*offs)
        self._check(self.L.sdlm_prefill(self.h, len(prompts), a, o))
        self.batch = len(prompts)

    def decode_step(self, ids: torch.Tensor, count: torch.Tensor, conf: Optional[torch.Tensor] = None,
                    logits: Optional[torch.Tensor] = None, static_scratch: bool = False) -> None:
        """static_scratch=True calls sdlm_decode_step_static (partial results in the library's static array)."""
        B, D = self.batch, self.D
        assert ids.dtype == torch.int32 and ids.numel() >= B * D and ids.is_cuda and ids.is_contiguous()
        assert count.dtype == torch.int32 and count.numel() >= B and count.is_cuda
        assert conf is None or (conf.dtype == torch.float32 and conf.numel() >= B * D and conf.is_cuda and conf.is_contiguous())
        assert logits is None or (logits.dtype == torch.float32 and logits.numel() >= B * D * self.m.vocab and
                                  logits.is_cuda and logits.is_contiguous())
        fn = self.L.sdlm_decode_step_static if static_scratch else self.L.sdlm_decode_step
        self._check(fn(self.h, _dp(ids), _dp(count), _dp(conf), _dp(logits)))

    def graph(self, enable: bool = True) -> None:
        """Replay decode_step as a HIP graph (the context must have been created on a non-default stream)."""
        self._check(self.L.sdlm_graph(self.h, 1 if enable else 0))

    def verify_step(self, rule: int = 0, ids_tilde: Optional[torch.Tensor] = None, count: Optional[torch.Tensor] = None,
                    logits: Optional[torch.Tensor] = None) -> None:
        """Self-speculative verification of the last decode_step; ids_tilde [batch, D] int32, count [batch] int32,
        logits [batch, D-1, vocab] fp32 (all optional, on the device)."""
        for t, n in ((ids_tilde, self.batch * self.D), (count, self.batch)):
            if t is not None:
                assert t.dtype == torch.int32 and t.is_cuda and t.is_contiguous() and t.numel() >= n
        if logits is not None:
            assert logits.dtype == torch.float32 and logits.is_cuda and logits.is_contiguous()
            assert logits.numel() >= self.batch * (self.D - 1) * self.m.vocab
        self._check(self.L.sdlm_verify_step(self.h, int(rule), _dp(ids_tilde), _dp(count), _dp(logits)))

    def kv_commit(self, ids_override: Optional[torch.Tensor] = None, count_override: Optional[torch.Tensor] = None) -> None:
        if ids_override is not None:
            assert ids_override.dtype == torch.int32 and ids_override.is_cuda and ids_override.is_contiguous()
            assert count_override is not None and count_override.dtype == torch.int32 and count_override.is_cuda
            assert ids_override.numel() >= self.batch * self.D and count_override.numel() >= self.batch
            self._order_inputs()
        self._check(self.L.sdlm_kv_commit(self.h, _dp(ids_override), _dp(count_override)))

    # -- state and debugging
    def get_lengths(self):
        n = torch.empty(self.batch, dtype=torch.int32, device=self.device)
        c = torch.empty(self.batch, dtype=torch.int32, device=self.device)
        self._check(self.L.sdlm_get_lengths(self.h, _dp(n), _dp(c)))
        return n.cpu(), c.cpu()

    def tap(self, layer: int, which: int, dst: Optional[torch.Tensor]) -> None:
        self._check(self.L.sdlm_debug_tap(self.h, layer, which, _dp(dst)))

    def rows(self):
        mr = self.max_rows
        out = [torch.empty(mr, dtype=torch.int32, device=self.device) for _ in range(4)]
        n = torch.empty(1, dtype=torch.int32, device=self.device)
        self._check(self.L.sdlm_debug_rows(self.h, *[_dp(t) for t in out], _dp(n)))
        torch.cuda.synchronize(self.device)
        R = int(n.item())
        return {k: t[:R].cpu() for k, t in zip(("tok", "pos", "seq", "kind"), out)}

    def read_kv(self, layer: int, seq: int, kv_head: int, pos0: int, count: int):
        d = self.m.head_dim
        k = torch.empty(count, d, dtype=torch.float32, device=self.device)
        v = torch.empty(count, d, dtype=torch.float32, device=self.device)
        self._check(self.L.sdlm_debug_read_kv(self.h, layer, seq, kv_head, pos0, count, _dp(k), _dp(v)))
        torch.cuda.synchronize(self.device)
        return k.cpu(), v.cpu()

    def profile(self, phases=None, every: int = 1) -> None:
        """phases: None/False -> off, True -> all, or an iterable of phase names to bracket with events; every: only
        every n-th launch of a phase is bracketed."""
        self._check(self.L.sdlm_profile_every(self.h, int(every)))
        if phases is None or phases is False:
            mask = 0
        elif phases is True:
            mask = -1
        else:
            mask = 0
            for p in phases:
                mask |= 1 << PHASES.index(p)
        self._check(self.L.sdlm_profile(self.h, mask))

    def profile_read(self):
        ms = (C.c_float * len(PHASES))()
        cnt = (C.c_int32 * len(PHASES))()
        self._check(self.L.sdlm_profile_read(self.h, ms, cnt))
        return {p: (float(ms[i]), int(cnt[i])) for i, p in enumerate(PHASES)}
