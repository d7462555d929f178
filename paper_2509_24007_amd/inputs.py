"""Seeded synthetic inputs for the SDLM block-decode step.

This module only manufactures *inputs* (weights, prompts, override tokens); it
holds none of the method's arithmetic and is the single piece of code that the
CPU oracle's tests and the HIP path's tests both use.  Everything is produced
by a counter-based generator built from exact 64-bit integer operations, so the
same (seed, tensor name, element index) gives the same bits on the CPU and on
the GPU, in any chunking:

    bits  = mix64(stream_key + index * ODD)          (SplitMix64 finaliser)
    value = QUANTILE[bits >> 48] * std               (normal draws)

QUANTILE is the standard normal inverse CDF at the 65536 midpoints
(u + 0.5) / 65536, evaluated once on the CPU in float64 and then used as a
lookup table on whichever device the tensor is generated on.  The paper trains
on Qwen-2.5 checkpoints and public SFT corpora (Sec. 4.1); neither is available
here, so only the *shapes* of those models are kept and weights are
N(0, 0.02^2) as the benchmark configuration prescribes.
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, List, Optional

import torch

_GOLDEN = -7046029254386353131      # 0x9E3779B97F4A7C15 as int64
_M1 = -4658895280553007687          # 0xBF58476D1CE4E5B9 as int64
_M2 = -7723592293110705685          # 0x94D049BB133111EB as int64


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 lanes."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def mix64(z: torch.Tensor) -> torch.Tensor:
    """SplitMix64 output function on int64 lanes (two's-complement wraparound)."""
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _mix64_int(z: int) -> int:
    mask = (1 << 64) - 1
    z &= mask
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    return z ^ (z >> 31)


def stream_key(seed: int, name: str) -> int:
    """A 64-bit key for the named stream of the given seed (as a signed int64)."""
    k = _mix64_int(seed * 0x9E3779B97F4A7C15 + zlib.crc32(name.encode()) + 0x1234567)
    k = _mix64_int(k + len(name))
    return k - (1 << 64) if k >= (1 << 63) else k


def raw_bits(seed: int, name: str, start: int, count: int, device="cpu") -> torch.Tensor:
    """64 pseudo-random bits (int64) for elements [start, start+count) of a stream."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return mix64(idx * _GOLDEN + stream_key(seed, name))


_QUANTILE_CPU: Optional[torch.Tensor] = None
_QUANTILE_DEV: Dict[str, torch.Tensor] = {}


def _quantile_table(device) -> torch.Tensor:
    global _QUANTILE_CPU
    if _QUANTILE_CPU is None:
        u = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
        _QUANTILE_CPU = torch.special.ndtri(u)
    key = str(device)
    if key not in _QUANTILE_DEV:
        _QUANTILE_DEV[key] = _QUANTILE_CPU.to(device)
    return _QUANTILE_DEV[key]


def normal(seed: int, name: str, shape, std: float, dtype=torch.float32,
           device="cpu", chunk: int = 1 << 25) -> torch.Tensor:
    """N(0, std^2) tensor of the given shape, rounded once to `dtype`."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=dtype, device=device)
    table = _quantile_table(device)
    for lo in range(0, n, chunk):
        cnt = min(chunk, n - lo)
        u = _lsr(raw_bits(seed, name, lo, cnt, device), 48)
        out[lo:lo + cnt] = (table[u] * std).to(torch.float32).to(dtype)
    return out.view(*shape)


def uniform_int(seed: int, name: str, count: int, lo: int, hi: int, device="cpu") -> torch.Tensor:
    """`count` integers uniform on [lo, hi] (inclusive), int32."""
    span = hi - lo + 1
    u = _lsr(raw_bits(seed, name, 0, count, device), 16)     # 48 non-negative bits
    return (u % span + lo).to(torch.int32)


# --------------------------------------------------------------------------
# Configurations (shapes of Qwen-2.5 decoders, Sec. 4.1; sizes of the five
# benchmark workloads).
# --------------------------------------------------------------------------

@dataclasses.dataclass
class ModelCfg:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6
    logit_scale: float = 8.0
    dtype: str = "bf16"            # "fp32" (debug / tiny) or "bf16"
    has_qkv_bias: bool = True
    mask_token_id: int = -1        # -1 -> vocab - 1
    block_causal: bool = False     # the "Causal Attention" ablation: causal instead of mutual attention inside the block

    def __post_init__(self):
        if self.mask_token_id < 0:
            self.mask_token_id = self.vocab - 1

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16


@dataclasses.dataclass
class RunCfg:
    batch: int
    prompt_lo: int
    prompt_hi: int
    block_D: int
    tau: float
    steps: int
    paged: bool = False
    page_size: int = 16
    taus: Optional[List[float]] = None


@dataclasses.dataclass
class Workload:
    name: str
    model: ModelCfg
    run: RunCfg
    seed: int = 0


def workloads() -> Dict[str, Workload]:
    w = {}
    w["C1"] = Workload("C1-tiny-fp32",
                       ModelCfg(2, 256, 4, 2, 64, 688, 4096, rope_theta=1.0e4, dtype="fp32",
                                has_qkv_bias=False),
                       RunCfg(1, 64, 64, 4, 0.5, 32))
    w["C2"] = Workload("C2-qwen2.5-1.5B-shaped",
                       ModelCfg(28, 1536, 12, 2, 128, 8960, 151936),
                       RunCfg(1, 512, 512, 4, 0.9, 256))
    w["C3"] = Workload("C3-qwen2.5-3B-shaped",
                       ModelCfg(36, 2048, 16, 2, 128, 11008, 151936),
                       RunCfg(16, 1024, 2048, 8, 0.9, 512))
    w["C4"] = Workload("C4-qwen2.5-7B-shaped",
                       ModelCfg(28, 3584, 28, 4, 128, 18944, 152064),
                       RunCfg(64, 2048, 4096, 4, 0.9, 512, paged=True, taus=[0.8, 0.9, 0.98]))
    w["C5"] = Workload("C5-qwen2.5-32B-shaped",
                       ModelCfg(64, 5120, 40, 8, 128, 27648, 152064),
                       RunCfg(32, 4096, 8192, 4, 0.9, 256, paged=True))
    return w


# --------------------------------------------------------------------------
# Weights and prompts
# --------------------------------------------------------------------------

LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "bq", "bk", "bv",
                 "ffn_norm", "w_gate", "w_up", "w_down")


def layer_shapes(m: ModelCfg) -> Dict[str, tuple]:
    qd, kd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    return {
        "attn_norm": (m.hidden,), "ffn_norm": (m.hidden,),
        "wq": (qd, m.hidden), "wk": (kd, m.hidden), "wv": (kd, m.hidden),
        "wo": (m.hidden, qd),
        "bq": (qd,), "bk": (kd,), "bv": (kd,),
        "w_gate": (m.ffn, m.hidden), "w_up": (m.ffn, m.hidden), "w_down": (m.hidden, m.ffn),
    }


def make_layer(m: ModelCfg, seed: int, layer: int, device="cpu", std: float = 0.02) -> Dict[str, Optional[torch.Tensor]]:
    """One decoder layer's tensors, [out_features, in_features] row-major.

    Norm gains are 1.0; biases are None when the model has no QKV bias.
    """
    dt = m.torch_dtype
    out: Dict[str, Optional[torch.Tensor]] = {}
    for name, shape in layer_shapes(m).items():
        if name in ("attn_norm", "ffn_norm"):
            out[name] = torch.ones(shape, dtype=dt, device=device)
        elif name in ("bq", "bk", "bv") and not m.has_qkv_bias:
            out[name] = None
        else:
            out[name] = normal(seed, f"L{layer}.{name}", shape, std, dt, device)
    return out


def make_globals(m: ModelCfg, seed: int, device="cpu", std: float = 0.02) -> Dict[str, torch.Tensor]:
    """Embedding table, (untied) LM head and final norm gain."""
    dt = m.torch_dtype
    return {
        "embed": normal(seed, "embed", (m.vocab, m.hidden), std, dt, device),
        "lm_head": normal(seed, "lm_head", (m.vocab, m.hidden), std, dt, device),
        "final_norm": torch.ones((m.hidden,), dtype=dt, device=device),
    }


def make_prompts(seed: int, batch: int, lo: int, hi: int, vocab: int) -> List[torch.Tensor]:
    """`batch` prompts with lengths uniform on [lo, hi] and ids uniform on [0, vocab)."""
    lens = uniform_int(seed, "prompt_len", batch, lo, hi)
    return [uniform_int(seed, f"prompt{b}", int(lens[b]), 0, vocab - 1) for b in range(batch)]


def make_overrides(seed: int, steps: int, batch: int, D: int, vocab: int):
    """Teacher-forcing material: per (step, sequence) a count in [1, D] and D token ids."""
    cnt = uniform_int(seed, "ovr_cnt", steps * batch, 1, D).view(steps, batch)
    ids = uniform_int(seed, "ovr_ids", steps * batch * D, 0, vocab - 1).view(steps, batch, D)
    return ids, cnt
