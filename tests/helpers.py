"""Shared test plumbing: small synthetic models for the oracle (and, in GPU tests, the HIP path)."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

from paper_2509_24007_amd import inputs as syn
from oracle import oracle as orc


def small_cfg(**kw):
    base = dict(n_layers=2, hidden=32, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn=48, vocab=64,
                rope_theta=1.0e4, dtype="fp32", has_qkv_bias=True)
    base.update(kw)
    return syn.ModelCfg(**base)


def make_model(mcfg, seed=0, std=0.02, device="cpu"):
    g = syn.make_globals(mcfg, seed, device=device, std=std)
    layers = [syn.make_layer(mcfg, seed, l, device=device, std=std) for l in range(mcfg.n_layers)]
    return g, layers


def oracle_model(mcfg, g, layers):
    return orc.model_from_inputs(mcfg, g, layers)


def rel_err(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))
