"""Pins for the CPU oracle: closed forms, hand-derived cases, a library cross-check.

Each test names the passage of the paper that fixes the behaviour.  None of these
tests touches the GPU path.
"""
import math
import os

import numpy as np
import pytest
import torch

from helpers import make_model, oracle_model, rel_err, small_cfg
from oracle import oracle as orc
from paper_2509_24007_amd import inputs as syn

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- sub-operations

def test_rmsnorm_constant_vector():
    # a constant vector c has mean square c^2, so RMSNorm gives g * c / sqrt(c^2 + eps)
    g = np.array([1.0, 2.0, -3.0, 0.5], dtype=np.float32)
    y = orc.probe_rmsnorm(np.full(4, 3.0), g, 1e-6)
    np.testing.assert_allclose(y, g.astype(np.float64) * 3.0 / math.sqrt(9.0 + 1e-6), rtol=1e-14)
    # 3-4-0-0: mean square 25/4
    y = orc.probe_rmsnorm(np.array([3.0, 4.0, 0.0, 0.0]), np.ones(4, np.float32), 0.0)
    np.testing.assert_allclose(y, np.array([3.0, 4.0, 0, 0]) / 2.5, rtol=1e-14)


def test_rope_closed_forms():
    rng = np.random.default_rng(1)
    v = rng.standard_normal(16)
    # position 0 is the identity
    np.testing.assert_array_equal(orc.probe_rope(v, 0, 1e4), v)
    # d = 2: a single plane rotated by `pos` radians, counter-clockwise
    r = orc.probe_rope(np.array([1.0, 0.0]), 3, 1e4)
    np.testing.assert_allclose(r, [math.cos(3.0), math.sin(3.0)], rtol=1e-14)
    # rotate-half pairing: element i pairs with i + d/2, frequency theta^(-2i/d)
    e = np.zeros(8)
    e[1] = 1.0
    r = orc.probe_rope(e, 5, 100.0)
    ang = 5.0 * 100.0 ** (-2.0 / 8.0)
    exp = np.zeros(8)
    exp[1], exp[5] = math.cos(ang), math.sin(ang)
    np.testing.assert_allclose(r, exp, atol=1e-15)
    # norms are preserved; the q.k product depends on the position difference only
    q, k = rng.standard_normal(16), rng.standard_normal(16)
    assert abs(np.linalg.norm(orc.probe_rope(q, 37, 1e4)) - np.linalg.norm(q)) < 1e-12
    a = orc.probe_rope(q, 40, 1e4) @ orc.probe_rope(k, 33, 1e4)
    b = orc.probe_rope(q, 107, 1e4) @ orc.probe_rope(k, 100, 1e4)
    assert abs(a - b) < 1e-10


def test_silu_values():
    assert orc.probe_silu(0.0) == 0.0
    assert abs(orc.probe_silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(orc.probe_silu(40.0) - 40.0) < 1e-12
    assert abs(orc.probe_silu(-40.0)) < 1e-12


def test_attention_probe_closed_forms():
    # zero query: uniform average of the values
    K = np.random.default_rng(0).standard_normal((5, 4))
    V = np.arange(20, dtype=np.float64).reshape(5, 4)
    np.testing.assert_allclose(orc.probe_attend(np.zeros(4), K, V), V.mean(0), rtol=1e-14)
    # two keys, scores differ by delta / sqrt(d): weights are a logistic of the scaled gap
    q = np.array([2.0, 0.0, 0.0, 0.0])
    K = np.array([[1.0, 0, 0, 0], [0.0, 0, 0, 0]])
    V = np.array([[1.0, 0, 0, 0], [0.0, 1, 0, 0]])
    p0 = 1.0 / (1.0 + math.exp(-2.0 / math.sqrt(4.0)))
    np.testing.assert_allclose(orc.probe_attend(q, K, V), [p0, 1 - p0, 0, 0], atol=1e-15)


# ---------------------------------------------------------------- confidence (Sec. 3.4 (1), (2))

def test_logit_confidence_closed_forms():
    V = 37
    assert abs(orc.conf_logit(np.full(V, 1.7)) - 1.0 / V) < 1e-15          # equal logits
    z = np.zeros(V)
    z[11] = 800.0
    assert orc.conf_logit(z) == 1.0 and orc.argmax(z) == 11                # one logit dominates
    assert abs(orc.conf_logit(np.array([0.3, 2.3])) - 1.0 / (1.0 + math.exp(-2.0))) < 1e-15
    # equals the softmax probability of the argmax token, computed by a library softmax
    z = np.random.default_rng(3).standard_normal(1000) * 4
    p = torch.softmax(torch.tensor(z), 0).numpy()
    assert abs(orc.conf_logit(z) - p.max()) < 1e-14 and orc.argmax(z) == int(p.argmax())
    # ties resolve to the lowest index
    assert orc.argmax(np.array([1.0, 5.0, 5.0, 2.0])) == 1


def test_entropy_confidence_closed_forms():
    V = 64
    assert abs(orc.conf_entropy(np.zeros(V))) < 1e-14                      # uniform: H = log V
    z = np.zeros(V)
    z[5] = 900.0
    assert abs(orc.conf_entropy(z) - 1.0) < 1e-14                          # one-hot: H = 0
    # two equally likely tokens among V: H = log 2
    z = np.full(V, -900.0)
    z[[3, 9]] = 0.0
    assert abs(orc.conf_entropy(z) - (1.0 - math.log(2) / math.log(V))) < 1e-14
    z = np.random.default_rng(4).standard_normal(V) * 3
    p = torch.softmax(torch.tensor(z), 0)
    H = float(torch.distributions.Categorical(probs=p).entropy())
    assert abs(orc.conf_entropy(z) - (1.0 - H / math.log(V))) < 1e-12


# ---------------------------------------------------------------- gamma_tau (Sec. 3.4, greedy decoding)

def test_gamma_hand_cases():
    # products 0.9, 0.81, 0.729, 0.6561
    c = [0.9, 0.9, 0.9, 0.9]
    assert orc.gamma(c, 0.95) == 1            # floor of 1 even though 0.9 < tau
    assert orc.gamma(c, 0.85) == 1
    assert orc.gamma(c, 0.80) == 2
    assert orc.gamma(c, 0.70) == 3
    assert orc.gamma(c, 0.60) == 4
    # a low first confidence blocks everything behind it
    assert orc.gamma([0.4, 1.0, 1.0, 1.0], 0.5) == 1
    assert orc.gamma([0.95, 0.5, 0.99, 0.99], 0.9) == 1
    # equality is accepted (>=): 0.5 * 0.5 = 0.25 exactly in binary
    assert orc.gamma([0.5, 0.5, 0.5], 0.25) == 2
    # per-position rule: every leading confidence >= tau
    assert orc.gamma(c, 0.85, rule=1) == 4
    assert orc.gamma([0.95, 0.5, 0.99, 0.99], 0.9, rule=1) == 1
    assert orc.gamma([0.3, 0.99], 0.9, rule=1) == 1


def test_gamma_properties():
    rng = np.random.default_rng(5)
    for _ in range(500):
        D = int(rng.integers(1, 9))
        conf = rng.uniform(0.0, 1.0, D).astype(np.float32) ** 0.3
        taus = np.sort(rng.uniform(0.0, 1.0, 6)).astype(np.float32)
        gs = [orc.gamma(conf, float(t)) for t in taus]
        assert all(1 <= g <= D for g in gs)                    # 1 <= gamma <= D (Sec. 3.2)
        assert all(a >= b for a, b in zip(gs, gs[1:]))         # non-increasing in tau
        assert orc.gamma(conf, 0.0) == D and orc.gamma(conf, -1.0) == D
        assert orc.gamma(conf, 1.5) == 1
        for t in taus:
            g0, g1 = orc.gamma(conf, float(t), 0), orc.gamma(conf, float(t), 1)
            assert g0 <= g1                                    # product rule is the stricter one
            # the accepted set is a prefix: gamma - 1 = number of j >= 2 passing, all of them leading
            cp = np.cumprod(conf, dtype=np.float32)
            passing = [j + 1 for j in range(D) if cp[j] >= t]
            assert g0 == max(passing + [1])


# ---------------------------------------------------------------- the mask (Sec. 3.3)

def test_block_mask_golden():
    # tests/golden/block_mask_n3_D3.txt was written by hand from the mask equation with block start s = n-1 = 2:
    # rows before s are causal, rows from s on see everything from s on as well.
    gold = np.loadtxt(os.path.join(GOLD, "block_mask_n3_D3.txt"), dtype=np.uint8, comments="#")
    np.testing.assert_array_equal(orc.block_mask(3, 3), gold)
    # D = 1 is the causal mask: next-token prediction (abstract; Sec. 3.3 first sentence)
    np.testing.assert_array_equal(orc.block_mask(6, 1), np.tril(np.ones((6, 6), np.uint8)))
    # n = 1: the whole sequence is the block, fully bidirectional
    np.testing.assert_array_equal(orc.block_mask(1, 4), np.ones((4, 4), np.uint8))


def _one_hot_model(T_tokens, n_layers=1):
    """A model whose forward can be done by counting.

    hidden = vocab = head_dim = Vv (one head).  embed = identity, wq = wk = 0 (all scores equal, so
    attention is the plain average of the visible values), wv = wo = identity, FFN = 0, lm_head = identity,
    logit_scale = 1, eps = 0.  Then for a row u holding token t_u, with vis(u) the visible rows,
        RMSNorm(e_t) = sqrt(Vv) e_t,   x_out[u] = e_{t_u} + sqrt(Vv) * mean_{v in vis(u)} e_{t_v},
        logits[u] = x_out[u] / rms(x_out[u]).
    """
    Vv = T_tokens
    eye = np.eye(Vv, dtype=np.float32)
    zero = np.zeros((Vv, Vv), dtype=np.float32)
    layer = dict(attn_norm=np.ones(Vv, np.float32), ffn_norm=np.ones(Vv, np.float32), wq=zero, wk=zero, wv=eye,
                 wo=eye, bq=None, bk=None, bv=None, w_gate=np.zeros((2, Vv), np.float32),
                 w_up=np.zeros((2, Vv), np.float32), w_down=np.zeros((Vv, 2), np.float32))
    g = dict(embed=eye, lm_head=eye, final_norm=np.ones(Vv, np.float32))
    return orc.Model(n_layers=n_layers, hidden=Vv, n_q_heads=1, n_kv_heads=1, head_dim=Vv, ffn=2, vocab=Vv,
                     rope_theta=1e4, rms_eps=0.0, logit_scale=1.0, mask_token_id=Vv - 1, has_qkv_bias=False,
                     globals_=g, layers=[layer] * n_layers)


def _counting_logits(ids, visible_sets, Vv):
    out = []
    for u, vis in enumerate(visible_sets):
        x = np.zeros(Vv)
        x[ids[u]] += 1.0
        for v in vis:
            x[ids[v]] += math.sqrt(Vv) / len(vis)
        out.append(x / math.sqrt(np.mean(x * x)))
    return np.array(out)


def test_counting_model_pins_visibility():
    """Hand-derivable micro model: logits reveal exactly which rows each row attended to."""
    Vv, D = 8, 3
    model = _one_hot_model(Vv)
    tokens = [2, 5, 0, 3]                      # n = 4 known tokens; mask id = 7
    n = len(tokens)
    ids = tokens + [7] * (D - 1)               # T = 6, block rows 3, 4, 5
    T, s = n + D - 1, n - 1
    vis = [list(range(u + 1)) if u < s else list(range(T)) for u in range(T)]
    want = _counting_logits(ids, vis, Vv)
    logits, out_ids, conf, gam = orc.brute_step(model, tokens, D, 0.5)
    np.testing.assert_allclose(logits, want[s:], rtol=1e-13, atol=1e-13)
    # a block row sees the masks to its right: its logit at the mask id (7) is non-zero for row s
    assert logits[0, 7] > 0.1
    # the same through the incremental route, prefix cached causally, block appended
    seq = orc.Seq(model, 16)
    seq.prefill(tokens)
    l2, ids2, conf2, g2 = seq.step(D, 0.5)
    np.testing.assert_allclose(l2, want[s:], rtol=1e-13, atol=1e-13)
    # prefix rows are strictly causal: read them through the general masked forward
    full = orc.forward_masked_logits(model, ids, orc.block_mask(n, D), 0, T)
    np.testing.assert_allclose(full, want, rtol=1e-13, atol=1e-13)


def test_block_rows_bidirectional_prefix_rows_causal():
    """'strict causality for u < i and full mutual attention for u, v >= i' (Sec. 3.3)."""
    m = small_cfg()
    g, layers = make_model(m, seed=3, std=0.3)
    model = oracle_model(m, g, layers)
    n, D = 7, 4
    toks = syn.uniform_int(1, "t", n, 0, m.vocab - 2).numpy()
    ids = np.concatenate([toks, np.full(D - 1, m.mask_token_id, np.int32)])
    T = n + D - 1
    mask = orc.block_mask(n, D)
    base = orc.forward_masked_logits(model, ids, mask, 0, T)
    for j in range(n, T):                      # perturb one in-block input token at a time
        ids2 = ids.copy()
        ids2[j] = (ids2[j] + 1 + j) % (m.vocab - 1)
        out = orc.forward_masked_logits(model, ids2, mask, 0, T)
        np.testing.assert_array_equal(out[:n - 1], base[:n - 1])          # prefix rows untouched
        for u in range(n - 1, T):                                          # every block row moves
            assert np.max(np.abs(out[u] - base[u])) > 1e-9


# ---------------------------------------------------------------- decoder forward vs library ops

def _torch_forward(m, g, layers, ids, mask_bool):
    """The same decoder written with torch library calls in float64 (sdpa, linear, silu, complex RoPE)."""
    F = torch.nn.functional
    dd = torch.float64
    T = len(ids)
    x = g["embed"].to(dd)[torch.as_tensor(ids, dtype=torch.long)]
    d, Hq, Hk = m.head_dim, m.n_q_heads, m.n_kv_heads
    pos = torch.arange(T, dtype=dd)
    inv = m.rope_theta ** (-torch.arange(0, d, 2, dtype=dd) / d)
    rot = torch.polar(torch.ones(T, d // 2, dtype=dd), pos[:, None] * inv[None, :])   # e^{i pos w}

    def rope(t):                                   # t: [T, H, d]; pairs (i, i + d/2) as complex numbers
        z = torch.complex(t[..., : d // 2], t[..., d // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    def norm(t, w):
        return t * torch.rsqrt(t.pow(2).mean(-1, keepdim=True) + m.rms_eps) * w.to(dd)

    for L in layers:
        xn = norm(x, L["attn_norm"])
        b = (lambda k: L[k].to(dd)) if m.has_qkv_bias else (lambda k: None)
        q = rope(F.linear(xn, L["wq"].to(dd), b("bq")).view(T, Hq, d))
        k = rope(F.linear(xn, L["wk"].to(dd), b("bk")).view(T, Hk, d))
        v = F.linear(xn, L["wv"].to(dd), b("bv")).view(T, Hk, d)
        k = k.repeat_interleave(Hq // Hk, dim=1)
        v = v.repeat_interleave(Hq // Hk, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           attn_mask=mask_bool[None, None])
        x = x + F.linear(a[0].transpose(0, 1).reshape(T, Hq * d), L["wo"].to(dd))
        xn = norm(x, L["ffn_norm"])
        x = x + F.linear(F.silu(F.linear(xn, L["w_gate"].to(dd))) * F.linear(xn, L["w_up"].to(dd)), L["w_down"].to(dd))
    return (m.logit_scale * F.linear(norm(x, g["final_norm"]), g["lm_head"].to(dd))).numpy()


@pytest.mark.parametrize("bias,dtype", [(True, "fp32"), (False, "fp32"), (True, "bf16")])
def test_forward_matches_library_decoder(bias, dtype):
    m = small_cfg(has_qkv_bias=bias, dtype=dtype, n_q_heads=6, n_kv_heads=2, hidden=48)
    g, layers = make_model(m, seed=7, std=0.25)
    model = oracle_model(m, g, layers)
    n, D = 9, 4
    ids = np.concatenate([syn.uniform_int(2, "t", n, 0, m.vocab - 1).numpy(), np.full(D - 1, m.mask_token_id)])
    mask = orc.block_mask(n, D)
    got = orc.forward_masked_logits(model, ids, mask, 0, len(ids))
    want = _torch_forward(m, g, layers, ids, torch.as_tensor(mask.astype(bool)))
    assert rel_err(got, want) < 1e-12
    # causal special case against the library's own causal flag
    causal = np.tril(np.ones((len(ids), len(ids)), np.uint8))
    got = orc.forward_masked_logits(model, ids, causal, 0, len(ids))
    want = _torch_forward(m, g, layers, ids, torch.as_tensor(causal.astype(bool)))
    assert rel_err(got, want) < 1e-12
    assert rel_err(orc.ntp_logits(model, ids), want[-1]) < 1e-12


def test_probes_match_forward_pieces():
    """Single-output probes agree with a library matmul on random data."""
    rng = np.random.default_rng(8)
    W = rng.standard_normal((7, 13)).astype(np.float32)
    b = rng.standard_normal(7).astype(np.float32)
    x = rng.standard_normal(13)
    for o in range(7):
        assert abs(orc.probe_linear(W, b, x, o) - (W[o].astype(np.float64) @ x + b[o])) < 1e-12
    Wb = torch.tensor(W).to(torch.bfloat16)
    Wb_np = Wb.view(torch.int16).numpy().view(np.uint16)
    assert abs(orc.probe_linear(Wb_np, None, x, 3) - (Wb.to(torch.float64).numpy()[3] @ x)) < 1e-12


def test_lm_head_probes_hand_case_and_scale():
    """The full-size LM-head reference (one logit, one row of logits): z_v = logit_scale * <xhat, W_lm[v]>
    (logits Z, Sec. 3.2; the scale is a configuration constant of the synthetic workloads).  Hand case: a one-hot
    xhat picks one column of W_lm; the scale multiplies it; rows and columns of W_lm are not interchangeable
    (V != h)."""
    m = small_cfg(vocab=11, hidden=8, ffn=16, n_q_heads=2, n_kv_heads=1, head_dim=4, logit_scale=3.0)
    g, layers = make_model(m, seed=5, std=0.5)
    model = oracle_model(m, g, layers)
    W = g["lm_head"].numpy().astype(np.float64)               # [V, h]
    for k in (0, 5, 7):
        e = np.zeros(m.hidden)
        e[k] = 1.0
        row = orc.probe_logits_row(model, e)
        np.testing.assert_allclose(row, 3.0 * W[:, k], rtol=1e-14)
        for v in (0, 4, 10):
            assert abs(orc.probe_logit(model, e, v) - 3.0 * W[v, k]) < 1e-14
    # linear in xhat; the scale is applied once
    x = np.random.default_rng(3).standard_normal(m.hidden)
    row = orc.probe_logits_row(model, x)
    np.testing.assert_allclose(row, 3.0 * (W @ x), rtol=1e-13)
    np.testing.assert_allclose([orc.probe_logit(model, x, v) for v in range(m.vocab)], row, rtol=1e-13)
    m1 = small_cfg(vocab=11, hidden=8, ffn=16, n_q_heads=2, n_kv_heads=1, head_dim=4, logit_scale=1.0)
    np.testing.assert_allclose(orc.probe_logits_row(oracle_model(m1, g, layers), x) * 3.0, row, rtol=1e-13)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_lm_head_probes_match_the_forward(dtype):
    """With zero output and down projections the residual stream that reaches the final norm is the embedding of
    the row's token, so the forward's logits (pinned above to the library decoder) must equal the probe applied to
    the normalised embedding, the normalisation written out here from its definition."""
    m = small_cfg(dtype=dtype, vocab=53, hidden=24, n_q_heads=4, n_kv_heads=2, head_dim=6, ffn=40, logit_scale=8.0)
    g, layers = make_model(m, seed=11, std=0.3)
    for L in layers:
        L["wo"] = torch.zeros_like(L["wo"])
        L["w_down"] = torch.zeros_like(L["w_down"])
    model = oracle_model(m, g, layers)
    ids = syn.uniform_int(4, "t", 6, 0, m.vocab - 1).numpy()
    causal = np.tril(np.ones((6, 6), np.uint8))
    Z = orc.forward_masked_logits(model, ids, causal, 0, 6)
    E = g["embed"].to(torch.float64).numpy()
    for r in range(6):
        x = E[ids[r]]
        xhat = x / math.sqrt(float(np.mean(x * x)) + m.rms_eps) * g["final_norm"].to(torch.float64).numpy()
        assert rel_err(orc.probe_logits_row(model, xhat), Z[r]) < 1e-13
        for v in (0, 17, 52):
            assert abs(orc.probe_logit(model, xhat, v) - Z[r, v]) <= 1e-12 * np.max(np.abs(Z[r]))
