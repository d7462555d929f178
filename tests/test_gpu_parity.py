"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI."""
import json
import os

import numpy as np
import pytest
import torch

from gpu_common import both_models, gpu_context, lockstep
from helpers import small_cfg
from oracle import oracle as orc
from paper_2509_24007_amd import inputs as syn

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def gpu_cfg(**kw):
    base = dict(hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=112, vocab=300)
    base.update(kw)
    return small_cfg(**base)


def test_c1_tiny_fp32_free_running():
    """configs[0]: 32 free-running steps, ids and gamma bit-exact against the stored oracle trajectory."""
    wl = syn.workloads()["C1"]
    m, r = wl.model, wl.run
    om, g_dev, layers_dev = both_models(m, wl.seed, 0.02)
    prompt = syn.make_prompts(wl.seed, 1, r.prompt_lo, r.prompt_hi, m.vocab)[0].numpy()
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=1, max_seq_len=64 + r.steps * r.block_D + r.block_D, D=r.block_D, tau=r.tau)
    assert ctx.kernel_info == "generic-fp32"
    st, seqs = lockstep(ctx, om, [prompt], r.block_D, r.tau, r.steps, logit_tol=1e-4, conf_tol=1e-5)
    print("C1", st)
    gold = json.load(open(os.path.join(GOLD, "c1_trajectory.json")))
    assert [int(t) for t in seqs[0].tokens] == gold["final_tokens"]
    assert st.id_near_tie == 0 and st.gamma_near_tie == 0
    ctx.close()


@pytest.mark.parametrize("D,tau,paged", [(1, 0.5, False), (2, 0.9, True), (4, 0.8, False), (4, 0.8, True), (8, 0.6, True), (16, 0.3, False)])
def test_small_fp32_ragged_batch(D, tau, paged):
    """Ragged batch, several block sizes, both cache layouts, override and own commits alternating."""
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=5, std=0.3)
    lens = [1, 2, 15, 16, 17, 33, 40]
    prompts = [syn.uniform_int(D, f"p{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 7
    ovr = syn.make_overrides(9, steps, len(lens), D, m.vocab)
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max_len, D=D, tau=tau, paged=paged, n_pages=n_pages,
                      prefill_rows=64)
    st, _ = lockstep(ctx, om, prompts, D, tau, steps, logit_tol=1e-4, conf_tol=1e-5, overrides=ovr, max_len=max_len)
    print(f"D={D} paged={paged}", st)
    if D >= 4:
        assert max(st.gammas) > 1
    ctx.close()


@pytest.mark.parametrize("conf_fn,rule", [(1, 0), (0, 1), (1, 1)])
def test_confidence_and_rule_variants(conf_fn, rule):
    m = gpu_cfg(has_qkv_bias=False, n_q_heads=6, n_kv_heads=2, hidden=96, head_dim=64)
    om, g_dev, layers_dev = both_models(m, seed=6, std=0.3)
    prompts = [syn.uniform_int(3, f"q{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate([5, 9, 30])]
    tau = 0.02 if conf_fn == 1 else 0.2
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=3, max_seq_len=80, D=4, tau=tau, conf_fn=conf_fn, accept_rule=rule)
    st, _ = lockstep(ctx, om, prompts, 4, tau, 5, logit_tol=1e-4, conf_tol=1e-5, conf_fn=conf_fn, rule=rule)
    print(st)
    ctx.close()


def test_small_bf16_generic_kernels():
    """bf16 storage through the shape-generic kernels (head_dim 64 is not served by the matrix-core path)."""
    m = gpu_cfg(dtype="bf16", head_dim=64, hidden=128, n_q_heads=4, n_kv_heads=2)
    om, g_dev, layers_dev = both_models(m, seed=7, std=0.08)
    prompts = [syn.uniform_int(4, f"b{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate([3, 20, 37])]
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=3, max_seq_len=80, D=4, tau=0.1, paged=True, n_pages=20)
    st, _ = lockstep(ctx, om, prompts, 4, 0.1, 6, logit_tol=2e-2, conf_tol=2e-2, bf16=True)
    print(st)
    ctx.close()


def test_step_is_repeatable_and_batch_independent():
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=8, std=0.3)
    prompts = [syn.uniform_int(5, f"r{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate([7, 21, 12])]
    D, V = 4, m.vocab
    outs = []
    for sel in ([0, 1, 2], [1], [2, 0]):
        ctx = gpu_context(m, g_dev, layers_dev, max_batch=3, max_seq_len=64, D=D, tau=0.05)
        ctx.prefill([prompts[i] for i in sel])
        B = len(sel)
        ids = torch.empty(B, D, dtype=torch.int32, device="cuda")
        cnt = torch.empty(B, dtype=torch.int32, device="cuda")
        logits = torch.empty(B * D, V, dtype=torch.float32, device="cuda")
        res = {}
        for t in range(3):
            ctx.decode_step(ids, cnt, None, logits)
            torch.cuda.synchronize()
            first = logits.clone()
            ctx.decode_step(ids, cnt, None, logits)          # repeated before commit: identical
            torch.cuda.synchronize()
            assert torch.equal(first, logits)
            for j, i in enumerate(sel):
                res[(i, t)] = logits.view(B, D, V)[j].cpu().clone()
            ctx.kv_commit()
        outs.append(res)
        ctx.close()
    for res in outs[1:]:
        for key, val in res.items():
            assert torch.equal(val, outs[0][key]), f"sequence {key[0]} step {key[1]} depends on its batch mates"


def test_cache_contents_match_oracle_cache():
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=10, std=0.3)
    prompts = [syn.uniform_int(6, f"k{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate([18, 5])]
    D = 4
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=64, D=D, tau=0.05, paged=True, n_pages=12)
    st, seqs = lockstep(ctx, om, prompts, D, 0.05, 4, logit_tol=1e-4, conf_tol=1e-5)
    for b, s in enumerate(seqs):
        for layer in range(m.n_layers):
            for hk in range(m.n_kv_heads):
                k, v = ctx.read_kv(layer, b, hk, 0, s.c)
                for pos in range(s.c):
                    ko, vo = s.read_kv(layer, pos, hk)
                    assert np.max(np.abs(k[pos].numpy() - ko)) < 1e-4 * max(1.0, np.max(np.abs(ko)))
                    assert np.max(np.abs(v[pos].numpy() - vo)) < 1e-4 * max(1.0, np.max(np.abs(vo)))
    ctx.close()


def test_error_paths():
    from paper_2509_24007_amd import sdlm
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=11, std=0.3)
    with pytest.raises(sdlm.SdlmError) as e:
        gpu_context(m, g_dev, layers_dev, max_batch=1, max_seq_len=32, D=17, tau=0.5)
    assert e.value.code == sdlm.EINVAL
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=24, D=4, tau=0.5)
    ids = torch.empty(2, 4, dtype=torch.int32, device="cuda")
    cnt = torch.empty(2, dtype=torch.int32, device="cuda")
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.decode_step(ids, cnt)
    assert e.value.code == sdlm.ESTATE
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.prefill([[1, 2, 3], []])
    assert e.value.code == sdlm.EINVAL
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.prefill([list(range(21))])                      # 21 + D > 24
    assert e.value.code == sdlm.ECAPACITY
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.prefill([[1, 2, m.vocab]])
    assert e.value.code == sdlm.EINVAL
    ctx.prefill([[1, 2, 3], [4, 5]])
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.kv_commit()
    assert e.value.code == sdlm.ESTATE
    four = torch.full((2,), 4, dtype=torch.int32, device="cuda")
    toks = torch.ones(2, 4, dtype=torch.int32, device="cuda")
    with pytest.raises(sdlm.SdlmError) as e:
        for _ in range(8):                                  # 3 + 4k tokens: capacity trips before any overflow
            ctx.decode_step(ids, cnt)
            ctx.kv_commit(toks, four)
    assert e.value.code == sdlm.ECAPACITY
    n, c = ctx.get_lengths()
    assert int(n.max()) + 4 > 24 and int(n.max()) <= 24
    # a clamped override count is reported
    ctx.prefill([[1, 2, 3]])
    ctx.decode_step(ids, cnt)
    ctx.kv_commit(toks, torch.full((2,), 9, dtype=torch.int32, device="cuda"))
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.get_lengths()
    assert e.value.code == sdlm.EINVAL
    # an override token outside the vocabulary is replaced and reported
    ctx.prefill([[1, 2, 3]])
    ctx.decode_step(ids, cnt)
    bad = torch.full((2, 4), m.vocab + 5, dtype=torch.int32, device="cuda")
    ctx.kv_commit(bad, torch.ones(2, dtype=torch.int32, device="cuda"))
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.get_lengths()
    assert e.value.code == sdlm.EINVAL
    ctx.decode_step(ids, cnt)                               # and the next step still runs on valid rows
    torch.cuda.synchronize()
    ctx.close()
    # paged pool too small for the prompts
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=64, D=4, tau=0.5, paged=True, n_pages=2)
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.prefill([list(range(20)), list(range(20))])
    assert e.value.code == sdlm.ECAPACITY
    ctx.prefill([list(range(14)), list(range(14))])
    with pytest.raises(sdlm.SdlmError) as e:
        for _ in range(4):
            ctx.decode_step(ids, cnt)
            ctx.kv_commit(toks, four)
    assert e.value.code == sdlm.ECAPACITY
    ctx.close()


@pytest.mark.parametrize("paged", [False, True])
def test_commit_at_the_capacity_edge(paged):
    """A step is admitted only if accepting all D tokens still fits (n + D <= max_seq_len), so a commit can never run
    out of positions or page-table entries on the device: with max_seq_len a multiple of the page size, a sequence
    that fills up exactly keeps every accepted token, reports no error, and the next step is refused on the host."""
    from paper_2509_24007_amd import sdlm
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=13, std=0.3)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=64, D=4, tau=0.5, paged=paged, n_pages=8 if paged else 0)
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.prefill([list(range(61)), [1, 2]])              # 61 + 4 > 64: all four tokens could not be kept
    assert e.value.code == sdlm.ECAPACITY
    prompts = [syn.uniform_int(13, "edge", 60, 0, m.vocab - 1).numpy(), np.array([3, 4], np.int32)]
    seqs = [orc.Seq(om, 64) for _ in prompts]
    for s, p in zip(seqs, prompts):
        s.prefill(p)
    ctx.prefill(prompts)
    ids = torch.empty(2, 4, dtype=torch.int32, device="cuda")
    cnt = torch.empty(2, dtype=torch.int32, device="cuda")
    logits = torch.empty(8, m.vocab, dtype=torch.float32, device="cuda")
    ctx.decode_step(ids, cnt, None, logits)
    toks = torch.tensor([[5, 6, 7, 8], [9, 10, 11, 12]], dtype=torch.int32, device="cuda")
    ctx.kv_commit(toks, torch.tensor([4, 1], dtype=torch.int32, device="cuda"))
    n, c = ctx.get_lengths()                                # no device-side error flag
    assert n.tolist() == [64, 3] and c.tolist() == [60, 2]
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.decode_step(ids, cnt)                           # 64 + 4 > 64
    assert e.value.code == sdlm.ECAPACITY
    ctx.close()
    # the same two sequences with room for one more step: the four committed tokens are really there (the step after
    # the commit matches the oracle, which was fed the same tokens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=80, D=4, tau=0.5, paged=paged, n_pages=10 if paged else 0)
    seqs = [orc.Seq(om, 80) for _ in prompts]
    for s, p in zip(seqs, prompts):
        s.prefill(p)
    ctx.prefill(prompts)
    ctx.decode_step(ids, cnt)
    for s in seqs:
        s.step(4, 0.5)
    ctx.kv_commit(toks, torch.tensor([4, 1], dtype=torch.int32, device="cuda"))
    assert seqs[0].commit([5, 6, 7, 8], 4) == 0 and seqs[1].commit([9], 1) == 0
    ctx.decode_step(ids, cnt, None, logits)
    torch.cuda.synchronize()
    z = logits.cpu().numpy().reshape(2, 4, -1)
    for b in range(2):
        lo, io, _, _ = seqs[b].step(4, 0.5)
        assert np.max(np.abs(z[b] - lo)) <= 1e-4 * np.max(np.abs(lo))
    ctx.close()


@pytest.mark.parametrize("dtype,hd", [("fp32", 32), ("bf16", 128)])
def test_nan_logits_still_give_valid_ids(dtype, hd):
    """Non-finite weights must not turn into out-of-range token ids (they would index the embedding table)."""
    m = gpu_cfg(dtype=dtype, head_dim=hd, hidden=128, ffn=128, n_q_heads=2, n_kv_heads=1) if dtype == "fp32" else mfma_cfg()
    om, g_dev, layers_dev = both_models(m, seed=12, std=0.05)
    g_dev = dict(g_dev)
    g_dev["lm_head"] = torch.full_like(g_dev["lm_head"], float("nan"))
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=64, D=4, tau=0.5)
    ctx.prefill([[1, 2, 3], [4]])
    ids = torch.empty(2, 4, dtype=torch.int32, device="cuda")
    cnt = torch.empty(2, dtype=torch.int32, device="cuda")
    for _ in range(3):
        ctx.decode_step(ids, cnt)
        ctx.kv_commit()
    torch.cuda.synchronize()
    assert int(ids.min()) >= 0 and int(ids.max()) < m.vocab
    assert int(cnt.min()) >= 1 and int(cnt.max()) <= 4
    ctx.close()


def test_generator_is_identical_on_cpu_and_gpu():
    a = syn.normal(3, "dev", (1000, 33), 0.02, torch.bfloat16, "cpu")
    b = syn.normal(3, "dev", (1000, 33), 0.02, torch.bfloat16, "cuda")
    assert torch.equal(a, b.cpu())
    assert torch.equal(syn.uniform_int(3, "u", 5000, 0, 151935), syn.uniform_int(3, "u", 5000, 0, 151935, device="cuda").cpu())


# ------------------------------------------------------------------ bf16 matrix-core path (head_dim 128)

def mfma_cfg(**kw):
    base = dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, ffn=512, vocab=2048, dtype="bf16",
                rope_theta=1.0e6, has_qkv_bias=True)
    base.update(kw)
    return syn.ModelCfg(**base)


@pytest.mark.parametrize("name,kw,lens,D,tau,paged", [
    ("g2", {}, [1, 9, 40, 100], 4, 0.6, True),
    ("g7-ragged-vocab", dict(n_q_heads=14, n_kv_heads=2, vocab=1000, ffn=320), [3, 17, 33, 64, 70], 4, 0.6, True),
    ("g8-D8-two-groups", dict(n_q_heads=16, n_kv_heads=2, hidden=512), [5, 130, 300], 8, 0.5, False),
    ("g6-D4-batch1-long", dict(n_q_heads=12, n_kv_heads=2, hidden=384, ffn=1024), [700], 4, 0.6, False),
    ("g4-batch20-128-row-tiles", dict(n_q_heads=8, n_kv_heads=2, vocab=4096 + 160), [3 + 7 * i for i in range(20)], 4, 0.6, True),
    ("g5-D16", dict(n_q_heads=10, n_kv_heads=2, hidden=320, ffn=640, has_qkv_bias=False), [2, 50], 16, 0.3, True),
    ("g4-batch36-192-row-gate-up-tile", dict(n_q_heads=8, n_kv_heads=2, hidden=256, ffn=24576), [3 + 2 * i for i in range(36)], 4, 0.6, True),
])
def test_bf16_mfma_path(name, kw, lens, D, tau, paged):
    """The bf16 product path: MFMA GEMMs, MFMA block-masked attention (split KV), fused LM-head reduction."""
    m = mfma_cfg(**kw)
    om, g_dev, layers_dev = both_models(m, seed=21, std=0.05)
    prompts = [syn.uniform_int(D, f"{name}{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 6
    ovr = syn.make_overrides(13, steps, len(lens), D, m.vocab)
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max_len, D=D, tau=tau, paged=paged, n_pages=n_pages,
                      prefill_rows=128)
    assert ctx.kernel_info == "mfma-bf16"
    st, _ = lockstep(ctx, om, prompts, D, tau, steps, logit_tol=2e-2, conf_tol=1e-3, overrides=ovr, bf16=True, max_len=max_len)
    print(name, st)
    ctx.close()


def test_bf16_mfma_entropy_confidence():
    m = mfma_cfg()
    om, g_dev, layers_dev = both_models(m, seed=22, std=0.05)
    prompts = [syn.uniform_int(1, f"e{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate([12, 31])]
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=80, D=4, tau=0.05, conf_fn=1)
    st, _ = lockstep(ctx, om, prompts, 4, 0.05, 4, logit_tol=2e-2, conf_tol=1e-3, conf_fn=1, bf16=True)
    print(st)
    ctx.close()


# ------------------------------------------------------------------ self-speculative verification (Sec. 3.4, Eq. 10)
@pytest.mark.parametrize("D,rule,paged", [(2, 0, False), (3, 1, True), (4, 0, True), (4, 1, False), (5, 0, False), (6, 0, True), (8, 0, False),
                                          (9, 1, False), (10, 0, True), (12, 1, False), (16, 0, True)])
def test_verify_small_fp32(D, rule, paged):
    """Second pass of a self-speculative step against the oracle's: logits of every verification input, ytilde,
    gamma_verify bit-exact, and the verified count is what an argument-less commit publishes.  The causal rows of the
    speculative tokens are computed once per sequence; D <= 4: all rows of a sequence share one staging tile, D >= 5: the
    causal rows and every input's block have tiles of their own and a block row reads two of them."""
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=6, std=0.3)
    lens = [1, 2, 15, 16, 17, 33]
    prompts = [syn.uniform_int(D, f"v{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 5
    ovr = syn.make_overrides(10, steps, len(lens), D, m.vocab)
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max_len, D=D, tau=0.5, paged=paged, n_pages=n_pages,
                      prefill_rows=64)
    st, _ = lockstep(ctx, om, prompts, D, 0.5, steps, logit_tol=1e-4, conf_tol=1e-5, overrides=ovr, max_len=max_len,
                     verify_rule=rule)
    print(f"verify D={D} rule={rule}", st, "verify rows", st.verify_rows, "gammas", np.bincount(st.verify_gammas))
    assert st.verify_rows == steps * len(lens) * (D - 1) and st.verify_skipped == 0 and st.verify_near_tie == 0
    ctx.close()


@pytest.mark.parametrize("paged,prefill_rows", [(True, 256), (False, 4096)])
def test_long_prefill_cache_matches_oracle_cache_bf16(paged, prefill_rows):
    """Prefill of long prompts on the matrix-core path (several passes when prefill_rows is below the prompt length,
    several KV chunks per attention work item, ragged last groups): every cached K and V vector of every layer, kv head
    and position against the oracle's cache, which by its pins holds the K/V of the real tokens under causal attention
    (Sec. 3.3: every block sees the real tokens before it causally).  The layers' inputs differ by bf16 rounding, so
    the comparison is per vector, relative to the vector's largest entry."""
    m = mfma_cfg(n_layers=3, n_q_heads=14, n_kv_heads=2, hidden=256, ffn=512)
    om, g_dev, layers_dev = both_models(m, seed=31, std=0.05)
    lens = [700, 1, 333, 1025]
    prompts = [syn.uniform_int(31, f"lp{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    D = 4
    n_pages = sum((n + 2 * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max(lens) + 2 * D, D=D, tau=0.5, paged=paged,
                      n_pages=n_pages if paged else 0, prefill_rows=prefill_rows)
    assert ctx.kernel_info == "mfma-bf16"
    ctx.prefill(prompts)
    n, c = ctx.get_lengths()
    assert n.tolist() == lens and c.tolist() == lens
    worst_k = worst_v = 0.0
    for b, p in enumerate(prompts):
        s = orc.Seq(om, len(p) + 2 * D)
        s.prefill(p)
        for layer in range(m.n_layers):
            for hk in range(m.n_kv_heads):
                k, v = ctx.read_kv(layer, b, hk, 0, len(p))
                k, v = k.numpy().astype(np.float64), v.numpy().astype(np.float64)
                for pos in range(len(p)):
                    ko, vo = s.read_kv(layer, pos, hk)
                    worst_k = max(worst_k, float(np.max(np.abs(k[pos] - ko)) / np.max(np.abs(ko))))
                    worst_v = max(worst_v, float(np.max(np.abs(v[pos] - vo)) / np.max(np.abs(vo))))
    print(f"long prefill paged={paged} rows/pass={prefill_rows}: worst relative K error {worst_k:.3e}, V {worst_v:.3e}")
    assert worst_k <= 2e-2 and worst_v <= 2e-2
    ctx.close()


@pytest.mark.parametrize("name,lens", [
    ("small-step", [9, 33]),                                   # at most 32 rows per step: QKV, RoPE and K/V placement are one launch
    ("larger-step", [3 + 5 * i for i in range(9)]),            # 72 rows: projection, then the RoPE + K/V placement kernel
])
def test_decode_cache_matches_oracle_cache_bf16(name, lens):
    """K/V written by decode steps on the matrix-core path: after several steps with forced acceptance counts, every cached K
    and V vector (prompt positions and the positions of the committed tokens, whose K/V came from the pending rows of
    later steps) against the oracle's clean cache (Sec. 3.3: only real tokens under causal attention are ever cached).
    Both QKV paths are covered: the fused launch of small steps and the separate kernels of larger ones."""
    m = mfma_cfg(n_q_heads=6, n_kv_heads=2, hidden=256, ffn=512)
    om, g_dev, layers_dev = both_models(m, seed=41, std=0.05)
    D, steps = 4, 5
    prompts = [syn.uniform_int(41, f"dc{name}{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    ovr = syn.make_overrides(17, steps, len(lens), D, m.vocab)   # forced tokens and counts on some steps: pending runs of every length
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max(lens) + (steps + 2) * D, D=D, tau=0.5, paged=True,
                      n_pages=sum((n + (steps + 2) * D + 15) // 16 + 1 for n in lens))
    assert ctx.kernel_info == "mfma-bf16"
    st, seqs = lockstep(ctx, om, prompts, D, 0.5, steps, logit_tol=2e-2, conf_tol=1e-5, overrides=ovr, bf16=True)
    worst_k = worst_v = 0.0
    grown = 0
    for b, s in enumerate(seqs):
        grown += s.c - len(prompts[b])
        for layer in range(m.n_layers):
            for hk in range(m.n_kv_heads):
                k, v = ctx.read_kv(layer, b, hk, 0, s.c)
                k, v = k.numpy().astype(np.float64), v.numpy().astype(np.float64)
                for pos in range(s.c):
                    ko, vo = s.read_kv(layer, pos, hk)
                    worst_k = max(worst_k, float(np.max(np.abs(k[pos] - ko)) / np.max(np.abs(ko))))
                    worst_v = max(worst_v, float(np.max(np.abs(v[pos] - vo)) / np.max(np.abs(vo))))
    print(f"decode cache {name}: {grown} positions written by pending rows, worst relative K error {worst_k:.3e}, V {worst_v:.3e}")
    assert grown >= steps * len(lens) - len(lens)   # every step but the last one's commit has left its tokens in the cache
    assert worst_k <= 2e-2 and worst_v <= 2e-2
    ctx.close()


def test_verify_position_independent_model_accepts_whole_block():
    """All-zero weights: every logit row is constant, arg-max is token 0 everywhere, so every position verifies."""
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=6, std=0.0)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=64, D=4, tau=2.0)
    ctx.prefill([np.array([4, 2, 7], dtype=np.int32), np.array([1], dtype=np.int32)])
    ids = torch.empty(2, 4, dtype=torch.int32, device="cuda")
    cnt = torch.empty(2, dtype=torch.int32, device="cuda")
    vid = torch.empty(2, 4, dtype=torch.int32, device="cuda")
    vc = torch.empty(2, dtype=torch.int32, device="cuda")
    ctx.decode_step(ids, cnt)
    ctx.verify_step(0, vid, vc)
    torch.cuda.synchronize()
    assert cnt.tolist() == [1, 1] and vc.tolist() == [4, 4]
    assert ids.cpu().eq(0).all() and vid.cpu().eq(0).all()
    ctx.kv_commit()
    n, c = ctx.get_lengths()
    assert n.tolist() == [3 + 4, 1 + 4]
    ctx.close()


def test_phase_timers_count_launches_and_sample():
    """The per-phase event timers report one launch per layer and step for a per-layer phase, every n-th of them when
    sampling, and the sampled steps produce the same tokens as the untimed ones."""
    m = mfma_cfg(n_layers=3)
    om, g_dev, layers_dev = both_models(m, seed=8, std=0.05)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=64, D=4, tau=0.5)
    prompts = [np.array([1, 2, 3], dtype=np.int32), np.array([4, 5], dtype=np.int32)]
    ids = torch.empty(3, 2, 4, dtype=torch.int32, device="cuda")
    cnt = torch.empty(3, 2, dtype=torch.int32, device="cuda")
    from paper_2509_24007_amd.sdlm import SdlmError
    for mode, (every, steps) in enumerate([(1, 2), (2, 3), (7, 2)]):
        ctx.prefill(prompts)
        ctx.profile(["gateup", "lmhead"], every=every)
        for _ in range(steps):
            ctx.decode_step(ids[mode], cnt[mode])
        got = ctx.profile_read()
        ctx.profile(None)
        assert got["gateup"][1] == -(-3 * steps // every) and got["lmhead"][1] == -(-steps // every)
        assert got["gateup"][0] > 0.0 and got["qkv"] == (0.0, 0)
    torch.cuda.synchronize()
    assert ids[0].eq(ids[1]).all() and ids[0].eq(ids[2]).all() and cnt[0].eq(cnt[1]).all() and cnt[0].eq(cnt[2]).all()
    with pytest.raises(SdlmError):
        ctx.profile(["gateup"], every=0)
    ctx.close()


def test_verify_error_paths():
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=6, std=0.3)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=1, max_seq_len=64, D=4, tau=0.5)
    ctx.prefill([np.array([1, 2, 3], dtype=np.int32)])
    from paper_2509_24007_amd.sdlm import SdlmError
    with pytest.raises(SdlmError):
        ctx.verify_step(0)              # no step yet
    ids = torch.empty(1, 4, dtype=torch.int32, device="cuda")
    cnt = torch.empty(1, dtype=torch.int32, device="cuda")
    ctx.decode_step(ids, cnt)
    with pytest.raises(SdlmError):
        ctx.verify_step(2)              # unknown rule
    ctx.verify_step(0)
    ctx.verify_step(1)                  # may be repeated before the commit
    ctx.kv_commit()
    with pytest.raises(SdlmError):
        ctx.verify_step(0)              # the step has been committed
    ctx.close()


@pytest.mark.parametrize("name,kw,lens,D", [
    ("vg2", {}, [1, 9, 40, 100], 4),
    ("vg7", dict(n_q_heads=14, n_kv_heads=2, vocab=1000, ffn=320), [3, 17, 33, 64, 70], 4),
    ("vg8-D8-two-groups-per-input", dict(n_q_heads=16, n_kv_heads=2, hidden=512), [5, 130, 300], 8),
    ("vg16-four-groups-across-inputs", dict(n_q_heads=16, n_kv_heads=1, hidden=256), [2, 31, 90], 4),
    ("vg4-D3", dict(n_q_heads=8, n_kv_heads=2), [7, 16, 49], 3),
    ("vg3-D5-two-staging-tiles", dict(n_q_heads=6, n_kv_heads=2), [4, 40], 5),
    ("vg7-D9", dict(n_q_heads=14, n_kv_heads=2, vocab=1000, ffn=320), [3, 70], 9),
    ("vg4-D16", dict(n_q_heads=8, n_kv_heads=2), [1, 33, 200], 16),
])
def test_verify_bf16_mfma(name, kw, lens, D):
    m = mfma_cfg(**kw)
    om, g_dev, layers_dev = both_models(m, seed=21, std=0.05)
    prompts = [syn.uniform_int(D, f"{name}{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 4
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max_len, D=D, tau=0.6, paged=True, n_pages=n_pages,
                      prefill_rows=128)
    assert ctx.kernel_info == "mfma-bf16"
    st, _ = lockstep(ctx, om, prompts, D, 0.6, steps, logit_tol=2e-2, conf_tol=1e-3, bf16=True, max_len=max_len, verify_rule=0)
    print(name, st, "verify rows", st.verify_rows, "skipped", st.verify_skipped, "near ties", st.verify_near_tie)
    assert st.verify_rows > 0
    ctx.close()


# ------------------------------------------------------------------ causal attention inside the block (Sec. 4.4 ablation)
@pytest.mark.parametrize("D,paged,verify", [(4, False, None), (8, True, None), (4, True, 0)])
def test_block_causal_small_fp32(D, paged, verify):
    m = gpu_cfg(block_causal=True)
    om, g_dev, layers_dev = both_models(m, seed=7, std=0.3)
    assert om.cfg.block_causal == 1
    lens = [1, 5, 16, 31]
    prompts = [syn.uniform_int(D, f"bc{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 5
    ovr = syn.make_overrides(11, steps, len(lens), D, m.vocab)
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max_len, D=D, tau=0.6, paged=paged, n_pages=n_pages,
                      prefill_rows=64)
    st, _ = lockstep(ctx, om, prompts, D, 0.6, steps, logit_tol=1e-4, conf_tol=1e-5, overrides=ovr, max_len=max_len,
                     verify_rule=verify)
    print(f"block-causal D={D}", st)
    assert st.id_near_tie == 0
    ctx.close()


def test_block_causal_bf16_mfma():
    m = mfma_cfg(block_causal=True)
    om, g_dev, layers_dev = both_models(m, seed=21, std=0.05)
    lens = [1, 9, 40, 100]
    prompts = [syn.uniform_int(4, f"bcm{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 4
    max_len = max(lens) + steps * 4 + 4
    n_pages = sum((n + steps * 4 + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max_len, D=4, tau=0.6, paged=True, n_pages=n_pages,
                      prefill_rows=128)
    assert ctx.kernel_info == "mfma-bf16"
    st, _ = lockstep(ctx, om, prompts, 4, 0.6, steps, logit_tol=2e-2, conf_tol=1e-3, bf16=True, max_len=max_len, verify_rule=0)
    print("block-causal mfma", st)
    ctx.close()


# ------------------------------------------------------------------ HIP-graph replay of the step
@pytest.mark.parametrize("kind", ["fp32", "mfma"])
def test_graph_replay_matches_oracle_and_eager(kind):
    """Every replay is checked against the oracle, with the library's eager commit kernels (own and override) and host
    synchronisations between replays; then a replayed and an eager context are compared bit for bit."""
    if kind == "fp32":
        m, std, tol, ctol, bf = gpu_cfg(), 0.3, 1e-4, 1e-5, False
    else:
        m, std, tol, ctol, bf = mfma_cfg(), 0.05, 2e-2, 1e-3, True
    om, g_dev, layers_dev = both_models(m, seed=8, std=std)
    lens = [1, 7, 16, 33, 40]
    D, tau, steps = 4, 0.6, 8
    prompts = [syn.uniform_int(3, f"gr{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    ovr = syn.make_overrides(12, steps, len(lens), D, m.vocab)
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    side = torch.cuda.Stream()
    kw = dict(max_batch=len(lens), max_seq_len=max_len, D=D, tau=tau, paged=True, n_pages=n_pages, prefill_rows=64)
    ctx = gpu_context(m, g_dev, layers_dev, stream=side, **kw)
    ctx.graph(True)
    st, _ = lockstep(ctx, om, prompts, D, tau, steps, logit_tol=tol, conf_tol=ctol, overrides=ovr, bf16=bf, max_len=max_len)
    print("graph", kind, st)
    # replayed vs eager, same inputs, fresh contexts: identical bits
    outs = []
    for use_graph in (True, False):
        c2 = gpu_context(m, g_dev, layers_dev, stream=side, **kw)
        if use_graph:
            c2.graph(True)
        c2.prefill(prompts)
        ids = torch.empty(steps, len(lens), D, dtype=torch.int32, device="cuda")
        cnt = torch.empty(steps, len(lens), dtype=torch.int32, device="cuda")
        conf = torch.empty(len(lens), D, dtype=torch.float32, device="cuda")
        logits = torch.empty(len(lens) * D, m.vocab, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        trace = []
        for t in range(steps):
            c2.decode_step(ids[t], cnt[t], conf, logits) if t % 3 else c2.decode_step(ids[t], cnt[t])   # the outputs change: re-capture
            torch.cuda.synchronize()
            trace.append((conf.clone(), logits.clone()) if t % 3 else None)
            c2.kv_commit()
        torch.cuda.synchronize()
        outs.append((ids.cpu(), cnt.cpu(), trace))
        c2.close()
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    for a, b in zip(outs[0][2], outs[1][2]):
        if a is not None:
            assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    ctx.close()


def test_graph_needs_a_real_stream():
    m = gpu_cfg()
    om, g_dev, layers_dev = both_models(m, seed=8, std=0.3)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=1, max_seq_len=32, D=2, tau=0.5)
    from paper_2509_24007_amd.sdlm import SdlmError
    if ctx.stream.cuda_stream == 0:
        with pytest.raises(SdlmError):
            ctx.graph(True)
    ctx.graph(False)
    ctx.close()


def test_mfma_row_blocks_beyond_the_sure_ones():
    """Every sequence is forced to accept D tokens, so the next step has the maximum B*2D rows: the row blocks the
    launch lists last (those that may be empty) all hold rows.  Alternating with single-token commits exercises the
    ragged and the empty case of the same launch shape."""
    m = mfma_cfg(n_q_heads=8, n_kv_heads=2)
    om, g_dev, layers_dev = both_models(m, seed=21, std=0.05)
    B, D, steps = 24, 4, 6
    lens = [3 + 5 * i for i in range(B)]
    prompts = [syn.uniform_int(4, f"rb{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    ids, cnt = syn.make_overrides(14, steps, B, D, m.vocab)
    cnt = cnt.clone()
    for t in range(steps):
        cnt[t] = D if (t // 2) % 2 == 0 else 1       # lockstep applies the overrides on odd steps
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=B, max_seq_len=max_len, D=D, tau=0.6, paged=True, n_pages=n_pages,
                      prefill_rows=128)
    assert ctx.kernel_info == "mfma-bf16"
    st, _ = lockstep(ctx, om, prompts, D, 0.6, steps, logit_tol=2e-2, conf_tol=1e-3, overrides=(ids, cnt), bf16=True, max_len=max_len)
    print("row blocks", st)
    ctx.close()


@pytest.mark.parametrize("B,D,hidden,ffn", [(1, 1, 128, 192), (1, 4, 320, 576), (3, 4, 448, 1088), (4, 4, 1088, 320), (2, 8, 192, 2112)])
def test_bf16_gate_up_of_at_most_32_rows(B, D, hidden, ffn):
    """Steps of at most 32 rows (B * 2D <= 32) take the gate/up kernel that splits k over the wavefronts of a workgroup:
    k extents whose per-wavefront share is shorter than, equal to and longer than the two register sets, not a multiple
    of a set, and row counts from 1 to the full 32."""
    m = mfma_cfg(n_q_heads=4, n_kv_heads=2, hidden=hidden, ffn=ffn, vocab=1000, has_qkv_bias=True)
    # (wide layers with weights of std 0.05 saturate the activations: bf16 noise alone then passes the logit bound, in
    # either gate/up kernel)
    om, g_dev, layers_dev = both_models(m, seed=70 + B + D, std=0.05 if hidden < 1000 else 0.03)
    lens = [5 + 7 * i for i in range(B)]
    prompts = [syn.uniform_int(5, f"sk{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 4
    ids, cnt = syn.make_overrides(21, steps, B, D, m.vocab)
    cnt = cnt.clone()
    cnt[1] = D                                       # the step after a full commit has B * 2D rows
    max_len = max(lens) + steps * D + D
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=B, max_seq_len=max_len, D=D, tau=0.5)
    assert ctx.kernel_info == "mfma-bf16"
    st, _ = lockstep(ctx, om, prompts, D, 0.5, steps, logit_tol=2e-2, conf_tol=1e-3, overrides=(ids, cnt), bf16=True, max_len=max_len)
    print("gate/up <= 32 rows", (B, D, hidden, ffn), st)
    ctx.close()


@pytest.mark.parametrize("hidden", [4100, 8200, 16384])
def test_fp32_wide_hidden_rows(hidden):
    """Rows wider than 4096 elements: the RMSNorm variants that hold 8 and 16 vectors of a row per thread (and the
    widest row the library accepts)."""
    m = gpu_cfg(hidden=hidden, n_layers=1, ffn=48, vocab=97)
    om, g_dev, layers_dev = both_models(m, seed=33, std=0.02)
    prompts = [np.array([3, 1, 4, 1, 5], dtype=np.int32), np.array([9, 2], dtype=np.int32)]
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=2, max_seq_len=32, D=3, tau=0.5)
    st, _ = lockstep(ctx, om, prompts, 3, 0.5, 3, logit_tol=1e-4, conf_tol=1e-5)
    print("wide rows", hidden, st)
    ctx.close()


# ------------------------------------------------------------------ seeded random shapes
def _random_case(seed):
    rng = np.random.RandomState(seed)
    G = int(rng.choice([1, 2, 3, 4, 7, 8]))
    Hk = int(rng.choice([1, 2, 3]))
    hidden = int(rng.choice([128, 192, 256, 320, 448]))
    ffn = int(rng.choice([192, 320, 576, 1088]))
    vocab = int(rng.choice([515, 1000, 2048, 3001]))
    D = int(rng.choice([1, 2, 3, 4, 5, 8]))
    B = int(rng.choice([1, 3, 9, 17, 30]))
    lens = [int(v) for v in rng.randint(1, 70, size=B)]
    paged = bool(rng.randint(0, 2))
    kw = dict(n_q_heads=G * Hk, n_kv_heads=Hk, hidden=hidden, ffn=ffn, vocab=vocab, has_qkv_bias=bool(rng.randint(0, 2)),
              block_causal=bool(rng.randint(0, 4) == 0))
    return kw, lens, D, paged


@pytest.mark.parametrize("seed", list(range(24)))
def test_bf16_mfma_random_shapes(seed):
    """Seeded random model shapes, batch sizes, block sizes and layouts through the matrix-core path: every tile
    policy branch (row-tile height, column-tile width, split counts, ragged and possibly-empty row blocks) sees shapes
    it was not tuned on."""
    kw, lens, D, paged = _random_case(seed)
    m = mfma_cfg(**kw)
    om, g_dev, layers_dev = both_models(m, seed=100 + seed, std=0.05)
    prompts = [syn.uniform_int(seed, f"rs{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 4
    ovr = syn.make_overrides(200 + seed, steps, len(lens), D, m.vocab)
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=len(lens), max_seq_len=max_len, D=D, tau=0.5, paged=paged, n_pages=n_pages,
                      prefill_rows=int(np.random.RandomState(seed).choice([32, 64, 200])))
    assert ctx.kernel_info == "mfma-bf16"
    verify = 0 if (D >= 2 and seed % 2 == 0) else None
    st, _ = lockstep(ctx, om, prompts, D, 0.5, steps, logit_tol=2e-2, conf_tol=1e-3, overrides=ovr, bf16=True, max_len=max_len,
                     verify_rule=verify)
    print(f"random shape {seed}: {kw} B={len(lens)} D={D} paged={paged} verify={verify}", st)
    ctx.close()


@pytest.mark.parametrize("seed", list(range(12)))
def test_fp32_generic_random_shapes(seed):
    """The same for the generic kernels (fp32 debug mode): head sizes 32..128, sizes that are not multiples of any
    tile, exact ids and gamma."""
    rng = np.random.RandomState(1000 + seed)
    Hk = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 5]))
    d = int(rng.choice([32, 64, 96, 128]))
    m = gpu_cfg(n_q_heads=G * Hk, n_kv_heads=Hk, head_dim=d, hidden=int(rng.choice([36, 64, 100, 132])),
                ffn=int(rng.choice([40, 112, 250])), vocab=int(rng.choice([97, 300, 1001])),
                has_qkv_bias=bool(rng.randint(0, 2)), block_causal=bool(rng.randint(0, 4) == 0))
    D = int(rng.choice([1, 2, 3, 4, 6, 9]))
    B = int(rng.choice([1, 2, 5, 11]))
    lens = [int(v) for v in rng.randint(1, 50, size=B)]
    paged = bool(rng.randint(0, 2))
    om, g_dev, layers_dev = both_models(m, seed=300 + seed, std=0.3)
    prompts = [syn.uniform_int(seed, f"rf{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 4
    ovr = syn.make_overrides(400 + seed, steps, B, D, m.vocab)
    max_len = max(lens) + steps * D + D
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=B, max_seq_len=max_len, D=D, tau=0.5, paged=paged, n_pages=n_pages,
                      prefill_rows=int(rng.choice([16, 64, 200])))
    verify = int(rng.randint(0, 2)) if D >= 2 and seed % 2 == 0 else None
    st, _ = lockstep(ctx, om, prompts, D, 0.5, steps, logit_tol=1e-4, conf_tol=1e-5, overrides=ovr, max_len=max_len, verify_rule=verify)
    print(f"random fp32 shape {seed}: B={B} D={D} d={d} paged={paged} verify={verify}", st)
    assert st.id_near_tie == 0
    ctx.close()


@pytest.mark.parametrize("seed", list(range(6)))
def test_bf16_mfma_random_long_contexts(seed):
    """Few sequences with contexts of a few hundred tokens: the KV chunking policy (chunk size halves until there are
    enough work items) and the merge of many chunks see lengths on both sides of every chunk boundary."""
    rng = np.random.RandomState(2000 + seed)
    G = int(rng.choice([1, 4, 7, 16]))
    m = mfma_cfg(n_q_heads=G * 2, n_kv_heads=2, hidden=int(rng.choice([128, 256])), ffn=256, vocab=1000)
    D = int(rng.choice([2, 4, 8]))
    B = int(rng.choice([1, 2, 3]))
    lens = [int(v) for v in rng.randint(100, 520, size=B)]
    om, g_dev, layers_dev = both_models(m, seed=500 + seed, std=0.05)
    prompts = [syn.uniform_int(seed, f"rl{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    steps = 3
    max_len = max(lens) + steps * D + D
    paged = bool(rng.randint(0, 2))
    n_pages = sum((n + steps * D + 15) // 16 + 1 for n in lens)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=B, max_seq_len=max_len, D=D, tau=0.5, paged=paged, n_pages=n_pages, prefill_rows=128)
    st, _ = lockstep(ctx, om, prompts, D, 0.5, steps, logit_tol=2e-2, conf_tol=1e-3, bf16=True, max_len=max_len)
    print(f"random long {seed}: G={G} B={B} D={D} lens={lens} paged={paged}", st)
    ctx.close()
