"""sdlm_decode_step_static (the step with its partial-result scratch in the library's static device array) against
sdlm_decode_step, through the C ABI: two calls in a row on one GPU, the second on a smaller input."""
import numpy as np
import pytest
import torch

from gpu_common import both_models, gpu_context
from helpers import small_cfg
from paper_2509_24007_amd import inputs as syn
from paper_2509_24007_amd import sdlm

pytestmark = pytest.mark.gpu


def _step_both(ctx, B, D, V):
    out = []
    for static in (False, True):
        ids = torch.full((B, D), -7, dtype=torch.int32, device="cuda")
        cnt = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        conf = torch.full((B, D), float("nan"), dtype=torch.float32, device="cuda")
        logits = torch.full((B * D, V), float("nan"), dtype=torch.float32, device="cuda")
        ctx.decode_step(ids, cnt, conf, logits, static_scratch=static)      # the step publishes nothing: it can be repeated
        torch.cuda.synchronize()
        out.append((ids.cpu().numpy(), cnt.cpu().numpy(), conf.cpu().numpy(), logits.cpu().numpy()))
    return out


def _compare(ref, got, logit_tol):
    (ri, rc, rf, rl), (gi, gc, gf, gl) = ref, got
    assert np.isfinite(gl).all() and np.isfinite(gf).all()
    err = np.max(np.abs(gl - rl), axis=1) / np.max(np.abs(rl), axis=1)
    assert err.max() <= logit_tol, err.max()
    # ids and gamma bit-exact, except where the existing entry point's own top-2 gap / product is inside the 1e-3 band
    top2 = np.sort(rl, axis=1)[:, -2:]
    gap = (top2[:, 1] - top2[:, 0]).reshape(ri.shape)
    assert ((gi == ri) | (gap < 1e-3)).all()
    if (gi == ri).all() and np.array_equal(gf, rf):
        assert np.array_equal(gc, rc)
    assert np.max(np.abs(np.log(gf) - np.log(rf))) <= 2 * np.max(np.abs(gl - rl)) + 1e-6
    return float(err.max())


@pytest.mark.parametrize("mode", ["fp32-generic", "bf16-mfma"])
def test_static_scratch_step_matches_the_workspace_step(mode):
    if mode == "fp32-generic":
        m = small_cfg(hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=112, vocab=300)
        std, tol = 0.3, 1e-4
    else:
        m = syn.ModelCfg(2, 512, 8, 2, 128, 1024, 3000, dtype="bf16")     # wide enough for split-k slabs and split-KV partials
        std, tol = 0.05, 2e-2
    D = 4
    om, g_dev, layers_dev = both_models(m, seed=21, std=std)
    ctx = gpu_context(m, g_dev, layers_dev, max_batch=5, max_seq_len=700, D=D, tau=0.3, paged=True, n_pages=5 * 45)
    assert ctx.kernel_info == ("generic-fp32" if mode == "fp32-generic" else "mfma-bf16")
    # call 1: five sequences, one of them long enough for several KV chunks, with pending rows
    lens = [600, 33, 1, 250, 97]
    prompts = [syn.uniform_int(21, f"na{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate(lens)]
    ctx.prefill(prompts)
    ids = torch.empty(5, D, dtype=torch.int32, device="cuda")
    cnt = torch.empty(5, dtype=torch.int32, device="cuda")
    ctx.decode_step(ids, cnt)
    ctx.kv_commit()
    ref, got = _step_both(ctx, 5, D, m.vocab)
    e1 = _compare(ref, got, tol)
    # call 2, right after it on the same GPU: a smaller input (two short sequences); the array still holds call 1's partials
    prompts = [syn.uniform_int(22, f"nb{i}", n, 0, m.vocab - 1).numpy() for i, n in enumerate([7, 40])]
    ctx.prefill(prompts)
    ref, got = _step_both(ctx, 2, D, m.vocab)
    e2 = _compare(ref, got, tol)
    # and the static step can be committed like any other
    ctx.kv_commit()
    n, c = ctx.get_lengths()
    assert (n.numpy() == np.array([7, 40]) + got[1]).all()
    print(mode, "static vs workspace step: max row-normalised logit difference", e1, e2)
    ctx.close()


def test_static_scratch_rejects_what_does_not_fit():
    m = small_cfg(hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=112, vocab=300000, dtype="fp32")
    # fp32 mode keeps batch x D x vocabulary logits in the scratch when the caller does not take them: 4 x 4 x 300000 x 4 B > 4 MiB
    ctx = sdlm.Context(sdlm.model_cfg(m), max_batch=4, max_seq_len=64, block_D=4, tau=0.5)
    g = syn.make_globals(m, 3, device="cuda")
    layers = {l: syn.make_layer(m, 3, l, device="cuda") for l in range(m.n_layers)}
    ctx.init_weights(g, layers)
    ctx.prefill([[1, 2, 3], [4], [5, 6], [7]])
    ids = torch.empty(4, 4, dtype=torch.int32, device="cuda")
    cnt = torch.empty(4, dtype=torch.int32, device="cuda")
    with pytest.raises(sdlm.SdlmError) as e:
        ctx.decode_step(ids, cnt, static_scratch=True)
    assert e.value.code == sdlm.ECAPACITY and "static" in str(e.value)
    ctx.decode_step(ids, cnt)                      # the workspace step still runs
    torch.cuda.synchronize()
    assert int(cnt.min()) >= 1
    ctx.close()
