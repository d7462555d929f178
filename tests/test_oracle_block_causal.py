"""Pins for the oracle's causal-in-block variant (Sec. 4.4, "Causal Attention": the block's bidirectional attention is
replaced by a causal mask).  With that mask the whole forward is a plain causal decoder over tokens ++ [m]*(D-1), so
every block row has a textbook definition the oracle's other routes can be held to."""
import numpy as np
import pytest

from helpers import make_model, oracle_model, rel_err, small_cfg
from oracle import oracle as orc
from paper_2509_24007_amd import inputs as syn


def test_causal_block_mask_is_the_lower_triangle():
    for n, D in ((1, 1), (3, 3), (5, 4), (2, 8)):
        T = n + D - 1
        np.testing.assert_array_equal(orc.block_mask(n, D, causal=True), np.tril(np.ones((T, T), np.uint8)))
    # and the default differs from it exactly on the block's upper triangle (hand-written for n=3, D=3)
    diff = orc.block_mask(3, 3).astype(int) - orc.block_mask(3, 3, causal=True).astype(int)
    want = np.zeros((5, 5), int)
    want[2, 3] = want[2, 4] = want[3, 4] = 1
    np.testing.assert_array_equal(diff, want)


@pytest.fixture(scope="module")
def models():
    m = small_cfg(block_causal=True)
    g, layers = make_model(m, seed=31, std=0.3)
    return m, oracle_model(m, g, layers), oracle_model(small_cfg(), g, layers)


@pytest.mark.parametrize("D", [1, 2, 4, 7])
def test_block_rows_equal_next_token_decoder_over_masks(models, D):
    """Block row t = the textbook causal decoder's next-token logits after tokens ++ [m]*t."""
    m, om, _ = models
    for plen in (1, 4, 11):
        prompt = syn.uniform_int(8, f"c{D}", plen, 0, m.vocab - 1).numpy()
        seq = orc.Seq(om, 64)
        seq.prefill(prompt)
        for step in range(3):
            hist = seq.tokens.copy()
            lc, ic, _, gc = seq.step(D, 0.3)
            lb, ib, _, gb = orc.brute_step(om, hist, D, 0.3)
            assert rel_err(lc, lb) < 1e-11 and gc == gb
            np.testing.assert_array_equal(ic, ib)
            for t in range(D):
                ext = np.concatenate([hist, np.full(t, m.mask_token_id, np.int32)]).astype(np.int32)
                assert rel_err(lc[t], orc.ntp_logits(om, ext)) < 1e-11
            assert seq.commit() == 0


def test_variants_share_the_first_row_only_when_the_block_is_one_token(models):
    m, om_c, om_b = models
    prompt = syn.uniform_int(9, "cv", 6, 0, m.vocab - 1).numpy()
    lc, _, _, _ = orc.brute_step(om_c, prompt, 1, 0.5)
    lb, _, _, _ = orc.brute_step(om_b, prompt, 1, 0.5)
    np.testing.assert_array_equal(lc, lb)
    lc, _, _, _ = orc.brute_step(om_c, prompt, 4, 0.5)
    lb, _, _, _ = orc.brute_step(om_b, prompt, 4, 0.5)
    assert rel_err(lc[0], lb[0]) > 1e-6            # bidirectional: x_last sees the masks; causal: it does not
    # the last row sees the whole block under both masks
    assert rel_err(lc[3], lb[3]) > 1e-6            # ... but the rows it attends to differ in their own inputs from layer 2 on


def test_verification_under_the_causal_variant(models):
    m, om, _ = models
    prompt = syn.uniform_int(10, "cw", 5, 0, m.vocab - 1).numpy()
    seq = orc.Seq(om, 64)
    seq.prefill(prompt)
    hist = seq.tokens.copy()
    _, yhat, _, _ = seq.step(4, 0.5)
    yt, gv = seq.verify()
    # causal block: the first row of input j is the plain next-token prediction after hist ++ yhat[:j-1]
    for j in range(1, 5):
        ext = np.concatenate([hist, yhat[: j - 1]]).astype(np.int32)
        assert int(np.argmax(orc.ntp_logits(om, ext))) == yt[j - 1]
