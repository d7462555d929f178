"""Pins for the oracle's self-speculative verification (Sec. 3.4, "Self-Speculative Decoding", Eq. 10).

The verification predictions are checked against a route that shares nothing with the cached one: a dense
forward without any cache over the explicitly extended token list under the explicit block mask.
"""
import itertools

import numpy as np
import pytest

from helpers import make_model, oracle_model, rel_err, small_cfg
from oracle import oracle as orc
from paper_2509_24007_amd import inputs as syn


def test_gamma_verify_hand_cases():
    # (yhat, ytilde, longest agreeing prefix, largest agreeing index) worked by hand
    cases = [
        ([5, 6, 7, 8], [5, 6, 7, 8], 4, 4),
        ([5, 6, 7, 8], [5, 6, 9, 8], 2, 4),
        ([5, 6, 7, 8], [5, 1, 7, 2], 1, 3),
        ([5, 6, 7, 8], [5, 1, 2, 3], 1, 1),
        ([5, 6, 7, 8], [4, 6, 7, 8], 1, 4),     # even a disagreeing first position still yields one token
        ([5, 6, 7, 8], [4, 1, 2, 3], 1, 1),
        ([3], [3], 1, 1),
        ([3], [2], 1, 1),
        ([1, 1, 1, 1, 1, 1, 1, 1], [1, 1, 1, 1, 1, 0, 1, 1], 5, 8),
    ]
    for yh, yt, prefix, printed in cases:
        assert orc.gamma_verify(yh, yt, 0) == prefix, (yh, yt)
        assert orc.gamma_verify(yh, yt, 1) == printed, (yh, yt)


def test_gamma_verify_exhaustive_small():
    # every pair of sequences over a 2-letter alphabet, D <= 4: bounds, ordering of the two rules, and the
    # defining property of each rule stated on the result rather than recomputed
    for D in (1, 2, 3, 4):
        for yh in itertools.product((0, 1), repeat=D):
            for yt in itertools.product((0, 1), repeat=D):
                g0, g1 = orc.gamma_verify(yh, yt, 0), orc.gamma_verify(yh, yt, 1)
                assert 1 <= g0 <= g1 <= D
                agree = [a == b for a, b in zip(yh, yt)]
                assert all(agree[1:g0]) or g0 == 1              # everything inside the accepted prefix agrees (position 1 is free)
                assert g0 == D or not agree[g0] or (g0 == 1 and not agree[0])   # and it cannot be extended
                assert g1 == 1 or agree[g1 - 1]
                assert not any(agree[max(g1, 1):])              # nothing beyond the printed rule's index agrees


@pytest.fixture(scope="module")
def model():
    m = small_cfg()
    g, layers = make_model(m, seed=23, std=0.3)
    return m, oracle_model(m, g, layers)


@pytest.mark.parametrize("D", [2, 4, 6])
def test_verification_predictions_equal_dense_recompute(model, D):
    m, om = model
    for plen in (1, 3, 9):
        prompt = syn.uniform_int(5, f"v{D}", plen, 0, m.vocab - 1).numpy()
        seq = orc.Seq(om, 96)
        seq.prefill(prompt)
        for step in range(3):
            hist = seq.tokens.copy()
            _, yhat, _, _ = seq.step(D, 0.5)
            yt, gv, z = seq.verify(rule=0, want_logits=True)
            assert yt[0] == yhat[0]
            for j in range(2, D + 1):
                ext = np.concatenate([hist, yhat[: j - 1]])       # verification input j: prefix yhat^1..yhat^{j-1}, masks follow
                lb, ib, _, _ = orc.brute_step(om, ext, D, 0.5)
                assert ib[0] == yt[j - 1]
                assert rel_err(z[j - 1], lb[0]) < 1e-11
            assert gv == orc.gamma_verify(yhat, yt, 0)
            yt1, gv1 = seq.verify(rule=1)
            np.testing.assert_array_equal(yt1, yt)
            assert gv1 == orc.gamma_verify(yhat, yt, 1) and gv1 >= gv
            # a commit without arguments now publishes the verified prefix of the speculative tokens
            seq.verify(rule=0)
            assert seq.commit() == 0
            assert seq.n == len(hist) + gv
            np.testing.assert_array_equal(seq.tokens[len(hist):], yhat[:gv])


def test_verification_leaves_the_sequence_untouched(model):
    m, om = model
    prompt = syn.uniform_int(6, "vu", 7, 0, m.vocab - 1).numpy()
    a, b = orc.Seq(om, 64), orc.Seq(om, 64)
    a.prefill(prompt); b.prefill(prompt)
    la, ia, _, _ = a.step(4, 0.5)
    lb, ib, _, _ = b.step(4, 0.5)
    a.verify()
    assert a.n == b.n and a.c == b.c
    # same override commit on both, then the next step must agree bit for bit: the verify pass left no trace
    assert a.commit(ia, 2) == 0 and b.commit(ib, 2) == 0
    l2a, _, _, _ = a.step(4, 0.5)
    l2b, _, _, _ = b.step(4, 0.5)
    np.testing.assert_array_equal(l2a, l2b)


def test_position_independent_model_verifies_everything():
    # all-zero weights: every logit row is constant, the arg-max rule picks token 0 everywhere, so the speculative
    # and the verification tokens agree at every position and the whole block is accepted
    m = small_cfg()
    g, layers = make_model(m, seed=3, std=0.0)
    om = oracle_model(m, g, layers)
    seq = orc.Seq(om, 64)
    seq.prefill(np.array([4, 2, 7], dtype=np.int32))
    _, yhat, _, _ = seq.step(4, 2.0)           # tau > 1: the confidence rule alone would accept a single token
    yt, gv = seq.verify()
    np.testing.assert_array_equal(yhat, 0)
    np.testing.assert_array_equal(yt, 0)
    assert gv == 4


def test_block_size_one_verification_is_trivial(model):
    m, om = model
    seq = orc.Seq(om, 32)
    seq.prefill(np.array([1, 2, 3], dtype=np.int32))
    _, yhat, _, _ = seq.step(1, 0.5)
    yt, gv = seq.verify()
    assert gv == 1 and yt[0] == yhat[0]
