"""The tiny fp32 workload (configs[0]) through the oracle: stored trajectory and full-recompute agreement."""
import json
import os

import numpy as np

from helpers import rel_err
from oracle import oracle as orc
from paper_2509_24007_amd import inputs as syn

GOLD = os.path.join(os.path.dirname(__file__), "golden", "c1_trajectory.json")


def test_c1_trajectory_and_brute_agreement():
    gold = json.load(open(GOLD))          # written by tests/golden/make_c1_golden.py (oracle only)
    wl = syn.workloads()["C1"]
    m, r = wl.model, wl.run
    g = syn.make_globals(m, wl.seed)
    layers = [syn.make_layer(m, wl.seed, l) for l in range(m.n_layers)]
    om = orc.model_from_inputs(m, g, layers)
    prompt = syn.make_prompts(wl.seed, 1, r.prompt_lo, r.prompt_hi, m.vocab)[0].numpy()
    assert len(prompt) == gold["prompt_len"] == 64
    seq = orc.Seq(om, 64 + r.steps * r.block_D + r.block_D)
    seq.prefill(prompt)
    for t, want in enumerate(gold["steps"]):
        hist = seq.tokens
        logits, ids, conf, gamma = seq.step(r.block_D, r.tau)
        assert [int(i) for i in ids] == want["ids"] and gamma == want["gamma"]
        np.testing.assert_allclose(conf, want["conf"], rtol=1e-6)
        if t in (0, 1, 15, 31):            # the cached step equals the full-attention recompute
            lb, ib, cb, gb = orc.brute_step(om, hist, r.block_D, r.tau)
            assert rel_err(logits, lb) < 1e-11 and gb == gamma
            np.testing.assert_array_equal(ib, ids)
        seq.commit()
    assert [int(x) for x in seq.tokens] == gold["final_tokens"]
