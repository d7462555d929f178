"""Writes tests/golden/c1_trajectory.json: the oracle's own free-running trajectory on the tiny fp32 workload
(2 layers, hidden 256, 4/2 heads of 64, FFN 688, vocab 4096, prompt 64, D=4, tau=0.5, 32 steps, seed 0).

Calls only oracle/ and the synthetic-input module.  Run from the repo root:
    python tests/golden/make_c1_golden.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle as orc                      # noqa: E402
from paper_2509_24007_amd import inputs as syn         # noqa: E402


def main():
    wl = syn.workloads()["C1"]
    m, r = wl.model, wl.run
    g = syn.make_globals(m, wl.seed)
    layers = [syn.make_layer(m, wl.seed, l) for l in range(m.n_layers)]
    om = orc.model_from_inputs(m, g, layers)
    prompt = syn.make_prompts(wl.seed, r.batch, r.prompt_lo, r.prompt_hi, m.vocab)[0].numpy()
    seq = orc.Seq(om, r.prompt_hi + r.steps * r.block_D + r.block_D)
    seq.prefill(prompt)
    steps = []
    for _ in range(r.steps):
        logits, ids, conf, gamma = seq.step(r.block_D, r.tau)
        top2 = [sorted(map(float, row))[-2:] for row in logits]
        steps.append({"ids": [int(i) for i in ids], "conf": [float(c) for c in conf], "gamma": gamma,
                      "top2_gap": [t[1] - t[0] for t in top2], "logit_max": [t[1] for t in top2]})
        seq.commit()
    out = {"workload": wl.name, "seed": wl.seed, "D": r.block_D, "tau": r.tau, "prompt_len": len(prompt),
           "steps": steps, "final_tokens": [int(t) for t in seq.tokens]}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_trajectory.json"), "w") as f:
        json.dump(out, f, indent=0)
    print("gammas", [s["gamma"] for s in steps])
    print("min conf-tau distance", min(abs(c - r.tau) for s in steps for c in s["conf"]))
    print("min top2 gap", min(min(s["top2_gap"]) for s in steps))


if __name__ == "__main__":
    main()
