"""Writes the stored expected values under tests/golden/ by running ONLY the CPU oracle (oracle/) on seeded
synthetic inputs (synth_inputs.py).  Nothing here touches the HIP library or a GPU.

The paper prints no worked example (its Fig. 2 and Fig. 3, the only step-by-step illustrations, are images that are not
part of the text; Section 3.2 and 3.3 describe them in words only), so no file here holds a value from the paper.
What is stored instead is the oracle's own decision trace on the smallest workload (C1: float32 pair, MTAD, gamma 4,
beam 2, prompt 32, seed 0) and on the same pair run as MMTAD, at tau = 0.3 and tau = 0, decisions taken in float32 as
the kernels take them.  The CPU suite checks that the oracle still reproduces these traces (a guard against an
unintended change of the oracle's arithmetic); the GPU suite checks the HIP path against them without running the oracle.

    python tests/golden/make_golden.py        # rewrites c1_traces.json
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import synth_inputs as si  # noqa: E402
from oracle import mtad, rng  # noqa: E402
from oracle.lm import CachedSession, DecoderLM  # noqa: E402

N_ITER = 6


def traces():
    w = si.WORKLOADS["C1"]
    wt, wd = si.make_weights(w.target, w.seed, "target"), si.make_weights(w.draft, w.seed, "draft")
    lm_p, lm_q = DecoderLM(w.target, wt), DecoderLM(w.draft, wd)
    prompt = [int(t) for t in si.make_prompt(w)[0]]
    out = {"workload": "C1", "seed": w.seed, "gamma": w.gamma, "beam": w.beam, "prompt": prompt, "runs": []}
    for mode in ("mtad", "mmtad"):
        for tau in (0.3, 0.0):
            sq, sp = CachedSession(lm_q, list(prompt)), CachedSession(lm_p, list(prompt))
            its = []
            for _ in range(N_ITER):
                tr = mtad.iteration(sq, sp, gamma=w.gamma, beam=w.beam, mode=mode, tau=tau, sample_bonus=True, seed=w.seed,
                                    dt=np.float32)
                h, t = tr["hist"], tr["tree"]
                its.append({
                    "beam_tok": np.asarray(h["tok"]).astype(int).tolist(),
                    "beam_parent": np.asarray(h["parent"]).astype(int).tolist(),
                    "tree_tok": np.asarray(t["tok"]).astype(int).tolist(),
                    "tree_parent": np.asarray(t["parent"]).astype(int).tolist(),
                    "eta": int(tr["eta"]), "node": int(tr["node"]), "bonus": int(tr["bonus"]),
                    "emitted": [int(x) for x in tr["emitted"]],
                    # smallest margin of any decision of this iteration: how far it is from flipping
                    "min_margin": float(min([float(np.min(h["margin"]))] + [abs(float(m)) for m in np.ravel(tr["accept_margins"])]
                                            + [float(tr["bonus_gap"])])),
                })
            out["runs"].append({"mode": mode, "tau": tau, "iterations": its})
    out["rng"] = {"hash_u64": [str(rng.hash_u64(7, s, p, i)) for s, p, i in ((0, 0, 0), (3, 41, 9), (6, 1000, 31999))],
                  "uniform": [float(rng.uniform(7, s, p, i)) for s, p, i in ((0, 0, 0), (3, 41, 9), (6, 1000, 31999))]}
    return out


if __name__ == "__main__":
    with open(os.path.join(HERE, "c1_traces.json"), "w") as f:
        json.dump(traces(), f, indent=1)
    print("wrote", os.path.join(HERE, "c1_traces.json"))
