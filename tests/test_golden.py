"""Stored decision traces (tests/golden/c1_traces.json, written by tests/golden/make_golden.py from the oracle alone).

CPU: the oracle still reproduces them (guards the oracle's arithmetic against unintended changes; an intended change
regenerates the file and says why in its commit).  GPU: the HIP path, run on its own through the C ABI, takes the same
decisions; every stored decision's margin is three orders of magnitude above the float32 path's logit error, so none may differ."""
import importlib.util
import json
import os

import numpy as np
import pytest

import synth_inputs as si

HERE = os.path.dirname(os.path.abspath(__file__))
GOLDEN = os.path.join(HERE, "golden", "c1_traces.json")


def _stored():
    with open(GOLDEN) as f:
        return json.load(f)


def test_oracle_reproduces_stored_traces():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now, want = mod.traces(), _stored()
    assert now["prompt"] == want["prompt"] and now["rng"]["hash_u64"] == want["rng"]["hash_u64"]
    assert np.allclose(now["rng"]["uniform"], want["rng"]["uniform"], rtol=0, atol=0)
    for a, b in zip(now["runs"], want["runs"]):
        assert (a["mode"], a["tau"]) == (b["mode"], b["tau"])
        for i, (x, y) in enumerate(zip(a["iterations"], b["iterations"])):
            for k in ("beam_tok", "beam_parent", "tree_tok", "tree_parent", "eta", "node", "bonus", "emitted"):
                assert x[k] == y[k], f"{a['mode']} tau={a['tau']} iteration {i}: {k}"
            assert abs(x["min_margin"] - y["min_margin"]) <= 1e-5 or x["min_margin"] == y["min_margin"]


def test_stored_margins_are_far_from_the_float32_error():
    for run in _stored()["runs"]:
        assert min(it["min_margin"] for it in run["iterations"]) > 1e-3   # measured float32 logit error of the HIP path: 3e-6


@pytest.mark.gpu
def test_hip_path_reproduces_stored_traces():
    import torch
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    from paper_2407_09722_amd import binding as mb
    want = _stored()
    w = si.WORKLOADS["C1"]
    wt, wd = si.make_weights(w.target, w.seed, "target"), si.make_weights(w.draft, w.seed, "draft")
    tm, dm = DeviceModel(w.target, wt, "cuda:0"), DeviceModel(w.draft, wd, "cuda:0")
    prompt = np.asarray(want["prompt"], np.int32)[None, :]
    assert np.array_equal(prompt, si.make_prompt(w))
    for run in want["runs"]:
        print(f"stored trace {run['mode']} tau={run['tau']}", flush=True)
        eng = Engine(tm, dm, batch=1, gamma=w.gamma, beam=w.beam, mode=run["mode"], max_context=128, device="cuda:0")
        eng.prefill(prompt)
        for i, it in enumerate(run["iterations"]):
            eng.draft_phase(seed=w.seed)
            eng.verify_phase()
            eng.accept_phase(run["tau"], True, w.seed)
            torch.cuda.synchronize()
            where = f"{run['mode']} tau={run['tau']} iteration {i}"
            assert eng.h_tok[0].cpu().tolist() == it["beam_tok"], where
            assert eng.h_parent[0].cpu().tolist() == it["beam_parent"], where
            assert eng.t_tok[0].cpu().tolist() == it["tree_tok"], where
            assert eng.t_parent[0].cpu().tolist() == it["tree_parent"], where
            assert int(eng.eta[0]) == it["eta"] and int(eng.bonus_row[0]) == it["node"] and int(eng.bonus_tok[0]) == it["bonus"], where
            eng.commit_phase()
            assert eng.emitted()[0] == it["emitted"], where
        assert mb.mtad_device_status(eng.ctx) == 0
        eng.close()
