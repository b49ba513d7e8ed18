"""GPU checks at the full size of the benchmark workload (C3: 32-layer 7B-shaped target, 2-layer draft, prompt 512), in the
launch configuration bench.py times.  The float64 oracle cannot run 32 layers at this width over a 512-token prompt in
seconds, so most of these are properties that hold at any size, each of them able to fail on a real mistake in the path:

* per-row normalisation: the fused logsumexp equals the logsumexp of the logits the pass wrote, and every conditional
  log-likelihood is the gathered logit minus its parent row's logsumexp;
* tau = 0 accepts every prefix (Section 3.2: tau in [0, 1)), so every iteration commits gamma + 1 tokens, while at the
  paper's tau random models disagree and exactly the bonus token is committed;
* a cache built by tree passes and commits equals a cache built by prefilling the same tokens: the next-token logits agree;
* the MMTAD tree contains the MTAD chain (the output beam, Section 3.3), so the conditional log-likelihoods along that
  path agree between the two passes although they run different kernels (5 rows against 17 rows under a tree mask).

The last test does compare with the oracle at full depth: all 32 layers at full width over a 24-token prompt (the oracle
holds the 6.6 G weights in float64, about 53 GB of host memory, and needs a few seconds per pass), two iterations of the
5-row chain (the one-launch pass) and two of the 17-row tree (one kernel per step), every logit within the tolerance.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-2  # the bf16 workloads' logit tolerance


@pytest.fixture(scope="module")
def models():
    from paper_2407_09722_amd.engine import DeviceModel
    w = si.WORKLOADS["C3"]
    print("C3 full depth: uploading weights", flush=True)
    tm = DeviceModel(w.target, lambda n: si.make_tensor(w.target, w.seed, "target", n), DEV, threads=16)
    dm = DeviceModel(w.draft, lambda n: si.make_tensor(w.draft, w.seed, "draft", n), DEV, threads=16)
    yield w, tm, dm
    del tm, dm
    torch.cuda.empty_cache()


def _engine(w, tm, dm, mode=None, beam=None, max_context=None):
    from paper_2407_09722_amd.engine import Engine
    return Engine(tm, dm, batch=w.batch, gamma=w.gamma, beam=beam or w.beam, mode=mode or w.mode,
                  max_context=max_context or (w.prompt_len + 128), device=DEV)


def _status(eng):
    from paper_2407_09722_amd import binding as mb
    return mb.mtad_device_status(eng.ctx)


def test_full_size_rows_are_normalised_and_gathered(models):
    w, tm, dm = models
    eng = _engine(w, tm, dm)
    print("C3 full: prefill + one verify", flush=True)
    eng.prefill(si.make_prompt(w))
    eng.draft_phase(seed=w.seed)
    eng.verify_phase()
    torch.cuda.synchronize()
    logits = eng.logits[0].double()
    assert torch.isfinite(logits).all()
    lse = torch.logsumexp(logits, dim=1)
    assert (lse - eng.row_lse[0].double()).abs().max().item() < 1e-4
    assert abs(float(logits.std()) - 3.0) < 0.5          # the unembedding is scaled for logit std 3
    par, tok = eng.t_parent[0].cpu().numpy(), eng.t_tok[0].cpu().numpy()
    got = eng.logp_cond[0].cpu().numpy()
    for c in range(1, eng.M):
        want = float(logits[par[c], tok[c]] - lse[par[c]])
        assert abs(got[c] - want) < 1e-4, (c, got[c], want)
    assert _status(eng) == 0
    eng.close()


def test_full_size_tau_extremes_and_cache_equivalence(models):
    w, tm, dm = models
    prompt = si.make_prompt(w)
    eng = _engine(w, tm, dm)
    eng.prefill(prompt)
    print("C3 full: tau = 0.3", flush=True)
    emitted = []
    for _ in range(3):
        eng.iteration(w.tau, seed=w.seed)
        out = eng.emitted()[0]
        assert len(out) == 1, "independent random models: only the bonus token passes at the paper's tau"
        emitted += out
    print("C3 full: tau = 0", flush=True)
    for _ in range(3):
        eng.iteration(0.0, seed=w.seed)
        out = eng.emitted()[0]
        assert len(out) == w.gamma + 1, "tau = 0 accepts the whole draft"
        emitted += out
    assert int(eng.tkv.len[0].item()) == prompt.shape[1] - 1 + len(emitted)
    assert all(0 <= t < w.target.vocab for t in emitted)
    # the same context prefilled from scratch: the next pass must see the same distribution at the root
    eng.draft_phase(seed=w.seed)
    eng.verify_phase()
    torch.cuda.synchronize()
    a = eng.logits[0, 0].clone()
    ref = _engine(w, tm, dm)
    full = np.concatenate([prompt, np.asarray(emitted, np.int32)[None, :]], axis=1)
    print("C3 full: prefill of the committed context", flush=True)
    ref.prefill(full)
    ref.draft_phase(seed=w.seed)
    ref.verify_phase()
    torch.cuda.synchronize()
    b = ref.logits[0, 0]
    err = (a - b).abs().max().item()
    print(f"C3 full: root logits, committed cache vs prefilled cache: max diff {err:.2e}")
    assert err < TOL
    assert _status(eng) == 0 and _status(ref) == 0
    eng.close()
    ref.close()


def test_full_size_tree_pass_contains_the_chain_pass(models):
    w, tm, dm = models
    prompt = si.make_prompt(w)
    chain = _engine(w, tm, dm, mode="mtad")
    tree = _engine(w, tm, dm, mode="mmtad")
    for eng in (chain, tree):
        eng.prefill(prompt)
        eng.draft_phase(seed=w.seed)     # deterministic top-b: the same beam history on both
        eng.verify_phase()
    torch.cuda.synchronize()
    assert torch.equal(chain.h_tok, tree.h_tok) and torch.equal(chain.h_parent, tree.h_parent)
    ct, tt = chain.t_tok[0].cpu().numpy(), tree.t_tok[0].cpu().numpy()
    tp, td = tree.t_parent[0].cpu().numpy(), tree.t_depth[0].cpu().numpy()
    # walk the chain's tokens down the tree
    node, worst = 0, 0.0
    for i in range(1, w.gamma + 1):
        kids = [c for c in range(1, tree.M) if tp[c] == node and td[c] == i and tt[c] == ct[i]]
        assert len(kids) == 1, f"depth {i}: the output beam's token is not a child of its predecessor in the tree"
        node = kids[0]
        d = abs(float(chain.logp_cond[0, i]) - float(tree.logp_cond[0, node]))
        worst = max(worst, d)
    print(f"C3 full: chain vs tree conditional log-likelihoods along the output beam: max diff {worst:.2e}")
    assert worst < TOL
    assert (chain.logits[0, 0] - tree.logits[0, 0]).abs().max().item() < TOL
    assert _status(chain) == 0 and _status(tree) == 0
    chain.close()
    tree.close()


def test_full_depth_c3_target_matches_oracle_on_a_short_prompt(models):
    """32 layers, d 4096, FFN 11008, vocabulary 32000 against the float64 oracle, element by element: MTAD (5 rows, the
    one-launch pass) and MMTAD (17 rows, three row groups, one kernel per step), in lock step."""
    from _parity import run_pair
    from oracle.lm import DecoderLM
    w, tm, dm = models
    print("C3 full depth: oracle weights (float64)", flush=True)
    wt = si.make_weights(w.target, w.seed, "target", threads=16)
    lm_p = DecoderLM(w.target, wt)
    del wt
    lm_q = DecoderLM(w.draft, si.make_weights(w.draft, w.seed, "draft", threads=16))
    prompt = si.make_prompt(w)[:, :24]
    for mode in ("mtad", "mmtad"):
        print(f"C3 full depth: {mode} against the oracle", flush=True)
        st = run_pair(w.target, w.draft, None, None, prompt, 2 * (w.gamma + 1), gamma=w.gamma, beam=w.beam, mode=mode, tau=0.0, seed=w.seed,
                      max_iters=2, lockstep=True, lms=(lm_p, lm_q), device_models=(tm, dm))
        print(f"C3 full depth {mode}: {st['iters']} iterations, {st['excused']} put back, max logit err {st['max_logit_err']:.2e}, parted: {st['events']}",
              flush=True)
        assert st["iters"] == 2 and st["iters"] - st["excused"] >= 1 and st["max_logit_err"] > 0
        assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


def test_full_depth_c5_pair_matches_oracle_on_a_short_prompt():
    """C5 at full depth and width against the float64 oracle, element by element: 40-layer 13B-shaped target (164 rows per
    pass: 4 trees of 8 beams x gamma 5 + root, the LDS-staged product kernels and 48-row attention items), 22-layer
    grouped-query draft, 4 sequences with their own 24-token prompts; one whole iteration.  The oracle holds the target in
    float64 (about 104 GB of host memory)."""
    from _parity import run_pair
    from oracle.lm import DecoderLM
    from paper_2407_09722_amd.engine import DeviceModel
    w = si.WORKLOADS["C5"]
    print("C5 full depth: weights", flush=True)
    wt = si.make_weights(w.target, w.seed, "target", threads=16)
    tm = DeviceModel(w.target, wt, DEV)
    lm_p = DecoderLM(w.target, wt)
    del wt
    wd = si.make_weights(w.draft, w.seed, "draft", threads=16)
    dm = DeviceModel(w.draft, wd, DEV)
    lm_q = DecoderLM(w.draft, wd)
    del wd
    prompt = si.make_prompt(w)[:, :24]
    print("C5 full depth: one iteration against the oracle", flush=True)
    st = run_pair(w.target, w.draft, None, None, prompt, w.gamma + 1, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=0.0, seed=w.seed,
                  max_iters=1, prefill_rows=32, lms=(lm_p, lm_q), device_models=(tm, dm))
    print(f"C5 full depth: {st['iters']} iteration, {st['excused']} of 4 sequences parted, max logit err {st['max_logit_err']:.2e}, parted: {st['events']}",
          flush=True)
    assert st["iters"] == 1 and st["excused"] <= 2 and st["max_logit_err"] > 0
    assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")
    del tm, dm, lm_p, lm_q
    torch.cuda.empty_cache()
