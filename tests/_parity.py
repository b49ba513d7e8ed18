"""Free-running parity of the HIP path against the oracle, iteration by iteration.

Both sides start from the same seeded weights and prompt and run on their own.  Every iteration the
beam history, tree, target logits, log-likelihoods, accept decision, bonus token and cache lengths
are compared.  Integer decisions must be identical; a difference is only excused when the oracle
reports that the decision's margin is below the logit tolerance (then the runs legitimately part
and the comparison stops).  Returns statistics of what was compared."""
import numpy as np
import torch

import synth_inputs as si
from oracle import mtad
from oracle.lm import CachedSession, DecoderLM


def logit_tolerance(dtype):
    # fp32: 1e-4 relative to max(1, |value|); bf16: 2e-2 absolute
    return (1e-4, 1e-4) if dtype == "fp32" else (0.0, 2e-2)


def close(got, want, dtype, what=""):
    rtol, atol = logit_tolerance(dtype)
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    same_inf = np.isinf(got) & (got == want)               # zero likelihoods (warped rows): equal infinities agree
    assert np.array_equal(np.isinf(got), np.isinf(want)), f"{what}: infinities in different places"
    got, want = np.where(same_inf, 0.0, got), np.where(same_inf, 0.0, want)
    err = np.abs(got - want)
    lim = atol + rtol * np.abs(want)
    assert np.all(err <= lim), f"{what}: max err {err.max():.3e} (limit {lim.flat[int(np.argmax(err - lim))]:.3e})"
    return float(err.max())


def run_pair(tshape, dshape, wt, wd, prompt, new_tokens, *, gamma, beam, mode, tau, sample_bonus=True,
             sample_beam=False, seed=0, max_context=None, page_size=16, prefill_rows=64, check_kv=False,
             max_iters=None, device="cuda:0", fused_pass=None, warp=None, method="mtad", lockstep=False, oracle_seqs=None, lms=None, device_models=None):
    """method "spd": vanilla speculative decoding (beam 1, chain, token-wise acceptance) instead of the joint rule.
    oracle_seqs: the sequences compared with the oracle (default all).  The others must then carry the prompt of
    oracle_seqs[0] and a deterministic run (no sampling): their trees and logits are checked against that sequence's.
    lms / device_models: prebuilt (target, draft) oracle models / uploaded models, for tests that run several
    configurations on one large pair of weight sets.
    lockstep (one sequence): where the runs part on an excused near-tie, the HIP side is put back on the oracle's context
    (cache lengths reset to the iteration's start, the oracle's tokens appended, its state set) and the comparison goes
    on, so every iteration of the run is compared up to the first decision that legitimately differs."""
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    prompt = np.asarray(prompt, np.int32)
    B, n0 = prompt.shape
    dtype = tshape.dtype
    M = 1 + (gamma if mode == "mtad" else gamma * beam)
    max_context = max_context or (n0 + new_tokens + 2 * (gamma + 1) + M + 8)
    tm, dm = device_models if device_models is not None else (DeviceModel(tshape, wt, device), DeviceModel(dshape, wd, device))
    eng = Engine(tm, dm, batch=B, gamma=gamma, beam=beam,
                 mode=mode, max_context=max_context, prefill_rows=prefill_rows, page_size=page_size, device=device, fused_pass=fused_pass,
                 warp=warp)
    lm_p, lm_q = lms if lms is not None else (DecoderLM(tshape, wt), DecoderLM(dshape, wd))
    sp = [CachedSession(lm_p, list(prompt[s])) for s in range(B)]
    sq = [CachedSession(lm_q, list(prompt[s])) for s in range(B)]
    oracle_seqs = list(range(B)) if oracle_seqs is None else list(oracle_seqs)
    if len(oracle_seqs) < B:
        assert not sample_beam and not sample_bonus and method == "mtad" and all(np.array_equal(prompt[s], prompt[oracle_seqs[0]]) for s in range(B))
    eng.prefill(prompt)
    stats = {"iters": 0, "excused": 0, "max_logit_err": 0.0, "eta": [], "tokens": [[] for _ in range(B)], "events": []}
    _, atol = logit_tolerance(dtype)
    margin_tol = max(atol, 1e-4) * 2
    alive = [s in oracle_seqs for s in range(B)]
    assert not lockstep or B == 1, "lock-step appends the same number of tokens to every sequence: one sequence only"
    stats["resyncs"] = 0

    def parted(s, tr):
        stats["excused"] += 1
        if lockstep:
            resync.append(s)
            stats["tokens"][s] += tr["emitted"]
        else:
            alive[s] = False

    while min(len(t) for t in stats["tokens"]) < new_tokens and (max_iters is None or stats["iters"] < max_iters):
        resync = []
        t_before = [len(x.context) - 1 for x in sp]
        d_before = [x.n_cached for x in sq]
        eng.draft_phase(sample_beam or method == "spd", seed)
        eng.verify_phase()
        if method == "spd":
            eng.accept_spd_phase(seed)
        else:
            eng.accept_phase(tau, sample_bonus, seed)
        torch.cuda.synchronize()
        g = {k: getattr(eng, k).cpu().numpy() for k in ("h_tok", "h_parent", "h_cum", "t_tok", "t_parent", "t_depth", "t_src",
                                                         "t_mask", "t_qref", "logp_cond", "row_lse", "logits", "eta", "path",
                                                         "bonus_row", "bonus_tok", "out_tok", "out_cnt")}
        eng.commit_phase()
        torch.cuda.synchronize()
        post = {k: getattr(eng, k).cpu().numpy() for k in ("root_tok", "catchup_tok", "catchup_cnt")}
        tlen, dlen = eng.tkv.len.cpu().numpy(), eng.dkv.len.cpu().numpy()
        for s in range(B):
            if s not in oracle_seqs:                   # a copy of the reference sequence: same tree, same logits, same decision
                r0 = oracle_seqs[0]
                for k in ("t_tok", "t_parent", "t_mask", "eta", "bonus_tok", "out_cnt"):
                    assert np.array_equal(g[k][s], g[k][r0]), f"sequence {s} differs from its copy {r0} in {k}"
                close(g["logits"][s], g["logits"][r0], dtype, f"logits of sequence {s} against its copy {r0}")
                stats["tokens"][s] += [int(t) for t in g["out_tok"][s, :g["out_cnt"][s]]]
                continue
            if not alive[s]:
                continue
            if method == "spd":
                tr = mtad.iteration_spd(sq[s], sp[s], gamma=gamma, seed=seed, seq_index=s, dt=np.float32, warp=warp)
            else:
                tr = mtad.iteration(sq[s], sp[s], gamma=gamma, beam=beam, mode=mode, tau=tau, stochastic_beam=sample_beam,
                                    sample_bonus=sample_bonus, seed=seed, seq_index=s, dt=np.float32, warp=warp)
            h = tr["hist"]
            # --- draft: beam history
            beams_differ = False
            for i in range(gamma):
                same = np.array_equal(g["h_tok"][s, i], h["tok"][i]) and np.array_equal(g["h_parent"][s, i], h["parent"][i])
                if not same:
                    assert h["margin"][i] < margin_tol or _near_tie(h["score"][i], margin_tol) or h["warp_margin"][i] < margin_tol, \
                        f"seq {s} iter {stats['iters']} beam step {i}: survivors differ, margin {h['margin'][i]}"
                    beams_differ = True
                    with np.errstate(invalid="ignore"):
                        diff = np.nanmax(np.abs(np.sort(g["h_cum"][s, i].astype(np.float64)) - np.sort(h["score"][i].astype(np.float64))))
                    stats["events"].append(("beam step", stats["iters"], i, float(h["margin"][i]), float(diff)))
                    break
                close(g["h_cum"][s, i], h["score"][i], dtype, f"cum_logq step {i}")
            if beams_differ:
                parted(s, tr)
                continue
            # --- tree
            t = tr["tree"]
            assert np.array_equal(g["t_tok"][s, 1:], t["tok"][1:]) and np.array_equal(g["t_parent"][s], t["parent"])
            assert np.array_equal(g["t_depth"][s], t["depth"]) and np.array_equal(g["t_src"][s, 1:], t["src_beam"][1:])
            assert np.array_equal(g["t_mask"][s].view(np.uint64), mtad.ancestor_masks(t["parent"]))
            close(g["t_qref"][s], t["qref"], dtype, "qref")
            # --- verify
            v = tr["verify"]
            if warp is not None and not np.array_equal(np.isinf(g["logits"][s]), np.isinf(v["logits"])):
                # a warped support differs: only where a top-k or top-p decision sits on its threshold
                assert v["warp_margin"] < margin_tol, f"warped supports differ with margin {v['warp_margin']}"
                stats["events"].append(("warp support", stats["iters"], float(v["warp_margin"])))
                parted(s, tr)
                continue
            stats["max_logit_err"] = max(stats["max_logit_err"], close(g["logits"][s], v["logits"], dtype, "target logits"))
            close(g["row_lse"][s], v["lse"], dtype, "row lse")
            close(g["logp_cond"][s], v["logp_cond"], dtype, "logp_cond")
            # --- accept + bonus
            if g["eta"][s] != tr["eta"] or g["bonus_row"][s] != tr["node"]:
                assert min(tr["accept_margins"]) < margin_tol * gamma, f"accept differs: {g['eta'][s]} vs {tr['eta']}"
                stats["events"].append(("accept", stats["iters"], float(min(tr["accept_margins"]))))
                parted(s, tr)
                continue
            assert list(g["path"][s, :tr["eta"]]) == tr["path_rows"] and np.all(g["path"][s, tr["eta"]:] == -1)
            if g["bonus_tok"][s] != tr["bonus"]:
                assert tr["bonus_gap"] < margin_tol, f"bonus token differs with gap {tr['bonus_gap']}"
                stats["events"].append(("bonus", stats["iters"], float(tr["bonus_gap"])))
                parted(s, tr)
                continue
            assert g["out_cnt"][s] == tr["eta"] + 1 and list(g["out_tok"][s, :tr["eta"] + 1]) == tr["emitted"]
            # --- commit: lengths and next-iteration state
            assert tlen[s] == len(sp[s].context) - 1
            pend = sq[s].context[sq[s].n_cached:]
            assert dlen[s] == sq[s].n_cached and post["catchup_cnt"][s] == len(pend)
            assert list(post["catchup_tok"][s, :len(pend)]) == pend and post["root_tok"][s] == sp[s].context[-1]
            if check_kv:
                _check_kv(eng.tkv, s, sp[s], dtype)
                _check_kv(eng.dkv, s, sq[s], dtype)
            stats["eta"].append(tr["eta"])
            stats["tokens"][s] += tr["emitted"]
        stats["iters"] += 1
        for s in resync:
            pend = sq[s].context[sq[s].n_cached:]
            eng.resync(t_before, d_before, [sp[s].context[t_before[s]:len(sp[s].context) - 1]], [sq[s].context[d_before[s]:sq[s].n_cached]],
                       [sp[s].context[-1]], [pend], [len(pend)])
            stats["resyncs"] += 1
        if not any(alive):
            break
    status = _status(eng)
    eng.close()
    assert status == 0, f"device status {status:#x}"
    return stats


def run_autoregressive(tshape, wt, prompt, new_tokens, *, sample=True, seed=0, warp=None, device="cuda:0"):
    """Plain decoding with the target alone on the HIP path against the oracle, token by token (free running; the runs
    may part only where the oracle reports a near-tie)."""
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    prompt = np.asarray(prompt, np.int32)
    B, n0 = prompt.shape
    dtype = tshape.dtype
    tm = DeviceModel(tshape, wt, device)
    eng = Engine(tm, tm, batch=B, gamma=1, beam=1, mode="mtad", max_context=n0 + new_tokens + 8, prefill_rows=16, device=device, warp=warp)
    lm = DecoderLM(tshape, wt)
    sp = [CachedSession(lm, list(prompt[s])) for s in range(B)]
    eng.prefill(prompt)
    _, atol = logit_tolerance(dtype)
    margin_tol = max(atol, 1e-4) * 2
    out = {"tokens": [[] for _ in range(B)], "excused": 0, "max_logit_err": 0.0}
    alive = [True] * B
    for it in range(new_tokens):
        eng.iteration_autoregressive(sample, seed)
        torch.cuda.synchronize()
        logits, tok, tlen = eng.logits.cpu().numpy().reshape(-1, tshape.vocab)[:B], eng.bonus_tok.cpu().numpy(), eng.tkv.len.cpu().numpy()
        for s in range(B):
            if not alive[s]:
                continue
            tr = mtad.autoregressive_step(sp[s], sample=sample, seed=seed, seq_index=s, dt=np.float32, warp=warp)
            if warp is not None and not np.array_equal(np.isinf(logits[s]), np.isinf(tr["logits"])):
                assert tr["warp_margin"] < margin_tol
                alive[s] = False
                out["excused"] += 1
                continue
            out["max_logit_err"] = max(out["max_logit_err"], close(logits[s], tr["logits"], dtype, "target row"))
            if tok[s] != tr["bonus"]:
                assert tr["bonus_gap"] < margin_tol, f"token differs with gap {tr['bonus_gap']}"
                alive[s] = False
                out["excused"] += 1
                continue
            assert tlen[s] == len(sp[s].context) - 1
            out["tokens"][s].append(int(tok[s]))
    status = _status(eng)
    eng.close()
    assert status == 0
    return out


def run_mtjd(tshape, wt, prompt, steps, *, K, beam, sample_beam=False, seed=0, warp=None, device="cuda:0"):
    """Multi-token joint decoding (beam sampling on the target itself) on the HIP path against the oracle, step by step."""
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    prompt = np.asarray(prompt, np.int32)
    B, n0 = prompt.shape
    dtype = tshape.dtype
    tm = DeviceModel(tshape, wt, device)
    eng = Engine(tm, tm, batch=B, gamma=K, beam=beam, mode="mtad", max_context=n0 + steps * K + 2 * K + 16, prefill_rows=16,
                 device=device, warp=warp)
    lm = DecoderLM(tshape, wt)
    sp = [CachedSession(lm, list(prompt[s])) for s in range(B)]
    eng.prefill(prompt)
    _, atol = logit_tolerance(dtype)
    margin_tol = max(atol, 1e-4) * 2
    out = {"tokens": [[] for _ in range(B)], "excused": 0}
    alive = [True] * B
    for it in range(steps):
        eng.iteration_mtjd(sample_beam, seed)
        torch.cuda.synchronize()
        g = {k: getattr(eng, k).cpu().numpy() for k in ("h_tok", "h_parent", "h_cum", "out_tok", "out_cnt", "catchup_tok", "catchup_cnt")}
        dlen = eng.dkv.len.cpu().numpy()
        for s in range(B):
            if not alive[s]:
                continue
            tr = mtad.iteration_mtjd(sp[s], K=K, beam=beam, stochastic=sample_beam, seed=seed, seq_index=s, dt=np.float32, warp=warp)
            h = tr["hist"]
            for i in range(K):
                same = np.array_equal(g["h_tok"][s, i], h["tok"][i]) and np.array_equal(g["h_parent"][s, i], h["parent"][i])
                if not same:
                    assert h["margin"][i] < margin_tol or _near_tie(h["score"][i], margin_tol) or h["warp_margin"][i] < margin_tol, \
                        f"seq {s} step {it} beam step {i}: survivors differ, margin {h['margin'][i]}"
                    alive[s] = False
                    break
                close(g["h_cum"][s, i], h["score"][i], dtype, f"cum_logq step {i}")
            if not alive[s]:
                out["excused"] += 1
                continue
            assert g["out_cnt"][s] == K and list(g["out_tok"][s, :K]) == tr["emitted"]
            pend = sp[s].context[sp[s].n_cached:]
            assert dlen[s] == sp[s].n_cached and g["catchup_cnt"][s] == len(pend) and list(g["catchup_tok"][s, :len(pend)]) == pend
            _check_kv(eng.dkv, s, sp[s], dtype)
            out["tokens"][s] += tr["emitted"]
    status = _status(eng)
    eng.close()
    assert status == 0
    return out


def _near_tie(scores, tol):
    s = np.sort(np.asarray(scores, np.float64))
    return len(s) > 1 and np.min(np.diff(s)) < tol


def _status(eng):
    from paper_2407_09722_amd import binding as mb
    return mb.mtad_device_status(eng.ctx)


def _check_kv(kv, s, sess, dtype):
    n = sess.n_cached
    if n == 0:
        return
    K, V = kv.gather(s, n)
    wantK = np.stack([k[:n] for k in sess.ck])
    wantV = np.stack([v[:n] for v in sess.cv])
    # A structural check (right slot, right row after the commit gather): a wrong row is off by O(1).  float32
    # caches agree to 1e-4; half-precision caches to a few grid steps (a rounding that lands on the other side of
    # a midpoint in an earlier layer moves every later value of that token a little)
    if dtype == "fp32":
        assert np.allclose(K, wantK, rtol=1e-4, atol=1e-5) and np.allclose(V, wantV, rtol=1e-4, atol=1e-5)
    else:
        for got, want in ((K, wantK), (V, wantV)):
            assert np.all(np.abs(got - want) <= np.abs(want) * 2 ** -8 + 4e-3), float(np.abs(got - want).max())
