"""Pins for oracle.mtad: beam sampling, verification, acceptance, bonus token, loop.

Toy models are explicit conditional tables over tiny vocabularies, so that every
gamma-token sequence can be enumerated (the joint distribution has |V|^gamma entries,
Section 3.2) and each rule can be re-evaluated in the probability domain, the form the
paper states it in."""
import itertools

import numpy as np
import pytest
from scipy import stats

import synth_inputs as si
from oracle import mtad
from oracle.lm import CachedSession, DecoderLM, RecomputeSession, TableSession


def table_lm(V, seed, temp=1.0):
    """Next-token log-probabilities that depend on the whole history (hash of the sequence)."""
    def fn(seq):
        g = np.random.default_rng([seed, len(seq)] + [int(t) for t in seq])
        logits = g.normal(size=V) * temp
        return logits - np.log(np.exp(logits).sum())
    return fn


def joint_logprob(fn, ctx, seq):
    lp, cur = 0.0, tuple(ctx)
    for t in seq:
        lp += fn(cur)[t]
        cur += (t,)
    return lp


# ---- beam sampling (Section 2.1) -----------------------------------------------------------

def test_wide_beam_finds_the_most_likely_sequence_by_enumeration():
    V, gamma = 6, 3
    fn = table_lm(V, 1, temp=2.0)
    ctx = (2, 4)
    hist = mtad.beam_search(TableSession(fn, ctx), gamma, V ** (gamma - 1))
    _, toks, q = mtad.output_beam(hist)
    allseq = list(itertools.product(range(V), repeat=gamma))
    scores = np.array([joint_logprob(fn, ctx, s) for s in allseq])
    best = allseq[int(np.argmax(scores))]
    assert tuple(toks) == best
    assert np.isclose(q[-1], scores.max())
    # the b final survivors are exactly the b best sequences, best first
    b = V ** (gamma - 1)
    want = np.sort(scores)[::-1][:b]
    assert np.allclose(hist["score"][-1], want)
    # stored prefix likelihoods are the joint likelihoods of the prefixes (Eq. 2 numerator)
    for i in range(gamma):
        assert np.isclose(q[i], joint_logprob(fn, ctx, toks[:i + 1]))


def test_width_one_beam_is_greedy_decoding():
    V, gamma = 7, 5
    fn = table_lm(V, 2)
    hist = mtad.beam_search(TableSession(fn, (1,)), gamma, 1)
    cur, want = (1,), []
    for _ in range(gamma):
        t = int(np.argmax(fn(cur)))
        want.append(t); cur += (t,)
    assert list(hist["tok"][:, 0]) == want


def test_beam_scores_and_parents_are_consistent_joint_likelihoods():
    V, gamma, b = 5, 4, 3
    fn = table_lm(V, 3)
    hist = mtad.beam_search(TableSession(fn, (0, 1)), gamma, b)
    for i in range(gamma):
        assert np.all(np.diff(hist["score"][i]) <= 0)            # listed best first
        for j in range(b):
            seq, jj = [], j
            for k in range(i, -1, -1):
                seq.append(int(hist["tok"][k][jj])); jj = int(hist["parent"][k][jj])
            assert np.isclose(hist["score"][i][j], joint_logprob(fn, (0, 1), seq[::-1]))


def test_topb_ties_go_to_lowest_flat_index():
    assert list(mtad.top_b(np.array([1.0, 3.0, 3.0, 0.0, 3.0]), 2)) == [1, 2]


def test_stochastic_width_one_is_ancestral_sampling():
    V, gamma = 3, 2
    fn = table_lm(V, 4)
    ctx = (1,)
    allseq = list(itertools.product(range(V), repeat=gamma))
    p = np.exp([joint_logprob(fn, ctx, s) for s in allseq])
    n = 6000
    counts = np.zeros(len(allseq))
    for seed in range(n):
        hist = mtad.beam_search(TableSession(fn, ctx), gamma, 1, stochastic=True, seed=seed)
        counts[allseq.index(tuple(int(t) for t in hist["tok"][:, 0]))] += 1
    assert stats.chisquare(counts, p / p.sum() * n).pvalue > 1e-4


def test_stochastic_beam_first_draw_follows_p_beam_and_draws_are_distinct():
    V, b = 4, 3
    fn = table_lm(V, 5)
    p = np.exp(fn((0,)))
    n = 6000
    counts = np.zeros(V)
    for seed in range(n):
        hist = mtad.beam_search(TableSession(fn, (0,)), 1, b, stochastic=True, seed=seed)
        toks = list(hist["tok"][0])
        assert len(set(toks)) == b
        counts[toks[0]] += 1
    assert stats.chisquare(counts, p * n).pvalue > 1e-4


# ---- verification (Section 3.3: one pass gives every node's conditional likelihood) -------------

def test_tree_verification_equals_branchwise_enumeration():
    V, gamma, b = 5, 3, 3
    fq, fp = table_lm(V, 6), table_lm(V, 7)
    ctx = (3, 1)
    hist = mtad.beam_search(TableSession(fq, ctx), gamma, b)
    for mode in ("mtad", "mmtad"):
        tree = mtad.build_tree(hist, mode)
        ver = mtad.verify(TableSession(fp, ctx), tree)
        assert np.allclose(np.exp(ver["logits"] - ver["lse"][:, None]).sum(axis=1), 1.0)
        for c in range(1, len(tree["tok"])):
            branch = [int(tree["tok"][r]) for r in mtad.branch_rows(tree, c)]
            assert len(branch) == tree["depth"][c]
            assert np.isclose(ver["logp_joint"][c], joint_logprob(fp, ctx, branch))
        assert len(tree["tok"]) == 1 + (gamma if mode == "mtad" else gamma * b)


def test_tree_rows_and_masks():
    hist = {"tok": np.array([[5, 6], [7, 8]]), "parent": np.array([[0, 0], [1, 1]]),
            "score": np.array([[-1.0, -2.0], [-3.0, -2.5]])}
    tree = mtad.build_tree(hist, "mmtad")
    assert list(tree["parent"]) == [-1, 0, 0, 2, 2] and list(tree["depth"]) == [0, 1, 1, 2, 2]
    assert list(mtad.ancestor_masks(tree["parent"])) == [0b1, 0b11, 0b101, 0b1101, 0b10101]
    # x** = final beam 1 (score -2.5), which extends step-0 beam 1
    assert tree["out_beams"] == [1, 1] and list(tree["qref"]) == [-2.0, -2.5]
    chain = mtad.build_tree(hist, "mtad")
    assert list(chain["tok"]) == [-1, 6, 8] and list(chain["parent"]) == [-1, 0, 1]


# ---- acceptance (Section 3.2, Algorithm 1; Section 3.3 Eq. 9) -----------------------------------

def _prob_domain_mtad(p, q, tau):
    eta = 0
    for i in range(len(p)):
        if min(1.0, np.prod(p[:i + 1]) / q[i]) > tau:
            eta = i + 1
    return eta


@pytest.mark.parametrize("tau", [0.0, 0.1, 0.3, 0.5, 0.9])
def test_mtad_accept_matches_probability_domain_rule_exhaustively(tau):
    # conditional target probabilities and joint draft probabilities on a grid: every outcome pattern occurs
    grid = [0.053, 0.21, 0.49, 0.87]          # generic values: no ratio lands exactly on a threshold
    gamma = 3
    tree = {"tok": np.arange(gamma + 1), "parent": np.arange(-1, gamma), "depth": np.arange(gamma + 1)}
    seen = set()
    for pc in itertools.product(grid, repeat=gamma):
        for qc in itertools.product(grid, repeat=gamma):
            q = np.cumprod(qc)
            tree["qref"] = np.log(q)
            joint = mtad.joint_from_cond(tree, np.log([1.0] + list(pc)))
            eta, node, _ = mtad.accept_mtad(tree, joint, tau)
            assert eta == _prob_domain_mtad(np.array(pc), q, tau) and node == eta
            seen.add(eta)
    assert seen == ({gamma} if tau == 0 else set(range(gamma + 1)))


def test_a_failing_prefix_does_not_block_a_longer_one():
    tree = {"tok": np.arange(4), "parent": np.arange(-1, 3), "depth": np.arange(4),
            "qref": np.log([0.5, 0.25, 0.1])}
    joint = np.log([1.0, 0.4, 0.01, 0.09])       # ratios 0.8, 0.04, 0.9
    assert mtad.accept_mtad(tree, joint, 0.3)[0] == 3
    assert mtad.accept_mtad(tree, np.log([1.0, 0.4, 0.01, 0.001]), 0.3)[0] == 1


def test_exact_tie_is_strict_for_the_chain_rule_and_inclusive_for_the_tree_rule():
    # Algorithm 1 tests tau < min(1, p/q); Eq. 9 tests p/q** >= tau
    tree = {"tok": np.arange(2), "parent": np.array([-1, 0]), "depth": np.array([0, 1]), "qref": np.log([0.5])}
    joint = np.array([0.0, np.log(0.25)])
    assert joint[1] - tree["qref"][0] == np.log(0.5)
    assert mtad.accept_mtad(tree, joint, 0.5)[0] == 0
    assert mtad.accept_mmtad(tree, joint, 0.5)[0] == 1


def test_identical_models_accept_everything_for_every_tau():
    V, gamma, b = 6, 4, 3
    fn = table_lm(V, 8)
    for tau in (0.0, 0.3, 0.9, 0.999999):
        for mode in ("mtad", "mmtad"):
            sq, sp = TableSession(fn, (1, 2)), TableSession(fn, (1, 2))
            tr = mtad.iteration(sq, sp, gamma=gamma, beam=b, mode=mode, tau=tau, sample_bonus=False)
            assert tr["eta"] == gamma and len(tr["emitted"]) == gamma + 1
            assert sq.context == sp.context == [1, 2] + tr["emitted"]


def test_tau_zero_accepts_all_and_overconfident_draft_accepts_none():
    V, gamma = 5, 3
    fq, fp = table_lm(V, 9, temp=4.0), table_lm(V, 10, temp=0.01)     # target ~ uniform, draft peaked
    tr = mtad.iteration(TableSession(fq, (0,)), TableSession(fp, (0,)), gamma=gamma, beam=2, mode="mtad",
                        tau=0.0, sample_bonus=False)
    assert tr["eta"] == gamma
    tr = mtad.iteration(TableSession(fq, (0,)), TableSession(fp, (0,)), gamma=gamma, beam=2, mode="mtad",
                        tau=0.999, sample_bonus=False)
    assert tr["eta"] == 0 and len(tr["emitted"]) == 1
    assert tr["emitted"][0] == int(np.argmax(fp((0,))))               # bonus token from the first row of P


def test_accepted_length_bound_of_theorem_3_6():
    # |log p - log q| <= U for every conditional  =>  every prefix of length <= |log tau| / U passes
    V, gamma, U = 6, 6, 0.2
    fp = table_lm(V, 11)

    def fq(seq):
        g = np.random.default_rng([77, len(seq)] + [int(t) for t in seq])
        shifted = fp(seq) + g.uniform(-U / 2, U / 2, V)                # renormalising moves each entry by <= U/2 more
        return shifted - np.log(np.exp(shifted).sum())
    for tau in (0.3, 0.5, 0.7):
        for ctx in ((0,), (1, 2), (3, 3, 3)):
            tr = mtad.iteration(TableSession(fq, ctx), TableSession(fp, ctx), gamma=gamma, beam=2, mode="mtad",
                                tau=tau, sample_bonus=False)
            assert tr["eta"] >= min(gamma, int(np.floor(abs(np.log(tau)) / U)))


@pytest.mark.parametrize("seed", range(6))
def test_tree_accepts_at_least_as_long_as_chain_theorem_3_7(seed):
    V, gamma, b = 5, 4, 3
    fq, fp = table_lm(V, 20 + seed, temp=1.5), table_lm(V, 40 + seed, temp=0.7)
    ctx = (seed % V,)
    hist = mtad.beam_search(TableSession(fq, ctx), gamma, b)
    for tau in (0.05, 0.1, 0.3, 0.5):
        res = {}
        for mode in ("mtad", "mmtad"):
            tree = mtad.build_tree(hist, mode)
            ver = mtad.verify(TableSession(fp, ctx), tree)
            acc = mtad.accept_mtad if mode == "mtad" else mtad.accept_mmtad
            res[mode] = acc(tree, ver["logp_joint"], tau) + (tree, ver)
        assert res["mmtad"][0] >= res["mtad"][0]
        # on x** itself both rules see the same ratio (same numerator and denominator)
        tree, ver = res["mmtad"][3], res["mmtad"][4]
        chain, cver = res["mtad"][3], res["mtad"][4]
        for i in range(gamma):
            row = 1 + i * b + tree["out_beams"][i]
            assert tree["tok"][row] == chain["tok"][i + 1]
            assert np.isclose(ver["logp_joint"][row], cver["logp_joint"][i + 1])


def test_mmtad_selection_longest_then_most_likely_by_enumeration():
    g = np.random.default_rng(0)
    gamma, b = 3, 3
    parent = [-1, 0, 0, 0] + [1 + int(g.integers(b)) for _ in range(b)] + [4 + int(g.integers(b)) for _ in range(b)]
    tree = {"tok": np.arange(10), "parent": np.array(parent), "depth": np.array([0] + [1] * 3 + [2] * 3 + [3] * 3)}
    for trial in range(300):
        cond = np.log(g.uniform(0.02, 1.0, 10)); cond[0] = 0.0
        tree["qref"] = np.log(np.sort(g.uniform(0.01, 1.0, gamma))[::-1])
        tau = float(g.choice([0.1, 0.3, 0.5, 0.9]))
        joint = mtad.joint_from_cond(tree, cond)
        eta, node, _ = mtad.accept_mmtad(tree, joint, tau)
        # definition in the probability domain
        P = np.exp(joint)
        ok = [c for c in range(1, 10) if P[c] / np.exp(tree["qref"][tree["depth"][c] - 1]) >= tau]
        if not ok:
            assert (eta, node) == (0, 0)
            continue
        deepest = max(tree["depth"][c] for c in ok)
        want = max((c for c in ok if tree["depth"][c] == deepest), key=lambda c: (P[c], -c))
        assert (eta, node) == (deepest, want)


# ---- bonus token and loop -------------------------------------------------------------------

def test_bonus_token_follows_target_row():
    logits = np.array([1.0, 0.0, -0.5, 2.2])
    p = np.exp(logits) / np.exp(logits).sum()
    n = 20000
    counts = np.zeros(4)
    for pos in range(n):
        counts[mtad.bonus_token(logits, sample=True, seed=3, position=pos)[0]] += 1
    assert stats.chisquare(counts, p * n).pvalue > 1e-4
    assert mtad.bonus_token(logits, sample=False)[0] == 3


def test_loop_lengths_and_accept_invariant():
    V, gamma, b, N = 8, 4, 3, 40
    fq, fp = table_lm(V, 60, temp=1.2), table_lm(V, 61, temp=1.0)
    for mode, tau in (("mtad", 0.3), ("mmtad", 0.3), ("mtad", 0.05)):
        toks, traces = mtad.generate(lambda c: TableSession(fq, c), lambda c: TableSession(fp, c), [1, 2, 3], N,
                                     gamma=gamma, beam=b, mode=mode, tau=tau, seed=5)
        assert len(toks) == N
        flat = [t for tr in traces for t in tr["emitted"]]
        assert flat[:N] == toks
        for tr in traces:
            assert 1 <= len(tr["emitted"]) <= gamma + 1 and len(tr["emitted"]) == tr["eta"] + 1
            if tr["eta"]:                                       # premise of Lemma A.1: accepted prefix has p/q >= tau
                i = tr["eta"]
                assert tr["joint"][tr["node"]] - tr["tree"]["qref"][i - 1] >= np.log(tau) - 1e-12
        assert any(tr["eta"] > 0 for tr in traces)


def test_identical_transformers_greedy_draft_reproduce_greedy_decoding():
    """draft == target, width-1 deterministic beam, argmax bonus: every iteration emits the
    gamma+1 greedy tokens, so the loop must reproduce plain greedy decoding (cache commit included)."""
    shape = si.ModelShape(2, 32, 4, 2, 8, 48, 40, "fp32")
    w = si.make_weights(shape, 3, "target", threads=1)
    lm = DecoderLM(shape, w)
    prompt, N = [5, 9, 1], 11
    want, cur = [], list(prompt)
    for _ in range(N):
        t = int(np.argmax(lm.logits_full(cur)[-1]))
        want.append(t); cur.append(t)
    for mode in ("mtad", "mmtad"):
        got, traces = mtad.generate(lambda c: CachedSession(lm, c), lambda c: CachedSession(lm, c), prompt, N,
                                    gamma=3, beam=1, mode=mode, tau=0.5, sample_bonus=False)
        assert got == want and all(tr["eta"] == 3 for tr in traces)


def test_cached_and_recompute_sessions_give_the_same_run():
    st, sd = si.ModelShape(2, 32, 4, 2, 8, 48, 40, "bf16"), si.ModelShape(1, 16, 2, 2, 8, 24, 40, "bf16")
    lp = DecoderLM(st, si.make_weights(st, 1, "target", threads=1))
    lq = DecoderLM(sd, si.make_weights(sd, 1, "draft", threads=1))
    kw = dict(gamma=3, beam=2, mode="mmtad", tau=0.0, seed=2)
    a, ta = mtad.generate(lambda c: CachedSession(lq, c), lambda c: CachedSession(lp, c), [1, 2, 3, 4], 9, **kw)
    b, tb = mtad.generate(lambda c: RecomputeSession(lq, c), lambda c: RecomputeSession(lp, c), [1, 2, 3, 4], 9, **kw)
    assert a == b
    for x, y in zip(ta, tb):
        assert np.allclose(x["verify"]["logits"], y["verify"]["logits"], atol=1e-9)
        assert np.allclose(x["hist"]["score"], y["hist"]["score"], atol=1e-9)


def test_perplexity_eq1():
    assert np.isclose(mtad.perplexity(np.log([0.5, 0.25, 0.5])), (0.5 * 0.25 * 0.5) ** (-1 / 3))


# ---- warped distributions (appendix "Hyper-parameter Details") --------------------------------

def test_warp_worked_example_by_hand():
    """12 tokens with the probabilities below.  Step 1 keeps the ten largest (their sum is 0.99) and normalises;
    the cumulative sums 0.40, 0.65, 0.80, 0.88, 0.92 (each / 0.99) first exceed 0.9 at the fifth token, so step 2
    keeps five tokens; normalised again they are 0.40, 0.25, 0.15, 0.08, 0.04 over 0.92."""
    p = np.array([0.02, 0.40, 0.005, 0.25, 0.01, 0.15, 0.08, 0.01, 0.04, 0.02, 0.01, 0.005])
    assert np.isclose(p.sum(), 1.0)
    lw, margin = mtad.warp_log_probs(np.log(p) + 2.5, 10, 0.9)       # any shift of the logits: the same distribution
    want = np.zeros(12)
    want[[1, 3, 5, 6, 8]] = np.array([0.40, 0.25, 0.15, 0.08, 0.04]) / 0.92
    assert np.allclose(np.exp(lw), want, atol=1e-12)
    assert np.all(np.isneginf(lw[want == 0]))
    assert np.isclose(margin, (0.88 / 0.99 - 0.9) * -1)             # the nearest cumulative sum is 0.88/0.99


def test_warp_support_matches_exact_rational_arithmetic():
    """Probabilities that are ratios of integers: the two integer decisions (which top_k tokens, how long the top_p
    prefix) are recomputed with exact fractions; the kept tokens keep their mutual ratios and sum to one."""
    from fractions import Fraction
    g = np.random.default_rng(5)
    for trial in range(200):
        V = int(g.integers(3, 40))
        top_k = int(g.integers(1, 14))
        top_p = Fraction(int(g.integers(1, 20)), 20)               # 0.05 .. 0.95
        n = g.permutation(np.arange(1, 5 * V + 1))[:V].astype(np.int64)   # distinct counts: no ties
        if trial % 4 == 0:
            n[int(g.integers(V))] = 50 * n.sum()                    # one token above every threshold: support of one
        lw, _ = mtad.warp_log_probs(np.log(n.astype(np.float64)), top_k, float(top_p))
        order = sorted(range(V), key=lambda i: -n[i])[:min(top_k, V)]
        tot = sum(int(n[i]) for i in order)
        cum, K = Fraction(0), len(order)
        for r, i in enumerate(order):
            cum += Fraction(int(n[i]), tot)
            if cum > top_p:
                K = r + 1
                break
        keep = order[:K]
        if any(abs(float(sum(Fraction(int(n[i]), tot) for i in order[:r + 1]) - top_p)) < 1e-9 for r in range(len(order))):
            continue                                                 # a cumulative sum exactly on the threshold: either side is rounding
        assert sorted(np.nonzero(np.isfinite(lw))[0]) == sorted(keep), (trial, V, top_k, top_p)
        kept = sum(int(n[i]) for i in keep)
        for i in keep:
            assert np.isclose(np.exp(lw[i]), n[i] / kept, rtol=1e-12)


def test_warp_ties_rank_by_token_id_and_short_vocabularies():
    lw, _ = mtad.warp_log_probs(np.zeros(6), 3, 0.99)               # six equal tokens, keep three: ids 0, 1, 2
    assert list(np.nonzero(np.isfinite(lw))[0]) == [0, 1, 2] and np.allclose(np.exp(lw[:3]), 1 / 3)
    lw, _ = mtad.warp_log_probs(np.array([0.3, -1.0]), 10, 0.5)     # fewer tokens than top_k
    assert np.isfinite(lw[0]) and np.isneginf(lw[1]) and lw[0] == 0.0


def test_warp_that_keeps_everything_is_the_unwarped_method():
    """top_k = |V| and a top_p no cumulative sum exceeds keep every token: p~ = p, and the warped iteration takes the
    decisions of the plain one (scores agree to rounding)."""
    V, gamma = 9, 3
    fq, fp = table_lm(V, 41, temp=1.5), table_lm(V, 42, temp=1.5)
    for mode in ("mtad", "mmtad"):
        for seed in range(5):
            kw = dict(gamma=gamma, beam=3, mode=mode, tau=0.3, stochastic_beam=True, sample_bonus=True, seed=seed)
            a = mtad.iteration(TableSession(fq, (1, 2)), TableSession(fp, (1, 2)), **kw)
            b = mtad.iteration(TableSession(fq, (1, 2)), TableSession(fp, (1, 2)), warp=(V, 1.5), **kw)
            assert np.array_equal(a["hist"]["tok"], b["hist"]["tok"]) and np.array_equal(a["hist"]["parent"], b["hist"]["parent"])
            assert np.allclose(a["hist"]["score"], b["hist"]["score"]) and np.allclose(a["joint"], b["joint"])
            assert a["eta"] == b["eta"] and a["node"] == b["node"] and a["emitted"] == b["emitted"]


def test_warped_iteration_stays_inside_the_supports():
    """Every drafted token lies in the draft's warped support of its step (finite score) as long as the beam is no
    wider than the support; a drafted token outside the target's support has zero target likelihood and cannot pass
    a positive threshold; the bonus token lies in the target's support of its row."""
    V, gamma, b = 30, 4, 2
    fq, fp = table_lm(V, 51, temp=3.0), table_lm(V, 52, temp=3.0)
    seen_reject = False
    for seed in range(40):
        tr = mtad.iteration(TableSession(fq, (3,)), TableSession(fp, (3,)), gamma=gamma, beam=b, mode="mmtad", tau=0.05,
                            stochastic_beam=True, sample_bonus=True, seed=seed, warp=(4, 0.8))
        assert np.isfinite(tr["verify"]["logits"][tr["node"], tr["bonus"]])
        finite = np.isfinite(tr["verify"]["logits"]).sum(axis=1)
        assert np.all(finite >= 1) and np.all(finite <= 4)
        assert np.allclose(np.exp(tr["verify"]["logits"]).sum(axis=1), 1.0)
        for c in range(1, len(tr["tree"]["tok"])):
            if np.isneginf(tr["joint"][c]):
                seen_reject = True
                assert c not in tr["path_rows"]
        for r in tr["path_rows"]:
            assert np.isfinite(tr["joint"][r])
    assert seen_reject


def test_autoregressive_step_is_ancestral_sampling_from_the_target():
    """Greedy: the argmax chain.  Sampled: first tokens over many seeds follow the target's first-row distribution
    (chi-square), warped or not."""
    V = 6
    fp = table_lm(V, 61, temp=1.5)
    sess = TableSession(fp, (2,))
    toks = [mtad.autoregressive_step(sess, sample=False)["bonus"] for _ in range(4)]
    cur = (2,)
    for t in toks:
        assert t == int(np.argmax(fp(cur)))
        cur += (t,)
    for warp in (None, (3, 0.95)):
        p = np.exp(fp((2,)))
        if warp:
            p = np.exp(mtad.warp_log_probs(fp((2,)), *warp)[0])
        N = 4000
        counts = np.zeros(V)
        for seed in range(N):
            counts[mtad.autoregressive_step(TableSession(fp, (2,)), sample=True, seed=seed, warp=warp)["bonus"]] += 1
        keep = p > 0
        assert np.all(counts[~keep] == 0)
        assert stats.chisquare(counts[keep], p[keep] * N).pvalue > 1e-3


# ---- vanilla speculative decoding (Section 2.2) ---------------------------------------------------

def test_speculative_decoding_keeps_the_target_distribution():
    """The property the method is built on (Section 2.2, last sentence: an identical sampling distribution): the first
    token an iteration emits, whether an accepted draft token or the correction token, follows the target's next-token
    distribution, for an unrelated draft model, warped or not; and so does the pair of the first two tokens."""
    V, gamma = 5, 3
    fq, fp = table_lm(V, 71, temp=1.5), table_lm(V, 72, temp=1.5)
    ctx = (1, 3)
    for warp in (None, (3, 0.95)):
        def dist(fn, c):
            lp = fn(c)
            return np.exp(mtad.warp_log_probs(lp, *warp)[0]) if warp else np.exp(lp)
        N = 6000
        first = np.zeros(V)
        pair = np.zeros((V, V))
        n_pair = 0
        for seed in range(N):
            tr = mtad.iteration_spd(TableSession(fq, ctx), TableSession(fp, ctx), gamma=gamma, seed=seed, warp=warp)
            first[tr["emitted"][0]] += 1
            if len(tr["emitted"]) >= 2:
                pair[tr["emitted"][0], tr["emitted"][1]] += 1
                n_pair += 1
        p1 = dist(fp, ctx)
        keep = p1 > 0
        assert np.all(first[~keep] == 0)
        assert stats.chisquare(first[keep], p1[keep] * N).pvalue > 1e-3
        # second token given the first: rows of the conditional table, each tested on its own sample
        for a in np.nonzero(keep)[0]:
            na = pair[a].sum()
            if na < 200:
                continue
            p2 = dist(fp, ctx + (int(a),))
            k2 = p2 > 0
            assert np.all(pair[a][~k2] == 0)
            # an iteration that rejects its first token emits one token only: among iterations that emit two, the second
            # token still follows the target given the first (the first was accepted, the second is accepted or corrected)
            assert stats.chisquare(pair[a][k2], p2[k2] * na).pvalue > 1e-4


def test_speculative_decoding_special_cases():
    """Identical models: every ratio is one, every token passes.  A draft whose mass lies where the target has none:
    the first token is always rejected and the correction is a plain draw from the target (the residual is p)."""
    V, gamma = 6, 4
    fn = table_lm(V, 81)
    for seed in range(20):
        tr = mtad.iteration_spd(TableSession(fn, (0,)), TableSession(fn, (0,)), gamma=gamma, seed=seed)
        assert tr["eta"] == gamma and len(tr["emitted"]) == gamma + 1
    def fq(seq):
        lp = np.full(V, -60.0); lp[:3] = np.log(1 / 3); return lp
    def fp(seq):
        lp = np.full(V, -60.0); lp[3:] = np.log(np.array([0.5, 0.3, 0.2])); return lp
    counts = np.zeros(V)
    for seed in range(3000):
        tr = mtad.iteration_spd(TableSession(fq, (0,)), TableSession(fp, (0,)), gamma=gamma, seed=seed)
        assert tr["eta"] == 0 and len(tr["emitted"]) == 1
        counts[tr["bonus"]] += 1
    assert np.all(counts[:3] == 0)
    assert stats.chisquare(counts[3:], np.array([0.5, 0.3, 0.2]) * 3000).pvalue > 1e-3


# ---- multi-token joint decoding (Section 3.1) -------------------------------------------------------

def test_mtjd_with_a_wide_beam_emits_the_most_likely_block_by_enumeration():
    """Deterministic, beam wide enough to hold every prefix: each iteration emits the K-token block with the highest
    joint likelihood under the model given everything emitted so far (all |V|^K blocks enumerated), twice in a row."""
    V, K = 5, 3
    fn = table_lm(V, 91, temp=2.0)
    sess = TableSession(fn, (4, 0))
    ctx = (4, 0)
    for _ in range(2):
        tr = mtad.iteration_mtjd(sess, K=K, beam=V ** (K - 1))
        blocks = list(itertools.product(range(V), repeat=K))
        scores = [joint_logprob(fn, ctx, b) for b in blocks]
        assert tuple(tr["emitted"]) == blocks[int(np.argmax(scores))]
        assert np.isclose(tr["logq"][-1], max(scores))
        ctx += tuple(tr["emitted"])
        assert tuple(sess.context) == ctx


def test_mtjd_with_one_token_per_step_is_single_token_decoding():
    """K = 1 (Section 3.1: equivalent to multinomial sampling): deterministic = greedy, stochastic = a draw from p."""
    V = 6
    fn = table_lm(V, 92, temp=1.5)
    sess = TableSession(fn, (1,))
    cur = (1,)
    for _ in range(3):
        t = mtad.iteration_mtjd(sess, K=1, beam=1)["emitted"]
        assert t == [int(np.argmax(fn(cur)))]
        cur += (t[0],)
    N, counts = 4000, np.zeros(V)
    for seed in range(N):
        counts[mtad.iteration_mtjd(TableSession(fn, (1,)), K=1, beam=1, stochastic=True, seed=seed)["emitted"][0]] += 1
    assert stats.chisquare(counts, np.exp(fn((1,))) * N).pvalue > 1e-3


def test_mtjd_blocks_are_at_least_as_likely_as_greedy_blocks():
    """The point of Section 3.1 on seeded tables: the block a width-4 beam chooses jointly is at least as likely as the greedy
    block (not a theorem for a finite beam: a fixed set of cases)."""
    V, K = 8, 4
    for seed in range(10):
        fn = table_lm(V, 100 + seed, temp=2.5)
        a = mtad.iteration_mtjd(TableSession(fn, (0,)), K=K, beam=4)
        g = mtad.iteration_mtjd(TableSession(fn, (0,)), K=K, beam=1)
        assert joint_logprob(fn, (0,), a["emitted"]) >= joint_logprob(fn, (0,), g["emitted"]) - 1e-12
