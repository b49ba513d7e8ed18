"""Oracle of one MTAD / MMTAD iteration and of the decoding loop.

TEST INFRASTRUCTURE (see the package header).  Steps follow Algorithm 1 of the paper
(appendix "Pseudocode of MTAD") and Section 3.3 for the multi-candidate variant, with
these readings of what the paper leaves open or misprints:

  * Algorithm 1 initialises eta to -1 and later sets it to the token id; read as: eta = 0
    when nothing passes (the bonus token then comes from the first row of P, so at least
    one token is produced, Section 3.2 item (3)) and eta = i for the longest passing prefix.
  * MTAD passes a prefix when min(1, p/q) > tau (strict, Section 3.2 and Algorithm 1);
    MMTAD passes a node when p/q** >= tau (Eq. 9).  tau = 0 is legal and passes everything.
  * All prefixes are examined: a failing prefix does not stop longer ones from passing.
  * q is the raw (unwarped) joint likelihood the beam search stored (Section 2.1), unless
    warping is asked for: then every next-token distribution of both models is warped as
    the appendix "Hyper-parameter Details" describes (keep the top_k most likely tokens
    and normalise; then, in descending order, keep the shortest prefix whose cumulative
    probability exceeds top_p; read as: and normalise again), the beam search scores with
    log q~, verification gathers log p~ (minus infinity for a draft token outside the
    target's support) and the bonus token is drawn from p~ (footnote of Section 3.2: it is
    equally valid to approximate p~ with q~).  A beam step with fewer than b candidates of
    non-zero likelihood fills the remaining beams with zero-likelihood candidates in index
    order; they can never be x**, and MMTAD judges them like any other node.
  * Deterministic beam search keeps the b best candidates (last sentence of Section 2.1);
    ties go to the lowest flat index beam*V + token; survivors are listed best first.
    Stochastic beam sampling draws b distinct candidates in proportion to p_beam (Eq. 2)
    by adding Gumbel noise to the joint log-likelihoods (the normaliser of Eq. 2 is common
    to all candidates of a step and cannot change the order).
  * x** is the final-step beam with the largest stored likelihood (Section 3.3); the
    denominator for a depth-i node is the likelihood stored at x**'s depth-i ancestor.
  * MMTAD judges every node on its own ratio; the longest passing node wins, ties go to the
    highest target likelihood (Section 3.3), then to the lowest row.
  * The bonus token is drawn from the target row of the accepted node (the root row when
    eta = 0), as argmax(logit + Gumbel noise) keyed by the token's absolute position, or as
    plain argmax in deterministic mode.

Decisions (top-b, thresholds, argmax) are taken in `dt`, float64 by default; tests that
compare integer decisions with the float32 kernels pass dt=np.float32 so that both sides
decide in the same precision.
"""
from __future__ import annotations

import numpy as np

from . import rng


def log_softmax_rows(logits):
    """Row-wise log-softmax; returns (log-probabilities, logsumexp per row)."""
    m = logits.max(axis=-1, keepdims=True)
    lse = m[..., 0] + np.log(np.exp(logits - m).sum(axis=-1))
    return logits - lse[..., None], lse


def perplexity(logp_tokens):
    """Eq. 1: exp of the mean negative log-likelihood of the generated tokens."""
    return float(np.exp(-np.mean(np.asarray(logp_tokens, dtype=np.float64))))


def warp_log_probs(logits_row, top_k, top_p, dt=np.float64):
    """log p~ of one next-token distribution (appendix "Hyper-parameter Details"): (1) the top_k most likely
    tokens keep their probabilities, the others get 0, normalise; (2) in descending order keep the first K tokens
    whose cumulative probability is larger than top_p (the smallest such K; all top_k tokens if it never is),
    the others get 0; normalise.  Equal logits rank by token id.  Sums run in descending order of probability.
    Returns (row of log p~ with -inf outside the support, margin): margin = how far the two integer decisions
    are from flipping (gap between the last kept and the first dropped logit of step 1, distance of the
    nearest cumulative probability from top_p)."""
    x = np.asarray(logits_row).astype(dt)
    V = x.size
    k = min(int(top_k), V)
    order = top_b(x, min(k + 1, V))
    gap = float(x[order[k - 1]] - x[order[k]]) if V > k else np.inf
    top = order[:k]
    e = np.exp(x[top] - x[top[0]])
    p = e / np.cumsum(e)[-1]                         # step 1: normalised over the top_k tokens
    c = np.cumsum(p)
    over = np.nonzero(c > dt(top_p))[0]
    K = int(over[0]) + 1 if over.size else k
    margin = min(gap, float(np.min(np.abs(c.astype(np.float64) - float(dt(top_p))))))
    out = np.full(V, -np.inf, dtype=dt)
    out[top[:K]] = np.log(p[:K] / np.cumsum(p[:K])[-1])
    return out, margin


def warp_rows(rows, warp, dt=np.float64):
    """warp_log_probs of every row; warp = (top_k, top_p).  Returns (rows of log p~, smallest margin)."""
    out = [warp_log_probs(r, warp[0], warp[1], dt) for r in rows]
    return np.stack([o[0] for o in out]), min(o[1] for o in out)


def top_b(keys, b):
    """Indices of the b largest keys, best first; equal keys: lowest index first."""
    keys = np.asarray(keys)
    order = np.lexsort((np.arange(keys.size), -keys))
    return order[:b]


# ---- draft: beam sampling on the auxiliary model (Section 2.1, Eq. 2) --------------------

def beam_search(session, gamma, b, *, stochastic=False, seed=0, seq_index=0, dt=np.float64, warp=None, keep_rows=False):
    """gamma beam steps from the session's context.  Returns a history dict with, per step
    i and survivor j: tok[i][j], parent[i][j] (index of the beam it extends in step i-1; 0 at
    step 0 where the only beam is the context), score[i][j] = log q(branch | context), and
    node[i][j] = the session node id (only for steps whose survivors were run, i < gamma-1)."""
    V = None
    rows, _ = session.tree_logits([], [])
    live_rows = rows[:1]
    live_score = np.zeros(1, dtype=dt)
    live_node = [-1]
    n0 = len(session.context)
    hist = {"tok": [], "parent": [], "score": [], "node": [], "margin": [], "warp_margin": [], "logq_rows": []}
    for i in range(gamma):
        logits = live_rows.astype(dt)
        V = logits.shape[1]
        if warp is None:
            _, lse = log_softmax_rows(live_rows)
            logq = logits - lse.astype(dt)[:, None]
            hist["warp_margin"].append(np.inf)
        else:
            logq, wm = warp_rows(logits, warp, dt)
            hist["warp_margin"].append(wm)
        if keep_rows:
            hist["logq_rows"].append(logq)                                   # log q(. | beam) of every live beam of this step
        cand = live_score[:, None] + logq                                    # joint log q of every extension
        flat = cand.ravel()
        if stochastic:
            g = rng.gumbel(seed, rng.stream_id(seq_index, rng.STREAM_BEAM), n0 + i, np.arange(flat.size))
            key = flat + g.astype(dt)
        else:
            key = flat
        k = min(b, flat.size)                    # a step has fewer than b candidates only if b > |V| (tests)
        sel = top_b(key, k + 1)
        with np.errstate(invalid="ignore"):
            margin = float(key[sel[k - 1]] - key[sel[k]]) if len(sel) > k else np.inf
        if not np.isfinite(margin):
            margin = np.inf if np.isfinite(key[sel[k - 1]]) else 0.0     # zero-likelihood beams: chosen by index alone
        sel = sel[:k]
        parent, tok = sel // V, sel % V
        score = flat[sel]
        pad = b - k
        hist["tok"].append(np.concatenate([tok, -np.ones(pad)]).astype(np.int32))
        hist["parent"].append(np.concatenate([parent, -np.ones(pad)]).astype(np.int32))
        hist["score"].append(np.concatenate([score, np.full(pad, -np.inf)]).astype(dt))
        hist["margin"].append(margin)
        if i < gamma - 1:
            rows, ids = session.tree_logits([live_node[p] for p in parent], tok)
            live_rows, live_node, live_score = rows[1:], ids, score
            hist["node"].append(list(ids) + [-1] * pad)
        else:
            hist["node"].append([-1] * b)
    for k in ("tok", "parent", "score"):
        hist[k] = np.stack(hist[k])
    return hist


def output_beam(hist):
    """x**: the final-step beam with the highest stored likelihood; returns the beam index
    at every depth (back-traced through the parents), its tokens and q_i = q(x**_{1:i})."""
    gamma = hist["tok"].shape[0]
    j = int(np.argmax(hist["score"][gamma - 1]))
    beams = [0] * gamma
    for i in range(gamma - 1, -1, -1):
        beams[i] = j
        j = int(hist["parent"][i][j])
    toks = [int(hist["tok"][i][beams[i]]) for i in range(gamma)]
    q = np.array([hist["score"][i][beams[i]] for i in range(gamma)])
    return beams, toks, q


def build_tree(hist, mode):
    """Rows of the target pass.  Row 0 is the root (the last context token).  MTAD: the chain
    of x**.  MMTAD: every survivor of every step, row 1 + i*b + j for step i, beam j."""
    gamma, b = hist["tok"].shape
    beams, toks, q = output_beam(hist)
    tok, parent, depth, src = [-1], [-1], [0], [-1]
    if mode == "mtad":
        for i in range(gamma):
            tok.append(toks[i]); parent.append(i); depth.append(i + 1); src.append(beams[i])
    elif mode == "mmtad":
        for i in range(gamma):
            for j in range(b):
                tok.append(int(hist["tok"][i][j]))
                parent.append(0 if i == 0 else 1 + (i - 1) * b + int(hist["parent"][i][j]))
                depth.append(i + 1); src.append(j)
    else:
        raise ValueError(mode)
    return {"tok": np.array(tok, np.int32), "parent": np.array(parent, np.int32),
            "depth": np.array(depth, np.int32), "src_beam": np.array(src, np.int32),
            "qref": q, "out_beams": beams}


def ancestor_masks(parent):
    """Bit j of mask[r] is set iff row j is r itself or an ancestor of r (the tree attention mask)."""
    masks = []
    for r in range(len(parent)):
        m, j = 0, r
        while j >= 0:
            m |= 1 << j
            j = int(parent[j])
        masks.append(m)
    return np.array(masks, dtype=np.uint64)


# ---- verification by the target model (Algorithm 1, P = M_p(input, X); Section 3.3) -------

def verify(session, tree, warp=None, dt=np.float64):
    """Target logits after the root and after every tree node, the conditional log-likelihood
    of every node's token given its branch, and the joint log p of every branch.  With warp =
    (top_k, top_p) the rows returned as "logits" are the rows of log p~ (their logsumexp is 0)."""
    M = len(tree["tok"])
    base = len(session.node_tok)                 # row r >= 1 becomes session node base + r - 1
    rows, ids = session.tree_logits([-1 if p == 0 else base + int(p) - 1 for p in tree["parent"][1:]],
                                    tree["tok"][1:])
    wm = np.inf
    if warp is None:
        logp, lse = log_softmax_rows(rows)
    else:
        rows, wm = warp_rows(np.asarray(rows).astype(dt), warp, dt)
        logp, lse = rows, np.zeros(len(rows))
    cond = np.zeros(M)
    joint = np.zeros(M)
    for c in range(1, M):
        p = int(tree["parent"][c])
        cond[c] = logp[p, tree["tok"][c]]
        joint[c] = joint[p] + cond[c]
    return {"logits": rows, "lse": lse, "logp_cond": cond, "logp_joint": joint, "node_ids": [-1] + list(ids), "warp_margin": wm}


def joint_from_cond(tree, cond, dt=np.float64):
    """Joint log-likelihood of every branch: conditionals summed from the root down."""
    M = len(tree["tok"])
    joint = np.zeros(M, dtype=dt)
    cond = np.asarray(cond, dtype=dt)
    for c in range(1, M):
        joint[c] = joint[int(tree["parent"][c])] + cond[c]
    return joint


def _log_tau(tau, dt):
    with np.errstate(divide="ignore"):
        return np.log(dt(tau)).astype(dt) if tau > 0 else dt(-np.inf)


def _margin(log_ratio, log_tau):
    """Distance of a log ratio from the threshold; infinite when either is (a zero likelihood cannot flip)."""
    d = float(log_ratio) - float(log_tau)
    return abs(d) if np.isfinite(d) else np.inf


def accept_mtad(tree, joint, tau, dt=np.float64):
    """Longest prefix i of the chain with min(1, p_i/q_i) > tau; eta = 0 if none."""
    log_tau = _log_tau(tau, dt)
    qref = np.asarray(tree["qref"], dtype=dt)
    joint = np.asarray(joint, dtype=dt)
    eta, node, margins = 0, 0, []
    for c in range(1, len(tree["tok"])):
        i = int(tree["depth"][c])
        ratio = min(dt(0), joint[c] - qref[i - 1])          # log min(1, p/q)
        margins.append(_margin(joint[c] - qref[i - 1], log_tau))
        if ratio > log_tau:
            eta, node = i, c                                  # all prefixes are examined; the longest wins
    return eta, node, margins


def accept_mmtad(tree, joint, tau, dt=np.float64):
    """Node (i, j) passes iff p(x^(j)_{1:i}) / q(x**_{1:i}) >= tau; longest, then highest p, then lowest row."""
    log_tau = _log_tau(tau, dt)
    qref = np.asarray(tree["qref"], dtype=dt)
    joint = np.asarray(joint, dtype=dt)
    best, margins = (0, -np.inf, 0), []
    for c in range(1, len(tree["tok"])):
        i = int(tree["depth"][c])
        margins.append(_margin(joint[c] - qref[i - 1], log_tau))
        if joint[c] - qref[i - 1] >= log_tau:
            if i > best[0] or (i == best[0] and joint[c] > best[1]):
                best = (i, joint[c], c)
    return best[0], best[2], margins


def branch_rows(tree, node):
    """Rows on the branch from the first level down to `node` (empty for the root)."""
    out = []
    while node > 0:
        out.append(int(node))
        node = int(tree["parent"][node])
    return out[::-1]


def bonus_token(logits_row, *, sample, seed=0, seq_index=0, position=0, dt=np.float64):
    """t ~ P_{eta+1}: argmax(logit + Gumbel) (a draw from softmax(logits)); plain argmax if not sampling.
    Returns (token, gap between the best and second-best key)."""
    key = np.asarray(logits_row).astype(dt)
    if sample:
        g = rng.gumbel(seed, rng.stream_id(seq_index, rng.STREAM_BONUS), position, np.arange(key.size))
        key = key + g.astype(dt)
    t = int(np.argmax(key))
    rest = np.delete(key, t)
    return t, float(key[t] - rest.max()) if rest.size else np.inf


# ---- one iteration and the loop -------------------------------------------------------------

def iteration(sq, sp, *, gamma, beam, mode, tau, stochastic_beam=False, sample_bonus=True, seed=0,
              seq_index=0, dt=np.float64, warp=None):
    """One iteration on draft session sq and target session sp (both hold the same context).
    Returns a trace; both sessions end with the context extended by [x_1..x_eta, t]."""
    assert sq.context == sp.context
    n = len(sp.context)
    hist = beam_search(sq, gamma, beam, stochastic=stochastic_beam, seed=seed, seq_index=seq_index, dt=dt, warp=warp)
    tree = build_tree(hist, mode)
    ver = verify(sp, tree, warp=warp, dt=dt)
    joint = joint_from_cond(tree, ver["logp_cond"].astype(dt), dt)
    eta, node, margins = (accept_mtad if mode == "mtad" else accept_mmtad)(tree, joint, tau, dt)
    rows = branch_rows(tree, node)
    t, gap = bonus_token(ver["logits"][node], sample=sample_bonus, seed=seed, seq_index=seq_index,
                         position=n + eta, dt=dt)
    accepted = _commit(sq, sp, hist, tree, ver, node, rows, eta, t, gamma)
    return {"hist": hist, "tree": tree, "verify": ver, "joint": joint, "eta": eta, "node": node,
            "path_rows": rows, "bonus": t, "bonus_gap": gap, "accept_margins": margins,
            "emitted": accepted + [t], "n_before": n}


def _commit(sq, sp, hist, tree, ver, node, rows, eta, t, gamma):
    """Both sessions take [x_1..x_eta, t]; returns the accepted tokens."""
    accepted = [int(tree["tok"][r]) for r in rows]
    sp.commit(ver["node_ids"][node] if node > 0 else None, [t])
    # the draft never ran its final-step tokens: commit what it has, hand over the rest as context
    keep = min(eta, gamma - 1)
    dnode = None
    if keep > 0:
        r = rows[keep - 1]
        dnode = hist["node"][keep - 1][int(tree["src_beam"][r])]
    sq.commit(dnode, accepted[keep:] + [t])
    return accepted


# ---- vanilla speculative decoding (Section 2.2), the baseline MTAD is compared with ---------------

def accept_tokenwise(tok, logp_rows, logq_rows, *, seed=0, seq_index=0, n=0, dt=np.float64):
    """Section 2.2 step 3: draft token x_t is accepted with probability min(1, p(x_t)/q(x_t)), each with its own
    uniform draw (keyed by the token's absolute position n + t - 1); the tokens before the first rejection are
    kept.  tok[t-1] = x_t; row t-1 of logp_rows / logq_rows is the distribution x_t was drawn from / is judged by.
    Returns (eta, margins): margin = distance of each examined draw from its threshold in the log domain."""
    gamma = len(tok)
    eta, margins = gamma, []
    for t in range(1, gamma + 1):
        u = rng.uniform(seed, rng.stream_id(seq_index, rng.STREAM_ACCEPT), n + t - 1, 0)
        log_u = np.log(dt(u))
        ratio = min(dt(0), dt(logp_rows[t - 1][tok[t - 1]]) - dt(logq_rows[t - 1][tok[t - 1]]))
        margins.append(_margin(log_u, ratio))
        if not log_u < ratio:
            eta = t - 1
            break
    return eta, margins


def residual_token(logp_row, logq_row, *, seed=0, seq_index=0, position=0, dt=np.float64):
    """The correction token after a rejection: a draw from the residual distribution norm(max(0, p - q)), as
    argmax(log weight + Gumbel noise).  Returns (token, gap between the best and second-best key)."""
    w = np.exp(np.asarray(logp_row).astype(dt)) - np.exp(np.asarray(logq_row).astype(dt))
    with np.errstate(divide="ignore"):
        key = np.where(w > 0, np.log(np.where(w > 0, w, dt(1))), dt(-np.inf)).astype(dt)
    g = rng.gumbel(seed, rng.stream_id(seq_index, rng.STREAM_BONUS), position, np.arange(key.size))
    key = key + g.astype(dt)
    t = int(np.argmax(key))
    rest = np.delete(key, t)
    return t, float(key[t] - rest.max()) if rest.size else np.inf


def iteration_spd(sq, sp, *, gamma, seed=0, seq_index=0, dt=np.float64, warp=None):
    """One iteration of vanilla speculative decoding: gamma tokens drawn one after the other from the draft model
    (beam sampling of width one is ancestral sampling), one target pass over the chain, token-wise acceptance, then the
    correction token from the residual distribution at the first rejection, or one more token from the target's next row
    if everything was accepted.  Same trace keys as `iteration`."""
    assert sq.context == sp.context
    n = len(sp.context)
    hist = beam_search(sq, gamma, 1, stochastic=True, seed=seed, seq_index=seq_index, dt=dt, warp=warp, keep_rows=True)
    tree = build_tree(hist, "mtad")
    ver = verify(sp, tree, warp=warp, dt=dt)
    logp_rows = np.asarray(ver["logits"]).astype(dt) - np.asarray(ver["lse"]).astype(dt)[:, None]
    logq_rows = [hist["logq_rows"][i][0] for i in range(gamma)]
    eta, margins = accept_tokenwise([int(t) for t in tree["tok"][1:]], logp_rows, logq_rows, seed=seed, seq_index=seq_index, n=n, dt=dt)
    if eta < gamma:
        t, gap = residual_token(logp_rows[eta], logq_rows[eta], seed=seed, seq_index=seq_index, position=n + eta, dt=dt)
    else:
        t, gap = bonus_token(logp_rows[gamma], sample=True, seed=seed, seq_index=seq_index, position=n + gamma, dt=dt)
    rows = list(range(1, eta + 1))
    accepted = _commit(sq, sp, hist, tree, ver, eta, rows, eta, t, gamma)
    return {"hist": hist, "tree": tree, "verify": ver, "joint": joint_from_cond(tree, ver["logp_cond"].astype(dt), dt), "eta": eta,
            "node": eta, "path_rows": rows, "bonus": t, "bonus_gap": gap, "accept_margins": margins, "emitted": accepted + [t],
            "n_before": n}


def iteration_mtjd(sp, *, K, beam, stochastic=False, seed=0, seq_index=0, dt=np.float64, warp=None):
    """Multi-token joint decoding (Section 3.1) as the paper runs it (Section 3.1, last paragraph: beam sampling
    approximates the draw from the joint distribution): K beam steps on the target model itself, then the K tokens of the
    final beam with the highest stored likelihood are the output.  K = 1 is single-token decoding.  The session's
    context grows by the K tokens.  Returns a trace."""
    n = len(sp.context)
    hist = beam_search(sp, K, beam, stochastic=stochastic, seed=seed, seq_index=seq_index, dt=dt, warp=warp)
    beams, toks, q = output_beam(hist)
    node = hist["node"][K - 2][beams[K - 2]] if K > 1 else None   # the last token was never run: it is handed over as context
    sp.commit(node, [toks[K - 1]])
    return {"hist": hist, "out_beams": beams, "emitted": toks, "logq": q, "n_before": n}


def autoregressive_step(sp, *, sample=True, seed=0, seq_index=0, dt=np.float64, warp=None):
    """Plain decoding with the target alone (the multinomial-sampling baseline of Section 2.2): one token from the
    target's next-token distribution (warped if asked), drawn like the bonus token of an iteration that accepted
    nothing.  Returns a trace; the session's context grows by the token."""
    n = len(sp.context)
    rows, _ = sp.tree_logits([], [])
    wm = np.inf
    if warp is not None:
        rows, wm = warp_rows(np.asarray(rows).astype(dt), warp, dt)
    t, gap = bonus_token(rows[0], sample=sample, seed=seed, seq_index=seq_index, position=n, dt=dt)
    sp.commit(None, [t])
    return {"logits": rows[0], "bonus": t, "bonus_gap": gap, "warp_margin": wm, "n_before": n}


def generate(make_sq, make_sp, prompt, new_tokens, **kw):
    """Decoding loop (Section 2.2 step 4 applied to MTAD): iterate until new_tokens tokens
    exist; the surplus of the last iteration is cut.  make_sq / make_sp build a session from
    a context.  Returns (tokens, traces)."""
    sq, sp = make_sq(list(prompt)), make_sp(list(prompt))
    out, traces = [], []
    while len(out) < new_tokens:
        tr = iteration(sq, sp, **kw)
        out += tr["emitted"]
        traces.append(tr)
    return out[:new_tokens], traces
