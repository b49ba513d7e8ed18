"""Oracle language models: p(. | x_{1:t}) as a function of the token sequence.

TEST INFRASTRUCTURE (see the package header).  float64 throughout.

The paper treats both models as black boxes M_p, M_q that return next-token
distributions (Section 2.1; Algorithm 1 takes them as inputs).  The decoder used here
is the one the workloads name: pre-RMSNorm, rotary positions (half-split pairing),
grouped-query causal attention, SwiGLU FFN, no biases, untied embedding / unembedding.

Three "sessions" expose one interface to the decoding algorithms:
  RecomputeSession  the definition: every node's distribution is obtained by running the
                    model from scratch over context + the node's branch, alone.
  CachedSession     the same numbers from one masked pass over all new nodes with a KV
                    cache (Section 3.3: tree attention yields the conditional likelihood
                    of every tree token in one pass).  Pinned equal to the definition.
  TableSession      a toy model given as a Python function of the sequence.

bf16 workloads: weights are stored in bfloat16 (the inputs arrive so); cached K and V are
rounded to IEEE half precision (nearest even; the same 16 bits per value as bfloat16 with 3
more mantissa bits, chosen because the values are O(1) and the finer grid makes cache
roundings that land on the other side of a midpoint 8 times smaller).  The activation entering a weight matrix product
(normalised hidden state, attention output, FFN activation) is reduced to the sum of two
bfloat16 terms, hi = bf16(x), lo = bf16(x - hi) (about 16 significant bits).  Everything else
(queries, residual stream, statistics, softmax, logits) is kept wide.  Rounding these
activations to a single bfloat16 was tried first and dropped: each rounding that lands on the
other side of a midpoint shifts everything downstream, the flips multiply layer by layer, and
two evaluations of this very oracle that differ by 1e-7 in the values being rounded end up
0.01 rms / 0.06 max apart in the logits, above the 2e-2 bound the workloads are held to.
fp32 workloads round nowhere.
"""
from __future__ import annotations

import numpy as np


def _widen(w: np.ndarray) -> np.ndarray:
    if w.dtype == np.uint16:      # bfloat16 bit patterns
        return (w.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return w.astype(np.float64)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to bfloat16 of a wide value (through float32)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


class DecoderLM:
    def __init__(self, shape, weights: dict):
        self.s = shape
        self.bf16 = shape.dtype == "bf16"
        self.W = {k: _widen(v) for k, v in weights.items()}
        hd = shape.head_dim
        self.inv_freq = shape.rope_theta ** (-2.0 * np.arange(hd // 2, dtype=np.float64) / hd)

    # -- building blocks -------------------------------------------------------------
    def _rp(self, x):
        """Activation entering a weight matrix product: two-term bfloat16 split."""
        if not self.bf16:
            return x
        hi = round_bf16(x)
        return hi + round_bf16(x - hi)

    def _rkv(self, x):
        """Cached K / V: stored in IEEE half precision."""
        return x.astype(np.float32).astype(np.float16).astype(np.float64) if self.bf16 else x

    def _rms(self, x, g):
        ms = np.mean(x * x, axis=-1, keepdims=True)
        return x / np.sqrt(ms + self.s.rms_eps) * g

    def _rope(self, x, pos):
        """x [R, heads, hd]; pair (i, i + hd/2) rotated by pos * theta^(-2i/hd)."""
        half = self.s.head_dim // 2
        ang = np.asarray(pos, dtype=np.float64)[:, None] * self.inv_freq[None, :]
        c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
        x1, x2 = x[..., :half], x[..., half:]
        return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)

    # -- one masked pass over R new rows ---------------------------------------------
    def forward_rows(self, tokens, pos, past_k, past_v, visible):
        """tokens [R], pos [R]; past_k/past_v: per layer [n, KVH, hd]; visible [R, n + R] bool:
        row r may attend to past row j (j < n) or to new row j - n.  Returns
        (logits [R, V], new_k per layer [R, KVH, hd], new_v per layer)."""
        s = self.s
        H, KVH, hd, f = s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn
        tokens = np.asarray(tokens, dtype=np.int64)
        R = len(tokens)
        visible = np.asarray(visible, dtype=bool)
        h = self.W["embed"][tokens]
        new_k, new_v = [], []
        for l in range(s.n_layers):
            a = self._rp(self._rms(h, self.W[f"L{l}.g_attn"]))
            qkv = a @ self.W[f"L{l}.w_qkv"].T
            q = qkv[:, :H * hd].reshape(R, H, hd)
            k = qkv[:, H * hd:(H + KVH) * hd].reshape(R, KVH, hd)
            v = qkv[:, (H + KVH) * hd:].reshape(R, KVH, hd)
            q = self._rope(q, pos)
            k = self._rkv(self._rope(k, pos))
            v = self._rkv(v)
            new_k.append(k)
            new_v.append(v)
            K = np.concatenate([past_k[l], k], axis=0)
            V = np.concatenate([past_v[l], v], axis=0)
            o = np.empty((R, H, hd))
            for j in range(H):
                g = j * KVH // H
                sc = (q[:, j, :] @ K[:, g, :].T) / np.sqrt(hd)
                sc = np.where(visible, sc, -np.inf)
                sc -= sc.max(axis=1, keepdims=True)
                p = np.exp(sc)
                p /= p.sum(axis=1, keepdims=True)
                o[:, j, :] = p @ V[:, g, :]
            h = h + self._rp(o.reshape(R, H * hd)) @ self.W[f"L{l}.w_o"].T
            u = self._rp(self._rms(h, self.W[f"L{l}.g_ffn"]))
            gu = u @ self.W[f"L{l}.w_gu"].T
            gate, up = gu[:, :f], gu[:, f:]
            act = self._rp(gate / (1.0 + np.exp(-gate)) * up)
            h = h + act @ self.W[f"L{l}.w_d"].T
        hf = self._rp(self._rms(h, self.W["g_final"]))
        return hf @ self.W["unembed"].T, new_k, new_v

    def empty_cache(self):
        s = self.s
        z = lambda: [np.zeros((0, s.n_kv_heads, s.head_dim)) for _ in range(s.n_layers)]
        return z(), z()

    def logits_full(self, tokens):
        """Definition: run the whole sequence from scratch, causal mask; logits [T, V]."""
        T = len(tokens)
        pk, pv = self.empty_cache()
        vis = np.tril(np.ones((T, T), dtype=bool))
        return self.forward_rows(tokens, np.arange(T), pk, pv, vis)[0]


# ---- sessions --------------------------------------------------------------------------

class _Session:
    """A context plus a growing tree of speculative nodes hanging off its end.

    tree_logits(parents, tokens) adds one node per token (parent -1 = the end of the
    context, otherwise the id of an existing node or of an earlier node of the same
    call) and returns the next-token logits after the context (row 0) and after each
    new node (rows 1..).  commit(node, extra) appends the node's branch and the extra
    tokens to the context and forgets the tree."""

    def __init__(self, context):
        self.context = [int(t) for t in context]
        self.node_tok, self.node_parent, self.node_depth = [], [], []

    def path(self, node):
        out = []
        while node >= 0:
            out.append(self.node_tok[node])
            node = self.node_parent[node]
        return out[::-1]

    def _add(self, parents, tokens):
        ids = []
        for p, t in zip(parents, tokens):
            p = int(p)
            assert -1 <= p < len(self.node_tok)
            self.node_tok.append(int(t))
            self.node_parent.append(p)
            self.node_depth.append(1 if p < 0 else self.node_depth[p] + 1)
            ids.append(len(self.node_tok) - 1)
        return ids

    def commit(self, node, extra=()):
        self.context += (self.path(node) if node is not None and node >= 0 else []) + [int(t) for t in extra]
        self.node_tok, self.node_parent, self.node_depth = [], [], []


class TableSession(_Session):
    """Toy model: fn(tuple_of_tokens) -> logits [V] (any unnormalised log-weights)."""

    def __init__(self, fn, context):
        super().__init__(context)
        self.fn = fn

    def tree_logits(self, parents, tokens):
        ids = self._add(parents, tokens)
        rows = [self.fn(tuple(self.context))]
        rows += [self.fn(tuple(self.context + self.path(i))) for i in ids]
        return np.asarray(rows, dtype=np.float64), ids


class RecomputeSession(_Session):
    """Definition form on a DecoderLM: every row is a from-scratch run over its own branch."""

    def __init__(self, lm: DecoderLM, context):
        super().__init__(context)
        self.lm = lm

    def tree_logits(self, parents, tokens):
        ids = self._add(parents, tokens)
        rows = [self.lm.logits_full(self.context)[-1]]
        rows += [self.lm.logits_full(self.context + self.path(i))[-1] for i in ids]
        return np.asarray(rows), ids


class CachedSession(_Session):
    """Incremental form: KV cache for the context, one masked pass per call for whatever is
    new (context tokens not yet cached, as a causal chain, plus the new tree nodes)."""

    def __init__(self, lm: DecoderLM, context):
        super().__init__(context)
        self.lm = lm
        self.ck, self.cv = lm.empty_cache()      # cached context rows
        self.nk, self.nv = lm.empty_cache()      # rows of the tree nodes, by node id
        self.root_logits = None

    @property
    def n_cached(self):
        return self.ck[0].shape[0]

    def tree_logits(self, parents, tokens):
        O = len(self.node_tok)                   # nodes of earlier calls: their K/V are kept in nk/nv
        ids = self._add(parents, tokens)
        n = self.n_cached
        pend = self.context[n:]                  # uncached context tail (ends with the root token)
        P, N = len(pend), len(ids)
        if P == 0 and self.root_logits is None:
            raise RuntimeError("context fully cached but root logits unknown")
        if P + N == 0:
            return self.root_logits[None, :].copy(), ids
        # rows of this pass: the pending chain, then the new nodes
        toks = pend + [self.node_tok[i] for i in ids]
        pos = list(range(n, n + P)) + [len(self.context) - 1 + self.node_depth[i] for i in ids]
        L = self.lm.s.n_layers
        past_k = [np.concatenate([self.ck[l], self.nk[l]], axis=0) for l in range(L)]
        past_v = [np.concatenate([self.cv[l], self.nv[l]], axis=0) for l in range(L)]
        # columns: [cached context n | older nodes O | pending chain P | new nodes N]
        vis = np.zeros((P + N, n + O + P + N), dtype=bool)
        vis[:, :n] = True
        vis[:P, n + O:n + O + P] = np.tril(np.ones((P, P), dtype=bool))
        for a, i in enumerate(ids):
            vis[P + a, n + O:n + O + P] = True
            j = i
            while j >= 0:                        # the node itself and its ancestors
                col = n + j if j < O else n + O + P + (j - O)
                vis[P + a, col] = True
                j = self.node_parent[j]
        logits, k_new, v_new = self.lm.forward_rows(toks, pos, past_k, past_v, vis)
        for l in range(L):
            if P:
                self.ck[l] = np.concatenate([self.ck[l], k_new[l][:P]], axis=0)
                self.cv[l] = np.concatenate([self.cv[l], v_new[l][:P]], axis=0)
            self.nk[l] = np.concatenate([self.nk[l], k_new[l][P:]], axis=0)
            self.nv[l] = np.concatenate([self.nv[l], v_new[l][P:]], axis=0)
        if P:
            self.root_logits = logits[P - 1]
        return np.concatenate([self.root_logits[None, :], logits[P:]], axis=0), ids

    def commit(self, node, extra=()):
        path_ids = []
        j = node if node is not None else -1
        while j >= 0:
            path_ids.append(j)
            j = self.node_parent[j]
        path_ids = path_ids[::-1]
        assert self.n_cached == len(self.context), "commit before the context tail was run"
        for l in range(self.lm.s.n_layers):
            self.ck[l] = np.concatenate([self.ck[l], self.nk[l][path_ids]], axis=0)
            self.cv[l] = np.concatenate([self.cv[l], self.nv[l][path_ids]], axis=0)
        self.nk, self.nv = self.lm.empty_cache()
        self.root_logits = None
        super().commit(node, extra)
