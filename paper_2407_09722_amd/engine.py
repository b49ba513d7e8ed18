"""Device-side harness around the C ABI: owns the torch allocations (weights, paged KV caches,
beam history, tree, accept outputs, state) and issues the calls of one MTAD/MMTAD iteration in
order.  No arithmetic of the method happens here."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as mb


def _dev(x, device):
    return torch.from_numpy(np.ascontiguousarray(x)).to(device)


class DeviceModel:
    """Weights of one decoder on the GPU plus the mtad_model descriptor pointing at them."""

    def __init__(self, shape, weights, device="cuda:0", threads=8):
        """weights: dict name -> array, or a callable name -> array (tensors are then produced a few at a
        time and dropped after the upload, so a 7B-shaped model never sits in host memory whole)."""
        self.shape = shape
        names = ["embed"]
        for l in range(shape.n_layers):
            names += [f"L{l}.{k}" for k in ("g_attn", "w_qkv", "w_o", "g_ffn", "w_gu", "w_d")]
        names += ["g_final", "unembed"]
        self.names = names

        def upload(n):
            w = weights(n) if callable(weights) else weights[n]
            if w.dtype != np.uint16:
                return _dev(w, device)
            t = _dev(w.view(np.int16), device)              # bfloat16 bit patterns; torch keeps them as raw 16-bit words
            kind = n.split(".")[-1]
            if kind == "embed":
                return t                                    # gathered by token id: stays row-major
            packed = torch.empty_like(t)                    # the layout the matrix-core kernels stream (done once)
            mode = {"w_qkv": mb.MTAD_PACK_QKV, "w_gu": mb.MTAD_PACK_GATE_UP}.get(kind, mb.MTAD_PACK_PLAIN)
            mb.mtad_pack_matrix(mode, t, packed, t.shape[0], t.shape[1], shape.head_dim)
            torch.cuda.current_stream().synchronize()
            return packed

        if callable(weights):
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=threads) as ex:
                self.tensors = list(ex.map(upload, names))
        else:
            self.tensors = [upload(n) for n in names]
        self._ptrs = (C.c_void_p * len(self.tensors))(*[t.data_ptr() for t in self.tensors])
        s = shape
        self.desc = mb.mtad_model(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab,
                                  1 if s.dtype == "bf16" else 0, s.rms_eps, s.rope_theta,
                                  C.cast(self._ptrs, C.POINTER(C.c_void_p)))

    def nbytes(self):
        return sum(t.numel() * t.element_size() for t in self.tensors)


class DeviceKV:
    """Paged KV cache of one model.  Physical pages are handed out in a seeded random order so that
    every access really goes through the page table."""

    def __init__(self, shape, batch, max_tokens, page_size=16, device="cuda:0", seed=0):
        self.shape, self.batch, self.page_size = shape, batch, page_size
        self.max_pages = (max_tokens + page_size - 1) // page_size
        self.n_pages = self.max_pages * batch
        dt = torch.float16 if shape.dtype == "bf16" else torch.float32
        dims = (shape.n_layers, self.n_pages, page_size, shape.n_kv_heads, shape.head_dim)
        self.k = torch.zeros(dims, dtype=dt, device=device)
        self.v = torch.zeros(dims, dtype=dt, device=device)
        perm = np.random.default_rng(seed).permutation(self.n_pages).astype(np.int32)
        self.page_table = _dev(perm.reshape(batch, self.max_pages), device)
        self.len = torch.zeros(batch, dtype=torch.int32, device=device)
        self.desc = mb.mtad_kv(mb.ptr(self.k), mb.ptr(self.v), mb.ptr(self.page_table), mb.ptr(self.len), page_size,
                               self.max_pages, self.n_pages)

    def gather(self, seq, n):
        """Host copy of the first n cached tokens of one sequence: (K, V) as float64 [L, n, KVH, hd]."""
        pt = self.page_table[seq].cpu().numpy()
        idx = torch.tensor([pt[t // self.page_size] * self.page_size + t % self.page_size for t in range(n)],
                           dtype=torch.long, device=self.k.device)
        out = []
        for x in (self.k, self.v):
            flat = x.reshape(x.shape[0], -1, x.shape[3], x.shape[4])[:, idx]
            out.append(flat.double().cpu().numpy())
        return out


class Engine:
    """One (target, draft) pair, one batch: buffers + the per-iteration call sequence."""

    def __init__(self, target: DeviceModel, draft: DeviceModel, *, batch, gamma, beam, mode, max_context,
                 prefill_rows=64, page_size=16, device="cuda:0", kv_seed=0, fused_pass=None, warp=None):
        self.target, self.draft = target, draft
        self.B, self.gamma, self.beam = batch, gamma, beam
        self.mode = mb.MTAD_MODE_MTAD if mode in ("mtad", 0) else mb.MTAD_MODE_MMTAD
        self.M = 1 + (gamma if self.mode == mb.MTAD_MODE_MTAD else gamma * beam)
        self.V = target.shape.vocab
        self.device = device
        cfg = mb.mtad_config(batch, gamma, beam, self.mode, prefill_rows, max_context)
        self.ctx = mb.mtad_create(cfg, target.desc, draft.desc)
        self.workspace = torch.empty(mb.mtad_workspace_bytes(self.ctx), dtype=torch.uint8, device=device)
        mb.mtad_bind_workspace(self.ctx, self.workspace)
        if fused_pass is not None:                          # 0 / False: one kernel per step; 1: one launch for large models; 2: always
            mb.mtad_set_fused_pass(self.ctx, int(fused_pass))
        if warp is not None:                                # (top_k, top_p): both models' distributions are warped
            mb.mtad_set_warp(self.ctx, warp[0], warp[1])
        self.tkv = DeviceKV(target.shape, batch, max_context, page_size, device, seed=kv_seed)
        self.dkv = DeviceKV(draft.shape, batch, max_context, page_size, device, seed=kv_seed + 1)
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        B, g, b, M = batch, gamma, beam, self.M
        self.h_tok, self.h_parent = torch.zeros(B, g, b, **i32), torch.zeros(B, g, b, **i32)
        self.h_cum = torch.zeros(B, g, b, **f32)
        self.hist = mb.mtad_beam(mb.ptr(self.h_tok), mb.ptr(self.h_parent), mb.ptr(self.h_cum))
        self.t_tok, self.t_parent, self.t_depth, self.t_src = (torch.zeros(B, M, **i32) for _ in range(4))
        self.t_mask = torch.zeros(B, M, dtype=torch.int64, device=device)
        self.t_qref = torch.zeros(B, g, **f32)
        self.tree = mb.mtad_tree(M, mb.ptr(self.t_tok), mb.ptr(self.t_parent), mb.ptr(self.t_depth), mb.ptr(self.t_src),
                                 mb.ptr(self.t_mask), mb.ptr(self.t_qref))
        self.logp_cond, self.row_lse = torch.zeros(B, M, **f32), torch.zeros(B, M, **f32)
        self.logits = torch.zeros(B, M, self.V, **f32)
        self.eta, self.bonus_row, self.bonus_tok, self.out_cnt = (torch.zeros(B, **i32) for _ in range(4))
        self.path = torch.zeros(B, g, **i32)
        self.out_tok = torch.zeros(B, g + 1, **i32)
        self.acc = mb.mtad_accept_out(mb.ptr(self.eta), mb.ptr(self.path), mb.ptr(self.bonus_row), mb.ptr(self.bonus_tok),
                                      mb.ptr(self.out_tok), mb.ptr(self.out_cnt))
        self.root_tok = torch.zeros(B, **i32)
        self.catchup_tok = torch.zeros(B, g + 1, **i32)
        self.catchup_cnt = torch.ones(B, **i32)
        self.state = mb.mtad_state(mb.ptr(self.root_tok), mb.ptr(self.catchup_tok), mb.ptr(self.catchup_cnt))

        # a one-row tree (the root alone) for plain autoregressive decoding on the same kernels
        self.ar_tok, self.ar_depth, self.ar_src = (torch.zeros(B, 1, **i32) for _ in range(3))
        self.ar_parent = torch.full((B, 1), -1, **i32)
        self.ar_mask = torch.ones(B, 1, dtype=torch.int64, device=device)
        self.ar_tree = mb.mtad_tree(1, mb.ptr(self.ar_tok), mb.ptr(self.ar_parent), mb.ptr(self.ar_depth), mb.ptr(self.ar_src),
                                    mb.ptr(self.ar_mask), mb.ptr(self.t_qref))

    def close(self):
        if self.ctx is not None:
            mb.mtad_destroy(self.ctx)
            self.ctx = None

    # -- context ------------------------------------------------------------------------------
    def prefill(self, prompt: np.ndarray, stream=None):
        """prompt int32 [B, n]: both caches take prompt[:, :n-1]; the last token becomes the root."""
        prompt = np.ascontiguousarray(prompt, dtype=np.int32)
        assert prompt.shape[0] == self.B and prompt.shape[1] >= 1
        n = prompt.shape[1]
        self.tkv.len.zero_()
        self.dkv.len.zero_()
        if n > 1:
            head = _dev(prompt[:, :n - 1], self.device)
            mb.mtad_prefill(self.ctx, self.target.desc, self.tkv.desc, head, n - 1, stream)
            mb.mtad_prefill(self.ctx, self.draft.desc, self.dkv.desc, head, n - 1, stream)
        self.set_state(prompt[:, -1], prompt[:, -1:], np.ones(self.B, np.int32))

    def set_state(self, root, catchup, cnt):
        """Host-provided state (used by lock-step tests that replay a reference context)."""
        self.root_tok.copy_(_dev(np.asarray(root, np.int32), self.device))
        cu = np.zeros((self.B, self.gamma + 1), np.int32)
        catchup = np.asarray(catchup, np.int32)
        cu[:, :catchup.shape[1]] = catchup
        self.catchup_tok.copy_(_dev(cu, self.device))
        self.catchup_cnt.copy_(_dev(np.asarray(cnt, np.int32), self.device))

    def resync(self, target_len, draft_len, target_tokens, draft_tokens, root, catchup, cnt):
        """Puts the caches and the state on a host-provided context (lock-step tests): the cache lengths are set to
        target_len / draft_len, then target_tokens / draft_tokens ([B, n], the same n for every sequence) are appended
        through the prefill path, then the state is set."""
        self.tkv.len.copy_(_dev(np.asarray(target_len, np.int32), self.device))
        self.dkv.len.copy_(_dev(np.asarray(draft_len, np.int32), self.device))
        for model, kv, toks in ((self.target, self.tkv, target_tokens), (self.draft, self.dkv, draft_tokens)):
            toks = np.ascontiguousarray(toks, dtype=np.int32).reshape(self.B, -1)
            if toks.shape[1]:
                mb.mtad_prefill(self.ctx, model.desc, kv.desc, _dev(toks, self.device), toks.shape[1], None)
        self.set_state(root, catchup, cnt)

    # -- one iteration (Algorithm 1 / Section 3.3), enqueue only ---------------------------------
    def draft_phase(self, sample_beam=False, seed=0, stream=None):
        for step in range(self.gamma):
            mb.mtad_draft_beam_step(self.ctx, self.draft.desc, self.dkv.desc, self.hist, step, self.state,
                                    int(sample_beam), seed, stream)
        mb.mtad_build_tree(self.ctx, self.hist, self.mode, self.tree, stream)

    def verify_phase(self, stream=None):
        mb.mtad_verify_tree(self.ctx, self.target.desc, self.tkv.desc, self.root_tok, self.tree, self.logp_cond,
                            self.row_lse, self.logits, stream)

    def accept_phase(self, tau, sample_bonus=True, seed=0, stream=None):
        mb.mtad_accept(self.ctx, self.tree, self.logp_cond, self.logits, self.V, self.tkv.desc, tau, self.mode,
                       int(sample_bonus), seed, self.acc, stream)

    def commit_phase(self, stream=None):
        mb.mtad_kv_commit(self.ctx, self.tkv.desc, self.dkv.desc, self.tree, self.acc, self.state, stream)

    def iteration(self, tau, sample_beam=False, sample_bonus=True, seed=0, stream=None):
        self.draft_phase(sample_beam, seed, stream)
        self.verify_phase(stream)
        self.accept_phase(tau, sample_bonus, seed, stream)
        self.commit_phase(stream)

    def accept_spd_phase(self, seed=0, stream=None):
        mb.mtad_accept_spd(self.ctx, self.tree, self.logits, self.row_lse, self.V, self.tkv.desc, seed, self.acc, stream)

    def iteration_spd(self, seed=0, stream=None):
        """One iteration of vanilla speculative decoding (Section 2.2; an engine built with beam = 1, mode "mtad"): the chain
        is drawn token by token from the draft, verified in one target pass, accepted token by token, and followed by the
        correction token (or one more target token when all passed)."""
        self.draft_phase(True, seed, stream)
        self.verify_phase(stream)
        self.accept_spd_phase(seed, stream)
        self.commit_phase(stream)

    def iteration_mtjd(self, sample_beam=False, seed=0, stream=None):
        """One step of multi-token joint decoding (Section 3.1; an engine whose draft model IS the target, mode "mtad"): gamma
        beam steps on that model, the chain of the most likely final beam is the output (`out_tok`, `out_cnt` = gamma), and
        its cache (`dkv`) takes the tokens.  The engine's target cache is not used."""
        self.draft_phase(sample_beam, seed, stream)
        mb.mtad_accept_chain(self.ctx, self.tree, self.acc, stream)
        mb.mtad_kv_commit(self.ctx, None, self.dkv.desc, self.tree, self.acc, self.state, stream)

    def iteration_autoregressive(self, sample=True, seed=0, stream=None):
        """One token of plain decoding with the target alone (the baseline MTAD is measured against, Section 2.2): a target
        pass over the root row, the token drawn from that row like a bonus token, the root's K/V committed.  The draft
        model and its cache are not touched.  Row 0 of `logits` / `row_lse` and `bonus_tok` hold the results."""
        mb.mtad_verify_tree(self.ctx, self.target.desc, self.tkv.desc, self.root_tok, self.ar_tree, self.logp_cond,
                            self.row_lse, self.logits, stream)
        mb.mtad_accept(self.ctx, self.ar_tree, self.logp_cond, self.logits, self.V, self.tkv.desc, 0.5, mb.MTAD_MODE_MTAD,
                       int(sample), seed, self.acc, stream)
        mb.mtad_kv_commit(self.ctx, self.tkv.desc, None, self.ar_tree, self.acc, self.state, stream)

    def capture_iteration(self, tau, sample_beam=False, sample_bonus=True, seed=0):
        """Records one iteration as a HIP graph and returns it (`graph.replay()` = one iteration on the current
        stream).  Everything that changes from one iteration to the next (lengths, root and catch-up tokens,
        beam history, the positions that key the random numbers) lives in device memory, and the calls allocate
        nothing, synchronise nothing and record no memset, so the same graph serves every iteration.  tau, seed and
        the two sampling switches are baked in."""
        side = torch.cuda.Stream(device=self.device)
        side.wait_stream(torch.cuda.current_stream(self.device))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            self.iteration(tau, sample_beam, sample_bonus, seed, stream=side)
        torch.cuda.current_stream(self.device).wait_stream(side)
        return graph

    def emitted(self):
        """Host copy of the tokens the last iteration produced, per sequence."""
        cnt = self.out_cnt.cpu().numpy()
        tok = self.out_tok.cpu().numpy()
        return [list(map(int, tok[s, :cnt[s]])) for s in range(self.B)]

    def generate(self, prompt, new_tokens, tau, **kw):
        """Decoding loop: iterate until every sequence has new_tokens tokens; surplus is cut."""
        self.prefill(prompt)
        out = [[] for _ in range(self.B)]
        iters = 0
        while min(len(o) for o in out) < new_tokens:
            self.iteration(tau, **kw)
            for s, e in enumerate(self.emitted()):
                out[s] += e
            iters += 1
        status = mb.mtad_device_status(self.ctx)
        if status:
            raise RuntimeError(f"device status bits {status:#x}")
        return [o[:new_tokens] for o in out], iters
