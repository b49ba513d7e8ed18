"""GPU parity at the real widths of the large workloads (reduced depth so that the float64 oracle stays
within a minute), and kernel-level decision tests fed the oracle's own float32 inputs."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import mtad
from tests._parity import run_pair

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(name, t_layers, d_layers, prompt_len, batch=None):
    w = si.reduced(si.WORKLOADS[name], t_layers, d_layers, prompt_len=prompt_len, batch=batch)
    wt = si.make_weights(w.target, w.seed, "target", threads=16)
    wd = si.make_weights(w.draft, w.seed, "draft", threads=16)
    return w, wt, wd


def test_c3_widths_two_layers_full_prompt():
    """7B-shaped target (d 4096, 32 heads of 128, FFN 11008, vocab 32000), chain of 5 rows, prompt 512."""
    w, wt, wd = _pair("C3", 2, 2, 512)
    print("C3-L2 oracle + GPU", flush=True)
    st = run_pair(w.target, w.draft, wt, wd, si.make_prompt(w), 8, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=w.tau, seed=w.seed,
                  lockstep=True)
    print(f"C3-L2: {st['iters']} iterations, {st['excused']} put back on the oracle's context, max logit err {st['max_logit_err']:.2e}, parted: {st['events']}")
    assert st["iters"] >= 4 and st["iters"] - st["excused"] >= 3 and len(st["tokens"][0]) >= 8
    # the runs may part only at a genuine near-tie: margin of the decision at the level of the measured error
    assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


def test_c4_widths_tree_of_17_rows():
    """Same widths, MMTAD: 4 beams x gamma 4 = 16 nodes + root under the tree mask; tau = 0 exercises the commit gather."""
    w, wt, wd = _pair("C4", 2, 2, 300)
    for tau in (w.tau, 0.0):
        print(f"C4-L2 tau={tau}", flush=True)
        st = run_pair(w.target, w.draft, wt, wd, si.make_prompt(w), 8, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=tau, seed=w.seed,
                      lockstep=True)
        assert st["iters"] - st["excused"] >= 2 and len(st["tokens"][0]) >= 8
        print(f"C4-L2 tau={tau}: {st['iters']} iterations, {st['excused']} put back on the oracle's context, mean eta {np.mean(st['eta']):.2f}, max logit err {st['max_logit_err']:.2e}, parted: {st['events']}")
        assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


@pytest.mark.parametrize("gamma,beam,mode", [(8, 2, "mtad"), (4, 3, "mmtad"), (7, 2, "mtad"), (3, 1, "mtad")])
def test_c3_widths_other_row_counts(gamma, beam, mode):
    """The same widths at 9 rows (two row groups on the three-strip product kernel), 13 rows (tree), 8 rows (a full row
    group) and 4 rows (the fewest rows that kernel takes): every fused epilogue at those shapes against the oracle."""
    w, wt, wd = _pair("C3", 1, 1, 96)
    print(f"C3-L1 gamma={gamma} beam={beam} {mode}", flush=True)
    st = run_pair(w.target, w.draft, wt, wd, si.make_prompt(w), 4, gamma=gamma, beam=beam, mode=mode, tau=0.0, seed=w.seed, max_iters=2)
    print(f"C3-L1 gamma={gamma} beam={beam} {mode}: max logit err {st['max_logit_err']:.2e}, parted: {st['events']}")
    assert st["iters"] >= 1
    assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


def test_c5_widths_batch4_tree_of_41_rows_gqa_draft():
    """13B-shaped target (d 5120, 40 heads), GQA draft (32 heads, 4 kv heads), batch 4, 8 beams x gamma 5 = 40 nodes + root."""
    w, wt, wd = _pair("C5", 1, 1, 70)
    print("C5-L1", flush=True)
    st = run_pair(w.target, w.draft, wt, wd, si.make_prompt(w), 6, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=0.0, seed=w.seed,
                  max_iters=2)
    print(f"C5-L1: max logit err {st['max_logit_err']:.2e}, parted: {st['events']}")
    assert st["iters"] >= 1
    assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


@pytest.mark.parametrize("mode", ["mtad", "mmtad"])
def test_long_context_with_more_key_splits_than_compute_units_need(mode):
    """12 heads of 128 x 8 sequences = 96 attention work items: three key splits already give every compute unit a
    workgroup, unevenly (288 on 256), so a context of more than 2048 keys is cut into four (the splits that fill the
    resident slots), with 5 rows (one row group per item) and with 17 (two)."""
    t = si.ModelShape(1, 1536, 12, 12, 128, 1536, 1024, "bf16")
    d = si.ModelShape(1, 256, 4, 4, 64, 512, 1024, "bf16")
    w = si.Workload("long", t, d, seed=11, batch=8, prompt_len=2100, new_tokens=4, gamma=4, beam=4, mode=mode, tau=0.0)
    wt = si.make_weights(t, w.seed, "target", threads=16)
    wd = si.make_weights(d, w.seed, "draft", threads=16)
    print(f"long context {mode}", flush=True)
    st = run_pair(t, d, wt, wd, si.make_prompt(w), 4, gamma=w.gamma, beam=w.beam, mode=mode, tau=0.0, seed=w.seed, max_iters=2,
                  prefill_rows=32)  # 8 sequences x 32 rows: the most a pass holds
    print(f"long context {mode}: max logit err {st['max_logit_err']:.2e}, parted: {st['events']}")
    assert st["iters"] >= 1
    assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


def test_attention_items_of_c4_32_rows_per_item_8_key_splits_over_2048_keys():
    """The attention launch of C4's verify step: 32 KV heads of 128 x 1 sequence = 32 work items of 17 rows (two 16-row
    groups per item), a context of more than 2048 keys cut into 8 splits (what fills 256 compute units from 32 items),
    then the split merge.  A one-layer model of those heads on a narrow residual stream keeps the oracle to seconds."""
    t = si.ModelShape(1, 512, 32, 32, 128, 512, 1024, "bf16")
    d = si.ModelShape(1, 256, 4, 4, 64, 512, 1024, "bf16")
    w = si.Workload("c4attn", t, d, seed=12, batch=1, prompt_len=2080, new_tokens=10, gamma=4, beam=4, mode="mmtad", tau=0.0)
    wt, wd = si.make_weights(t, w.seed, "target", threads=16), si.make_weights(d, w.seed, "draft", threads=16)
    print("attention at C4's item shape", flush=True)
    st = run_pair(t, d, wt, wd, si.make_prompt(w), 10, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=0.0, seed=w.seed, max_iters=2,
                  max_context=2048 + 128 + 17)
    print(f"attention at C4's item shape: max logit err {st['max_logit_err']:.2e}, parted: {st['events']}")
    assert st["iters"] >= 1 and st["max_logit_err"] > 0
    assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


def test_attention_items_of_c5_48_rows_per_item_3_key_splits_over_4096_keys():
    """The attention launch of C5's verify step: 40 KV heads of 128 x 4 sequences = 160 work items of 41 rows (three
    16-row groups per item), a context of more than 4096 keys in 3 splits (480 workgroups: every resident slot of 256
    compute units at two per unit).  The four sequences carry one prompt and the run is deterministic, so one oracle run
    (float64 attention over 4100 x 4100 scores per head) serves all four: sequence 0 is compared with the oracle,
    the other three with sequence 0."""
    t = si.ModelShape(1, 256, 40, 40, 128, 256, 1024, "bf16")
    d = si.ModelShape(1, 256, 4, 4, 64, 512, 1024, "bf16")
    w = si.Workload("c5attn", t, d, seed=13, batch=1, prompt_len=4100, new_tokens=6, gamma=5, beam=8, mode="mmtad", tau=0.0)
    wt, wd = si.make_weights(t, w.seed, "target", threads=16), si.make_weights(d, w.seed, "draft", threads=16)
    prompt = np.repeat(si.make_prompt(w), 4, axis=0)
    print("attention at C5's item shape", flush=True)
    st = run_pair(t, d, wt, wd, prompt, 6, gamma=w.gamma, beam=w.beam, mode=w.mode, tau=0.0, sample_bonus=False, seed=w.seed, max_iters=1,
                  max_context=4096 + 256, prefill_rows=32, oracle_seqs=[0])
    print(f"attention at C5's item shape: max logit err {st['max_logit_err']:.2e}, parted: {st['events']}")
    assert st["iters"] >= 1 and st["max_logit_err"] > 0
    assert all(ev[3] < 5e-3 for ev in st["events"] if ev[0] == "beam step") and all(ev[-1] < 5e-3 for ev in st["events"] if ev[0] != "beam step")


# ---- decision kernels on the oracle's float32 inputs: integers must be identical -------------------------------------

def _engine(B, gamma, beam, mode, V):
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    shape = si.ModelShape(1, 64, 1, 1, 64, 96, V, "fp32")
    w = si.make_weights(shape, 1, "target", threads=1)
    m = DeviceModel(shape, w, DEV)
    return Engine(m, m, batch=B, gamma=gamma, beam=beam, mode=mode, max_context=256, device=DEV)


@pytest.mark.parametrize("mode", ["mtad", "mmtad"])
def test_accept_kernel_bit_exact_on_oracle_inputs(mode):
    from paper_2407_09722_amd import binding as mb
    B, gamma, beam, V = 3, 4, 3, 1024
    eng = _engine(B, gamma, beam, mode, V)
    g = np.random.default_rng(7)
    M = eng.M
    for trial in range(40):
        tau = float(g.choice([0.0, 0.1, 0.3, 0.5, 0.9]))
        sample = bool(trial % 2)
        trees, conds, logits = [], [], g.standard_normal((B, M, V)).astype(np.float32) * 3
        hist_all = []
        for s in range(B):
            hist = {"tok": g.integers(0, V, (gamma, beam)).astype(np.int32), "parent": np.zeros((gamma, beam), np.int32),
                    "score": -np.sort(g.uniform(0.1, 6, (gamma, beam)).astype(np.float32), axis=1)}
            hist["parent"][1:] = g.integers(0, beam, (gamma - 1, beam))
            hist["score"] = np.cumsum(hist["score"], axis=0).astype(np.float32) * -1 * -1
            hist["score"] = -np.abs(hist["score"])
            tree = mtad.build_tree(hist, mode)
            cond = -g.uniform(0.05, 3.0, M).astype(np.float32)
            cond[0] = 0
            trees.append(tree); conds.append(cond); hist_all.append(hist)
        eng.t_tok.copy_(torch.from_numpy(np.stack([t["tok"] for t in trees])).to(DEV))
        eng.t_parent.copy_(torch.from_numpy(np.stack([t["parent"] for t in trees])).to(DEV))
        eng.t_depth.copy_(torch.from_numpy(np.stack([t["depth"] for t in trees])).to(DEV))
        eng.t_src.copy_(torch.from_numpy(np.stack([t["src_beam"] for t in trees])).to(DEV))
        eng.t_qref.copy_(torch.from_numpy(np.stack([t["qref"] for t in trees]).astype(np.float32)).to(DEV))
        eng.logp_cond.copy_(torch.from_numpy(np.stack(conds)).to(DEV))
        eng.logits.copy_(torch.from_numpy(logits).to(DEV))
        eng.tkv.len.fill_(17 + trial)
        eng.accept_phase(tau, sample_bonus=sample, seed=trial)
        torch.cuda.synchronize()
        eta, row, tok, path = (x.cpu().numpy() for x in (eng.eta, eng.bonus_row, eng.bonus_tok, eng.path))
        for s in range(B):
            joint = mtad.joint_from_cond(trees[s], conds[s], np.float32)
            acc = mtad.accept_mtad if mode == "mtad" else mtad.accept_mmtad
            e, node, _ = acc(trees[s], joint, tau, np.float32)
            assert (eta[s], row[s]) == (e, node), (trial, s, tau)
            assert list(path[s, :e]) == mtad.branch_rows(trees[s], node)
            t, gap = mtad.bonus_token(logits[s, node], sample=sample, seed=trial, seq_index=s, position=17 + trial + 1 + e,
                                      dt=np.float32)
            assert tok[s] == t or gap < 1e-5, (trial, s, gap)
    eng.close()


@pytest.mark.parametrize("sample", [False, True])
def test_beam_topb_kernel_bit_exact_on_oracle_inputs(sample):
    from paper_2407_09722_amd import binding as mb
    B, gamma, beam, V = 2, 3, 4, 32000
    eng = _engine(B, gamma, beam, "mmtad", V)
    g = np.random.default_rng(11)
    for step in range(gamma):
        R = gamma + 1 if step == 0 else beam
        logits = (g.standard_normal((B, R, V)) * 3).astype(np.float32)
        if step == 1:
            logits[:, 1] = logits[:, 0]                       # duplicated rows: ties across beams go to the lowest flat index
        lse = np.log(np.exp(logits.astype(np.float64)).sum(-1)).astype(np.float32)
        cnt = np.array([1, 2], np.int32)
        prev = -np.abs(g.standard_normal((B, beam))).astype(np.float32)
        if step == 1:
            prev[:, 1] = prev[:, 0]
        if step > 0:
            eng.h_cum[:, step - 1].copy_(torch.from_numpy(prev).to(DEV))
        dl, dlse = torch.from_numpy(logits).to(DEV), torch.from_numpy(lse).to(DEV)
        length = torch.tensor([40, 41], dtype=torch.int32, device=DEV)
        mb.mtad_k_beam_topb(eng.ctx, dl, dlse, eng.hist, step, torch.from_numpy(cnt).to(DEV), length, R, V, int(sample), 5)
        torch.cuda.synchronize()
        tok, par, cum = (x.cpu().numpy() for x in (eng.h_tok, eng.h_parent, eng.h_cum))
        for s in range(B):
            if step == 0:
                rows, live = logits[s, cnt[s] - 1:cnt[s]], np.zeros(1, np.float32)
            else:
                rows, live = logits[s, :beam], prev[s]
            ls = lse[s, cnt[s] - 1:cnt[s]] if step == 0 else lse[s, :beam]
            flat = (live[:, None] + (rows - ls[:, None])).astype(np.float32).ravel()
            key = flat
            if sample:
                from oracle import rng
                key = flat + rng.gumbel(5, rng.stream_id(s, rng.STREAM_BEAM), int(length[s]) + cnt[s] + step,
                                        np.arange(flat.size)).astype(np.float32)
            sel = mtad.top_b(key, beam + 1)
            margin = key[sel[beam - 1]] - key[sel[beam]]
            sel = sel[:beam]
            same = list(tok[s, step]) == list(sel % V) and list(par[s, step]) == list(sel // V)
            assert same or (sample and margin < 1e-5), (step, s)
            if same:
                assert np.array_equal(cum[s, step], flat[sel])     # same float32 formula, same bits
    eng.close()


def test_kv_capacity_overflow_sets_status_instead_of_faulting():
    from paper_2407_09722_amd import binding as mb
    from paper_2407_09722_amd.engine import DeviceModel, Engine
    shape = si.ModelShape(1, 64, 1, 1, 64, 96, 1024, "fp32")
    m = DeviceModel(shape, si.make_weights(shape, 1, "target", threads=1), DEV)
    eng = Engine(m, m, batch=1, gamma=2, beam=2, mode="mtad", max_context=16, page_size=16, device=DEV)
    eng.prefill(np.arange(12, dtype=np.int32)[None, :])
    assert mb.mtad_device_status(eng.ctx) == 0
    for _ in range(4):                                          # 11 cached + 3 rows per pass soon exceeds 16 slots
        eng.iteration(0.0)
    assert mb.mtad_device_status(eng.ctx) & 1
    with pytest.raises(mb.MtadError):
        mb.mtad_prefill(eng.ctx, m.desc, eng.tkv.desc, eng.root_tok, 17)     # more tokens than the cache holds: refused on the host
    eng.close()
