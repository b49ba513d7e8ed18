"""ctypes binding of libmtad.so: the same names as include/mtad.h, argument marshalling only.

PyTorch is imported for device memory and streams; every step of the path runs in the HIP
kernels of libmtad.  There is no fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

import torch  # noqa: F401  (loaded first so that libmtad binds to the HIP runtime torch uses)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmtad.so")

MTAD_OK, MTAD_EINVAL, MTAD_ESHAPE, MTAD_ECAP, MTAD_EHIP, MTAD_ENOSYS = 0, -1, -2, -3, -4, -5
MTAD_MODE_MTAD, MTAD_MODE_MMTAD = 0, 1
MTAD_MAX_ROWS, MTAD_MAX_BEAM = 64, 8

EXPORTS = ["mtad_create", "mtad_destroy", "mtad_workspace_bytes", "mtad_bind_workspace", "mtad_strerror",
           "mtad_last_hip_error", "mtad_device_status", "mtad_set_fused_pass", "mtad_set_warp", "mtad_pack_matrix", "mtad_prefill", "mtad_draft_beam_step", "mtad_build_tree",
           "mtad_verify_tree", "mtad_accept", "mtad_accept_spd", "mtad_accept_chain", "mtad_kv_commit",
           "mtad_k_gemm", "mtad_k_gemm_x", "mtad_k_rmsnorm", "mtad_k_row_lse", "mtad_k_warp_rows", "mtad_k_beam_topb", "mtad_k_beam_topb_static", "mtad_k_copy"]

i32, u64, f32, vp = C.c_int32, C.c_uint64, C.c_float, C.c_void_p


class mtad_model(C.Structure):
    _fields_ = [(n, i32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "dtype")] + \
               [("rms_eps", f32), ("rope_theta", f32), ("weights", C.POINTER(vp))]


class mtad_kv(C.Structure):
    _fields_ = [("k", vp), ("v", vp), ("page_table", vp), ("len", vp), ("page_size", i32), ("max_pages", i32), ("n_pages", i32)]


class mtad_beam(C.Structure):
    _fields_ = [("tok", vp), ("parent", vp), ("cum_logq", vp)]


class mtad_tree(C.Structure):
    _fields_ = [("M", i32), ("tok", vp), ("parent", vp), ("depth", vp), ("src_beam", vp), ("anc_mask", vp), ("qref", vp)]


class mtad_accept_out(C.Structure):
    _fields_ = [(n, vp) for n in ("eta", "path", "bonus_row", "bonus_tok", "out_tok", "out_cnt")]


class mtad_state(C.Structure):
    _fields_ = [("root_tok", vp), ("catchup_tok", vp), ("catchup_cnt", vp)]


class mtad_config(C.Structure):
    _fields_ = [(n, i32) for n in ("batch", "gamma", "beam", "mode", "prefill_rows", "max_context")]


class MtadError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__(f"{fn} failed: {status} ({lib().mtad_strerror(status).decode()})")


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_09722_amd.build` "
                               "(or __graft_entry__.build()); the HIP library is the only implementation")
        L = C.CDLL(LIB_PATH)
        P = C.POINTER
        L.mtad_create.argtypes = [P(vp), P(mtad_config), P(mtad_model), P(mtad_model)]
        L.mtad_destroy.argtypes = [vp]
        L.mtad_destroy.restype = None
        L.mtad_workspace_bytes.argtypes = [vp]
        L.mtad_workspace_bytes.restype = C.c_size_t
        L.mtad_bind_workspace.argtypes = [vp, vp, C.c_size_t]
        L.mtad_strerror.argtypes = [C.c_int]
        L.mtad_strerror.restype = C.c_char_p
        L.mtad_last_hip_error.argtypes = [vp]
        L.mtad_device_status.argtypes = [vp, P(C.c_uint32), vp]
        L.mtad_set_fused_pass.argtypes = [vp, i32]
        L.mtad_set_warp.argtypes = [vp, i32, f32]
        L.mtad_pack_matrix.argtypes = [i32, vp, vp, i32, i32, i32, vp]
        L.mtad_prefill.argtypes = [vp, P(mtad_model), P(mtad_kv), vp, i32, vp]
        L.mtad_draft_beam_step.argtypes = [vp, P(mtad_model), P(mtad_kv), P(mtad_beam), i32, P(mtad_state), i32, u64, vp]
        L.mtad_build_tree.argtypes = [vp, P(mtad_beam), i32, P(mtad_tree), vp]
        L.mtad_verify_tree.argtypes = [vp, P(mtad_model), P(mtad_kv), vp, P(mtad_tree), vp, vp, vp, vp]
        L.mtad_accept.argtypes = [vp, P(mtad_tree), vp, vp, i32, P(mtad_kv), f32, i32, i32, u64, P(mtad_accept_out), vp]
        L.mtad_accept_chain.argtypes = [vp, P(mtad_tree), P(mtad_accept_out), vp]
        L.mtad_accept_spd.argtypes = [vp, P(mtad_tree), vp, vp, i32, P(mtad_kv), u64, P(mtad_accept_out), vp]
        L.mtad_kv_commit.argtypes = [vp, P(mtad_kv), P(mtad_kv), P(mtad_tree), P(mtad_accept_out), P(mtad_state), vp]
        L.mtad_k_gemm.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.mtad_k_gemm_x.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
        L.mtad_k_rmsnorm.argtypes = [i32, vp, vp, vp, i32, i32, f32, vp]
        L.mtad_k_row_lse.argtypes = [vp, vp, i32, i32, vp]
        L.mtad_k_warp_rows.argtypes = [vp, vp, i32, i32, i32, f32, vp]
        L.mtad_k_copy.argtypes = [vp, vp, C.c_int64, vp]
        L.mtad_k_beam_topb.argtypes = [vp, vp, vp, P(mtad_beam), i32, vp, vp, i32, i32, i32, u64, vp]
        L.mtad_k_beam_topb_static.argtypes = [vp, vp, P(mtad_beam), i32, i32, i32, i32, vp, vp, i32, i32, i32, u64, vp]
        for name in EXPORTS:
            fn = getattr(L, name)
            if name not in ("mtad_destroy", "mtad_workspace_bytes", "mtad_strerror"):
                fn.restype = C.c_int
        _lib = L
    return _lib


def _check(fn, status):
    if status != MTAD_OK:
        raise MtadError(fn, status)


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return vp(stream.cuda_stream)


def ptr(t):
    """Device (or host) address of a tensor as void*."""
    return vp(t.data_ptr()) if t is not None else vp(0)


# ---- same names as the C ABI --------------------------------------------------------------------

def mtad_create(cfg: mtad_config, target: mtad_model, draft: mtad_model):
    h = vp()
    _check("mtad_create", lib().mtad_create(C.byref(h), C.byref(cfg), C.byref(target), C.byref(draft)))
    return h


def mtad_destroy(ctx):
    lib().mtad_destroy(ctx)


def mtad_workspace_bytes(ctx) -> int:
    return int(lib().mtad_workspace_bytes(ctx))


def mtad_bind_workspace(ctx, buf: torch.Tensor):
    _check("mtad_bind_workspace", lib().mtad_bind_workspace(ctx, ptr(buf), buf.numel() * buf.element_size()))


def mtad_set_warp(ctx, top_k: int, top_p: float):
    _check("mtad_set_warp", lib().mtad_set_warp(ctx, int(top_k), f32(top_p)))


def mtad_k_warp_rows(logits, lse, rows, vocab, top_k, top_p, stream=None):
    _check("mtad_k_warp_rows", lib().mtad_k_warp_rows(ptr(logits), ptr(lse), rows, vocab, int(top_k), f32(top_p), _stream_ptr(stream)))


def mtad_set_fused_pass(ctx, on: bool):
    _check("mtad_set_fused_pass", lib().mtad_set_fused_pass(ctx, int(on)))


def mtad_device_status(ctx, stream=None) -> int:
    bits = C.c_uint32(0)
    _check("mtad_device_status", lib().mtad_device_status(ctx, C.byref(bits), _stream_ptr(stream)))
    return bits.value


MTAD_PACK_PLAIN, MTAD_PACK_QKV, MTAD_PACK_GATE_UP = 0, 1, 2
MTAD_X_PLANES, MTAD_X_FRAGMENTS = 0, 1


def mtad_pack_matrix(kind, src, dst, N, K, head_dim=0, stream=None):
    _check("mtad_pack_matrix", lib().mtad_pack_matrix(kind, ptr(src), ptr(dst), N, K, head_dim, _stream_ptr(stream)))


def mtad_prefill(ctx, model, kv, tokens: torch.Tensor, n_tokens: int, stream=None):
    _check("mtad_prefill", lib().mtad_prefill(ctx, C.byref(model), C.byref(kv), ptr(tokens), n_tokens, _stream_ptr(stream)))


def mtad_draft_beam_step(ctx, draft, dkv, hist, step, st, sample_beam=0, seed=0, stream=None):
    _check("mtad_draft_beam_step", lib().mtad_draft_beam_step(ctx, C.byref(draft), C.byref(dkv), C.byref(hist), step, C.byref(st),
                                                             int(sample_beam), u64(seed), _stream_ptr(stream)))


def mtad_build_tree(ctx, hist, mode, tree, stream=None):
    _check("mtad_build_tree", lib().mtad_build_tree(ctx, C.byref(hist), mode, C.byref(tree), _stream_ptr(stream)))


def mtad_verify_tree(ctx, target, tkv, root_tok, tree, logp_cond, row_lse, logits, stream=None):
    _check("mtad_verify_tree", lib().mtad_verify_tree(ctx, C.byref(target), C.byref(tkv), ptr(root_tok), C.byref(tree), ptr(logp_cond),
                                                     ptr(row_lse), ptr(logits), _stream_ptr(stream)))


def mtad_accept(ctx, tree, logp_cond, logits, vocab, tkv, tau, mode, sample_bonus, seed, out, stream=None):
    _check("mtad_accept", lib().mtad_accept(ctx, C.byref(tree), ptr(logp_cond), ptr(logits), vocab, C.byref(tkv), f32(tau), mode,
                                           int(sample_bonus), u64(seed), C.byref(out), _stream_ptr(stream)))


def mtad_accept_chain(ctx, tree, out, stream=None):
    _check("mtad_accept_chain", lib().mtad_accept_chain(ctx, C.byref(tree), C.byref(out), _stream_ptr(stream)))


def mtad_accept_spd(ctx, tree, logits, row_lse, vocab, tkv, seed, out, stream=None):
    _check("mtad_accept_spd", lib().mtad_accept_spd(ctx, C.byref(tree), ptr(logits), ptr(row_lse), vocab, C.byref(tkv), u64(seed),
                                                   C.byref(out), _stream_ptr(stream)))


def mtad_kv_commit(ctx, tkv, dkv, tree, acc, st, stream=None):
    _check("mtad_kv_commit", lib().mtad_kv_commit(ctx, C.byref(tkv) if tkv is not None else None, C.byref(dkv) if dkv is not None else None, C.byref(tree),
                                                 C.byref(acc), C.byref(st), _stream_ptr(stream)))


def mtad_k_gemm(dtype, W, X, Y, R, N, K, ldy, accumulate=False, stream=None, ctx=None, x_order=0):
    if x_order:
        _check("mtad_k_gemm_x", lib().mtad_k_gemm_x(ctx, dtype, ptr(W), ptr(X), ptr(Y), R, N, K, ldy, int(accumulate), x_order, _stream_ptr(stream)))
    else:
        _check("mtad_k_gemm", lib().mtad_k_gemm(ctx, dtype, ptr(W), ptr(X), ptr(Y), R, N, K, ldy, int(accumulate), _stream_ptr(stream)))



def mtad_k_rmsnorm(dtype, h, g, out, rows, d, eps, stream=None):
    _check("mtad_k_rmsnorm", lib().mtad_k_rmsnorm(dtype, ptr(h), ptr(g), ptr(out), rows, d, f32(eps), _stream_ptr(stream)))


def mtad_k_row_lse(logits, lse, rows, vocab, stream=None):
    _check("mtad_k_row_lse", lib().mtad_k_row_lse(ptr(logits), ptr(lse), rows, vocab, _stream_ptr(stream)))


def mtad_k_beam_topb(ctx, logits, lse, hist, step, catchup_cnt, length, rows_per_seq, vocab, sample_beam=0, seed=0, stream=None):
    _check("mtad_k_beam_topb", lib().mtad_k_beam_topb(ctx, ptr(logits), ptr(lse), C.byref(hist), step, ptr(catchup_cnt), ptr(length),
                                                     rows_per_seq, vocab, int(sample_beam), u64(seed), _stream_ptr(stream)))


MTAD_STATIC_TOPB_MAX_BATCH = 64


def mtad_k_beam_topb_static(logits, lse, hist, batch, gamma, beam, step, catchup_cnt, length, rows_per_seq, vocab, sample_beam=0, seed=0,
                            stream=None):
    _check("mtad_k_beam_topb_static", lib().mtad_k_beam_topb_static(ptr(logits), ptr(lse), C.byref(hist), batch, gamma, beam, step,
                                                                   ptr(catchup_cnt), ptr(length), rows_per_seq, vocab, int(sample_beam),
                                                                   u64(seed), _stream_ptr(stream)))


def mtad_k_copy(src, dst, nbytes, stream=None):
    _check("mtad_k_copy", lib().mtad_k_copy(ptr(src), ptr(dst), nbytes, _stream_ptr(stream)))
