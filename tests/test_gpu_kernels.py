"""GPU parity of single kernels against the oracle's arithmetic (float64 numpy) on the same seeded inputs."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _mb():
    from paper_2407_09722_amd import binding as mb
    mb.lib()
    return mb


def _bits(x):
    return torch.from_numpy(si.f32_to_bf16_bits(x).view(np.int16)).to(DEV)


def _fragment_order(planes):
    """[2][R][K] bfloat16 bit planes -> the operand-fragment order mtad_k_gemm_x documents (written out from that text)."""
    _, R, K = planes.shape
    G = (R + 7) // 8
    rows = R if R <= 24 else 8 * G
    out = np.zeros(2 * rows * K, dtype=planes.dtype)
    plane, r, k = np.meshgrid(np.arange(2), np.arange(R), np.arange(K), indexing="ij")
    kt, kg, e = k // 32, (k % 32) // 8, k % 8
    if R <= 24:
        off = ((((kt * 4 + kg) * 2 + plane) * R + r) * 8) + e
    else:
        off = (((kt * G + r // 8) * 64 + kg * 16 + plane * 8 + r % 8) * 8) + e
    out[off.ravel()] = planes.ravel()
    return out


def _gemm_case(mb, R, N, K, dtype, seed, accumulate=False, ldy=None, ctx=None, x_order=0):
    g = np.random.default_rng(seed)
    W = (g.standard_normal((N, K)) * 0.05).astype(np.float32)
    X = g.standard_normal((R, K)).astype(np.float32)
    ldy = ldy or N
    Y0 = g.standard_normal((R, ldy)).astype(np.float32)
    if dtype == 1:
        hi = si.bf16_bits_to_f32(si.f32_to_bf16_bits(X))
        lo = si.bf16_bits_to_f32(si.f32_to_bf16_bits(X - hi))
        Wrow, Xd = _bits(W), _bits(np.stack([hi, lo]))                   # activation = hi + lo planes
        if x_order:
            Xd = torch.from_numpy(_fragment_order(Xd.cpu().numpy().reshape(2, R, K))).to(DEV)
        Wd = torch.empty_like(Wrow)
        mb.mtad_pack_matrix(mb.MTAD_PACK_PLAIN, Wrow, Wd, N, K)          # the layout the kernel streams
        W, X = si.bf16_bits_to_f32(si.f32_to_bf16_bits(W)), hi.astype(np.float64) + lo
    else:
        Wd, Xd = torch.from_numpy(W).to(DEV), torch.from_numpy(X).to(DEV)
    Yd = torch.from_numpy(Y0).to(DEV)
    mb.mtad_k_gemm(dtype, Wd, Xd, Yd, R, N, K, ldy, accumulate, ctx=ctx, x_order=x_order)
    torch.cuda.synchronize()
    got = Yd.cpu().numpy().astype(np.float64)
    want = Y0.astype(np.float64)
    prod = X.astype(np.float64) @ W.astype(np.float64).T
    want[:, :N] = (want[:, :N] + prod) if accumulate else prod
    scale = np.abs(X).astype(np.float64) @ np.abs(W).astype(np.float64).T      # bound on the sum of |terms|
    err = np.abs(got[:, :N] - want[:, :N])
    assert np.all(err <= 2e-6 * scale + 1e-6), f"R{R} N{N} K{K}: max err {err.max()}"
    assert np.array_equal(got[:, N:], want[:, N:])                            # padding columns untouched


@pytest.mark.parametrize("R,N,K", [(1, 16, 32), (5, 48, 1376), (5, 2304, 768), (16, 64, 4096), (17, 4096, 4096),
                                   (5, 12288, 4096), (5, 4096, 11008), (33, 80, 96), (41, 512, 2048), (100, 96, 160),
                                   (164, 640, 5120), (200, 32, 64), (256, 1024, 1376),
                                   # more than 8 rows and more strips than compute units: several strips per workgroup
                                   (17, 12288, 4096), (9, 22016, 256), (30, 12304, 128), (41, 8192, 96), (24, 4112, 64),
                                   # 4 to 8 rows and at least two strips per compute unit: three strips per workgroup; strip
                                   # counts that leave the last workgroup one or two strips, odd k tile counts
                                   (5, 22016, 4096), (8, 8208, 160), (4, 8224, 96), (7, 8240, 1056), (6, 32000, 352),
                                   # 9 to 24 rows on the same kernel with two or three row groups
                                   (10, 12288, 4096), (16, 8208, 160), (9, 8224, 96), (13, 32000, 352), (17, 22016, 4096), (24, 8240, 96), (19, 8208, 1056),
                                   # many rows: activations staged through LDS, 4 or 8 strips per workgroup, 8 / 16 / 24 column groups
                                   (164, 16400, 256), (64, 16384, 160), (128, 16384, 96), (70, 16, 32), (190, 48, 1056), (77, 2000, 352), (25, 16400, 288), (32, 32000, 2048)])
def test_gemm_bf16_matches_float64(R, N, K):
    mb = _mb()
    print(f"gemm bf16 R={R} N={N} K={K}", flush=True)
    _gemm_case(mb, R, N, K, 1, seed=R * 7 + N)


@pytest.mark.parametrize("R,N,K", [(17, 4096, 4096), (17, 4096, 11008), (64, 4096, 4096), (41, 5120, 5120), (9, 2064, 2048), (30, 4112, 2080),
                                   (164, 5120, 5120), (164, 16384, 2048), (100, 4112, 1056), (256, 4096, 1024),
                                   # many rows (with a context's scratch): 4 or 8 strips per workgroup, 4 / 8 / 16 / 24 column
                                   # groups, ragged strips, rows and k tiles
                                   (164, 16400, 256), (64, 16384, 160), (128, 16384, 96), (70, 16, 32), (190, 48, 1056),
                                   (77, 2000, 352), (25, 16400, 288), (32, 32000, 2048), (100, 96, 160), (200, 32, 64)])
def test_gemm_bf16_with_context_workspace(R, N, K):
    """With a context's workspace: few output strips and more than 8 rows cut the reduction dimension over workgroups and
    the last one to arrive adds the ranges; passes of many rows take the kernel that stages both operands through LDS.
    Twice in a row, so that the arrival counters are seen to return to zero."""
    mb = _mb()
    shape = si.ModelShape(1, 4096, 32, 32, 128, 11008, 32000, "bf16")
    draft = si.ModelShape(1, 5120, 40, 40, 128, 8192, 32000, "bf16")
    desc = lambda s: mb.mtad_model(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 1, s.rms_eps, s.rope_theta, None)
    ctx = mb.mtad_create(mb.mtad_config(1, 4, 4, 1, 64, 256), desc(shape), desc(draft))
    ws = torch.empty(mb.mtad_workspace_bytes(ctx), dtype=torch.uint8, device=DEV)
    mb.mtad_bind_workspace(ctx, ws)
    for rep in range(2):
        print(f"gemm bf16 k-split R={R} N={N} K={K} rep {rep}", flush=True)
        _gemm_case(mb, R, N, K, 1, seed=R + N + rep, ctx=ctx)
    mb.mtad_destroy(ctx)


@pytest.mark.parametrize("R,N,K", [(1, 64, 96), (2, 8208, 160), (5, 12288, 4096), (5, 4096, 11008), (8, 22016, 256), (7, 48, 1056),
                                   (9, 4096, 4096), (17, 12288, 4096), (24, 4112, 64), (41, 8192, 96), (64, 4096, 1024),
                                   (25, 16400, 288), (100, 4112, 1056), (164, 5120, 5120), (190, 48, 1056)])
def test_gemm_bf16_fragment_order_input(R, N, K):
    """The activation layouts of the kernel-per-step passes (fragments without unused row slots up to 8 rows, whole 8-row
    fragments beyond) through every product kernel: one strip, three strips, several strips, k split, LDS-staged."""
    mb = _mb()
    shape = si.ModelShape(1, 4096, 32, 32, 128, 11008, 32000, "bf16")
    draft = si.ModelShape(1, 5120, 40, 40, 128, 8192, 32000, "bf16")
    desc = lambda s: mb.mtad_model(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 1, s.rms_eps, s.rope_theta, None)
    ctx = mb.mtad_create(mb.mtad_config(1, 4, 4, 1, 64, 256), desc(shape), desc(draft))
    ws = torch.empty(mb.mtad_workspace_bytes(ctx), dtype=torch.uint8, device=DEV)
    mb.mtad_bind_workspace(ctx, ws)
    print(f"gemm bf16 fragment order R={R} N={N} K={K}", flush=True)
    _gemm_case(mb, R, N, K, 1, seed=R * 3 + N, ctx=ctx, x_order=mb.MTAD_X_FRAGMENTS)
    _gemm_case(mb, R, N, K, 1, seed=R * 3 + N + 1, x_order=mb.MTAD_X_FRAGMENTS)      # without a context: the skinny kernels only
    mb.mtad_destroy(ctx)


def test_gemm_bf16_c5_gate_up_product_at_full_size():
    """The largest product of C5's target pass at its real size: 164 rows (4 trees of 41) x 27648 gate/up features x 5120,
    activations in fragment order, on the kernel the pass takes for it (8 strips per workgroup, 24 column groups, 64 KiB
    of LDS): every element against the float64 product."""
    mb = _mb()
    w = si.WORKLOADS["C5"]
    desc = lambda s: mb.mtad_model(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 1, s.rms_eps, s.rope_theta, None)
    ctx = mb.mtad_create(mb.mtad_config(w.batch, w.gamma, w.beam, 1, 32, 256), desc(w.target), desc(w.draft))
    ws = torch.empty(mb.mtad_workspace_bytes(ctx), dtype=torch.uint8, device=DEV)
    mb.mtad_bind_workspace(ctx, ws)
    R, N, K = w.batch * w.tree_rows, 2 * w.target.d_ffn, w.target.d_model
    print(f"gemm bf16 C5 gate/up R={R} N={N} K={K}", flush=True)
    _gemm_case(mb, R, N, K, 1, seed=5, ctx=ctx, x_order=mb.MTAD_X_FRAGMENTS)
    mb.mtad_destroy(ctx)


def test_gemm_accumulate_and_padded_rows():
    mb = _mb()
    _gemm_case(mb, 5, 64, 96, 1, seed=1, accumulate=True)
    _gemm_case(mb, 20, 48, 64, 1, seed=2, accumulate=True, ldy=52)
    _gemm_case(mb, 7, 30, 44, 0, seed=3, accumulate=True, ldy=32)


@pytest.mark.parametrize("R,N,K", [(1, 4, 4), (5, 1024, 256), (9, 688 * 2, 256), (5, 256, 688), (32, 37, 344), (64, 1024, 128)])
def test_gemm_fp32_matches_float64(R, N, K):
    mb = _mb()
    _gemm_case(mb, R, N, K, 0, seed=R + N + K)


@pytest.mark.parametrize("rows,V,top_k,top_p", [(37, 32000, 10, 0.9), (5, 1000, 10, 0.9), (3, 7, 10, 0.9), (9, 4099, 16, 0.5), (4, 32000, 1, 0.9), (3, 40001, 10, 0.9),
                                                (6, 2048, 10, 1.0)])
def test_warp_rows_matches_oracle(rows, V, top_k, top_p):
    """Rows of logits -> rows of log p~: same support as the oracle (float32 decisions) unless the oracle reports a decision
    on its threshold, values to 1e-5, minus infinity elsewhere, lse = 0.  Rows with exact ties, a dominant token
    (support of one) and NaN entries included."""
    from oracle import mtad
    mb = _mb()
    g = np.random.default_rng(rows * 31 + V)
    x = (g.standard_normal((rows, V)) * 3.0).astype(np.float32)
    x[0, : min(V, 12)] = x[0].max() + 1.0                      # twelve-way tie at the top: token ids decide
    if rows > 1:
        x[1, V // 2] = x[1].max() + 30.0                       # one token holds all the mass
    if rows > 2 and V > 20:
        x[2, 5] = np.nan                                       # ranks last
    xd = torch.from_numpy(x).to(DEV)
    lse = torch.full((rows,), 7.0, dtype=torch.float32, device=DEV)
    mb.mtad_k_warp_rows(xd, lse, rows, V, top_k, top_p)
    torch.cuda.synchronize()
    got = xd.cpu().numpy()
    assert torch.all(lse == 0).item()
    for r in range(rows):
        ref = np.where(np.isnan(x[r]), -np.inf, x[r]).astype(np.float32)
        want, margin = mtad.warp_log_probs(ref, top_k, top_p, dt=np.float32)
        if not np.array_equal(np.isfinite(got[r]), np.isfinite(want)):
            assert margin < 1e-5, f"row {r}: supports differ with margin {margin}"
            continue
        sup = np.isfinite(want)
        assert np.all(np.isneginf(got[r][~sup]))
        assert np.allclose(got[r][sup], want[sup], rtol=1e-5, atol=1e-5), (r, got[r][sup], want[sup])
        assert abs(np.exp(got[r][sup].astype(np.float64)).sum() - 1.0) < 1e-5


def test_lm_head_shape_full_vocab():
    """The 7B-shaped lm_head at its real size, checked on every output."""
    mb = _mb()
    _gemm_case(mb, 5, 32000, 4096, 1, seed=11)


@pytest.mark.parametrize("dtype", [0, 1])
def test_rmsnorm(dtype):
    mb = _mb()
    g = np.random.default_rng(3)
    for rows, d in ((1, 128), (5, 4096), (17, 768), (41, 5120)):
        h = (g.standard_normal((rows, d)) * 3).astype(np.float32)
        gain = (1 + 0.1 * g.standard_normal(d)).astype(np.float32)
        out = torch.zeros((2, rows, d) if dtype else (rows, d), dtype=torch.int16 if dtype else torch.float32, device=DEV)
        mb.mtad_k_rmsnorm(dtype, torch.from_numpy(h).to(DEV), torch.from_numpy(gain).to(DEV), out, rows, d, 1e-5)
        torch.cuda.synchronize()
        x = h.astype(np.float64)
        want = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + 1e-5) * gain
        if dtype:
            planes = si.bf16_bits_to_f32(out.cpu().numpy().view(np.uint16)).astype(np.float64)
            got = planes[0] + planes[1]
            assert np.all(np.abs(planes[0] - want) <= np.abs(want) * 2 ** -8)        # hi = nearest bfloat16
            assert np.all(np.abs(got - want) <= np.abs(want) * 2 ** -15)             # hi + lo: ~16 significant bits
        else:
            got = out.cpu().numpy().astype(np.float64)
            assert np.allclose(got, want, rtol=2e-6, atol=1e-7)


def test_row_lse():
    mb = _mb()
    g = np.random.default_rng(4)
    for rows, V in ((1, 7), (5, 1024), (17, 32000)):
        x = (g.standard_normal((rows, V)) * 3).astype(np.float32)
        lse = torch.zeros(rows, dtype=torch.float32, device=DEV)
        mb.mtad_k_row_lse(torch.from_numpy(x).to(DEV), lse, rows, V)
        torch.cuda.synchronize()
        xx = x.astype(np.float64)
        want = xx.max(1) + np.log(np.exp(xx - xx.max(1, keepdims=True)).sum(1))
        assert np.allclose(lse.cpu().numpy(), want, rtol=1e-6, atol=1e-6)
