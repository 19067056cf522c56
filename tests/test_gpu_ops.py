"""GPU parity of the single operations (the kernels one by one) against the oracle's primitives,
at shapes that span several tiles plus ragged tails, through the C ABI."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import stage_oracle as O
from tests import harness as hz

pytestmark = pytest.mark.gpu


def _randn(role, shape, std=1.0, seed=0, dtype="bf16"):
    return si.round_to(si.normal(si.stream_key(seed, role, *shape), shape, std), dtype)


def _f32_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


GEMM_SHAPES = [
    # (M, N, K)
    (256, 256, 128),       # one 256 tile / 4 tiles of 128
    (512, 768, 320),       # several tiles, K = 5 slices
    (2048, 2048, 512),     # 64 tiles of 256 -> 128 path; 256 tiles of 128
    (1024, 12288, 256),    # 192 tiles of 256
    (200, 264, 136),       # ragged everywhere (multiples of 8)
    (130, 72, 64),         # smaller than a tile
]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("form", ["fwd", "dgrad", "wgrad"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_gemm_forms(M, N, K, form, dtype):
    import torch
    import paper_2410_19367_amd as bp
    if dtype == "f32" and M * N * K > 512 * 768 * 320:
        pytest.skip("fp32 path is exercised on the small shapes")
    dt = bp.BP_BF16 if dtype == "bf16" else bp.BP_F32
    tol = hz.TOL[dtype] if dtype == "f32" else 1e-2
    if form == "fwd":            # Y[M,N] = X[M,K] W[K,N] + b + R
        X = _randn("gx", (M, K), dtype=dtype); W = _randn("gw", (K, N), 0.05, dtype=dtype)
        b = _randn("gb", (N,), 0.5, dtype="f32"); R = _randn("gr", (M, N), dtype=dtype)
        ref = O.linear_fwd(X.astype(np.float64), W.astype(np.float64), b.astype(np.float64), R.astype(np.float64))
        out = hz.empty_like_dev((M, N), dtype)
        bp.bp_op_gemm(dt, 0, 0, M, N, K, hz.to_dev(X, dtype), K, hz.to_dev(W, dtype), N, out, N,
                      bias=_f32_dev(b), residual=hz.to_dev(R, dtype))
        got = hz.to_host(out)
    elif form == "dgrad":        # dX[M,N] = dY[M,K] W[N,K]^T
        dY = _randn("gdy", (M, K), dtype=dtype); W = _randn("gw2", (N, K), 0.05, dtype=dtype)
        ref = O.linear_dgrad(dY.astype(np.float64), W.astype(np.float64))
        out = hz.empty_like_dev((M, N), dtype)
        bp.bp_op_gemm(dt, 0, 1, M, N, K, hz.to_dev(dY, dtype), K, hz.to_dev(W, dtype), K, out, N)
        got = hz.to_host(out)
    else:                        # dW[M,N] += X[K,M]^T dY[K,N]   (K = tokens)
        X = _randn("gx3", (K, M), dtype=dtype); dY = _randn("gdy3", (K, N), dtype=dtype)
        C0 = _randn("gc0", (M, N), 3.0, dtype="f32")
        dW, _ = O.linear_wgrad(X.astype(np.float64), dY.astype(np.float64))
        ref = C0.astype(np.float64) + dW
        out = _f32_dev(C0)
        bp.bp_op_gemm(dt, 1, 0, M, N, K, hz.to_dev(X, dtype), M, hz.to_dev(dY, dtype), N, out, N, accumulate=1)
        got = hz.to_host(out)
    torch.cuda.synchronize()
    err = hz.rel_err(got, ref)
    assert err <= tol, (form, M, N, K, err)


@pytest.mark.parametrize("T,H", [(64, 128), (300, 1024), (260, 2048), (77, 5120), (33, 8192), (5, 8)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_layernorm_fwd_bwd(T, H, dtype):
    import torch
    import paper_2410_19367_amd as bp
    dt = bp.BP_BF16 if dtype == "bf16" else bp.BP_F32
    x = _randn("lx", (T, H), 2.0, dtype=dtype) + np.float32(0.5)
    x = si.round_to(x, dtype)
    g = _randn("lg", (H,), 0.3, dtype="f32") + 1.0
    b = _randn("lb", (H,), 0.3, dtype="f32")
    dout = _randn("ld", (T, H), dtype=dtype)
    res = _randn("lr", (T, H), dtype=dtype)
    eps = 1e-5
    x64 = x.astype(np.float64)
    ref, xhat, rstd = O.layer_norm_fwd(x64, g.astype(np.float64), b.astype(np.float64), eps)
    dx_ref, dg_ref, db_ref = O.layer_norm_bwd(dout.astype(np.float64), xhat, rstd, g.astype(np.float64))
    dx_ref = dx_ref + res
    xd, gd, bd = hz.to_dev(x, dtype), _f32_dev(g), _f32_dev(b)
    out = hz.empty_like_dev((T, H), dtype)
    mean = torch.empty(T, device="cuda"); rs = torch.empty(T, device="cuda")
    bp.bp_op_layernorm_fwd(dt, T, H, xd, gd, bd, eps, out, mean, rs)
    dx = hz.empty_like_dev((T, H), dtype)
    dg0 = _randn("ldg0", (H,), dtype="f32"); db0 = _randn("ldb0", (H,), dtype="f32")
    dgd, dbd = _f32_dev(dg0), _f32_dev(db0)
    ws = torch.empty(2 * bp.bp_op_colsum_workspace(T, H), device="cuda")
    bp.bp_op_layernorm_bwd(dt, T, H, hz.to_dev(dout, dtype), xd, mean, rs, gd, hz.to_dev(res, dtype),
                           dx, dgd, dbd, ws)
    torch.cuda.synchronize()
    tol = 1e-2 if dtype == "bf16" else 1e-5
    assert hz.rel_err(hz.to_host(out), ref) <= tol
    assert hz.rel_err(hz.to_host(mean), x64.mean(-1)) <= 1e-5
    assert hz.rel_err(hz.to_host(rs), rstd[:, 0]) <= 1e-5
    assert hz.rel_err(hz.to_host(dx), dx_ref) <= tol
    assert hz.rel_err(hz.to_host(dgd), dg0 + dg_ref) <= 1e-4
    assert hz.rel_err(hz.to_host(dbd), db0 + db_ref) <= 1e-4


@pytest.mark.parametrize("T,F", [(64, 512), (300, 4096), (100, 8192), (37, 520)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_bias_gelu_fwd_bwd(T, F, dtype):
    import torch
    import paper_2410_19367_amd as bp
    dt = bp.BP_BF16 if dtype == "bf16" else bp.BP_F32
    u = _randn("gu", (T, F), 2.0, dtype=dtype)
    b = _randn("gbias", (F,), 0.5, dtype="f32")
    dg = _randn("gdg", (T, F), dtype=dtype)
    h = u.astype(np.float64) + b
    g_ref = O.gelu(h)
    du_ref = dg * O.gelu_grad(h)
    db0 = _randn("gdb0", (F,), dtype="f32")
    ud, bd = hz.to_dev(u, dtype), _f32_dev(b)
    g = hz.empty_like_dev((T, F), dtype)
    bp.bp_op_bias_gelu_fwd(dt, T, F, ud, bd, g)
    du = hz.empty_like_dev((T, F), dtype)
    dbd = _f32_dev(db0)
    ws = torch.empty(bp.bp_op_colsum_workspace(T, F), device="cuda")
    bp.bp_op_bias_gelu_bwd(dt, T, F, hz.to_dev(dg, dtype), ud, bd, du, dbd, ws)
    torch.cuda.synchronize()
    tol = 1e-2 if dtype == "bf16" else 1e-5
    assert hz.rel_err(hz.to_host(g), g_ref) <= tol
    assert hz.rel_err(hz.to_host(du), du_ref) <= tol
    assert hz.rel_err(hz.to_host(dbd), db0 + du_ref.sum(0)) <= (2e-3 if dtype == "bf16" else 1e-5)


ATTN_CASES = [
    # B, S, heads, d, causal, lens
    (2, 64, 2, 64, True, None),
    (1, 200, 2, 128, True, None),
    (2, 384, 3, 64, True, None),
    (1, 512, 2, 128, True, None),
    (3, 160, 2, 64, False, [160, 41, 97]),
    (2, 256, 2, 128, False, [256, 130]),
    (2, 96, 2, 64, False, None),
    (1, 72, 1, 32, True, None),
    (3, 128, 2, 64, False, [128, 41, 97]),
    (2, 256, 2, 64, False, None),
    (1, 640, 2, 128, False, [333]),
    (2, 1024, 1, 128, True, None),
    (2, 192, 2, 64, True, None),
    (1, 320, 3, 128, False, [200]),
    (2, 64, 2, 128, True, None),
    # head widths below the tile width (padded inside the MFMA kernels): the paper's 40 and 96, and others
    (2, 128, 4, 40, False, [128, 77]),
    (1, 256, 2, 96, True, None),
    (2, 192, 2, 40, True, None),
    (1, 128, 3, 96, False, [100]),
    (1, 192, 2, 32, True, None),
    (1, 128, 2, 112, False, None),
    (1, 128, 2, 48, True, None),
    (1, 64, 2, 8, True, None),
    # long enough for the eight-wave forward (two tiles per step), padded widths
    (1, 512, 2, 112, True, None),
    (1, 512, 2, 40, False, [300]),
    # the eight-wave forward with an odd number of 64-key tiles, so that the last step holds one tile only
    (1, 576, 2, 64, True, None),
    (1, 704, 1, 96, True, None),
    (1, 576, 2, 128, False, [500]),
]


@pytest.mark.parametrize("B,S,heads,d,causal,lens", ATTN_CASES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_fwd_bwd(B, S, heads, d, causal, lens, dtype):
    import torch
    import paper_2410_19367_amd as bp
    dt = bp.BP_BF16 if dtype == "bf16" else bp.BP_F32
    H = heads * d
    qkv = _randn("aqkv", (B, S, 3 * H), 1.0, dtype=dtype)
    dctx = _randn("adctx", (B, S, H), dtype=dtype)
    q64 = qkv.astype(np.float64)
    q = O._split_heads(q64[..., :H], heads); k = O._split_heads(q64[..., H:2 * H], heads)
    v = O._split_heads(q64[..., 2 * H:], heads)
    la = None if lens is None else np.array(lens)
    ctx_h, p = O.attention_fwd(q, k, v, causal, la)
    ctx_ref = O._merge_heads(ctx_h)
    dq, dk, dv = O.attention_bwd(O._split_heads(dctx.astype(np.float64), heads), q, k, v, p)
    dqkv_ref = np.concatenate([O._merge_heads(dq), O._merge_heads(dk), O._merge_heads(dv)], -1)
    # log-sum-exp of the scaled, masked scores, from the definition
    lse_ref = np.empty((B, heads, S))
    for b in range(B):
        ok = O.allowed_mask(S, causal, None if la is None else la[b])
        for h in range(heads):
            s = np.where(ok, q[b, h] @ k[b, h].T / np.sqrt(d), -np.inf)
            mx = s.max(-1)
            lse_ref[b, h] = mx + np.log(np.exp(s - mx[:, None]).sum(-1))
    qd = hz.to_dev(qkv, dtype)
    ctx = hz.empty_like_dev((B, S, H), dtype)
    lse = torch.empty((B, heads, S), device="cuda")
    lens_d = None if lens is None else torch.tensor(lens, dtype=torch.int32, device="cuda")
    bp.bp_op_attention_fwd(dt, B, S, heads, d, causal, lens_d, qd, ctx, lse)
    dqkv = hz.empty_like_dev((B, S, 3 * H), dtype)
    delta = torch.empty((B, heads, S), device="cuda")
    # the backward consumes the oracle's ctx (rounded to the storage type), not the GPU's
    ctx_in = hz.to_dev(si.round_to(ctx_ref, dtype), dtype)
    bp.bp_op_attention_bwd(dt, B, S, heads, d, causal, lens_d, qd, ctx_in, lse, hz.to_dev(dctx, dtype), dqkv, delta)
    torch.cuda.synchronize()
    tol = 1e-2 if dtype == "bf16" else 2e-5
    assert hz.rel_err(hz.to_host(ctx), ctx_ref) <= tol
    assert np.max(np.abs(hz.to_host(lse) - lse_ref)) <= (1e-4 if dtype == "f32" else 2e-3)
    got = hz.to_host(dqkv)
    for name, sl in (("dq", slice(0, H)), ("dk", slice(H, 2 * H)), ("dv", slice(2 * H, 3 * H))):
        err = hz.rel_err(got[..., sl], dqkv_ref[..., sl])
        assert err <= (2e-2 if dtype == "bf16" else 5e-5), (name, err)


@pytest.mark.parametrize("B,S,heads,d,causal", [(1, 512, 2, 128, True), (2, 256, 2, 64, False), (1, 1024, 1, 128, True)])
def test_attention_wide_score_range(B, S, heads, d, causal):
    """Scores whose magnitude grows along the key axis (std up to ~16, maxima tens of binary orders
    apart between tiles): the running softmax reference has to move many times, by large and by
    small amounts, and the result must still match the definition."""
    import torch
    import paper_2410_19367_amd as bp
    H = heads * d
    qkv = _randn("wqkv", (B, S, 3 * H), 1.0, dtype="f32").astype(np.float64)
    ramp = 1.0 + 7.0 * np.arange(S) / S
    qkv[..., :H] *= 2.0
    qkv[..., H:2 * H] *= ramp[None, :, None]
    qkv = si.round_to(qkv, "bf16")
    dctx = _randn("wdctx", (B, S, H), dtype="bf16")
    q64 = qkv.astype(np.float64)
    q = O._split_heads(q64[..., :H], heads); k = O._split_heads(q64[..., H:2 * H], heads)
    v = O._split_heads(q64[..., 2 * H:], heads)
    ctx_h, p = O.attention_fwd(q, k, v, causal, None)
    ctx_ref = O._merge_heads(ctx_h)
    dq, dk, dv = O.attention_bwd(O._split_heads(dctx.astype(np.float64), heads), q, k, v, p)
    dqkv_ref = np.concatenate([O._merge_heads(dq), O._merge_heads(dk), O._merge_heads(dv)], -1)
    qd = hz.to_dev(qkv, "bf16")
    ctx = hz.empty_like_dev((B, S, H), "bf16")
    lse = torch.empty((B, heads, S), device="cuda")
    bp.bp_op_attention_fwd(bp.BP_BF16, B, S, heads, d, causal, None, qd, ctx, lse)
    dqkv = hz.empty_like_dev((B, S, 3 * H), "bf16")
    delta = torch.empty((B, heads, S), device="cuda")
    ctx_in = hz.to_dev(si.round_to(ctx_ref, "bf16"), "bf16")
    bp.bp_op_attention_bwd(bp.BP_BF16, B, S, heads, d, causal, None, qd, ctx_in, lse, hz.to_dev(dctx, "bf16"), dqkv,
                           delta)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(hz.to_host(ctx)))
    assert hz.rel_err(hz.to_host(ctx), ctx_ref) <= 1e-2
    got = hz.to_host(dqkv)
    for name, sl in (("dq", slice(0, H)), ("dk", slice(H, 2 * H)), ("dv", slice(2 * H, 3 * H))):
        err = hz.rel_err(got[..., sl], dqkv_ref[..., sl])
        assert err <= 2e-2, (name, err)


@pytest.mark.parametrize("M,N,T,n", [
    (512, 768, 256, 2),        # 128-tile direct-to-LDS kernel, segment change between slices
    (2048, 6144, 192, 3),      # 256x192 tiles
    (4096, 4096, 128, 4),      # 256x256 tiles, four segments of two slices
    (256, 256, 64, 4),         # one slice per segment
    (256, 256, 64, 8),         # the most segments
    (2048, 2048, 128, 8),      # 256x256 tiles, eight segments of two slices
    (200, 264, 136, 3),        # ragged: one launch per segment
    (512, 768, 256, 1),
    (2048, 2048, 1024, 4),     # with a workspace: 64 tiles x 4 token slices, one per segment
    (2048, 2048, 2048, 2),     # with a workspace: 4 token slices, two per segment
    (2048, 2048, 1536, 2),     # with a workspace: 3072 tokens -> 3 slices, boundaries inside segments
    (4096, 5120, 2048, 2),     # with a workspace: 320 tiles, the last 64 cut into 4 token slices
    (512, 768, 1024, 2),       # with a workspace: 24 tiles of 128 x 128, two token slices, K steps of 128
    (512, 768, 1088, 2),       # the same with K steps of 64 (1088 = 17 * 64)
    (2048, 2560, 1664, 2),     # with a workspace: 80 tiles x 3 token slices of 18, 17, 17 steps
    (512, 768, 1600, 2),       # with a workspace: 24 small tiles x 3 token slices of 17, 17, 16 steps
    (2048, 1152, 2048, 2),     # with a workspace, N a multiple of 128 and 192 but not of 256
])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("overwrite", [0, 1])
def test_wgrad_group(M, N, T, n, dtype, overwrite):
    """dW (+)= sum_i X_i^T dY_i over a group of micro-batches in one call."""
    import torch
    import paper_2410_19367_amd as bp
    if dtype == "f32" and M * N > 2 ** 21:
        pytest.skip("fp32 generic kernel: small shapes only")
    dt = bp.BP_BF16 if dtype == "bf16" else bp.BP_F32
    xs = [_randn(f"gx{i}", (T, M), dtype=dtype) for i in range(n)]
    ys = [_randn(f"gy{i}", (T, N), dtype=dtype) for i in range(n)]
    w0 = _randn("gw0", (M, N), dtype="f32")
    ref = sum(x.astype(np.float64).T @ y.astype(np.float64) for x, y in zip(xs, ys))
    if not overwrite:
        ref = ref + w0
    xd = [hz.to_dev(x, dtype) for x in xs]
    yd = [hz.to_dev(y, dtype) for y in ys]
    wd = _f32_dev(w0)
    ws = torch.empty(4 * M * N, device="cuda") if T >= 1024 else None
    bp.bp_op_wgrad_group(dt, M, N, T, xd, yd, wd, overwrite, ws, 0 if ws is None else ws.numel())
    torch.cuda.synchronize()
    err = hz.rel_err(wd.cpu().numpy().astype(np.float64), ref)
    assert err <= (2e-3 if dtype == "bf16" else 1e-5), err
