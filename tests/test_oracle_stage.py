"""Pins for the numpy stage oracle against things other than itself: brute-force scalar loops,
closed forms, invariants, finite differences, the synchronous-semantics invariant (sum over
micro-batches under any valid order == full-batch gradient), and the paper's parameter counts."""
import math
import os
import random

import numpy as np
import pytest

import synth_inputs as si
from oracle import schedule_oracle as so
from oracle import stage_oracle as O


def _rand_params(rng, H, F, scale=0.3):
    P = {}
    for n in O.PARAM_NAMES:
        shp = O.param_shape(H, F, n)
        if n in ("ln1_g", "ln2_g"):
            P[n] = 1.0 + 0.3 * rng.standard_normal(shp)
        else:
            P[n] = scale * rng.standard_normal(shp)
    return P


# ------------------------------------------------------------------ brute force, scalar loops

def _brute_layer(x, P, heads, causal, lens, eps):
    """Whole layer with python scalars only (tiny shapes)."""
    B, S, H = x.shape
    F = P["w1"].shape[1]
    d = H // heads

    def ln(row, g, b):
        mu = sum(row) / H
        var = sum((v - mu) ** 2 for v in row) / H
        return [(row[j] - mu) / math.sqrt(var + eps) * g[j] + b[j] for j in range(H)]

    def gelu(v):
        return 0.5 * v * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))

    z = np.zeros_like(x)
    for b in range(B):
        a = [ln(list(x[b, s]), P["ln1_g"], P["ln1_b"]) for s in range(S)]
        qkv = [[sum(a[s][i] * P["wqkv"][i, o] for i in range(H)) + P["bqkv"][o]
                for o in range(3 * H)] for s in range(S)]
        ctx = [[0.0] * H for _ in range(S)]
        for hh in range(heads):
            for i in range(S):
                js = [j for j in range(S)
                      if (not causal or j <= i) and (lens is None or j < lens[b])]
                sc = [sum(qkv[i][hh * d + c] * qkv[j][H + hh * d + c] for c in range(d)) / math.sqrt(d)
                      for j in js]
                mx = max(sc)
                e = [math.exp(v - mx) for v in sc]
                tot = sum(e)
                for c in range(d):
                    ctx[i][hh * d + c] = sum(e[t] / tot * qkv[j][2 * H + hh * d + c]
                                             for t, j in enumerate(js))
        for s in range(S):
            y = [x[b, s, o] + sum(ctx[s][i] * P["wo"][i, o] for i in range(H)) + P["bo"][o]
                 for o in range(H)]
            m = ln(y, P["ln2_g"], P["ln2_b"])
            g = [gelu(sum(m[i] * P["w1"][i, o] for i in range(H)) + P["b1"][o]) for o in range(F)]
            for o in range(H):
                z[b, s, o] = y[o] + sum(g[i] * P["w2"][i, o] for i in range(F)) + P["b2"][o]
    return z


@pytest.mark.parametrize("causal,lens", [(True, None), (False, [2, 3]), (False, None)])
def test_layer_forward_matches_scalar_brute_force(causal, lens):
    rng = np.random.default_rng(1)
    B, S, H, heads, F = 2, 3, 4, 2, 6
    P = _rand_params(rng, H, F)
    x = rng.standard_normal((B, S, H))
    z, _ = O.layer_forward(x, P, heads, causal, None if lens is None else np.array(lens), 1e-5)
    zb = _brute_layer(x, P, heads, causal, lens, 1e-5)
    np.testing.assert_allclose(z, zb, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ attention special cases

def test_attention_special_cases():
    rng = np.random.default_rng(2)
    B, h, S, d = 2, 2, 5, 3
    q, k, v = (rng.standard_normal((B, h, S, d)) for _ in range(3))
    # S = 1: the only key gets probability 1
    c1, p1 = O.attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1], True, None)
    np.testing.assert_allclose(c1, v[:, :, :1])
    # causal: row 0 attends only itself; rows sum to one; nothing above the diagonal
    ctx, p = O.attention_fwd(q, k, v, True, None)
    np.testing.assert_allclose(ctx[:, :, 0], v[:, :, 0])
    np.testing.assert_allclose(p.sum(-1), 1.0)
    assert np.all(np.triu(p[0, 0], 1) == 0.0)
    # identical keys -> uniform weights -> running mean of v under the causal mask
    kk = np.broadcast_to(k[:, :, :1], k.shape)
    ctx_u, _ = O.attention_fwd(q, kk, v, True, None)
    run_mean = np.cumsum(v, axis=2) / np.arange(1, S + 1)[None, None, :, None]
    np.testing.assert_allclose(ctx_u, run_mean, rtol=1e-12)
    # padding with len = S equals no mask; len < S zeroes the masked keys exactly
    full, _ = O.attention_fwd(q, k, v, False, np.array([S, S]))
    none, _ = O.attention_fwd(q, k, v, False, None)
    np.testing.assert_array_equal(full, none)
    _, pp = O.attention_fwd(q, k, v, False, np.array([3, 5]))
    assert np.all(pp[0, :, :, 3:] == 0.0) and np.all(pp[1] > 0.0)
    # padded result equals attention over the truncated key/value set
    ctx_pad, _ = O.attention_fwd(q, k, v, False, np.array([3, 5]))
    s = q[0, 1] @ k[0, 1, :3].T / math.sqrt(d)
    e = np.exp(s - s.max(-1, keepdims=True))
    np.testing.assert_allclose(ctx_pad[0, 1], (e / e.sum(-1, keepdims=True)) @ v[0, 1, :3], rtol=1e-12)


def test_attention_scale_is_one_over_sqrt_d():
    # two keys, scores differ by exactly q.(k0-k1)/sqrt(d): closed-form logistic weight
    d = 4
    q = np.zeros((1, 1, 2, d)); k = np.zeros((1, 1, 2, d)); v = np.zeros((1, 1, 2, d))
    q[0, 0, :, 0] = 2.0
    k[0, 0, 0, 0] = 1.0
    k[0, 0, 1, 0] = -1.0
    v[0, 0, 0, 0] = 1.0
    ctx, p = O.attention_fwd(q, k, v, False, None)
    delta = 2.0 * (1.0 - (-1.0)) / math.sqrt(d)
    assert abs(p[0, 0, 0, 0] - 1.0 / (1.0 + math.exp(-delta))) < 1e-15


# ------------------------------------------------------------------ LayerNorm / GELU / linear

def test_layernorm_invariants():
    rng = np.random.default_rng(3)
    H = 16
    x = 3.0 * rng.standard_normal((2, 5, H)) + 1.5
    eps = 1e-5
    out, xhat, rstd = O.layer_norm_fwd(x, np.ones(H), np.zeros(H), eps)
    np.testing.assert_allclose(out.mean(-1), 0.0, atol=1e-14)
    var = x.var(-1)                       # numpy's default is the biased variance
    np.testing.assert_allclose(out.var(-1), var / (var + eps), rtol=1e-12)
    # affine: out = xhat * g + b
    g, b = rng.standard_normal(H), rng.standard_normal(H)
    out2, _, _ = O.layer_norm_fwd(x, g, b, eps)
    np.testing.assert_allclose(out2, out * g + b, rtol=1e-13)
    # invariance to a per-row shift, and to a per-row scale as eps -> 0
    out3, _, _ = O.layer_norm_fwd(x + 7.0, np.ones(H), np.zeros(H), eps)
    np.testing.assert_allclose(out3, out, atol=1e-12)
    o4a, _, _ = O.layer_norm_fwd(x, np.ones(H), np.zeros(H), 0.0)
    o4b, _, _ = O.layer_norm_fwd(x * 5.0, np.ones(H), np.zeros(H), 0.0)
    np.testing.assert_allclose(o4a, o4b, rtol=1e-12, atol=1e-12)
    # backward with gamma = 1: dx rows sum to zero and are orthogonal to xhat
    # (exactly so at eps = 0, where xhat has unit variance)
    dout = rng.standard_normal(x.shape)
    _, xhat, rstd = O.layer_norm_fwd(x, np.ones(H), np.zeros(H), 0.0)
    dx, dgam, dbet = O.layer_norm_bwd(dout, xhat, rstd, np.ones(H))
    np.testing.assert_allclose(dx.sum(-1), 0.0, atol=1e-13)
    np.testing.assert_allclose((dx * xhat).sum(-1), 0.0, atol=1e-12)
    np.testing.assert_allclose(dbet, dout.reshape(-1, H).sum(0))


def test_gelu_closed_forms():
    assert O.gelu(np.array(0.0)) == 0.0
    assert O.gelu_grad(np.array(0.0)) == 0.5
    x = np.linspace(-6, 6, 241)
    # tanh form tracks the erf form to ~1e-3 absolute and tends to relu for large |x|
    erf_form = np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in x])
    assert np.max(np.abs(O.gelu(x) - erf_form)) < 1.1e-3
    assert abs(O.gelu(np.array(10.0)) - 10.0) < 1e-12 and abs(O.gelu(np.array(-10.0))) < 1e-12
    # printed constant of the tanh form: at x = 1 the value is 0.8411919906...
    assert abs(float(O.gelu(np.array(1.0))) - 0.8411919906082768) < 1e-12
    # derivative against central differences
    hstep = 1e-6
    fd = (O.gelu(x + hstep) - O.gelu(x - hstep)) / (2 * hstep)
    np.testing.assert_allclose(O.gelu_grad(x), fd, rtol=1e-8, atol=1e-9)


def test_linear_steps_match_loop_nest():
    """The oracle's matmuls with [in,out] weights against a differently ordered scalar loop nest
    (catches a transposed operand)."""
    rng = np.random.default_rng(4)
    B, S, H, heads, F = 1, 2, 4, 1, 8
    P = _rand_params(rng, H, F)
    x = rng.standard_normal((B, S, H))
    z, c = O.layer_forward(x, P, heads, True, None, 1e-5)
    for o in range(3 * H):
        for s in range(S):
            acc = P["bqkv"][o]
            for i in range(H):
                acc += c["a"][0, s, i] * P["wqkv"][i, o]
            got = np.concatenate([c["q"][0, 0, s], c["k"][0, 0, s], c["v"][0, 0, s]])[o]
            assert abs(acc - got) < 1e-13
    h1 = np.zeros((S, F))
    for o in range(F):
        for s in range(S):
            h1[s, o] = P["b1"][o] + sum(c["m"][0, s, i] * P["w1"][i, o] for i in range(H))
    np.testing.assert_allclose(c["h1"][0], h1, rtol=1e-13)


def _loop_linear(x, W, b, res):
    """y[t][o] = sum_i x[t][i] W[i][o] + b[o] + res[t][o], output-column-major loop order, python floats."""
    T, I = len(x), len(x[0])
    Oo = len(W[0])
    y = [[0.0] * Oo for _ in range(T)]
    for o in range(Oo):
        for i in range(I):
            w = float(W[i][o])
            for t in range(T):
                y[t][o] += float(x[t][i]) * w
    for t in range(T):
        for o in range(Oo):
            y[t][o] += (float(b[o]) if b is not None else 0.0) + (float(res[t][o]) if res is not None else 0.0)
    return np.array(y)


def test_linear_primitives_match_scalar_loops_and_adjoint_identity():
    """linear_fwd / linear_dgrad / linear_wgrad, the expected values of every GEMM parity case,
    pinned three ways that do not call a matmul: (1) scalar loop nests in another loop order over
    non-square shapes (a transposed or swapped operand cannot even be evaluated or gives other
    numbers), (2) the adjoint identity <dy, x W> = <dy W^T, x> = <x^T dy, W>, (3) one-hot inputs
    that read single rows / columns of W."""
    rng = np.random.default_rng(40)
    T, I, Oo = 5, 3, 7                      # all different: every transposition changes a shape
    x = rng.standard_normal((T, I)); W = rng.standard_normal((I, Oo))
    b = rng.standard_normal(Oo); res = rng.standard_normal((T, Oo)); dy = rng.standard_normal((T, Oo))
    # (1) forward, with and without bias / residual
    np.testing.assert_allclose(O.linear_fwd(x, W), _loop_linear(x, W, None, None), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(O.linear_fwd(x, W, b, res), _loop_linear(x, W, b, res), rtol=1e-13, atol=1e-13)
    # dgrad: dx[t][i] = sum_o dy[t][o] W[i][o]   (loop order i, t, o)
    dx = np.zeros((T, I))
    for i in range(I):
        for t in range(T):
            acc = 0.0
            for o in range(Oo):
                acc += float(dy[t, o]) * float(W[i, o])
            dx[t, i] = acc
    got_dx = O.linear_dgrad(dy, W)
    assert got_dx.shape == (T, I)
    np.testing.assert_allclose(got_dx, dx, rtol=1e-13, atol=1e-13)
    # wgrad: dW[i][o] = sum_t x[t][i] dy[t][o], db[o] = sum_t dy[t][o]   (loop order t outermost)
    dW = np.zeros((I, Oo)); db = np.zeros(Oo)
    for t in range(T):
        for o in range(Oo):
            db[o] += float(dy[t, o])
            for i in range(I):
                dW[i, o] += float(x[t, i]) * float(dy[t, o])
    got_dW, got_db = O.linear_wgrad(x, dy)
    assert got_dW.shape == (I, Oo) and got_db.shape == (Oo,)
    np.testing.assert_allclose(got_dW, dW, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(got_db, db, rtol=1e-13, atol=1e-13)
    # a leading batch axis is flattened into tokens
    x3 = rng.standard_normal((2, T, I)); dy3 = rng.standard_normal((2, T, Oo))
    gW3, gb3 = O.linear_wgrad(x3, dy3)
    np.testing.assert_allclose(gW3, sum(O.linear_wgrad(x3[i], dy3[i])[0] for i in range(2)), rtol=1e-13)
    np.testing.assert_allclose(gb3, dy3.sum(axis=(0, 1)), rtol=1e-13)
    # (2) adjoint identity, evaluated with element-wise sums only
    lhs = float((dy * O.linear_fwd(x, W)).sum())
    assert abs(lhs - float((got_dx * x).sum())) < 1e-12 * max(1.0, abs(lhs))
    assert abs(lhs - float((got_dW * W).sum())) < 1e-12 * max(1.0, abs(lhs))
    # (3) one-hot probes: a unit input row picks a row of W, a unit output gradient picks W's column
    for i in range(I):
        e = np.zeros((1, I)); e[0, i] = 1.0
        np.testing.assert_array_equal(O.linear_fwd(e, W)[0], W[i])
    for o in range(Oo):
        e = np.zeros((1, Oo)); e[0, o] = 1.0
        np.testing.assert_array_equal(O.linear_dgrad(e, W)[0], W[:, o])
    # the finite-difference meaning of the three: d<R, x W + b>/dx, /dW, /db
    R = rng.standard_normal((T, Oo)); h = 1e-6
    f = lambda xv, Wv, bv: float((R * O.linear_fwd(xv, Wv, bv)).sum())
    gW, gb = O.linear_wgrad(x, R)
    for idx in [(0, 0), (2, 5), (1, 6)]:
        Wp = W.copy(); Wp[idx] += h; Wm = W.copy(); Wm[idx] -= h
        assert abs((f(x, Wp, b) - f(x, Wm, b)) / (2 * h) - gW[idx]) < 1e-7
    for idx in [(0, 0), (4, 2)]:
        xp = x.copy(); xp[idx] += h; xm = x.copy(); xm[idx] -= h
        assert abs((f(xp, W, b) - f(xm, W, b)) / (2 * h) - O.linear_dgrad(R, W)[idx]) < 1e-7
    bp_ = b.copy(); bp_[3] += h; bm_ = b.copy(); bm_[3] -= h
    assert abs((f(x, W, bp_) - f(x, W, bm_)) / (2 * h) - gb[3]) < 1e-7


def test_linear_pins_catch_a_transposed_operand():
    """Planted mistakes (on the CPU, in copies of the oracle's formulas): with square shapes a
    transposed weight or swapped wgrad operands still evaluate, and the scalar-loop pin rejects them."""
    rng = np.random.default_rng(41)
    T = I = Oo = 4
    x = rng.standard_normal((T, I)); W = rng.standard_normal((I, Oo)); dy = rng.standard_normal((T, Oo))
    good = _loop_linear(x, W, None, None)
    assert np.max(np.abs(O.linear_fwd(x, W) - good)) < 1e-12
    assert np.max(np.abs(O.linear_fwd(x, W.T) - good)) > 1e-2          # weight read as [out, in]
    ref_dx = np.array([[sum(dy[t, o] * W[i, o] for o in range(Oo)) for i in range(I)] for t in range(T)])
    assert np.max(np.abs(O.linear_dgrad(dy, W) - ref_dx)) < 1e-12
    assert np.max(np.abs(O.linear_dgrad(dy, W.T) - ref_dx)) > 1e-2     # forgot the transpose in dgrad
    ref_dW = np.array([[sum(x[t, i] * dy[t, o] for t in range(T)) for o in range(Oo)] for i in range(I)])
    assert np.max(np.abs(O.linear_wgrad(x, dy)[0] - ref_dW)) < 1e-12
    assert np.max(np.abs(O.linear_wgrad(dy, x)[0] - ref_dW)) > 1e-2    # operands swapped: dW^T


# ------------------------------------------------------------------ finite differences

def _make_stage(rng, L, H, heads, S, B, causal, n_chunks=1, F=0):
    st = O.StageOracle(L, H, heads, S, B, causal, n_chunks=n_chunks, mlp=F)
    for c in range(n_chunks):
        for l in range(L):
            P = _rand_params(rng, H, st.F)
            for n in O.PARAM_NAMES:
                st.set_param(c, l, n, P[n])
    return st


@pytest.mark.parametrize("causal,lens", [(True, None), (False, [3, 5])])
def test_gradients_match_central_differences(causal, lens):
    rng = np.random.default_rng(5)
    L, H, heads, S, B, F = 2, 8, 2, 5, 2, 12
    st = _make_stage(rng, L, H, heads, S, B, causal, F=F)
    if lens is not None:
        st.set_seqlens(0, lens)
    x = rng.standard_normal((B, S, H))
    R = rng.standard_normal((B, S, H))

    def loss_of(xv):
        st.stash.clear()
        return float((st.forward(0, 0, xv) * R).sum())

    st.zero_grad()
    st.stash.clear()
    st.forward(0, 0, x)
    dx = st.backward(0, 0, R)
    # inputs
    eps = 1e-5
    fd = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp = x.copy(); xp[idx] += eps
        xm = x.copy(); xm[idx] -= eps
        fd[idx] = (loss_of(xp) - loss_of(xm)) / (2 * eps)
    np.testing.assert_allclose(dx, fd, rtol=2e-6, atol=1e-8)
    # every parameter tensor of every layer (a sample of entries for the matrices)
    pick = random.Random(0)
    for l in range(L):
        for n in O.PARAM_NAMES:
            W = st.params[0][l][n]
            G = st.get_grad(0, l, n)
            idxs = list(np.ndindex(*W.shape))
            if len(idxs) > 24:
                idxs = pick.sample(idxs, 24)
            for idx in idxs:
                old = W[idx]
                W[idx] = old + eps
                lp = loss_of(x)
                W[idx] = old - eps
                lm = loss_of(x)
                W[idx] = old
                fdv = (lp - lm) / (2 * eps)
                assert abs(G[idx] - fdv) <= 2e-6 * max(1.0, abs(fdv)), (l, n, idx, G[idx], fdv)


def test_planted_mistakes_would_be_caught():
    """The finite-difference pin is sensitive: dropping the residual path or the softmax
    correction term from the adjoint changes dx by far more than the pin's tolerance."""
    rng = np.random.default_rng(6)
    H, heads, S, B, F = 8, 2, 4, 1, 12
    P = _rand_params(rng, H, F)
    x = rng.standard_normal((B, S, H))
    R = rng.standard_normal((B, S, H))
    z, c = O.layer_forward(x, P, heads, True, None, 1e-5)
    G = {n: np.zeros_like(P[n]) for n in O.PARAM_NAMES}
    dx = O.layer_backward(R, c, P, G)
    c_bad = dict(c)
    c_bad["p"] = c["p"].transpose(0, 1, 3, 2).copy()       # a transposed operand
    G2 = {n: np.zeros_like(P[n]) for n in O.PARAM_NAMES}
    dx_bad = O.layer_backward(R, c_bad, P, G2)
    assert np.max(np.abs(dx - dx_bad)) > 1e-3


# ------------------------------------------------------------------ synchronous semantics

def _setup_pipeline(D, N, causal=True, lens=False, seed=7):
    rng = np.random.default_rng(seed)
    L, H, heads, S, B, F = 1, 8, 2, 4, 2, 16
    st = _make_stage(rng, L, H, heads, S, B, causal, n_chunks=2 * D, F=F)
    inputs = rng.standard_normal((N, B, S, H))
    targets = rng.standard_normal((N, B, S, H))
    ll = None
    if lens:
        ll = rng.integers(2, S + 1, size=(N, B))
        for m in range(N):
            st.set_seqlens(m, ll[m])
    return st, inputs, targets, ll


@pytest.mark.parametrize("causal,lens", [(True, False), (False, True)])
def test_microbatch_sum_equals_full_batch_under_v_schedule(causal, lens):
    D, N = 2, 4
    st, inputs, targets, ll = _setup_pipeline(D, N, causal, lens)
    order = so.generate(D, N)
    loss = st.run_schedule(order, inputs, targets)
    loss_fb, G, _ = st.full_batch_reference(inputs, targets, ll)
    assert abs(loss - loss_fb) <= 1e-12 * abs(loss_fb)
    for c in range(2 * D):
        for n in O.PARAM_NAMES:
            a, b = st.get_grad(c, 0, n), G[c][0][n]
            assert np.max(np.abs(a - b)) <= 1e-11 * max(1e-30, np.max(np.abs(b))), (c, n)


def test_gradients_do_not_depend_on_the_order():
    D, N = 2, 4
    st, inputs, targets, _ = _setup_pipeline(D, N)
    base = so.generate(D, N)
    st.run_schedule(base, inputs, targets)
    ref = {(c, n): st.get_grad(c, 0, n).copy() for c in range(2 * D) for n in O.PARAM_NAMES}
    rng = random.Random(1)
    for _ in range(3):
        pending, seen, order = list(base), set(), []
        while pending:
            ready = [o for o in pending if
                     (o.kind == "F" and (o.stage == 0 or ("F", o.stage - 1, o.mb) in seen)) or
                     (o.kind == "B" and ("F", o.stage, o.mb) in seen and
                      (o.stage == 2 * D - 1 or ("B", o.stage + 1, o.mb) in seen))]
            o = rng.choice(ready)
            pending.remove(o); seen.add((o.kind, o.stage, o.mb)); order.append(o)
        st.run_schedule(order, inputs, targets)
        for (c, n), g in ref.items():
            assert np.max(np.abs(st.get_grad(c, 0, n) - g)) <= 1e-12 * max(1e-30, np.max(np.abs(g)))


def test_stage_composition_equals_one_deep_stage():
    """Eight one-layer stages run in sequence == one eight-layer stage (bit for bit)."""
    rng = np.random.default_rng(8)
    H, heads, S, B, F = 8, 2, 4, 2, 16
    deep = _make_stage(rng, 8, H, heads, S, B, True, F=F)
    chain = O.StageOracle(1, H, heads, S, B, True, n_chunks=8, mlp=F)
    for l in range(8):
        for n in O.PARAM_NAMES:
            chain.set_param(l, 0, n, deep.params[0][l][n])
    x = rng.standard_normal((B, S, H))
    g = rng.standard_normal((B, S, H))
    z = deep.forward(0, 0, x)
    dx = deep.backward(0, 0, g)
    a = x
    for c in range(8):
        a = chain.forward(c, 0, a)
    np.testing.assert_array_equal(a, z)
    d = g
    for c in reversed(range(8)):
        d = chain.backward(c, 0, d)
    np.testing.assert_array_equal(d, dx)
    for l in range(8):
        np.testing.assert_array_equal(chain.get_grad(l, 0, "wqkv"), deep.get_grad(0, l, "wqkv"))


def test_accumulation_persists_until_zero_grad_and_state_errors():
    rng = np.random.default_rng(9)
    st = _make_stage(rng, 1, 8, 2, 4, 1, True, F=16)
    x = rng.standard_normal((1, 4, 8)); g = rng.standard_normal((1, 4, 8))
    st.forward(0, 0, x); st.backward(0, 0, g)
    g1 = st.get_grad(0, 0, "w1").copy()
    st.forward(0, 1, x); st.backward(0, 1, g)
    np.testing.assert_allclose(st.get_grad(0, 0, "w1"), 2 * g1, rtol=1e-14)
    st.zero_grad()
    assert np.all(st.get_grad(0, 0, "w1") == 0)
    with pytest.raises(O.StageError):
        st.backward(0, 0, g)
    st.forward(0, 0, x)
    with pytest.raises(O.StageError):
        st.forward(0, 0, x)


def test_loss_gradient_is_its_derivative():
    rng = np.random.default_rng(10)
    z = rng.standard_normal((2, 3, 4)); y = rng.standard_normal((2, 3, 4))
    l0, g = O.StageOracle.loss_and_grad(z, y, 5)
    assert abs(l0 - 0.5 * ((z - y) ** 2).sum() / (5 * 2 * 3)) < 1e-15
    zp = z.copy(); zp[1, 2, 3] += 1e-6
    lp, _ = O.StageOracle.loss_and_grad(zp, y, 5)
    assert abs((lp - l0) / 1e-6 - g[1, 2, 3]) < 1e-6


# ------------------------------------------------------------------ the paper's model sizes

def test_parameter_count_matches_table_3():
    p = os.path.join(os.path.dirname(__file__), "golden", "paper_table3_models.txt")
    rows = [l.split() for l in open(p) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for name, L, heads, H, S, billions in rows:
        L, H, billions = int(L), int(H), int(billions)
        per_layer = O.params_per_layer(H)
        assert per_layer == 12 * H * H + 13 * H
        assert round(L * per_layer / 1e9) == billions, name


# ------------------------------------------------------------------ the input generator

def test_synthetic_inputs_are_reproducible_and_shaped():
    cfg = si.CONFIGS[0]
    a = si.make_activation(cfg, "act_in", 0)
    b = si.make_activation(cfg, "act_in", 0)
    c = si.make_activation(cfg, "act_in", 1)
    assert a.shape == (2, 64, 128) and np.array_equal(a, b) and not np.array_equal(a, c)
    assert abs(a.mean()) < 0.05 and abs(a.std() - 1.0) < 0.05
    P = si.make_params(cfg)
    assert abs(P[0][0]["wqkv"].std() - 0.02) < 0.002
    assert np.all(P[0][1]["ln1_g"] == 1.0) and np.all(P[0][1]["ln2_b"] == 0.0)
    # bf16 rounding: representable values are fixed points, ties go to even
    x = np.array([1.0, 1.00390625, 1.005859375, -3.140625], dtype=np.float32)
    r = si.round_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0078125 and r[3] == -3.140625
    assert np.array_equal(si.from_bf16_bits(si.to_bf16_bits(r)), r)
    lens = si.make_seqlens(si.CONFIGS[2], 3)
    assert lens.shape == (8,) and lens.min() >= 256 and lens.max() <= 512
    assert si.CONFIGS[1].flops_per_microbatch() == pytest.approx(2.680e12, rel=1e-3)
    assert si.CONFIGS[3].flops_per_microbatch() == pytest.approx(1.598e13, rel=1e-3)
