"""CPU oracle for one pipeline stage's chunk(s) of pre-LN transformer layers (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This is the plain definition of what the GPU library must compute,
written out step by step with materialised attention scores and textbook formulas; nothing here
is tiled, fused or reordered, and nothing is shared with the HIP path.  Only tests/, the smoke
check and the bench's cpu_baseline leg may import it.

What the paper fixes (BitPipe, arXiv 2410.19367):
  * a stage is a contiguous chunk of transformer layers; the schedule's unit of work is one
    forward or one backward of a chunk on one micro-batch (Section 3.2, Section 3.3, Appendix B
    Eq. 1 where their costs are t_f and t_b);
  * training is synchronous: gradients of all micro-batches of an iteration are accumulated and
    the pipeline is flushed before the update (Section 1, Section 2), so the sum over
    micro-batches under any valid order equals the full-batch gradient;
  * the two directions' replicas of a stage hold the same weights and their gradients are
    summed by an all-reduce (Section 3.4, Appendix C);
  * 12*L*H^2 parameters for (L,H) = (64,2560) -> 5B and (96,3072) -> 11B (Table 3), i.e. a fused
    3H-wide QKV projection, an H x H output projection and a 4H-wide MLP.
The layer equations themselves are the standard pre-LN GPT/BERT block (the paper builds on
Megatron-LM, Section 4.1, and never writes them): see `layer_forward`.

Readings taken where the paper is silent: LayerNorm uses the biased variance and eps = 1e-5;
GELU is the tanh form; attention scores are scaled by 1/sqrt(d); masked keys get exactly zero
probability; the causal mask keeps j <= i; padding masks keys only (j < len_b) and padded query
rows are computed like any other; no dropout; all four linear layers have a bias.

Pins (tests/test_oracle_*.py): central finite differences for every gradient, brute-force
attention loops, LayerNorm/GELU closed forms and invariants, matmul against a second loop nest,
micro-batch-sum == full-batch, order invariance, stage composition, Table 3's parameter counts.
"""
from __future__ import annotations

import math

import numpy as np

PARAM_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")

_GELU_C = math.sqrt(2.0 / math.pi)
_GELU_A = 0.044715


# ----------------------------------------------------------------------------- primitives

def layer_norm_fwd(x, gamma, beta, eps):
    """Row-wise LayerNorm over the last axis: biased variance, then affine.
    Returns (out, xhat, rstd)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, xhat, rstd


def layer_norm_bwd(dout, xhat, rstd, gamma):
    """Adjoint of layer_norm_fwd.  Returns (dx, dgamma, dbeta)."""
    red = tuple(range(dout.ndim - 1))
    dgamma = (dout * xhat).sum(axis=red)
    dbeta = dout.sum(axis=red)
    dxhat = dout * gamma
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dxhat - m1 - xhat * m2)
    return dx, dgamma, dbeta


def linear_fwd(x, W, b=None, residual=None):
    """y = x W (+ b) (+ residual) with W row-major [in, out]."""
    y = x @ W
    if b is not None:
        y = y + b
    if residual is not None:
        y = y + residual
    return y


def linear_dgrad(dy, W):
    """dx = dy W^T."""
    return dy @ W.T


def linear_wgrad(x, dy):
    """dW = x^T dy over all rows (tokens); db = column sums of dy."""
    x2 = x.reshape(-1, x.shape[-1])
    d2 = dy.reshape(-1, dy.shape[-1])
    return x2.T @ d2, d2.sum(axis=0)


def gelu(x):
    """tanh-form GELU: 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    return 0.5 * x * (1.0 + np.tanh(_GELU_C * (x + _GELU_A * x ** 3)))


def gelu_grad(x):
    """d gelu / dx of the tanh form."""
    t = np.tanh(_GELU_C * (x + _GELU_A * x ** 3))
    du = _GELU_C * (1.0 + 3.0 * _GELU_A * x ** 2)
    return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * du


def allowed_mask(S, causal, length):
    """[S, S] boolean: may query i attend key j?  causal: j <= i; padding: j < length."""
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    ok = np.ones((S, S), dtype=bool)
    if causal:
        ok &= (j <= i)
    if length is not None:
        ok &= (j < int(length))
    return ok


def attention_fwd(q, k, v, causal, lens):
    """q, k, v: [B, h, S, d].  Returns (ctx [B,h,S,d], p [B,h,S,S]) with the full probability
    matrix materialised.  Softmax runs over allowed keys only; masked keys get probability 0."""
    B, h, S, d = q.shape
    ctx = np.empty_like(q)
    p = np.empty((B, h, S, S))
    for b in range(B):
        ok = allowed_mask(S, causal, None if lens is None else lens[b])
        for hh in range(h):
            s = (q[b, hh] @ k[b, hh].T) / math.sqrt(d)
            s = np.where(ok, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            e = np.exp(s)
            pp = e / e.sum(axis=-1, keepdims=True)
            p[b, hh] = pp
            ctx[b, hh] = pp @ v[b, hh]
    return ctx, p


def attention_bwd(dctx, q, k, v, p):
    """Adjoint of attention_fwd.  Returns (dq, dk, dv), each [B, h, S, d]."""
    B, h, S, d = q.shape
    dq = np.empty_like(q)
    dk = np.empty_like(q)
    dv = np.empty_like(q)
    for b in range(B):
        for hh in range(h):
            pp = p[b, hh]
            do = dctx[b, hh]
            dv[b, hh] = pp.T @ do
            dp = do @ v[b, hh].T
            ds = pp * (dp - (dp * pp).sum(axis=-1, keepdims=True))
            dq[b, hh] = (ds @ k[b, hh]) / math.sqrt(d)
            dk[b, hh] = (ds.T @ q[b, hh]) / math.sqrt(d)
    return dq, dk, dv


def _split_heads(t, heads):
    """[B, S, H] -> [B, h, S, d]; head hh owns columns hh*d .. hh*d+d-1."""
    B, S, H = t.shape
    return t.reshape(B, S, heads, H // heads).transpose(0, 2, 1, 3)


def _merge_heads(t):
    """[B, h, S, d] -> [B, S, H]."""
    B, h, S, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(B, S, h * d)


# ----------------------------------------------------------------------------- one layer

def layer_forward(x, P, heads, causal, lens, eps):
    """One pre-LN transformer layer.  x: [B, S, H] fp64.  P: dict of the 12 parameter tensors.

        a   = LN(x; ln1_g, ln1_b)            qkv = a Wqkv + bqkv   (columns [q | k | v])
        ctx = softmax(q k^T / sqrt(d) + mask) v
        y   = x + ctx Wo + bo
        m   = LN(y; ln2_g, ln2_b)            h1 = m W1 + b1,  g = GELU(h1)
        z   = y + g W2 + b2

    Returns (z, cache) where cache holds what the adjoint needs."""
    H = x.shape[-1]
    a, xhat1, rstd1 = layer_norm_fwd(x, P["ln1_g"], P["ln1_b"], eps)
    qkv = a @ P["wqkv"] + P["bqkv"]
    q = _split_heads(qkv[..., 0:H], heads)
    k = _split_heads(qkv[..., H:2 * H], heads)
    v = _split_heads(qkv[..., 2 * H:3 * H], heads)
    ctx_h, p = attention_fwd(q, k, v, causal, lens)
    ctx = _merge_heads(ctx_h)
    y = x + ctx @ P["wo"] + P["bo"]
    m, xhat2, rstd2 = layer_norm_fwd(y, P["ln2_g"], P["ln2_b"], eps)
    h1 = m @ P["w1"] + P["b1"]
    g = gelu(h1)
    z = y + g @ P["w2"] + P["b2"]
    cache = dict(xhat1=xhat1, rstd1=rstd1, a=a, q=q, k=k, v=v, p=p, ctx=ctx,
                 xhat2=xhat2, rstd2=rstd2, m=m, h1=h1, g=g)
    return z, cache


def layer_backward(dz, cache, P, G):
    """Adjoint of layer_forward.  dz: [B, S, H].  Adds parameter gradients into dict G
    (G[name] += ...) and returns dx."""
    H = dz.shape[-1]
    flat = lambda t: t.reshape(-1, t.shape[-1])
    c = cache
    # z = y + g W2 + b2
    G["w2"] += flat(c["g"]).T @ flat(dz)
    G["b2"] += flat(dz).sum(axis=0)
    dg = dz @ P["w2"].T
    dy = dz.copy()
    # g = GELU(h1), h1 = m W1 + b1
    dh1 = dg * gelu_grad(c["h1"])
    G["w1"] += flat(c["m"]).T @ flat(dh1)
    G["b1"] += flat(dh1).sum(axis=0)
    dm = dh1 @ P["w1"].T
    # m = LN(y)
    dy_ln, dgam, dbet = layer_norm_bwd(dm, c["xhat2"], c["rstd2"], P["ln2_g"])
    G["ln2_g"] += dgam
    G["ln2_b"] += dbet
    dy = dy + dy_ln
    # y = x + ctx Wo + bo
    G["wo"] += flat(c["ctx"]).T @ flat(dy)
    G["bo"] += flat(dy).sum(axis=0)
    dctx = dy @ P["wo"].T
    dx = dy.copy()
    # attention
    heads = c["q"].shape[1]
    dq, dk, dv = attention_bwd(_split_heads(dctx, heads), c["q"], c["k"], c["v"], c["p"])
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)
    # qkv = a Wqkv + bqkv
    G["wqkv"] += flat(c["a"]).T @ flat(dqkv)
    G["bqkv"] += flat(dqkv).sum(axis=0)
    da = dqkv @ P["wqkv"].T
    # a = LN(x)
    dx_ln, dgam, dbet = layer_norm_bwd(da, c["xhat1"], c["rstd1"], P["ln1_g"])
    G["ln1_g"] += dgam
    G["ln1_b"] += dbet
    return dx + dx_ln


# ----------------------------------------------------------------------------- the stage

def param_shape(hidden, mlp, name):
    H, F = hidden, mlp
    return {"ln1_g": (H,), "ln1_b": (H,), "wqkv": (H, 3 * H), "bqkv": (3 * H,),
            "wo": (H, H), "bo": (H,), "ln2_g": (H,), "ln2_b": (H,),
            "w1": (H, F), "b1": (F,), "w2": (F, H), "b2": (H,)}[name]


def params_per_layer(hidden, mlp=0):
    """Parameter count of one layer (12 H^2 + 13 H when mlp = 4H)."""
    mlp = mlp or 4 * hidden
    return sum(int(np.prod(param_shape(hidden, mlp, n))) for n in PARAM_NAMES)


class StageError(Exception):
    """State or dependency misuse (double forward, backward without forward, bad order)."""


class StageOracle:
    """n_chunks chunks of `layers` layers each; mirrors the library's calls:
    forward(chunk, mb, act_in) -> act_out, backward(chunk, mb, grad_out) -> grad_in with
    gradient accumulation across micro-batches, and run_schedule(order, ...)."""

    def __init__(self, layers, hidden, heads, seq, microbatch, causal,
                 n_chunks=1, mlp=0, ln_eps=1e-5):
        assert hidden % heads == 0
        self.L, self.H, self.h, self.S, self.B = layers, hidden, heads, seq, microbatch
        self.causal = bool(causal)
        self.n_chunks = n_chunks
        self.F = mlp or 4 * hidden
        self.eps = ln_eps
        self.params = [[{n: np.zeros(param_shape(self.H, self.F, n)) for n in PARAM_NAMES}
                        for _ in range(layers)] for _ in range(n_chunks)]
        for c in range(n_chunks):
            for l in range(layers):
                self.params[c][l]["ln1_g"][:] = 1.0
                self.params[c][l]["ln2_g"][:] = 1.0
        self.lens = {}
        self.stash = {}
        self.zero_grad()

    # -- parameters and gradients
    def set_param(self, chunk, layer, name, value):
        value = np.asarray(value, dtype=np.float64)
        assert value.shape == self.params[chunk][layer][name].shape
        self.params[chunk][layer][name] = value.copy()

    def load_params(self, params):
        for c in range(self.n_chunks):
            for l in range(self.L):
                for n in PARAM_NAMES:
                    self.set_param(c, l, n, params[c][l][n])

    def zero_grad(self):
        # two accumulators, one per pipeline direction (the two replicas of Section 3.4)
        self.grads = [[[{n: np.zeros(param_shape(self.H, self.F, n)) for n in PARAM_NAMES}
                        for _ in range(self.L)] for _ in range(self.n_chunks)] for _ in range(2)]

    def get_grad(self, chunk, layer, name):
        return self.grads[0][chunk][layer][name]

    def set_seqlens(self, mb, lens):
        self.lens[mb] = None if lens is None else np.asarray(lens, dtype=np.int64)

    # -- one chunk, one micro-batch
    def forward(self, chunk, mb, act_in):
        if (chunk, mb) in self.stash:
            raise StageError(f"forward({chunk},{mb}) while its stash is still live")
        x = np.asarray(act_in, dtype=np.float64)
        caches = []
        lens = self.lens.get(mb)
        for l in range(self.L):
            x, cache = layer_forward(x, self.params[chunk][l], self.h, self.causal, lens, self.eps)
            caches.append(cache)
        self.stash[(chunk, mb)] = caches
        return x

    def backward(self, chunk, mb, grad_out, direction=0):
        if (chunk, mb) not in self.stash:
            raise StageError(f"backward({chunk},{mb}) without a stashed forward")
        caches = self.stash.pop((chunk, mb))
        d = np.asarray(grad_out, dtype=np.float64)
        for l in reversed(range(self.L)):
            d = layer_backward(d, caches[l], self.params[chunk][l], self.grads[direction][chunk][l])
        return d

    # -- loss on the last stage's output (synthetic: the paper's LM loss needs its datasets)
    @staticmethod
    def loss_and_grad(z, target, n_micro):
        """L_m = 1/(N*B*S) * sum_{b,s} 0.5 * ||z - Y||^2 ; returns (L_m, dL/dz)."""
        B, S, _ = z.shape
        diff = z - target
        scale = 1.0 / (n_micro * B * S)
        return 0.5 * scale * float((diff * diff).sum()), diff * scale

    def merge_directions(self):
        """The emulated all-reduce between the two replicas: grads(down) += grads(up)."""
        for c in range(self.n_chunks):
            for l in range(self.L):
                for n in PARAM_NAMES:
                    self.grads[0][c][l][n] += self.grads[1][c][l][n]
                    self.grads[1][c][l][n][:] = 0.0

    def run_schedule(self, order, inputs, targets):
        """Execute a serial list of ops (kind 'F'|'B', direction, vdev, stage, mb) over all
        n_chunks stages (stage index == chunk index), handing each stage's output to the next.
        inputs, targets: [N, B, S, H].  Returns the loss summed over micro-batches.  Raises
        StageError if an op's inputs are not there yet."""
        N = inputs.shape[0]
        last = self.n_chunks - 1
        act, grad = {}, {}
        loss = 0.0
        self.zero_grad()
        for op in order:
            kind, direction, stage, mb = op.kind, op.direction, op.stage, op.mb
            if kind == "F":
                if stage == 0:
                    xin = inputs[mb]
                elif (stage - 1, mb) in act:
                    xin = act[(stage - 1, mb)]
                else:
                    raise StageError(f"F(stage {stage}, mb {mb}) before its producer")
                out = self.forward(stage, mb, xin)
                act[(stage, mb)] = out
                if stage == last:
                    lm, g = self.loss_and_grad(out, targets[mb], N)
                    loss += lm
                    grad[(stage + 1, mb)] = g
            else:
                if (stage + 1, mb) not in grad:
                    raise StageError(f"B(stage {stage}, mb {mb}) before its upstream gradient")
                grad[(stage, mb)] = self.backward(stage, mb, grad.pop((stage + 1, mb)), direction)
        if self.stash:
            raise StageError("order leaves forwards without a backward")
        self.merge_directions()
        return loss

    def full_batch_reference(self, inputs, targets, lens=None):
        """Non-pipelined reference: concatenate all N micro-batches into one batch of N*B
        sequences, run every chunk back to back, one backward.  lens: [N, B] or None.
        Returns (loss, grads) with grads[chunk][layer][name]; does not touch self.grads."""
        N, B, S, H = inputs.shape
        x = inputs.reshape(N * B, S, H).astype(np.float64)
        ll = None if lens is None else np.asarray(lens).reshape(N * B)
        caches = []
        for c in range(self.n_chunks):
            for l in range(self.L):
                x, cache = layer_forward(x, self.params[c][l], self.h, self.causal, ll, self.eps)
                caches.append((c, l, cache))
        diff = x - targets.reshape(N * B, S, H)
        scale = 1.0 / (N * B * S)
        loss = 0.5 * scale * float((diff * diff).sum())
        d = diff * scale
        G = [[{n: np.zeros(param_shape(self.H, self.F, n)) for n in PARAM_NAMES}
              for _ in range(self.L)] for _ in range(self.n_chunks)]
        for c, l, cache in reversed(caches):
            d = layer_backward(d, cache, self.params[c][l], G[c][l])
        return loss, G, d.reshape(N, B, S, H)
