"""Seeded synthetic inputs shared by the CPU oracle tests, the GPU parity tests and bench.py.

This module holds no transformer or schedule arithmetic.  It only produces reproducible
tensors: a counter-based integer hash (the splitmix64 finaliser) feeds Box-Muller for normal
values, and helpers round values to what bf16 / fp32 can represent so that both sides of a
parity test consume bit-identical inputs.

Workload recipe (all configs): activations and upstream gradients ~ N(0,1); weight matrices
and biases ~ N(0,0.02); LayerNorm gamma = 1, beta = 0 (optionally jittered for tests that
need every term exercised); BERT-style valid lengths uniform on an integer range.
Each tensor has its own stream, keyed by (seed, a string naming its role, integer indices).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass

import numpy as np

_MASK64 = np.uint64(0xFFFFFFFFFFFFFFFF)

# order of the per-layer parameter tensors; the index is the C-ABI's tensor id
PARAM_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """Bijective 64-bit mixer applied element-wise (uint64 in, uint64 out)."""
    with np.errstate(over="ignore"):
        x = (x + np.uint64(0x9E3779B97F4A7C15)) & _MASK64
        x = ((x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK64
        x = ((x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK64
        return x ^ (x >> np.uint64(31))


def stream_key(seed: int, role: str, *idx: int) -> np.uint64:
    """64-bit key of one tensor's stream."""
    k = np.array([(seed & 0xFFFFFFFF) | (zlib.crc32(role.encode()) << 32)], dtype=np.uint64)
    k = _splitmix64(k)
    for i in idx:
        k = _splitmix64(k ^ np.uint64((int(i) + 0x632BE59BD9B4E019) & 0xFFFFFFFFFFFFFFFF))
    return k[0]


def uniform01(key: np.uint64, n: int, offset: int = 0) -> np.ndarray:
    """n doubles in (0,1): counter `offset + i` hashed with the key, top 53 bits used."""
    ctr = np.arange(offset, offset + n, dtype=np.uint64)
    bits = _splitmix64(ctr ^ key)
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(key: np.uint64, shape, std: float = 1.0) -> np.ndarray:
    """fp64 N(0, std^2) tensor of the given shape via Box-Muller on two counter streams."""
    n = int(np.prod(shape))
    m = (n + 1) // 2
    u1 = uniform01(key, m, 0)
    u2 = uniform01(key, m, 1 << 40)
    r = np.sqrt(-2.0 * np.log(u1))
    z = np.concatenate([r * np.cos(2.0 * np.pi * u2), r * np.sin(2.0 * np.pi * u2)])[:n]
    return (z * std).reshape(shape)


def integers(key: np.uint64, n: int, lo: int, hi: int) -> np.ndarray:
    """n int32 values uniform on [lo, hi] inclusive."""
    u = uniform01(key, n)
    return np.minimum(lo + np.floor(u * (hi - lo + 1)), hi).astype(np.int32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16-representable value (ties to even); returns float32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    if np.all(np.isfinite(f)):
        # the rounding increment cannot carry out of 32 bits for a finite value
        b = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
        return b.view(np.float32).reshape(f.shape)
    b = b.astype(np.uint64)
    b = (b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return b.astype(np.uint32).view(np.float32).reshape(f.shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of round_bf16(x) (what a device bf16 buffer holds)."""
    return (round_bf16(x).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """float32 values of uint16 bf16 bit patterns."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to what `dtype` ('f32' | 'bf16') represents; returns float32."""
    if dtype == "bf16":
        return round_bf16(x)
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32)
    raise ValueError(dtype)


@dataclass(frozen=True)
class StageConfig:
    """Shape of one pipeline stage's chunk(s) of pre-LN transformer layers."""
    name: str
    layers: int          # layers per chunk
    hidden: int
    heads: int
    seq: int
    microbatch: int      # sequences per micro-batch (B)
    causal: bool
    dtype: str           # 'f32' | 'bf16'
    n_micro: int         # micro-batches per run (N)
    n_chunks: int = 1
    mlp: int = 0         # 0 -> 4*hidden
    len_lo: int = 0      # BERT-style valid-length range (inclusive); 0 -> no padding
    len_hi: int = 0
    ln_eps: float = 1e-5

    @property
    def F(self) -> int:
        return self.mlp or 4 * self.hidden

    @property
    def T(self) -> int:
        return self.microbatch * self.seq

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    def flops_per_microbatch(self, lens=None) -> float:
        """Algorithmic fwd+bwd flops of one chunk on one micro-batch (no recompute counted):
        linear layers 3 * 2*T*(3H^2 + H^2 + 2*H*F), attention 3 * 4*T*S*H*c with c = 1/2 causal,
        1 bidirectional (nominal, padded keys counted).  With `lens` (valid key counts per sequence
        of a bidirectional micro-batch) the attention term counts only unmasked keys: c_b = len_b/S."""
        T, H, S, Fm = self.T, self.hidden, self.seq, self.F
        gemm = 6.0 * T * (4 * H * H + 2 * H * Fm)
        if lens is not None and not self.causal:
            attn = 12.0 * S * H * float(np.sum(np.asarray(lens, dtype=np.float64)))
        else:
            attn = 12.0 * T * S * H * (0.5 if self.causal else 1.0)
        return self.layers * (gemm + attn)


# The five workloads of the baseline file, in its order, followed by one stage of each of the
# paper's two large models at their own shapes (Table 3: BERT-64 with 64 heads of width 40,
# GPT-96 with 32 heads of width 96; micro-batch sizes of Section 4.2).
CONFIGS = (
    StageConfig("cfg0_tiny_gpt_f32", 2, 128, 2, 64, 2, True, "f32", 4),
    StageConfig("cfg1_gpt_h2048", 4, 2048, 16, 2048, 1, True, "bf16", 8),
    StageConfig("cfg2_bert_h1024", 6, 1024, 16, 512, 8, False, "bf16", 8, len_lo=256, len_hi=512),
    StageConfig("cfg3_gpt_h5120", 2, 5120, 40, 2048, 2, True, "bf16", 16),
    StageConfig("cfg4_vsched_h1024", 2, 1024, 16, 1024, 1, True, "bf16", 8, n_chunks=8),
    StageConfig("cfg5_bert64_stage_h2560_d40", 4, 2560, 64, 512, 4, False, "bf16", 8, len_lo=256, len_hi=512),
    StageConfig("cfg6_gpt96_stage_h3072_d96", 6, 3072, 32, 1024, 1, True, "bf16", 8),
)


def param_shape(cfg: StageConfig, name: str):
    H, Fm = cfg.hidden, cfg.F
    return {"ln1_g": (H,), "ln1_b": (H,), "wqkv": (H, 3 * H), "bqkv": (3 * H,),
            "wo": (H, H), "bo": (H,), "ln2_g": (H,), "ln2_b": (H,),
            "w1": (H, Fm), "b1": (Fm,), "w2": (Fm, H), "b2": (H,)}[name]


def normal_bulk(key: np.uint64, shape, std: float = 1.0) -> np.ndarray:
    """float32 N(0, std^2) tensor from numpy's counter-based Philox generator keyed by the stream
    key: the same distribution as `normal`, about 30 times faster, for benchmark-sized tensors
    whose individual values no test compares (the two generators give different streams)."""
    rng = np.random.Generator(np.random.Philox(key=int(key)))
    out = rng.standard_normal(int(np.prod(shape)), dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out.reshape(shape)


def make_params(cfg: StageConfig, seed: int = 0, ln_jitter: float = 0.0, bulk: bool = False):
    """params[chunk][layer][name] -> float32 array already rounded to cfg.dtype.

    Weight matrices are row-major [in, out]; wqkv's columns are [q | k | v], head-major inside.
    ln_jitter > 0 perturbs gamma/beta away from (1, 0) so tests exercise the affine terms.
    bulk: for benchmarks, whose values no test compares: the same recipe from the faster generator
    `normal_bulk`, drawn once per tensor name; the other layers get that tensor with its rows rotated
    and its sign alternating (distinct values, same distribution), and the values are left unrounded
    (the library rounds weight matrices to the storage dtype itself).
    """
    if bulk:
        base = {}
        for ti, name in enumerate(PARAM_NAMES):
            shp = param_shape(cfg, name)
            key = stream_key(seed, "param:" + cfg.name, 0, 0, ti)
            if name in ("ln1_g", "ln2_g"):
                base[name] = (1.0 + ln_jitter * normal_bulk(key, shp)).astype(np.float32)
            elif name in ("ln1_b", "ln2_b"):
                base[name] = (ln_jitter * normal_bulk(key, shp)).astype(np.float32)
            else:
                base[name] = normal_bulk(key, shp, 0.02)
        out = []
        for c in range(cfg.n_chunks):
            layers = []
            for l in range(cfg.layers):
                i = c * cfg.layers + l
                p = {}
                for name in PARAM_NAMES:
                    if i == 0 or name in ("ln1_g", "ln2_g", "ln1_b", "ln2_b"):
                        p[name] = base[name]
                    else:
                        v = np.roll(base[name], 977 * i, axis=0)
                        p[name] = -v if i & 1 else v
                layers.append(p)
            out.append(layers)
        return out
    draw = normal
    out = []
    for c in range(cfg.n_chunks):
        layers = []
        for l in range(cfg.layers):
            p = {}
            for ti, name in enumerate(PARAM_NAMES):
                shp = param_shape(cfg, name)
                key = stream_key(seed, "param:" + cfg.name, c, l, ti)
                if name in ("ln1_g", "ln2_g"):
                    v = 1.0 + ln_jitter * draw(key, shp)
                elif name in ("ln1_b", "ln2_b"):
                    v = ln_jitter * draw(key, shp)
                else:
                    v = draw(key, shp, 0.02)
                p[name] = round_to(v, cfg.dtype)
            layers.append(p)
        out.append(layers)
    return out


def make_activation(cfg: StageConfig, role: str, mb: int, seed: int = 0, std: float = 1.0, bulk: bool = False):
    """[B, S, H] float32 tensor (rounded to cfg.dtype): role 'act_in' | 'grad_out' | 'target'."""
    key = stream_key(seed, role + ":" + cfg.name, mb)
    draw = normal_bulk if bulk else normal
    return round_to(draw(key, (cfg.microbatch, cfg.seq, cfg.hidden), std), cfg.dtype)


def make_seqlens(cfg: StageConfig, mb: int, seed: int = 0):
    """int32 [B] valid lengths for BERT-style key padding, or None when the config has none."""
    if cfg.len_hi <= 0:
        return None
    return integers(stream_key(seed, "lens:" + cfg.name, mb), cfg.microbatch, cfg.len_lo, cfg.len_hi)


def scaled(cfg: StageConfig, **kw) -> StageConfig:
    """A copy of cfg with some fields replaced (reduced shapes for fast tests)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return StageConfig(**d)
