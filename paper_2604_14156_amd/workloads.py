"""Seeded synthetic inputs for the five workload shapes.

This module only draws inputs (weights, dictionaries, planted usage vectors,
caches, noise).  It holds none of the method's arithmetic: no sketching, no
recovery, no layer execution.  Both the CPU oracle's tests and the GPU tests
feed from it, so the two sides always see identical inputs.

Recipes
-------
dictionary   : per unit g a profile pi_g ~ N(0,1)^b; Psi_g = pi_g / ||pi_g||
               (block-diagonal, one atom per unit, rb = 1).
planted usage: z = sum_{g in S*} a_g pi_g + background,  S* uniform k-of-G.
               "unit"    : a_g = 1           (active entries are exactly N(0,1))
               "laplace" : a_g ~ Laplace(0,1) (heavy-tailed block magnitudes)
               background ~ N(0, bg^2)^n (the tail sigma_t of Assumption 1).
head usage   : k_h active entries N(0,1) + N(0, 0.05^2) background, identity
               dictionary.
saliency     : mask ~ Bernoulli(0.25); score ~ N(3,1) if active else N(0,1).
weights      : N(0, std^2), rounded to the storage type.
"""
from dataclasses import dataclass, field
import numpy as np

GAUSS = 0
RADEMACHER = 1
SRHT = 2


# ----------------------------------------------------------------------------
# bf16 storage helpers (data preparation only)
# ----------------------------------------------------------------------------
def to_bf16_bits(a):
    """float array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    # finite inputs only: the 32-bit add cannot wrap below the largest finite float
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def from_bf16_bits(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_bf16(a):
    """float array -> float32 array holding bf16-representable values."""
    return from_bf16_bits(to_bf16_bits(a))


# ----------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class FFNShape:
    d: int
    G: int
    b: int
    k: int
    m: int
    ens: int
    dtype: str            # "f32" | "bf16"
    wstd: float
    amp: str              # "unit" | "laplace"
    bg: float             # dense background std on z
    noise: float          # measurement noise std on y

    @property
    def n(self):
        return self.G * self.b


@dataclass(frozen=True)
class HeadShape:
    H: int = 32
    dh: int = 128
    kh: int = 12
    m: int = 16
    L: int = 4096
    ens: int = GAUSS
    bg: float = 0.05


CFG1 = FFNShape(d=256, G=16, b=64, k=4, m=64, ens=GAUSS, dtype="f32",
                wstd=1.0 / 16.0, amp="unit", bg=0.0, noise=0.01)
CFG2 = FFNShape(d=4096, G=172, b=64, k=43, m=256, ens=RADEMACHER, dtype="bf16",
                wstd=0.02, amp="laplace", bg=0.05, noise=0.0)
CFG3_HEADS = HeadShape()
CFG4 = FFNShape(d=8192, G=448, b=64, k=112, m=512, ens=GAUSS, dtype="bf16",
                wstd=0.02, amp="laplace", bg=0.0, noise=0.0)
CFG5_TOK = dict(n_tok=8192, m_tok=512, k_tok=2048, ens=RADEMACHER, p_active=0.25)


def scaled(shape, **kw):
    """A reduced copy of a shape (for tests that must finish in seconds)."""
    vals = {f: getattr(shape, f) for f in shape.__dataclass_fields__}
    vals.update(kw)
    return type(shape)(**vals)


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------
def rng_for(seed):
    return np.random.Generator(np.random.PCG64(seed))


def make_profiles(rng, G, b):
    """pi [G, b] ~ N(0,1) and the unit-norm dictionary psi [G, b, 1] (fp32 values)."""
    pi = rng.standard_normal((G, b))
    psi = (pi / np.linalg.norm(pi, axis=1, keepdims=True)).astype(np.float32)
    return pi, psi.reshape(G, b, 1)


def plant_usage(rng, pi, k, B, amp, bg):
    """B planted usage vectors.  Returns z [B, n] (fp32 values) and S* [B, k] ascending."""
    G, b = pi.shape
    z = np.zeros((B, G * b))
    supports = np.empty((B, k), dtype=np.int32)
    for t in range(B):
        S = np.sort(rng.choice(G, size=k, replace=False))
        supports[t] = S
        a = np.ones(k) if amp == "unit" else rng.laplace(0.0, 1.0, size=k)
        for j, g in enumerate(S):
            z[t, g * b:(g + 1) * b] = a[j] * pi[g]
        if bg > 0.0:
            z[t] += bg * rng.standard_normal(G * b)
    return z.astype(np.float32), supports


def drift_supports(rng, supports, G, swaps):
    """Next-token supports: every row of `supports` [B, k] has `swaps` of its units replaced by
    units it did not hold (planted support drift of 2*swaps units).  Rows come back ascending."""
    out = np.empty_like(supports)
    for t in range(supports.shape[0]):
        S = supports[t].tolist()
        leave = set(rng.choice(len(S), size=swaps, replace=False).tolist())
        pool = np.setdiff1d(np.arange(G), np.array(S))
        enter = rng.choice(pool, size=swaps, replace=False).tolist()
        out[t] = np.sort(np.array([g for i, g in enumerate(S) if i not in leave] + enter))
    return out


def plant_usage_on(rng, pi, supports, amp, bg):
    """Planted usage vectors on given supports [B, k] (same value recipe as plant_usage)."""
    G, b = pi.shape
    B, k = supports.shape
    z = np.zeros((B, G * b))
    for t in range(B):
        a = np.ones(k) if amp == "unit" else rng.laplace(0.0, 1.0, size=k)
        for j, g in enumerate(supports[t]):
            z[t, g * b:(g + 1) * b] = a[j] * pi[g]
        if bg > 0.0:
            z[t] += bg * rng.standard_normal(G * b)
    return z.astype(np.float32)


def plant_usage_literal(rng, G, b, k, B, amp, bg):
    """The literal reading: every active entry is its own draw (z is not in the
    span of any rank-1 dictionary).  Used for timing and parity only."""
    z = np.zeros((B, G * b))
    supports = np.empty((B, k), dtype=np.int32)
    for t in range(B):
        S = np.sort(rng.choice(G, size=k, replace=False))
        supports[t] = S
        for g in S:
            z[t, g * b:(g + 1) * b] = (rng.standard_normal(b) if amp == "unit"
                                       else rng.laplace(0.0, 1.0, size=b))
        if bg > 0.0:
            z[t] += bg * rng.standard_normal(G * b)
    return z.astype(np.float32), supports


def plant_head_usage(rng, hs, B):
    u = hs.bg * rng.standard_normal((B, hs.H))
    supports = np.empty((B, hs.kh), dtype=np.int32)
    for t in range(B):
        S = np.sort(rng.choice(hs.H, size=hs.kh, replace=False))
        supports[t] = S
        u[t, S] += rng.standard_normal(hs.kh)
    return u.astype(np.float32), supports


def plant_saliency(rng, n_tok, p_active):
    mask = rng.random(n_tok) < p_active
    s = np.where(mask, rng.normal(3.0, 1.0, n_tok), rng.normal(0.0, 1.0, n_tok))
    return s.astype(np.float32), mask


def plant_token_usage(rng, pi, S_star, mask, k, amp, bg):
    """Per-token usage vectors of a prompt [n_tok, n]: salient tokens (mask true) all use the support
    S_star with their own magnitudes, every other token uses k random units of its own."""
    G, b = pi.shape
    n_tok = mask.shape[0]
    z = np.zeros((n_tok, G * b), dtype=np.float32)
    for t in range(n_tok):
        S = S_star if mask[t] else np.sort(rng.choice(G, size=k, replace=False))
        a = np.ones(k) if amp == "unit" else rng.laplace(0.0, 1.0, size=k)
        row = np.zeros(G * b)
        for j, g in enumerate(S):
            row[g * b:(g + 1) * b] = a[j] * pi[g]
        if bg > 0.0:
            row += bg * rng.standard_normal(G * b)
        z[t] = row
    return z


def make_ffn_weights(rng, G, b, d, std, dtype):
    """Wg, Wu as [G, b, d]; Wd as [G, d, b]; values representable in `dtype`."""
    def draw(shape):
        w = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        return round_bf16(w) if dtype == "bf16" else w
    return draw((G, b, d)), draw((G, b, d)), draw((G, d, b))


def make_tokens(rng, T, d, dtype):
    x = rng.standard_normal((T, d), dtype=np.float32)
    return round_bf16(x) if dtype == "bf16" else x


def make_kv(rng, B, H, L, dh):
    q = round_bf16(rng.standard_normal((B, H, dh), dtype=np.float32))
    K = round_bf16(rng.standard_normal((B, H, L, dh), dtype=np.float32))
    V = round_bf16(rng.standard_normal((B, H, L, dh), dtype=np.float32))
    return q, K, V


def random_supports(rng, G, k, B):
    return np.stack([np.sort(rng.choice(G, size=k, replace=False)) for _ in range(B)]).astype(np.int32)
