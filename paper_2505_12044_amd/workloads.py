"""Seeded synthetic inputs for the five benchmark configurations.

This module holds input generation only: random draws, the closed-form / SVD factor
construction that turns a bias into the factors the library consumes, and storage-type
rounding.  It contains none of the attention arithmetic and imports neither the HIP
binding nor the CPU oracle, so both sides can be fed from it.

Every array is returned as float32 holding values that are exactly representable in the
configuration's storage type (bf16 configurations are rounded to bf16 with
round-to-nearest-even first), so the GPU kernels and the float64 oracle see identical
numbers.

The five shapes stand in for the workloads the paper measures on (a GPT-2-style ALiBi
decoder, Swin window attention, Pairformer triangle attention, long-sequence training);
no item of those datasets or models is reproduced here.

Generator: numpy.random.default_rng(1000 + config number); draw order q, k, v, bias
source, dout.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

__all__ = ["Workload", "make_workload", "CONFIG_NAMES", "round_bf16", "f32_to_bf16_bits",
           "bf16_bits_to_f32", "alibi_factors", "swin_table_bias", "pair_bias", "distance_factors",
           "distance_factors_rank5", "make_pde_workload"]

CONFIG_NAMES = ("tiny_fp32", "alibi_causal", "vision_relpos", "pairformer", "long_train")


# ---------------------------------------------------------------------------------
# storage-type rounding
# ---------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even; inputs must be finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(np.shape(x))


def _store(x, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return round_bf16(x) if dtype == "bf16" else x


# ---------------------------------------------------------------------------------
# bias sources
# ---------------------------------------------------------------------------------
def alibi_slopes_f32(num_heads: int):
    """Head slopes m_h = 2^(-8 (h+1) / num_heads) of the decoder workload, float32 [H]."""
    h = np.arange(num_heads, dtype=np.float64)
    return (2.0 ** (-8.0 * (h + 1.0) / num_heads)).astype(np.float32)


def alibi_factors(num_heads: int, n: int):
    """Exact rank-2 factors of the ALiBi bias -m_h (i - j) (Example 3.4, with the slope and
    sign of the decoder workload): phi_q(i) = [-m_h i, m_h], phi_k(j) = [1, j], 0-based,
    m_h = 2^(-8 (h+1) / num_heads).  Returned in float32: [1,H,n,2] each."""
    h = np.arange(num_heads, dtype=np.float64)
    m = 2.0 ** (-8.0 * (h + 1.0) / num_heads)
    pos = np.arange(n, dtype=np.float64)
    phi_q = np.empty((1, num_heads, n, 2), dtype=np.float64)
    phi_k = np.empty((1, num_heads, n, 2), dtype=np.float64)
    phi_q[0, :, :, 0] = -m[:, None] * pos[None, :]
    phi_q[0, :, :, 1] = m[:, None]
    phi_k[0, :, :, 0] = 1.0
    phi_k[0, :, :, 1] = pos[None, :]
    return phi_q.astype(np.float32), phi_k.astype(np.float32)


def distance_factors(x: np.ndarray, alpha: np.ndarray, strength: float):
    """Exact rank-9 factors of the weighted squared-distance bias
    b_ij = -strength * alpha_i * ||x_i - x_j||^2 for 3-D positions x [n,3] (Example 3.5 with
    the token-wise weight of the PDE-solver experiment, Sec. 4.3): per axis a the three
    columns [x_a^2, 1, -2 x_a] on the query side against [1, y_a^2, y_a] on the key side; the
    weight multiplies the query side.  alpha: [H, n].  Returns float32 [1,H,n,9] each."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    uq = np.empty((n, 9)); uk = np.empty((n, 9))
    for a in range(3):
        uq[:, 3 * a] = x[:, a] ** 2; uq[:, 3 * a + 1] = 1.0; uq[:, 3 * a + 2] = -2.0 * x[:, a]
        uk[:, 3 * a] = 1.0; uk[:, 3 * a + 1] = x[:, a] ** 2; uk[:, 3 * a + 2] = x[:, a]
    w = -float(strength) * np.asarray(alpha, dtype=np.float64)          # [H, n]
    phi_q = (w[:, :, None] * uq[None]).astype(np.float32)[None]
    phi_k = np.broadcast_to(uk.astype(np.float32), (1, w.shape[0], n, 9)).copy()
    return phi_q, phi_k


def distance_factors_rank5(x: np.ndarray, alpha: np.ndarray, strength: float):
    """The same bias as distance_factors with the per-axis constants merged:
    ||x - y||^2 = |x|^2 + |y|^2 - 2 x.y, i.e. [|x|^2, 1, -2 x_0, -2 x_1, -2 x_2] against
    [1, |y|^2, y_0, y_1, y_2] (rank 5 instead of the nine printed columns of Example 3.5).
    Returns float32 [1,H,n,5] each."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    n2 = np.sum(x * x, axis=1)
    uq = np.concatenate([n2[:, None], np.ones((n, 1)), -2.0 * x], axis=1)
    uk = np.concatenate([np.ones((n, 1)), n2[:, None], x], axis=1)
    w = -float(strength) * np.asarray(alpha, dtype=np.float64)
    phi_q = (w[:, :, None] * uq[None]).astype(np.float32)[None]
    phi_k = np.broadcast_to(uk.astype(np.float32), (1, w.shape[0], n, 5)).copy()
    return phi_q, phi_k


def swin_table_bias(rng, num_heads: int, grid: int, sigma: float = 4.0) -> np.ndarray:
    """Relative-position bias of window attention on a grid x grid window: per head a smooth
    random (2 grid - 1)^2 table (unit-variance Gaussian noise, separable Gaussian blur of
    width sigma truncated at 4 sigma with reflecting borders, rescaled to unit standard
    deviation), indexed by the offset between two tokens.  Returns float64 [H, N, N]."""
    from scipy.ndimage import gaussian_filter

    side = 2 * grid - 1
    n = grid * grid
    y, x = np.divmod(np.arange(n), grid)
    dy = y[:, None] - y[None, :] + (grid - 1)
    dx = x[:, None] - x[None, :] + (grid - 1)
    out = np.empty((num_heads, n, n), dtype=np.float64)
    for h in range(num_heads):
        t = rng.standard_normal((side, side))
        t = gaussian_filter(t, sigma=sigma, mode="reflect", truncate=4.0)
        t = t / np.std(t)
        out[h] = t[dy, dx]
    return out


def pair_bias(rng, num_heads: int, n: int, channels: int = 128, noise: float = 0.1) -> np.ndarray:
    """Pairformer-style bias projected from a pair representation z [n,n,channels]:
    z_jk = a_j b_k (broadcast over channels) + noise * N(0,1); b[h] = z . w_h with
    w_h ~ N(0, 1/channels).  Returns float64 [H, n, n]."""
    a = rng.standard_normal(n)
    b = rng.standard_normal(n)
    eps = rng.standard_normal((n, n, channels))
    w = rng.standard_normal((num_heads, channels)) / np.sqrt(channels)
    z = a[:, None, None] * b[None, :, None] + noise * eps
    return np.einsum("jkc,hc->hjk", z, w)


def _svd_factors(bias: np.ndarray, rank: int):
    """Truncated SVD with the singular values split evenly between the two factors."""
    u, s, vt = np.linalg.svd(bias, full_matrices=False)
    root = np.sqrt(s[:rank])
    return u[:, :rank] * root, vt[:rank].T * root


# ---------------------------------------------------------------------------------
# workloads
# ---------------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    B: int
    H: int
    N: int
    C: int
    R: int
    causal: bool
    dtype: str                    # storage / MFMA input type of q, k, v, out: "f32" | "bf16"
    phi_dtype: str                # storage type of the factors: "f32" | "bf16"
    q: np.ndarray                 # [B,H,N,C]
    k: np.ndarray
    v: np.ndarray
    phi_q: np.ndarray             # [Bp,H,N,R], Bp in {1, B}
    phi_k: np.ndarray
    dout: Optional[np.ndarray] = None          # [B,H,N,C] upstream gradient
    bias: Optional[np.ndarray] = None          # dense [Bp,H,N,N] for the baseline (may be None)
    bias_exact: Optional[np.ndarray] = None    # float64 unrounded source bias, when one exists
    notes: dict = field(default_factory=dict)

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.C))

    @property
    def phi_broadcast(self) -> bool:
        return self.phi_q.shape[0] == 1 and self.B > 1

    @property
    def pairs(self) -> int:
        n = self.N
        per = n * (n + 1) // 2 if self.causal else n * n
        return self.B * self.H * per

    def fwd_flops(self) -> float:
        """Algorithmic forward flop: 2 (C + R) per pair for the scores, 2 C for the values."""
        return 2.0 * (2 * self.C + self.R) * self.pairs

    def bwd_flops(self) -> float:
        return 2.0 * (5 * self.C + 3 * self.R) * self.pairs


_DEFAULTS = {
    "tiny_fp32":     dict(B=1,   H=2,  N=256,   C=64,  R=4,  causal=False, dtype="f32",  phi_dtype="f32"),
    "alibi_causal":  dict(B=4,   H=16, N=4096,  C=128, R=2,  causal=True,  dtype="bf16", phi_dtype="f32"),
    "vision_relpos": dict(B=8,   H=12, N=1024,  C=64,  R=32, causal=False, dtype="bf16", phi_dtype="bf16"),
    "pairformer":    dict(B=384, H=4,  N=384,   C=32,  R=16, causal=False, dtype="bf16", phi_dtype="bf16"),
    "long_train":    dict(B=2,   H=8,  N=16384, C=128, R=8,  causal=False, dtype="bf16", phi_dtype="bf16"),
}


def make_workload(name: str, dense: bool = False, with_dout: Optional[bool] = None,
                  **overrides) -> Workload:
    """Build one configuration.  `overrides` may shrink B, H, N (and grid for vision_relpos
    via N = grid^2) for tests; the recipe is otherwise unchanged.  `dense=True` also
    materialises the dense bias for the baseline kernel (never for long_train at full size
    unless asked: it is 8.6 GB)."""
    if name not in _DEFAULTS:
        raise KeyError(f"unknown workload {name!r}; choose from {CONFIG_NAMES}")
    p = dict(_DEFAULTS[name])
    p.update(overrides)
    B, H, N, C, R = p["B"], p["H"], p["N"], p["C"], p["R"]
    dtype, phi_dtype = p["dtype"], p["phi_dtype"]
    idx = CONFIG_NAMES.index(name) + 1
    rng = np.random.default_rng(1000 + idx)
    if with_dout is None:
        with_dout = name == "long_train"

    def draw(shape):
        return _store(rng.standard_normal(shape), dtype)

    q = draw((B, H, N, C))
    k = draw((B, H, N, C))
    v = draw((B, H, N, C))
    bias = None
    bias_exact = None
    notes = {}

    if name == "tiny_fp32":
        phi_q = _store(0.5 * rng.standard_normal((1 if B == 1 else B, H, N, R)), phi_dtype)
        phi_k = _store(0.5 * rng.standard_normal((1 if B == 1 else B, H, N, R)), phi_dtype)
        if dense:
            bias = _store(np.einsum("bhir,bhjr->bhij", phi_q.astype(np.float64),
                                    phi_k.astype(np.float64)), dtype)
    elif name == "alibi_causal":
        phi_q, phi_k = alibi_factors(H, N)
        phi_q, phi_k = _store(phi_q, phi_dtype), _store(phi_k, phi_dtype)
        if dense:
            h = np.arange(H, dtype=np.float64)
            m = 2.0 ** (-8.0 * (h + 1.0) / H)
            pos = np.arange(N, dtype=np.float64)
            d = pos[:, None] - pos[None, :]
            bias = np.empty((1, H, N, N), dtype=np.float32)
            for hh in range(H):
                bias[0, hh] = _store(-m[hh] * d, dtype)
    elif name == "vision_relpos":
        grid = int(round(np.sqrt(N)))
        if grid * grid != N:
            raise ValueError("vision_relpos needs N to be a square")
        bias_exact = swin_table_bias(rng, H, grid)[None]          # [1,H,N,N]
        fq = np.empty((1, H, N, R)); fk = np.empty((1, H, N, R))
        for hh in range(H):
            fq[0, hh], fk[0, hh] = _svd_factors(bias_exact[0, hh], R)
        phi_q, phi_k = _store(fq, phi_dtype), _store(fk, phi_dtype)
        if dense:
            bias = _store(bias_exact, dtype)
    elif name == "pairformer":
        bias_exact = pair_bias(rng, H, N)[None]                   # [1,H,N,N]
        fq = np.empty((1, H, N, R)); fk = np.empty((1, H, N, R))
        for hh in range(H):
            fq[0, hh], fk[0, hh] = _svd_factors(bias_exact[0, hh], R)
        phi_q, phi_k = _store(fq, phi_dtype), _store(fk, phi_dtype)
        if dense:
            bias = _store(bias_exact, dtype)
    elif name == "long_train":
        sigma = float(R) ** -0.25 if R > 0 else 0.0      # Var(phi_q . phi_k) = R sigma^4 = 1
        phi_q = _store(sigma * rng.standard_normal((B, H, N, R)), phi_dtype)
        phi_k = _store(sigma * rng.standard_normal((B, H, N, R)), phi_dtype)
        if dense:
            bias = np.empty((B, H, N, N), dtype=np.float32)
            for b in range(B):
                for hh in range(H):
                    bias[b, hh] = _store(phi_q[b, hh].astype(np.float64) @ phi_k[b, hh].astype(np.float64).T, dtype)
    dout = draw((B, H, N, C)) if with_dout else None
    return Workload(name=name, B=B, H=H, N=N, C=C, R=R, causal=p["causal"], dtype=dtype,
                    phi_dtype=phi_dtype, q=q, k=k, v=v, phi_q=phi_q, phi_k=phi_k, dout=dout,
                    bias=bias, bias_exact=bias_exact, notes=notes)


def make_pde_workload(B: int = 1, H: int = 8, N: int = 32186, C: int = 16, strength: float = 4.0,
                      seed: int = 1006, rank5: bool = False) -> Workload:
    """The shape of the paper's PDE-solver attention (Sec. 4.3): N = 32186 mesh points, 8 heads
    of 16 channels, bias -s alpha_i ||x_i - x_j||^2 as rank-9 fp32 factors shared over the
    batch.  Points are uniform in the unit cube, alpha ~ U(0.5, 1.5) per head and point;
    q, k, v, dout ~ N(0,1) rounded to bf16.  A stand-in for the mesh of the paper's dataset,
    which is not reproduced.  rank5 supplies the same bias as five merged columns."""
    rng = np.random.default_rng(seed)
    q, k, v = (_store(rng.standard_normal((B, H, N, C)), "bf16") for _ in range(3))
    x = rng.random((N, 3))
    alpha = 0.5 + rng.random((H, N))
    phi_q, phi_k = (distance_factors_rank5 if rank5 else distance_factors)(x, alpha, strength)
    dout = _store(rng.standard_normal((B, H, N, C)), "bf16")
    return Workload(name="pde_distance", B=B, H=H, N=N, C=C, R=phi_q.shape[-1], causal=False, dtype="bf16",
                    phi_dtype="f32", q=q, k=k, v=v, phi_q=phi_q, phi_k=phi_k, dout=dout,
                    notes={"x": x, "alpha": alpha, "strength": strength})
