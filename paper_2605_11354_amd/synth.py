"""Seeded synthetic multi-view token tensors for the SLA forward.

This module only *draws inputs*; it contains none of the attention arithmetic and is the
one piece of code that both the CPU oracle's tests and the HIP path's tests/bench use, so
that both sides see bit-identical tensors.  Everything is generated on the host with a
counter-based generator (splitmix64 hash of (key, counter) -> Box-Muller), so a tensor
element depends only on (seed, stream, index) and never on chunking or library versions.

Recipe (stands in for VGGT / DA3-Large activations, which need weights and datasets that
are not available): per batch item a cluster id is drawn uniformly per token and shared by
Q, K and all heads; every head has its own Gaussian cluster centres; Q and K are
0.5*centre + independent N(0,1) noise, V is N(0,1); all rounded to bf16
(round-to-nearest-even) with magnitudes below 2^-20 flushed to zero.  The optional FP8 path
quantises each (head, token block) with the scaled E4M3 quantiser of the paper's App. B.2
(scale = max(amax, 1e-8)/448, clamp to +-448, round to nearest even), block = the pooling
block of the tensor (bq rows for Q, bk rows for K and V).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


@dataclass(frozen=True)
class SLAConfig:
    """Shape of one SLA workload (the five benchmark configurations use this)."""
    name: str
    B: int
    H: int
    N: int
    D: int
    bq: int
    bk: int
    crit_frac: float
    neg_frac: float
    dtype: str            # "bf16" or "fp8"
    n_clusters: int
    centres_per_batch: bool   # True: every batch item (frame) draws its own centre set
    proj_per_head: bool
    seed: int = 0

    def with_(self, **kw) -> "SLAConfig":
        return replace(self, **kw)


CONFIGS = [
    SLAConfig("c0_tiny", 1, 2, 512, 64, 64, 64, 0.125, 0.50, "bf16", 16, False, False),
    SLAConfig("c1_global8", 1, 16, 8 * 1374, 64, 64, 64, 0.05, 0.75, "bf16", 256, False, True),
    SLAConfig("c2_global32", 1, 16, 32 * 1374, 64, 128, 64, 0.05, 0.80, "bf16", 256, False, True),
    SLAConfig("c3_frame32", 32, 16, 1374, 64, 64, 64, 0.10, 0.60, "bf16", 64, True, True),
    SLAConfig("c4_fp8_global100", 1, 16, 100 * 1374, 64, 128, 64, 0.03, 0.85, "fp8", 256, False, True),
]

# stream identifiers of the counter-based generator
_S_CLUSTER, _S_CENTRE, _S_NQ, _S_NK, _S_V, _S_W = 1, 2, 3, 4, 5, 6


def _mix(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on uint64 arrays (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def _key(seed: int, stream: int, a: int = 0, b: int = 0) -> np.uint64:
    k = np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    for v in (stream, a, b):
        k = _mix(k ^ np.uint64(v))
    return k[0]


def _uniform(key: np.uint64, counter: np.ndarray) -> np.ndarray:
    """U[0,1) with 53 bits from hash(key, counter)."""
    with np.errstate(over="ignore"):
        z = _mix(_mix(counter.astype(np.uint64)) ^ key)
    return (z >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normals(key: np.uint64, n: int, start: int = 0) -> np.ndarray:
    """n standard normals, element i a function of (key, start+i) only."""
    idx = np.arange(start, start + n, dtype=np.uint64)
    u1 = _uniform(key, idx * np.uint64(2))
    u2 = _uniform(key, idx * np.uint64(2) + np.uint64(1))
    return np.sqrt(-2.0 * np.log1p(-u1)) * np.cos(2.0 * np.pi * u2)


def uniform_ints(key: np.uint64, n: int, hi: int) -> np.ndarray:
    return np.minimum((_uniform(key, np.arange(n, dtype=np.uint64)) * hi).astype(np.int64), hi - 1)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float -> bf16 bit pattern (uint16), round-to-nearest-even, |x| < 2^-20 flushed to 0."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    bits = r.astype(np.uint16)
    small = np.abs(bf16_bits_to_f32(bits)) < 2.0 ** -20
    bits[small] = 0
    return bits


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- E4M3 (OCP "fn")
def e4m3_code_values() -> np.ndarray:
    """Value of each of the 256 E4M3 codes (1-4-3, bias 7, no inf, 0x7f/0xff = NaN)."""
    c = np.arange(256)
    s = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 7).astype(np.float64)
    v = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))
    v = s * v
    v[(c & 0x7F) == 0x7F] = np.nan
    return v


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """fp32 values already clamped to [-448, 448] -> E4M3 codes, round-to-nearest-even.

    Works on the value grid: within a binade 2^e the spacing is 2^(e-3) (e >= -6), below
    2^-6 the spacing is 2^-9; np.rint rounds half to even, which on these grids is the same
    as even mantissa.
    """
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    a = np.abs(x)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6, 8)
    step = 2.0 ** (e - 3)
    q = np.rint(a / step) * step          # may round up into the next binade: still on grid
    q = np.minimum(q, 448.0)
    # q -> code
    with np.errstate(divide="ignore"):
        eq = np.floor(np.log2(np.where(q > 0, q, 1.0)))
    sub = q < 2.0 ** -6
    eq = np.where(sub, -6, eq)
    mant = np.where(sub, q / 2.0 ** -9, (q / 2.0 ** eq - 1.0) * 8.0)
    code = np.where(sub, 0, (eq + 7).astype(np.int64) << 3) + mant.astype(np.int64)
    code = code.astype(np.uint8)
    code |= (np.signbit(x).astype(np.uint8) << 7)
    return code


def quantise_e4m3_blocks(bits: np.ndarray, blk: int):
    """bf16 bits [..., N, D] -> (codes uint8 [..., N, D], scales fp32 [..., ceil(N/blk)]).

    Scaled quantiser of App. B.2 applied per block of `blk` consecutive tokens:
    scale = max(amax, 1e-8)/448 in fp32, x/scale in fp32, clamp, cast RNE.
    """
    x = bf16_bits_to_f32(bits)
    N = x.shape[-2]
    nb = (N + blk - 1) // blk
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(x.shape[:-2] + (nb,), dtype=np.float32)
    for j in range(nb):
        sl = slice(j * blk, min(N, (j + 1) * blk))
        xb = x[..., sl, :]
        amax = np.abs(xb).max(axis=(-1, -2)).astype(np.float32)
        sc = (np.maximum(amax, np.float32(1e-8)) / np.float32(448.0)).astype(np.float32)
        scales[..., j] = sc
        y = (xb / sc[..., None, None]).astype(np.float32)
        codes[..., sl, :] = e4m3_encode(np.clip(y, -448.0, 448.0))
    return codes, scales


# --------------------------------------------------------------------------- tensors
def make_inputs(cfg: SLAConfig) -> dict:
    """Draw Q, K, V, W_proj for a configuration.

    Returns a dict with numpy arrays:
      Q, K, V : uint16 bf16 bit patterns [B,H,N,D]   (dtype "bf16"), or
                uint8 E4M3 codes                       (dtype "fp8") plus
      sQ, sK, sV : float32 per-block scales [B,H,Nqb] / [B,H,Nkb] / [B,H,Nkb] (fp8 only)
      W : uint16 bf16 bits [D,D] or [H,D,D]  (row-major [D_in, D_out])
    """
    B, H, N, D = cfg.B, cfg.H, cfg.N, cfg.D
    Q = np.empty((B, H, N, D), dtype=np.uint16)
    K = np.empty((B, H, N, D), dtype=np.uint16)
    V = np.empty((B, H, N, D), dtype=np.uint16)
    for b in range(B):
        cl = uniform_ints(_key(cfg.seed, _S_CLUSTER, b), N, cfg.n_clusters)
        cb = b if cfg.centres_per_batch else 0
        for h in range(H):
            cen = normals(_key(cfg.seed, _S_CENTRE, cb, h), cfg.n_clusters * D).reshape(cfg.n_clusters, D)
            base = 0.5 * cen[cl]
            Q[b, h] = to_bf16_bits(base + normals(_key(cfg.seed, _S_NQ, b, h), N * D).reshape(N, D))
            K[b, h] = to_bf16_bits(base + normals(_key(cfg.seed, _S_NK, b, h), N * D).reshape(N, D))
            V[b, h] = to_bf16_bits(normals(_key(cfg.seed, _S_V, b, h), N * D).reshape(N, D))
    nW = H if cfg.proj_per_head else 1
    W = to_bf16_bits(normals(_key(cfg.seed, _S_W), nW * D * D).reshape(nW, D, D) / 8.0)
    if not cfg.proj_per_head:
        W = W[0]
    out = {"W": W, "cfg": cfg}
    if cfg.dtype == "fp8":
        out["Q"], out["sQ"] = quantise_e4m3_blocks(Q, cfg.bq)
        out["K"], out["sK"] = quantise_e4m3_blocks(K, cfg.bk)
        out["V"], out["sV"] = quantise_e4m3_blocks(V, cfg.bk)
    else:
        out["Q"], out["K"], out["V"] = Q, K, V
        out["sQ"] = out["sK"] = out["sV"] = None
    return out
