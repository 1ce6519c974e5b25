"""ctypes wrapper around the fp64 CPU oracle (oracle/sla_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  It never imports the GPU package and the GPU package never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sla_oracle.c")
_LIB = os.path.join(_HERE, "libsla_oracle.so")
_lib = None


class Params(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("N", C.c_int32), ("D", C.c_int32),
                ("bq", C.c_int32), ("bk", C.c_int32), ("k_crit", C.c_int32), ("k_neg", C.c_int32),
                ("dtype", C.c_int32), ("proj_per_head", C.c_int32), ("sm_scale", C.c_double), ("phi", C.c_int32)]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction; fma() is explicit)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off", "-mfma",
               "-Wall", "-Wextra", "-Werror", _SRC, "-o", _LIB, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.sla_oracle_threads.restype = C.c_int
        for f in (_lib.sla_oracle_classify, _lib.sla_oracle_states_head, _lib.sla_oracle_attend):
            f.restype = C.c_int
    return _lib


def threads() -> int:
    return int(lib().sla_oracle_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def counts(crit_frac: float, neg_frac: float, Nkb: int):
    kc, kn = C.c_int32(), C.c_int32()
    lib().sla_oracle_counts(C.c_double(crit_frac), C.c_double(neg_frac), C.c_int32(Nkb), C.byref(kc), C.byref(kn))
    return kc.value, kn.value


def make_params(B, H, N, bq, bk, k_crit, k_neg, dtype="bf16", proj_per_head=False, sm_scale=None, D=64, phi="softmax"):
    """phi: feature map of the linear branch, "softmax" (over the channels) or "elu1" (ELU(x)+1, Alg. 1 step 6)."""
    return Params(B, H, N, D, bq, bk, k_crit, k_neg, 0 if dtype == "bf16" else 1,
                  1 if proj_per_head else 0, (1.0 / np.sqrt(D)) if sm_scale is None else sm_scale,
                  {"softmax": 0, "elu1": 1}[phi])


def _chk(x, dt):
    assert x is None or (x.dtype == dt and x.flags["C_CONTIGUOUS"]), (None if x is None else x.dtype, dt)


def classify(p: Params, Q, K, sQ=None, sK=None, want_scores=False, want_pc=False, want_means=False):
    """Steps 1-4.  Returns dict(labels, scores?, Pc?, qbar?, kbar?)."""
    dt = np.uint16 if p.dtype == 0 else np.uint8
    _chk(Q, dt), _chk(K, dt), _chk(sQ, np.float32), _chk(sK, np.float32)
    Nqb, Nkb = -(-p.N // p.bq), -(-p.N // p.bk)
    shp = (p.B, p.H, Nqb, Nkb)
    out = {"labels": np.zeros(shp, np.int8)}
    out["scores"] = np.zeros(shp, np.float64) if want_scores else None
    out["Pc"] = np.zeros(shp, np.float64) if want_pc else None
    out["qbar"] = np.zeros((p.B, p.H, Nqb, 64)) if want_means else None
    out["kbar"] = np.zeros((p.B, p.H, Nkb, 64)) if want_means else None
    rc = lib().sla_oracle_classify(C.byref(p), _p(Q), _p(K), _p(sQ), _p(sK), _p(out["labels"]),
                                   _p(out["scores"]), _p(out["Pc"]), _p(out["qbar"]), _p(out["kbar"]))
    assert rc == 0, rc
    return out


def states_head(p: Params, K, V, sK, sV, bh: int):
    """Step 6a for one (b,h): h [Nkb,64,64] (h[j][d][e]), z [Nkb,64]."""
    Nkb = -(-p.N // p.bk)
    h = np.zeros((Nkb, 64, 64)); z = np.zeros((Nkb, 64))
    rc = lib().sla_oracle_states_head(C.byref(p), _p(K), _p(V), _p(sK), _p(sV), C.c_int32(bh), _p(h), _p(z))
    assert rc == 0, rc
    return h, z


def attend(p: Params, Q, K, V, W, labels, sel=None, sQ=None, sK=None, sV=None, want_parts=False):
    """Steps 5-7 on the query blocks in `sel` (list of (bh, i)); None = all blocks.

    Returns dict(O [n_sel,bq,64], O_sparse?, O_lin?, sel)."""
    dt = np.uint16 if p.dtype == 0 else np.uint8
    _chk(Q, dt), _chk(K, dt), _chk(V, dt), _chk(W, np.uint16), _chk(labels, np.int8)
    Nqb = -(-p.N // p.bq)
    if sel is None:
        sel = [(bh, i) for bh in range(p.B * p.H) for i in range(Nqb)]
    sel_bh = np.ascontiguousarray([s[0] for s in sel], dtype=np.int32)
    sel_i = np.ascontiguousarray([s[1] for s in sel], dtype=np.int32)
    n = len(sel)
    O = np.zeros((n, p.bq, 64))
    Osp = np.zeros((n, p.bq, 64)) if want_parts else None
    Olin = np.zeros((n, p.bq, 64)) if want_parts else None
    rc = lib().sla_oracle_attend(C.byref(p), _p(Q), _p(K), _p(V), _p(sQ), _p(sK), _p(sV), _p(W), _p(labels),
                                 C.c_int32(n), _p(sel_bh), _p(sel_i), _p(O), _p(Osp), _p(Olin))
    assert rc == 0, rc
    return {"O": O, "O_sparse": Osp, "O_lin": Olin, "sel": sel}


def forward(p: Params, Q, K, V, W, sQ=None, sK=None, sV=None, sel=None, want_parts=False):
    """Whole SLA forward: classify, then attend.  With sel=None, O is scattered to [B,H,N,64]."""
    c = classify(p, Q, K, sQ, sK)
    a = attend(p, Q, K, V, W, c["labels"], sel, sQ, sK, sV, want_parts)
    a["labels"] = c["labels"]
    if sel is None:
        Nqb = -(-p.N // p.bq)
        for k in ("O", "O_sparse", "O_lin"):
            if a[k] is not None:
                a[k] = a[k].reshape(p.B, p.H, Nqb * p.bq, 64)[:, :, :p.N, :]
    return a


def grad_wproj(p: Params, Q, K, V, labels, dO, sQ=None, sK=None, sV=None):
    """Gradient of L = sum(O * dO) with respect to the projection of the linear branch.

    Alg. 1 step 10 / eq. (1): O = O_sparse + O_lin W_O, and W_O is the only parameter the method
    trains (section 3.3), so dL/dW_O = sum over the tokens (and over every (b,h) that uses the matrix)
    of O_lin[t]^T dO[t], with O_lin the normalised linear output before the projection.  No gradient
    flows through the block masks or into Q, K, V.

    dO: float64 [B,H,N,64].  Returns dW float64 [nW,64,64] ([D_in, D_out]), nW = H if the projection
    is per head, else 1."""
    _chk(labels, np.int8)
    dO = np.ascontiguousarray(dO, dtype=np.float64)
    assert dO.shape == (p.B, p.H, p.N, 64), dO.shape
    Wzero = np.zeros((p.H if p.proj_per_head else 1, 64, 64), np.uint16)      # the projection itself does not enter
    parts = attend(p, Q, K, V, Wzero, labels, None, sQ, sK, sV, want_parts=True)
    Nqb = -(-p.N // p.bq)
    olin = parts["O_lin"].reshape(p.B, p.H, Nqb * p.bq, 64)[:, :, :p.N, :]
    if p.proj_per_head:
        return np.einsum("bhtd,bhte->hde", olin, dO)
    return np.einsum("bhtd,bhte->de", olin, dO)[None]


def _e4m3_grid():
    """The 127 non-negative finite E4M3 values in ascending order (codes 0..126), from the C oracle's decoder."""
    dec = lib().sla_oracle_decode_e4m3
    dec.restype = C.c_double
    grid = np.array([dec(C.c_uint8(c)) for c in range(127)], dtype=np.float64)
    assert np.all(np.diff(grid) > 0) and grid[-1] == 448.0
    return grid


def _e4m3_cast(y):
    """fp32 values in [-448, 448] -> E4M3 codes: nearest representable value, a value exactly half-way between two
    neighbours goes to the one with an even code (round to nearest even on this grid)."""
    grid = _e4m3_grid()
    a = np.abs(y).astype(np.float64)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 0, 126)                       # first grid value >= a
    lo = np.maximum(hi - 1, 0)
    dlo, dhi = a - grid[lo], grid[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return code | (np.signbit(y).astype(np.uint8) << 7)


def quantise_e4m3_blocks(bits, blk: int):
    """Scaled FP8 quantiser of App. B.2 (eqs. for scale, clamp and cast) applied per block of `blk` consecutive
    tokens of every (b, h), the granularity configuration 4 uses for Q, K and V:
        scale = max(amax, 1e-8) / 448        (fp32; the 1e-8 is the paper's epsilon against division by zero)
        code  = E4M3(clamp(x / scale, -448, 448))   with round-to-nearest-even
    bits: uint16 bf16 bit patterns [..., N, D].  Returns (codes uint8 [..., N, D], scales fp32 [..., ceil(N/blk)]).

    The cast is written from the format's definition: the 127 non-negative finite E4M3 values (decoded by the C
    oracle's table routine) are searched for the nearest one; a value exactly half-way between two neighbours goes
    to the one with an even code."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    x = (bits.astype(np.uint32) << 16).view(np.float32)
    N = x.shape[-2]
    nb = -(-N // blk)
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(x.shape[:-2] + (nb,), dtype=np.float32)
    for j in range(nb):
        sl = slice(j * blk, min(N, (j + 1) * blk))
        xb = x[..., sl, :]
        amax = np.abs(xb).max(axis=(-2, -1)).astype(np.float32)
        scale = (np.maximum(amax, np.float32(1e-8)) / np.float32(448.0)).astype(np.float32)
        scales[..., j] = scale
        y = (xb / scale[..., None, None]).astype(np.float32)                          # fp32 division, correctly rounded
        y = np.clip(y, np.float32(-448.0), np.float32(448.0))
        code = _e4m3_cast(y)
        codes[..., sl, :] = code
    return codes, scales


def quantise_e4m3_rows(bits):
    """Scaled FP8 quantiser of App. B.2 / B.3 with one scale per row (per token for activations, per output channel
    for weights): bits uint16 bf16 [R, C] -> (codes uint8 [R, C], scales fp32 [R]); scale = max(amax, 1e-8) / 448."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    x = (bits.astype(np.uint32) << 16).view(np.float32)
    amax = np.abs(x).max(axis=-1).astype(np.float32)
    scale = (np.maximum(amax, np.float32(1e-8)) / np.float32(448.0)).astype(np.float32)
    y = np.clip((x / scale[:, None]).astype(np.float32), np.float32(-448.0), np.float32(448.0))
    return _e4m3_cast(y), scale


def fp8_linear(x_bits, W_bits, bias_bits=None):
    """Forward value of the FP8 fake-quantised linear layer (Alg. 2): activations quantised per token, weights per
    output channel, y = x_fp8 W_fp8^T + b with x_fp8 = E4M3(clamp(x / scale_x)) * scale_x (likewise W).
    x [N, d_in], W [d_out, d_in], bias [d_out]: uint16 bf16 bit patterns.  Returns y float64 [N, d_out]."""
    grid = _e4m3_grid()
    deq = lambda c, s: np.where(c & 0x80, -1.0, 1.0) * grid[(c & 0x7F).astype(np.int64)] * s.astype(np.float64)[:, None]
    cx, sx = quantise_e4m3_rows(x_bits)
    cw, sw = quantise_e4m3_rows(W_bits)
    y = deq(cx, sx) @ deq(cw, sw).T
    if bias_bits is not None:
        y = y + (np.asarray(bias_bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)[None, :]
    return y


def alg1_token_level(Q, K, V, W_O, lam: float, sm_scale=None, phi: str = "elu1"):
    """Alg. 1 exactly as the paper prints it, for one head, in fp64 (quadratic in N: small inputs only).

    Token-level selection and a linear branch over ALL keys, where the block-level module above selects key blocks per
    query block and restricts the linear branch to the marginal blocks.  Steps, in the algorithm's notation
    (step 1, the frozen projections, is outside: Q, K, V are given):
      2  S = Q K^T / sqrt(d)                        (sm_scale overrides 1/sqrt(d))
      3  M = TopKMask(S, lambda): per query row the ceil(lambda N) largest scores are kept; equal scores are ordered
         by key index, lowest first (the tie rule of the block-level classifier).  lambda = 0 keeps nothing.
      4  A_sparse = Softmax(S (.) M): dropped entries are excluded from the softmax (a 0/1 product would leave
         exp(0) of mass on them); a row that keeps nothing gives 0
      5  O_sparse = A_sparse V
      6  phi(Q), phi(K): ELU(x) + 1 elementwise (phi="softmax": the channel softmax of the benchmark configurations)
      7  T = phi(K)^T V
      8  z = phi(K)^T 1_N
      9  O_lin = (phi(Q) T) ./ (phi(Q) z)
      10 O = O_sparse + O_lin W_O
    Q, K, V: float64 [N, d]; W_O: float64 [d, d].  Returns dict(O, O_sparse, O_lin, M) with M the boolean mask [N, N]."""
    Q, K, V, W_O = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, W_O))
    N, d = Q.shape
    scale = (1.0 / np.sqrt(d)) if sm_scale is None else float(sm_scale)
    S = (Q @ K.T) * scale                                                   # step 2
    keep = int(np.ceil(lam * N - 1e-12)) if lam > 0 else 0
    keep = min(max(keep, 0), N)
    M = np.zeros((N, N), dtype=bool)                                        # step 3
    if keep > 0:
        order = np.argsort(-S, axis=1, kind="stable")                       # score descending, equal scores by key index
        np.put_along_axis(M, order[:, :keep], True, axis=1)
    O_sparse = np.zeros((N, V.shape[1]))
    if keep > 0:                                                            # steps 4-5
        Sm = np.where(M, S, -np.inf)
        E = np.where(M, np.exp(Sm - Sm.max(axis=1, keepdims=True)), 0.0)
        O_sparse = (E / E.sum(axis=1, keepdims=True)) @ V
    if phi == "elu1":                                                       # step 6
        f = lambda X: np.where(X > 0, X + 1.0, np.exp(np.minimum(X, 0.0)))
    else:
        def f(X):
            Ex = np.exp(X - X.max(axis=-1, keepdims=True))
            return Ex / Ex.sum(axis=-1, keepdims=True)
    fQ, fK = f(Q), f(K)
    T = fK.T @ V                                                            # step 7
    z = fK.T @ np.ones(N)                                                   # step 8
    O_lin = (fQ @ T) / (fQ @ z)[:, None]                                    # step 9
    return {"O": O_sparse + O_lin @ W_O, "O_sparse": O_sparse, "O_lin": O_lin, "M": M}    # step 10
