"""Helpers shared by the GPU parity tests: upload seeded inputs, run the C-ABI entry points,
fetch results, and evaluate the oracle on the same inputs."""
from __future__ import annotations

import numpy as np
import torch

from paper_2605_11354_amd import binding as B
from paper_2605_11354_amd import synth

TOL = {"bf16": 2e-2, "fp8": 6e-2}      # max-abs error relative to the RMS of the oracle output


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def dev_u8(codes: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(codes).cuda()


def dev_f32(x):
    return None if x is None else torch.from_numpy(x).cuda()


def bf16_tensor_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


class Case:
    """One workload: host arrays (for the oracle) and device tensors (for the library)."""

    def __init__(self, cfg: synth.SLAConfig, inputs: dict | None = None, k_crit=-1, k_neg=-1, sm_scale=0.0, phi="softmax"):
        self.cfg = cfg
        self.d = inputs if inputs is not None else synth.make_inputs(cfg)
        self.fp8 = cfg.dtype == "fp8"
        self.Nqb = -(-cfg.N // cfg.bq)
        self.Nkb = -(-cfg.N // cfg.bk)
        self.sm_scale = sm_scale                      # 0: the default 1/sqrt(D) on both sides
        self.p = B.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, cfg.crit_frac, cfg.neg_frac, k_crit, k_neg,
                               cfg.dtype, cfg.proj_per_head, sm_scale, phi=phi)
        self.phi = phi
        self.k_c, self.k_n = B.sla_resolve_counts(self.p)
        up = dev_u8 if self.fp8 else dev_bf16
        self.Q, self.K, self.V = up(self.d["Q"]), up(self.d["K"]), up(self.d["V"])
        self.sQ, self.sK, self.sV = dev_f32(self.d["sQ"]), dev_f32(self.d["sK"]), dev_f32(self.d["sV"])
        self.W = dev_bf16(self.d["W"])
        self.ws = B.alloc_workspace(self.p)

    def oracle_params(self, oracle):
        c = self.cfg
        return oracle.make_params(c.B, c.H, c.N, c.bq, c.bk, self.k_c, self.k_n, c.dtype, c.proj_per_head,
                                  self.sm_scale if self.sm_scale > 0 else None, phi=self.phi)

    # ---- library calls
    def forward(self, want_labels=True):
        c = self.cfg
        O = torch.empty((c.B, c.H, c.N, 64), dtype=torch.bfloat16, device="cuda")
        lab = torch.empty((c.B, c.H, self.Nqb, self.Nkb), dtype=torch.int8, device="cuda") if want_labels else None
        B.sla_forward(self.p, self.Q, self.K, self.V, self.W, O, lab, self.sQ, self.sK, self.sV, self.ws)
        torch.cuda.synchronize()
        return O, lab

    def classify(self, want=("crit_idx", "Pc", "qbar", "kbar", "scores")):
        c = self.cfg
        shp = (c.B, c.H, self.Nqb, self.Nkb)
        out = {"labels": torch.empty(shp, dtype=torch.int8, device="cuda")}
        out["crit_idx"] = torch.full((c.B, c.H, self.Nqb, max(self.k_c, 1)), -7, dtype=torch.int32, device="cuda") if "crit_idx" in want else None
        out["Pc"] = torch.empty(shp, dtype=torch.float32, device="cuda") if "Pc" in want else None
        out["qbar"] = torch.empty((c.B, c.H, self.Nqb, 64), dtype=torch.float64, device="cuda") if "qbar" in want else None
        out["kbar"] = torch.empty((c.B, c.H, self.Nkb, 64), dtype=torch.float64, device="cuda") if "kbar" in want else None
        out["scores"] = torch.empty(shp, dtype=torch.float64, device="cuda") if "scores" in want else None
        B.sla_pool_classify(self.p, self.Q, self.K, out["labels"], out["crit_idx"], out["Pc"], out["qbar"], out["kbar"],
                            out["scores"], self.sQ, self.sK, self.ws)
        torch.cuda.synchronize()
        return {k: (None if v is None else v.cpu().numpy()) for k, v in out.items()}

    def states(self):
        c = self.cfg
        hT = torch.empty((c.B, c.H, self.Nkb, B.STATE_ROWS, 64), dtype=torch.bfloat16, device="cuda")
        B.sla_linear_states(self.p, self.K, self.V, hT, self.sK, self.sV)
        torch.cuda.synchronize()
        return hT

    def aggregate(self, labels_dev, hT):
        c = self.cfg
        Hq = torch.empty((c.B, c.H, self.Nqb, B.STATE_ROWS, 64), dtype=torch.bfloat16, device="cuda")
        B.sla_marginal_aggregate(self.p, labels_dev, hT, Hq, self.ws)
        torch.cuda.synchronize()
        return Hq

    def sparse_combine(self, labels_dev, Hq):
        c = self.cfg
        O = torch.empty((c.B, c.H, c.N, 64), dtype=torch.bfloat16, device="cuda")
        B.sla_sparse_combine(self.p, self.Q, self.K, self.V, self.W if Hq is not None else None, labels_dev, Hq, O,
                             self.sQ, self.sK, self.sV, self.ws)
        torch.cuda.synchronize()
        return O

    # ---- oracle calls
    def oracle_classify(self, oracle, **kw):
        return oracle.classify(self.oracle_params(oracle), self.d["Q"], self.d["K"], self.d["sQ"], self.d["sK"], **kw)

    def oracle_attend(self, oracle, labels, sel=None, want_parts=False):
        d = self.d
        return oracle.attend(self.oracle_params(oracle), d["Q"], d["K"], d["V"], d["W"], labels, sel,
                             d["sQ"], d["sK"], d["sV"], want_parts)


def gather_blocks(O_full: np.ndarray, sel, bq: int, H: int) -> np.ndarray:
    """[B,H,N,64] -> [n_sel,bq,64] (rows past N zero) in the oracle's compact layout."""
    N = O_full.shape[2]
    out = np.zeros((len(sel), bq, 64))
    for s, (bh, i) in enumerate(sel):
        rows = min(N, (i + 1) * bq) - i * bq
        out[s, :rows] = O_full[bh // H, bh % H, i * bq:i * bq + rows]
    return out


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max-abs error over all elements, relative to the RMS of the reference."""
    rms = float(np.sqrt(np.mean(ref ** 2)))
    return float(np.abs(got - ref).max() / max(rms, 1e-30))


def bf16_half_ulp(x: np.ndarray) -> np.ndarray:
    """Half the spacing of bf16 (8 significant bits) at each |x|: the error a correctly rounded store may add."""
    ax = np.abs(x)
    e = np.floor(np.log2(np.where(ax > 0, ax, 1.0)))
    return np.where(ax > 0, 2.0 ** (e - 8), 0.0)


def output_error(got: np.ndarray, ref: np.ndarray):
    """(strict, arithmetic) errors of a bf16 output tensor, both relative to RMS(ref).

    strict     = max |got - ref|                                  (includes the final bf16 store)
    arithmetic = max (|got - ref| - half_ulp_bf16(ref)), >= 0     (what the kernels' arithmetic adds on
                 top of the one rounding any bf16 output must make)
    """
    rms = max(float(np.sqrt(np.mean(ref ** 2))), 1e-30)
    diff = np.abs(got - ref)
    return float(diff.max() / rms), float(np.maximum(diff - bf16_half_ulp(ref), 0.0).max() / rms)


def assert_output(got, ref, dtype, what=""):
    strict, arith = output_error(got, ref)
    print(f"[parity] {what}: strict max-abs/RMS = {strict:.4e}, beyond the bf16 store = {arith:.4e} (bar {TOL[dtype]:.0e})")
    assert arith <= TOL[dtype], (what, strict, arith)
    return strict, arith
