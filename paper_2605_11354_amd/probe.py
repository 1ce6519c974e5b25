"""Phase timing of the two MFMA kernels from inside the kernels.

Runs libsla_probe.so, the library compiled with -DSLA_PROBE_TIME: one wave of one workgroup of attend_kernel (and of the
fp8 GEMM) writes the shader-clock counter at the boundaries of its phases and, at its start and end, the 100 MHz
counter.  The ratio of the two is the clock the wave really ran at; the differences are cycles per phase.  A probe
point costs the wave about 80 cycles, so phase sums are slightly above the unprobed kernel's; results are unchanged.

    python3 -m paper_2605_11354_amd.probe --config 2          # attend_kernel on configuration 2
    python3 -m paper_2605_11354_amd.probe --gemm 44032        # the q/k/v projection GEMM on 44032 rows

The lists of configuration 3 go to attend_short_kernel, which carries no phase probe.
"""
from __future__ import annotations

import argparse
import ctypes
import os

import numpy as np
import torch

from . import binding as B
from . import synth

PROBE_LIB = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsla_probe.so")


def _use_probe_library() -> ctypes.CDLL:
    if not os.path.exists(PROBE_LIB):
        raise ImportError(f"{PROBE_LIB} is missing: run `python -m paper_2605_11354_amd.build`")
    B._lib = None
    B.LIB_PATH = PROBE_LIB
    return ctypes.CDLL(PROBE_LIB)


def probe_attend(idx: int, per_tile: bool) -> None:
    cfg = synth.CONFIGS[idx]
    L = _use_probe_library()
    d = synth.make_inputs(cfg)
    fp8 = cfg.dtype == "fp8"
    up16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    up = (lambda a: torch.from_numpy(a).cuda()) if fp8 else up16
    Q, K, V = up(d["Q"]), up(d["K"]), up(d["V"])
    sc = [torch.from_numpy(d[k]).cuda() if fp8 else None for k in ("sQ", "sK", "sV")]
    W = up16(d["W"])
    O = torch.empty((cfg.B, cfg.H, cfg.N, 64), dtype=torch.bfloat16, device="cuda")
    p = B.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, cfg.crit_frac, cfg.neg_frac, -1, -1, cfg.dtype, cfg.proj_per_head)
    k_c, _ = B.sla_resolve_counts(p)
    if k_c <= 2:
        raise SystemExit(f"{cfg.name}: lists of {k_c} blocks run in attend_short_kernel, which has no phase probe")
    ws = B.alloc_workspace(p)
    for _ in range(5):
        r = B.sla_forward_profiled(p, Q, K, V, W, O, None, *sc, ws)
    torch.cuda.synchronize()
    buf = (ctypes.c_ulonglong * 512)()
    if L.sla_probe_read(buf) != 0:
        raise RuntimeError("sla_probe_read failed")
    t = np.array(buf[:], dtype=np.uint64).reshape(64, 8).astype(np.int64)
    nk = min(k_c, 61)                                  # the probe keeps the first 61 blocks of the list
    print(f"{cfg.name}: lists of {k_c} key blocks; stage times of this launch (ms):", {k: round(v, 4) for k, v in r.items()})
    print("wave life: %d shader-clock ticks in %d ticks of 100 MHz -> %.3f GHz" % (t[63, 6], t[63, 7], t[63, 6] / max(1, t[63, 7]) * 0.1))
    rows, prev = [], None
    for c in range(nk):
        row = t[c]
        gap = row[0] - prev if prev is not None else 0
        rows.append([gap, row[1] - row[0], row[2] - row[1], row[3] - row[2], row[4] - row[3]])
        if per_tile:
            print("block %2d: loop-back %5d | wait+barrier %5d | requests %5d | first half %5d | second half %5d" % tuple(rows[-1]))
        prev = row[4]
    R = np.array(rows)[3:-2] if nk > 8 else np.array(rows)[1:]
    m = np.median(R, axis=0)
    print("per key block (64 keys), median over the middle of the list, cycles: loop-back %d, wait+barrier %d, requests %d, "
          "first half %d, second half %d; sum %d" % (*m, m.sum()))
    pr, ep = t[62], t[61]
    print("prologue, cycles: start -> list length %d | -> copies requested %d | -> scales requested %d | -> all landed + barrier %d | "
          "-> first S %d | -> block 0 %d" % (pr[1] - pr[0], pr[2] - pr[1], pr[3] - pr[2], pr[4] - pr[3], pr[5] - pr[4], t[0, 0] - pr[5]))
    print("epilogue, cycles: last block -> loop exit %d | last PV + 1/l %d | phi(Q) %d | linear-branch MFMAs %d | barrier %d | store %d"
          % (ep[0] - t[nk - 1, 4] if nk == k_c else -1, ep[1] - ep[0], ep[2] - ep[1], ep[3] - ep[2], ep[4] - ep[3], ep[5] - ep[4]))
    probe_select_report(L, (cfg.N + cfg.bk - 1) // cfg.bk)
    nwg = min(32768, cfg.B * cfg.H * ((cfg.N + cfg.bq - 1) // cfg.bq))
    wb = (ctypes.c_ulonglong * (2 * nwg))()
    if L.sla_probe_read_wg(wb, nwg) != 0:
        raise RuntimeError("sla_probe_read_wg failed")
    w = np.array(wb[:], dtype=np.uint64).reshape(nwg, 2).astype(np.int64)
    life = (w[:, 1] - w[:, 0]) / 100.0
    span = (w[:, 1].max() - w[:, 0].min()) / 100.0
    print("workgroups (first %d): life median %.1f us, 10%% %.1f, 90%% %.1f; first start to last end %.1f us"
          % (nwg, np.median(life), np.percentile(life, 10), np.percentile(life, 90), span))


def probe_select_report(L: ctypes.CDLL, nkb: int) -> None:
    """Phases of select_keys_kernel (rows of more than 256 key blocks) for one row in the middle of the launch."""
    if nkb <= 256:
        return
    buf = (ctypes.c_ulonglong * 32)()
    if L.sla_probe_read_select(buf) != 0:
        raise RuntimeError("sla_probe_read_select failed")
    t = [int(x) for x in buf]
    out = ["load keys + min/max %d" % (t[1] - t[0]), "spread over the row's range %d" % (t[2] - t[1])]
    last = t[2]
    for p in range(4):
        a, b, c = t[4 + 3 * p], t[5 + 3 * p], t[6 + 3 * p]
        if a == 0:
            break
        out.append("pass %d: clear %d, count %d, scan + cut %d" % (p, a - last, b - a, c - b))
        last = c
    out += ["labels, lists, masks %d" % (t[17] - t[16]), "mask store %d" % (t[18] - t[17]), "whole row %d" % (t[18] - t[0])]
    print("select_keys_kernel, one row of %d keys, cycles: " % nkb + " | ".join(out))


def probe_gemm(M: int) -> None:
    L = _use_probe_library()
    d_in, d_out = 1024, 3072
    g = torch.Generator(device="cuda").manual_seed(1)
    x = torch.randn((M, d_in), device="cuda", generator=g).to(torch.bfloat16)
    W = (torch.randn((d_out, d_in), device="cuda", generator=g) / 32).to(torch.bfloat16)
    b = torch.randn((d_out,), device="cuda", generator=g).to(torch.bfloat16)
    y = torch.empty((M, d_out), dtype=torch.bfloat16, device="cuda")
    for _ in range(8):
        B.sla_fp8_linear(x, W, b, y)
    torch.cuda.synchronize()
    buf = (ctypes.c_ulonglong * 16)()
    if L.sla_probe_read_gemm(buf) != 0:
        raise RuntimeError("sla_probe_read_gemm failed")
    t = list(buf)
    c, r = t[:8], t[8:]
    print(f"fp8 GEMM [{M} x {d_in}] x [{d_in} x {d_out}], one wave of one workgroup:")
    names = ["start -> first tiles landed", "main loop", "last barrier", "accumulators -> LDS (scale, bias, bf16)", "stores (issue + completion)"]
    for i, n in enumerate(names):
        print("  %-42s %7d cycles  %6.2f us" % (n, c[i + 1] - c[i], (r[i + 1] - r[i]) / 100.0))
    print("  tile total %d cycles in %.2f us -> %.3f GHz" % (c[5] - c[0], (r[5] - r[0]) / 100.0, (c[5] - c[0]) / max(1, r[5] - r[0]) * 0.1))
    print("  inside the main loop: waiting for copies %d cycles, then for the barrier %d cycles (about 100 of probe per step included)" % (c[6], c[7]))


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__.splitlines()[0])
    ap.add_argument("--config", type=int, default=None, help="index into synth.CONFIGS (1, 2 or 4)")
    ap.add_argument("--gemm", type=int, default=None, metavar="M", help="rows of the projection GEMM")
    ap.add_argument("--per-tile", action="store_true", help="print every block of the probed list")
    a = ap.parse_args()
    if a.config is None and a.gemm is None:
        ap.error("give --config or --gemm")
    if not torch.cuda.is_available():
        raise SystemExit("the probe needs a GPU")
    if a.config is not None:
        probe_attend(a.config, a.per_tile)
    if a.gemm is not None:
        probe_gemm(a.gemm)


if __name__ == "__main__":
    main()
