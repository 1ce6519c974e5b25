"""Thin ctypes binding of libsla.so: argument marshalling only.

Every function has the name and the semantics of the C entry point declared in
include/sla.h; tensors are torch CUDA tensors used purely as device memory (their
data_ptr() is passed through), the stream is torch's current stream.  There is no CPU
fallback: if the HIP library has not been built, importing the symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsla.so")

SLA_OK, SLA_ERR_INVALID_ARG, SLA_ERR_UNSUPPORTED, SLA_ERR_WORKSPACE, SLA_ERR_HIP = 0, -1, -2, -3, -4
SLA_BF16, SLA_FP8_E4M3 = 0, 1
STATE_ROWS = 65          # rows of one block state: 64 rows of h^T and one row of z
EXPORTS = ["sla_resolve_counts", "sla_workspace_bytes", "sla_forward", "sla_pool_classify", "sla_linear_states",
           "sla_marginal_aggregate", "sla_sparse_combine", "sla_forward_profiled", "sla_wproj_grad", "sla_quantise_e4m3",
           "sla_forward_with_labels", "sla_fp8_linear_workspace_bytes", "sla_fp8_linear", "sla_forward_static", "sla_sparse_combine_f32", "sla_fp8_linear_qkv",
           "sla_strerror", "sla_last_error", "sla_stage_name"]
STATIC_WORKSPACE_BYTES = 96 * 1024 * 1024
NUM_STAGES = 6


class SlaParams(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("N", C.c_int32), ("D", C.c_int32),
                ("bq", C.c_int32), ("bk", C.c_int32),
                ("crit_frac", C.c_double), ("neg_frac", C.c_double),
                ("k_crit", C.c_int32), ("k_neg", C.c_int32),
                ("dtype", C.c_int32), ("phi", C.c_int32), ("proj_per_head", C.c_int32),
                ("sm_scale", C.c_float), ("layout", C.c_int32)]


class SlaError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__(f"{where}: status {status}: {detail}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Loads the HIP library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2605_11354_amd.build` "
                              "(the SLA forward has no CPU or PyTorch fallback)")
        _lib = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(_lib, name)                      # raises AttributeError on a missing export
        _lib.sla_strerror.restype = C.c_char_p
        _lib.sla_last_error.restype = C.c_char_p
        _lib.sla_stage_name.restype = C.c_char_p
        for name in EXPORTS[:16]:
            getattr(_lib, name).restype = C.c_int
    return _lib


def make_params(B, H, N, bq, bk, crit_frac=0.0, neg_frac=0.0, k_crit=-1, k_neg=-1, dtype="bf16",
                proj_per_head=False, sm_scale=0.0, D=64, phi="softmax", layout="bhnd") -> SlaParams:
    """layout: "bhnd" = Q, K, V, O are [B,H,N,D]; "bnhd" = [B,N,H,D] (rows of a head H*D elements apart)."""
    return SlaParams(B, H, N, D, bq, bk, crit_frac, neg_frac, k_crit, k_neg,
                     SLA_BF16 if dtype == "bf16" else SLA_FP8_E4M3, {"softmax": 0, "elu1": 1}[phi],
                     1 if proj_per_head else 0, sm_scale, {"bhnd": 0, "bnhd": 1}[layout])


def _check(status: int, where: str):
    if status != SLA_OK:
        raise SlaError(status, where, lib().sla_last_error().decode())


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def sla_resolve_counts(p: SlaParams):
    kc, kn = C.c_int32(), C.c_int32()
    _check(lib().sla_resolve_counts(C.byref(p), C.byref(kc), C.byref(kn)), "sla_resolve_counts")
    return kc.value, kn.value


def sla_workspace_bytes(p: SlaParams) -> int:
    n = C.c_size_t()
    _check(lib().sla_workspace_bytes(C.byref(p), C.byref(n)), "sla_workspace_bytes")
    return n.value


def alloc_workspace(p: SlaParams, device="cuda:0") -> torch.Tensor:
    return torch.empty(max(256, sla_workspace_bytes(p)), dtype=torch.uint8, device=device)


def sla_forward(p, Q, K, V, W_proj, O, labels=None, sQ=None, sK=None, sV=None, workspace=None):
    ws = workspace if workspace is not None else alloc_workspace(p, Q.device)
    _check(lib().sla_forward(C.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(sQ), _ptr(sK), _ptr(sV), _ptr(W_proj),
                             _ptr(O), _ptr(labels), _ptr(ws), C.c_size_t(ws.numel()), _stream()), "sla_forward")
    return O


def sla_forward_static(p, Q, K, V, W_proj, O, labels=None, sQ=None, sK=None, sV=None):
    """sla_forward on the library's own workspace (no allocation; shapes up to STATIC_WORKSPACE_BYTES of workspace)."""
    _check(lib().sla_forward_static(C.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(sQ), _ptr(sK), _ptr(sV), _ptr(W_proj),
                                    _ptr(O), _ptr(labels), _stream()), "sla_forward_static")
    return O


def sla_forward_profiled(p, Q, K, V, W_proj, O, labels=None, sQ=None, sK=None, sV=None, workspace=None):
    """Returns {stage name: milliseconds} for one forward (synchronises the stream)."""
    ws = workspace if workspace is not None else alloc_workspace(p, Q.device)
    ms = (C.c_float * NUM_STAGES)()
    _check(lib().sla_forward_profiled(C.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(sQ), _ptr(sK), _ptr(sV), _ptr(W_proj),
                                      _ptr(O), _ptr(labels), _ptr(ws), C.c_size_t(ws.numel()), _stream(), ms),
           "sla_forward_profiled")
    return {lib().sla_stage_name(i).decode(): float(ms[i]) for i in range(NUM_STAGES)}


def sla_pool_classify(p, Q, K, labels, crit_idx=None, Pc=None, qbar=None, kbar=None, scores=None,
                      sQ=None, sK=None, workspace=None):
    ws = workspace if workspace is not None else alloc_workspace(p, Q.device)
    _check(lib().sla_pool_classify(C.byref(p), _ptr(Q), _ptr(K), _ptr(sQ), _ptr(sK), _ptr(labels), _ptr(crit_idx),
                                   _ptr(Pc), _ptr(qbar), _ptr(kbar), _ptr(scores), _ptr(ws), C.c_size_t(ws.numel()),
                                   _stream()), "sla_pool_classify")
    return labels


def sla_linear_states(p, K, V, hT, sK=None, sV=None):
    _check(lib().sla_linear_states(C.byref(p), _ptr(K), _ptr(V), _ptr(sK), _ptr(sV), _ptr(hT), _stream()),
           "sla_linear_states")
    return hT


def sla_marginal_aggregate(p, labels, hT, Hq, workspace=None):
    ws = workspace if workspace is not None else alloc_workspace(p, hT.device)
    _check(lib().sla_marginal_aggregate(C.byref(p), _ptr(labels), _ptr(hT), _ptr(Hq), _ptr(ws), C.c_size_t(ws.numel()),
                                        _stream()), "sla_marginal_aggregate")
    return Hq


def sla_forward_with_labels(p, Q, K, V, W_proj, labels, O, sQ=None, sK=None, sV=None, workspace=None):
    ws = workspace if workspace is not None else alloc_workspace(p, Q.device)
    _check(lib().sla_forward_with_labels(C.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(sQ), _ptr(sK), _ptr(sV), _ptr(W_proj),
                                         _ptr(labels), _ptr(O), _ptr(ws), C.c_size_t(ws.numel()), _stream()),
           "sla_forward_with_labels")
    return O


def sla_fp8_linear(x, W, bias, y, workspace=None):
    """y bf16 [N,d_out] <- FP8 fake-quantised linear layer of x bf16 [N,d_in] with W bf16 [d_out,d_in] and bias (or None)."""
    import torch
    N, d_in = x.shape
    d_out = W.shape[0]
    n = C.c_size_t(0)
    _check(lib().sla_fp8_linear_workspace_bytes(C.c_int32(N), C.c_int32(d_in), C.c_int32(d_out), C.byref(n)), "sla_fp8_linear_workspace_bytes")
    ws = workspace if workspace is not None else torch.empty(max(n.value, 256), dtype=torch.uint8, device=x.device)
    _check(lib().sla_fp8_linear(_ptr(x), _ptr(W), _ptr(bias), C.c_int32(N), C.c_int32(d_in), C.c_int32(d_out), _ptr(y), _ptr(ws),
                                C.c_size_t(ws.numel()), _stream()), "sla_fp8_linear")
    return y


def sla_quantise_e4m3(X, blk, codes, scales, layout="bhnd"):
    """X bf16 [B,H,N,64] ([B,N,H,64] with layout "bnhd") -> codes uint8 of the same layout, scales fp32 [B,H,ceil(N/blk)]."""
    if layout == "bhnd":
        Bn, H, N, D = X.shape
    else:
        Bn, N, H, D = X.shape
    assert D == 64
    _check(lib().sla_quantise_e4m3(_ptr(X), C.c_int32(Bn), C.c_int32(H), C.c_int32(N), C.c_int32(blk),
                                   C.c_int32({"bhnd": 0, "bnhd": 1}[layout]), _ptr(codes), _ptr(scales), _stream()),
           "sla_quantise_e4m3")
    return codes, scales


def sla_wproj_grad(p, Q, dO, dW, workspace, sQ=None):
    """dW (fp32 [nW,64,64]) <- gradient of sum(O * dO) w.r.t. W_proj; `workspace` is the one sla_forward just used."""
    _check(lib().sla_wproj_grad(C.byref(p), _ptr(Q), _ptr(sQ), _ptr(dO), _ptr(dW), _ptr(workspace),
                                C.c_size_t(workspace.numel()), _stream()), "sla_wproj_grad")
    return dW


def sla_sparse_combine(p, Q, K, V, W_proj, labels, Hq, O, sQ=None, sK=None, sV=None, workspace=None):
    ws = workspace if workspace is not None else alloc_workspace(p, Q.device)
    _check(lib().sla_sparse_combine(C.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(sQ), _ptr(sK), _ptr(sV), _ptr(W_proj),
                                    _ptr(labels), _ptr(Hq), _ptr(O), _ptr(ws), C.c_size_t(ws.numel()), _stream()),
           "sla_sparse_combine")
    return O


def sla_sparse_combine_f32(p, Q, K, V, W_proj, labels, Hq, O32, sQ=None, sK=None, sV=None, workspace=None):
    """sla_sparse_combine with the result in fp32 (O32: float32 tensor of the shape of O)."""
    ws = workspace if workspace is not None else alloc_workspace(p, Q.device)
    _check(lib().sla_sparse_combine_f32(C.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(sQ), _ptr(sK), _ptr(sV), _ptr(W_proj),
                                        _ptr(labels), _ptr(Hq), _ptr(O32), _ptr(ws), C.c_size_t(ws.numel()), _stream()),
           "sla_sparse_combine_f32")
    return O32


def sla_fp8_linear_qkv(x, W, bias, B_, N, H, bq, Q8, K8, V8, sQ, sK, sV, workspace=None):
    """qkv projection with the per-block E4M3 quantiser in the GEMM's epilogue: x [B*N, d_in], W [3*H*64, d_in]."""
    import torch
    d_in = x.shape[1]
    if workspace is None:
        n = C.c_size_t()
        _check(lib().sla_fp8_linear_workspace_bytes(C.c_int32(B_ * N), C.c_int32(d_in), C.c_int32(3 * H * 64), C.byref(n)),
               "sla_fp8_linear_workspace_bytes")
        workspace = torch.empty(max(256, n.value), dtype=torch.uint8, device=x.device)
    _check(lib().sla_fp8_linear_qkv(_ptr(x), _ptr(W), _ptr(bias), C.c_int32(B_), C.c_int32(N), C.c_int32(H), C.c_int32(d_in),
                                    C.c_int32(bq), _ptr(Q8), _ptr(K8), _ptr(V8), _ptr(sQ), _ptr(sK), _ptr(sV),
                                    _ptr(workspace), C.c_size_t(workspace.numel()), _stream()), "sla_fp8_linear_qkv")
