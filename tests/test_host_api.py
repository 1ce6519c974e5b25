"""Host-side logic of the C-ABI library (no GPU needed): exports, count rule, validation, workspace."""
import ctypes as C
import os
import re

import pytest

from paper_2605_11354_amd import binding as B
from paper_2605_11354_amd import build as libbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        libbuild.build()
    return B.lib()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "sla.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(sla_[a-z0-9_]+)\s*\(", header))
    assert {"sla_forward", "sla_pool_classify", "sla_linear_states", "sla_marginal_aggregate", "sla_sparse_combine",
            "sla_workspace_bytes", "sla_resolve_counts", "sla_strerror", "sla_last_error"} <= names
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in sla.h but not exported"
    assert set(B.EXPORTS) == names


def test_count_rule_matches_golden_table(lib):
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "block_counts.txt")) if l[0] != "#"]
    for name, nkb, fc, fn, kc, kn, km in rows:
        p = B.make_params(1, 1, int(nkb) * 64, 64, 64, float(fc), float(fn))
        assert B.sla_resolve_counts(p) == (int(kc), int(kn)), name
    assert B.sla_resolve_counts(B.make_params(1, 1, 640, 64, 64, 0.0, 1.0)) == (0, 10)
    assert B.sla_resolve_counts(B.make_params(1, 1, 640, 64, 64, 0.001, 0.999)) == (1, 9)
    assert B.sla_resolve_counts(B.make_params(1, 1, 640, 64, 64, k_crit=3, k_neg=2)) == (3, 2)


@pytest.mark.parametrize("kw,status", [
    (dict(D=32), B.SLA_ERR_UNSUPPORTED), (dict(bk=32), B.SLA_ERR_UNSUPPORTED), (dict(bq=96), B.SLA_ERR_UNSUPPORTED),
    (dict(crit_frac=0.7, neg_frac=0.5), B.SLA_ERR_INVALID_ARG), (dict(crit_frac=-0.1), B.SLA_ERR_INVALID_ARG),
    (dict(k_crit=5, k_neg=-1), B.SLA_ERR_INVALID_ARG), (dict(k_crit=9, k_neg=9), B.SLA_ERR_INVALID_ARG),
    (dict(N=64 * 5000), B.SLA_ERR_UNSUPPORTED), (dict(B=-1), B.SLA_ERR_INVALID_ARG), (dict(sm_scale=-1.0), B.SLA_ERR_INVALID_ARG), (dict(phi=2), B.SLA_ERR_INVALID_ARG),
])
def test_invalid_parameters_are_rejected_on_the_host(lib, kw, status):
    base = dict(B=1, H=2, N=640, bq=64, bk=64, crit_frac=0.1, neg_frac=0.5)
    base.update(kw)
    phi = base.pop("phi", None)
    p = B.make_params(**base)
    if phi is not None:
        p.phi = phi                                         # a value outside sla_phi_t
    with pytest.raises(B.SlaError) as e:
        B.sla_workspace_bytes(p)
    assert e.value.status == status
    assert len(lib.sla_last_error()) > 0 and lib.sla_strerror(status)


def test_null_and_misaligned_pointers_fail_before_any_launch(lib):
    p = B.make_params(1, 2, 640, 64, 64, 0.1, 0.5)
    null = C.c_void_p(0)
    rc = lib.sla_forward(C.byref(p), null, null, null, null, null, null, null, null, null, null, C.c_size_t(0), null)
    assert rc == B.SLA_ERR_INVALID_ARG and b"NULL" in lib.sla_last_error()
    rc = lib.sla_linear_states(C.byref(p), C.c_void_p(8), C.c_void_p(16), null, null, C.c_void_p(16), null)
    assert rc == B.SLA_ERR_INVALID_ARG and b"aligned" in lib.sla_last_error()
    fp8 = B.make_params(1, 2, 640, 64, 64, 0.1, 0.5, dtype="fp8")
    rc = lib.sla_linear_states(C.byref(fp8), C.c_void_p(16), C.c_void_p(16), null, null, C.c_void_p(16), null)
    assert rc == B.SLA_ERR_INVALID_ARG                      # e4m3 inputs need their scales
    assert lib.sla_forward(None, null, null, null, null, null, null, null, null, null, null, C.c_size_t(0), null) == B.SLA_ERR_INVALID_ARG


def test_empty_problem_is_a_no_op(lib):
    p = B.make_params(0, 2, 640, 64, 64, 0.1, 0.5)
    null = C.c_void_p(0)
    assert lib.sla_forward(C.byref(p), null, null, null, null, null, null, null, null, null, null, C.c_size_t(0), null) == B.SLA_OK


def test_workspace_size_covers_every_slice(lib):
    for N, bq in [(512, 64), (10992, 64), (43968, 128), (137400, 128)]:
        p = B.make_params(1, 16, N, bq, 64, 0.05, 0.8)
        nqb, nkb = -(-N // bq), -(-N // 64)
        need = 16 * (nqb * 64 * 8 + nkb * 64 * 8 + nqb * nkb * 8 + nqb * nkb + (nqb + nkb) * 65 * 64 * 2)
        assert B.sla_workspace_bytes(p) >= need


def test_wproj_grad_rejects_bad_pointers_before_any_launch(lib):
    p = B.make_params(1, 2, 640, 64, 64, 0.1, 0.5)
    null = C.c_void_p(0)
    rc = lib.sla_wproj_grad(C.byref(p), C.c_void_p(16), null, C.c_void_p(16), null, C.c_void_p(256), C.c_size_t(1 << 30), null)
    assert rc == B.SLA_ERR_INVALID_ARG and b"dW" in lib.sla_last_error()
    rc = lib.sla_wproj_grad(C.byref(p), null, null, C.c_void_p(16), C.c_void_p(16), C.c_void_p(256), C.c_size_t(1 << 30), null)
    assert rc == B.SLA_ERR_INVALID_ARG
    rc = lib.sla_wproj_grad(C.byref(p), C.c_void_p(16), null, C.c_void_p(16), C.c_void_p(16), C.c_void_p(256), C.c_size_t(64), null)
    assert rc == B.SLA_ERR_WORKSPACE
    fp8 = B.make_params(1, 2, 640, 64, 64, 0.1, 0.5, dtype="fp8")
    rc = lib.sla_wproj_grad(C.byref(fp8), C.c_void_p(16), null, C.c_void_p(16), C.c_void_p(16), C.c_void_p(256), C.c_size_t(1 << 30), null)
    assert rc == B.SLA_ERR_INVALID_ARG                      # e4m3 Q needs its scales


def test_fp8_linear_and_quantiser_validate_on_the_host(lib):
    null = C.c_void_p(0)
    n = C.c_size_t(0)
    assert lib.sla_fp8_linear_workspace_bytes(C.c_int32(1000), C.c_int32(1024), C.c_int32(3072), C.byref(n)) == B.SLA_OK
    assert n.value >= 1000 * 1024 + 3072 * 1024 + 4 * (1000 + 3072)
    assert lib.sla_fp8_linear_workspace_bytes(C.c_int32(1000), C.c_int32(1000), C.c_int32(3072), C.byref(n)) == B.SLA_ERR_UNSUPPORTED
    assert lib.sla_fp8_linear_workspace_bytes(C.c_int32(1000), C.c_int32(1024), C.c_int32(3070), C.byref(n)) == B.SLA_ERR_UNSUPPORTED
    assert lib.sla_fp8_linear_workspace_bytes(C.c_int32(-1), C.c_int32(1024), C.c_int32(3072), C.byref(n)) == B.SLA_ERR_INVALID_ARG
    # no tokens: nothing to do, nothing dereferenced
    assert lib.sla_fp8_linear(null, null, null, C.c_int32(0), C.c_int32(128), C.c_int32(8), null, null, C.c_size_t(0), null) == B.SLA_OK
    rc = lib.sla_fp8_linear(C.c_void_p(16), C.c_void_p(16), null, C.c_int32(4), C.c_int32(128), C.c_int32(8), C.c_void_p(16), null, C.c_size_t(0), null)
    assert rc == B.SLA_ERR_WORKSPACE
    rc = lib.sla_quantise_e4m3(C.c_void_p(16), C.c_int32(1), C.c_int32(2), C.c_int32(640), C.c_int32(96), C.c_int32(0), C.c_void_p(16), C.c_void_p(16), null)
    assert rc == B.SLA_ERR_UNSUPPORTED and b"block" in lib.sla_last_error()
    rc = lib.sla_quantise_e4m3(C.c_void_p(16), C.c_int32(1), C.c_int32(2), C.c_int32(640), C.c_int32(64), C.c_int32(7), C.c_void_p(16), C.c_void_p(16), null)
    assert rc == B.SLA_ERR_INVALID_ARG
    assert lib.sla_quantise_e4m3(null, C.c_int32(0), C.c_int32(2), C.c_int32(640), C.c_int32(64), C.c_int32(0), null, null, null) == B.SLA_OK
