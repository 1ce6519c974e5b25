"""sla_forward_static (the entry point that allocates nothing) against sla_forward, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2605_11354_amd import binding as B
from paper_2605_11354_amd import synth
from tests.gpu_util import Case

pytestmark = pytest.mark.gpu


def _run_both(cfg):
    c = Case(cfg)
    O_ref, lab_ref = c.forward()
    O = torch.full_like(O_ref, float("nan"))
    lab = torch.full_like(lab_ref, -7)
    B.sla_forward_static(c.p, c.Q, c.K, c.V, c.W, O, lab, c.sQ, c.sK, c.sV)
    torch.cuda.synchronize()
    assert torch.equal(lab, lab_ref), "labels differ between sla_forward_static and sla_forward"
    assert torch.equal(O.view(torch.int16), O_ref.view(torch.int16)), "outputs differ bit for bit"


def test_static_workspace_forward_matches_forward_twice_in_a_row():
    """Two calls in a row on the library's own workspace, the second on a smaller input (the array keeps the first
    call's contents): both must reproduce sla_forward bit for bit (same kernels, same order of operations)."""
    big = synth.CONFIGS[1].with_(H=4, N=5 * 1374)            # ragged tails, per-head projection, 64-row query blocks
    small = synth.CONFIGS[0].with_(N=330)                     # smaller in every slice of the workspace
    assert B.sla_workspace_bytes(Case(big).p) <= B.STATIC_WORKSPACE_BYTES
    _run_both(big)
    _run_both(small)
    fp8 = synth.CONFIGS[4].with_(H=2, N=1500)
    _run_both(fp8)


def test_static_workspace_rejects_shapes_beyond_its_size():
    cfg = synth.CONFIGS[2]
    p = B.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, cfg.crit_frac, cfg.neg_frac, -1, -1, cfg.dtype, cfg.proj_per_head)
    assert B.sla_workspace_bytes(p) > B.STATIC_WORKSPACE_BYTES
    dummy = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.SlaError) as e:
        B.sla_forward_static(p, dummy, dummy, dummy, dummy, dummy)          # rejected on the host before any pointer is used
    assert e.value.status == B.SLA_ERR_WORKSPACE and "sla_forward_static holds" in str(e.value)
