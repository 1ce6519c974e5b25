"""The long-row classifier that stores 32-bit keys instead of fp64 logits (rows of more than 256 key blocks, neither
logits nor block-score softmax asked for): labels, critical lists and marginal masks must be those of the exact fp64
order (Alg. 1 steps 2-3 on block means; logit descending, index ascending), also where a threshold cuts through blocks
whose logits agree in their leading 32 bits, or exactly."""
import numpy as np
import pytest
import torch

from paper_2605_11354_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu
C0 = synth.CONFIGS[0]


def _bf16(x):
    return synth.to_bf16_bits(np.asarray(x, dtype=np.float32))


def _variants(cfg, d):
    """plain; groups of four key blocks whose means differ by far less than 2^-20 relative (two of them exactly equal);
    a run of all-zero key blocks (logit exactly 0: a large group of exact ties in the middle of the order); Q = 0 (all tie);
    runs of blocks with tiny distinct logits (below)."""
    yield "plain", d
    K = d["K"].copy()
    nkb = cfg.N // 64                                         # whole blocks only
    for j0 in range(0, nkb - 3, 4):
        base = K[:, :, j0 * 64:(j0 + 1) * 64].copy()
        base[:, :, 5, 3] = 0
        base[:, :, 9, 7] = 0
        b1 = base.copy(); b1[:, :, 5, 3] = _bf16(2.0 ** -38)
        b3 = base.copy(); b3[:, :, 9, 7] = _bf16(-(2.0 ** -37))
        K[:, :, j0 * 64:(j0 + 1) * 64] = base
        K[:, :, (j0 + 1) * 64:(j0 + 2) * 64] = b1
        K[:, :, (j0 + 2) * 64:(j0 + 3) * 64] = base
        K[:, :, (j0 + 3) * 64:(j0 + 4) * 64] = b3
    yield "near_ties", dict(d, K=K)
    K = d["K"].copy()
    K[:, :, 40 * 64:(40 + nkb // 3) * 64] = 0
    yield "zero_run", dict(d, K=K)
    yield "all_tie", dict(d, Q=np.zeros_like(d["Q"]))
    # a run of key blocks with tiny, distinct logits (one non-zero element of 2^-(40 + j mod 30), alternating sign): next to
    # the row's range they are all one value, but their keys differ in sign and exponent -- a tied group of the ranked
    # 32-bit values whose members are told apart by the upper halves of their exact keys, some pairs only by the index
    K = d["K"].copy()
    for t, j in enumerate(range(40, 40 + nkb // 3)):
        K[:, :, j * 64:(j + 1) * 64] = 0
        K[:, :, j * 64, 3] = _bf16((-1.0) ** t * 2.0 ** -(40 + t % 30))
    yield "tiny_run", dict(d, K=K)
    K = d["K"].copy()                                          # the same with a short run (a group of at most 64 blocks)
    for t, j in enumerate(range(40, 40 + min(40, nkb // 4))):
        K[:, :, j * 64:(j + 1) * 64] = 0
        K[:, :, j * 64, 3] = _bf16((-1.0) ** t * 2.0 ** -(40 + t % 13))
    yield "tiny_short_run", dict(d, K=K)


@pytest.mark.parametrize("nkb,bq,kc,kn", [(300, 64, 15, 200), (300, 128, 1, 299), (300, 64, 299, 1), (300, 64, 0, 150), (300, 64, 7, 0),
                                          (700, 128, 35, 560), (1000, 64, 50, 500), (1100, 128, 3, 1000), (1700, 128, 40, 1100),
                                          (2147, 128, 64, 1400), (2500, 128, 100, 2000), (4000, 128, 120, 2500), (3000, 64, 90, 2400)])
def test_key_classifier_equals_the_exact_order(oracle, nkb, bq, kc, kn):
    from paper_2605_11354_amd import binding as B
    cfg = C0.with_(H=2 if nkb <= 1100 else 1, N=nkb * 64 - 17, bq=bq, n_clusters=256)
    d = synth.make_inputs(cfg)
    for name, dd in _variants(cfg, d):
        case = G.Case(cfg, dd, k_crit=kc, k_neg=kn)
        got = case.classify(want=("crit_idx",))                # no logits, no softmax: the 32-bit key path
        ref = case.oracle_classify(oracle)
        bad = np.argwhere(got["labels"] != ref["labels"])
        assert bad.size == 0, (name, len(bad), bad[:4])
        if kc > 0:
            for idx in np.ndindex(got["labels"].shape[:3]):
                assert np.array_equal(got["crit_idx"][idx], np.nonzero(ref["labels"][idx] == 2)[0]), (name, idx)
        old = case.classify(want=("scores",))                  # the fp64 path of the same library
        assert np.array_equal(old["labels"], got["labels"]), name
        # the marginal mask the aggregation reads: run the forward with and without given labels
        O1, lab1 = case.forward()
        assert np.array_equal(lab1.cpu().numpy(), ref["labels"]), name
        O2 = torch.empty_like(O1)
        B.sla_forward_with_labels(case.p, case.Q, case.K, case.V, case.W, lab1, O2, case.sQ, case.sK, case.sV, case.ws)
        torch.cuda.synchronize()
        assert torch.equal(O1.view(torch.int16), O2.view(torch.int16)), name


def test_key_classifier_e4m3_inputs(oracle):
    cfg = synth.CONFIGS[4].with_(H=2, N=700 * 64 - 30)
    case = G.Case(cfg)
    got = case.classify(want=("crit_idx",))
    ref = case.oracle_classify(oracle)
    assert np.array_equal(got["labels"], ref["labels"])


@pytest.mark.parametrize("nkb,kc,kn", [(100, 5, 60), (100, 40, 30), (250, 12, 150), (250, 60, 100)])
def test_short_rows_with_tied_groups(oracle, nkb, kc, kn):
    """Rows of at most 256 key blocks (the fused classifier) look for both ranks among the same 32-bit spread of the logits
    and fall back to the exact keys where a group is not taken whole: the same variants as above."""
    cfg = C0.with_(H=2, N=nkb * 64 - 17, bq=64, n_clusters=64)
    d = synth.make_inputs(cfg)
    for name, dd in _variants(cfg, d):
        case = G.Case(cfg, dd, k_crit=kc, k_neg=kn)
        got = case.classify(want=("crit_idx",))
        ref = case.oracle_classify(oracle)
        assert np.array_equal(got["labels"], ref["labels"]), name
        for idx in np.ndindex(got["labels"].shape[:3]):
            assert np.array_equal(got["crit_idx"][idx], np.nonzero(ref["labels"][idx] == 2)[0]), (name, idx)
        O1, lab1 = case.forward()
        assert np.array_equal(lab1.cpu().numpy(), ref["labels"]), name
