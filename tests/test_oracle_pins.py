"""Pins of the fp64 oracle against what the paper and the mathematics fix (CPU only).

Each test names the passage it pins:
  * section 3.3 (A_full) and Alg. 1 steps 2-5  -> all-critical limit = dense softmax attention
  * Alg. 1 steps 6-10                           -> all-marginal limit = linear attention
  * eq. (1)                                     -> O = O_sparse + O_lin W
  * Alg. 1 step 3 at block level                -> rank definition, counts, ties
The paper prints no worked numeric example of SLA, so the pins are closed forms, limits that
reduce to textbook operators (written independently in tests/bruteforce.py), invariants and
brute force on small inputs.
"""
from fractions import Fraction

import numpy as np
import pytest

from paper_2605_11354_amd import synth
from tests import bruteforce as bf


def _rand_bits(rng, shape, scale=1.0):
    return synth.to_bf16_bits(rng.standard_normal(shape) * scale)


def _small(rng, B=1, H=2, N=150, per_head=True):
    Q = _rand_bits(rng, (B, H, N, 64)); K = _rand_bits(rng, (B, H, N, 64)); V = _rand_bits(rng, (B, H, N, 64))
    W = _rand_bits(rng, (H, 64, 64) if per_head else (64, 64), 0.125)
    return Q, K, V, W


@pytest.mark.parametrize("N,bq,bk", [(512, 64, 64), (150, 64, 64), (300, 128, 64), (64, 64, 64), (1, 64, 64)])
def test_all_critical_equals_dense_attention(oracle, N, bq, bk):
    rng = np.random.default_rng(1)
    Q, K, V, W = _small(rng, N=N)
    Nkb = -(-N // bk)
    p = oracle.make_params(1, 2, N, bq, bk, Nkb, 0, proj_per_head=True)
    r = oracle.forward(p, Q, K, V, W, want_parts=True)
    assert (r["labels"] == 2).all()
    for h in range(2):
        ref = bf.dense_attention(bf.bf16_bits_to_f64(Q[0, h]), bf.bf16_bits_to_f64(K[0, h]),
                                 bf.bf16_bits_to_f64(V[0, h]), 0.125)
        np.testing.assert_allclose(r["O"][0, h], ref, rtol=0, atol=1e-12)
        assert np.abs(r["O_lin"][0, h]).max() == 0.0     # linear branch contributes exactly 0


@pytest.mark.parametrize("scale", [0.25, 0.03, 1.0])
def test_softmax_scale_other_than_the_default_reaches_the_sparse_branch(oracle, scale):
    """sm_scale != 1/sqrt(D): all blocks critical must equal dense softmax attention at THAT scale (section 3.3 fixes
    only the default), and a general label pattern the token-level masked form at that scale."""
    rng = np.random.default_rng(8)
    Q, K, V, W = _small(rng, N=300)
    p = oracle.make_params(1, 2, 300, 128, 64, 5, 0, proj_per_head=True, sm_scale=scale)
    r = oracle.forward(p, Q, K, V, W)
    for h in range(2):
        ref = bf.dense_attention(*(bf.bf16_bits_to_f64(x[0, h]) for x in (Q, K, V)), scale)
        np.testing.assert_allclose(r["O"][0, h], ref, rtol=0, atol=1e-12)
    p = oracle.make_params(1, 2, 300, 64, 64, 2, 1, proj_per_head=True, sm_scale=scale)
    r = oracle.forward(p, Q, K, V, W)
    for h in range(2):
        ref, _, _ = bf.sla_tokenlevel(*(bf.bf16_bits_to_f64(x[0, h]) for x in (Q, K, V)), bf.bf16_bits_to_f64(W[h]),
                                      r["labels"][0, h], 64, 64, scale)
        np.testing.assert_allclose(r["O"][0, h], ref, rtol=0, atol=1e-11)


def test_all_critical_on_config0(oracle):
    cfg = synth.CONFIGS[0]
    d = synth.make_inputs(cfg)
    p = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, 8, 0)
    r = oracle.forward(p, d["Q"], d["K"], d["V"], d["W"])
    for h in range(cfg.H):
        ref = bf.dense_attention(*(bf.bf16_bits_to_f64(d[k][0, h]) for k in "QKV"), 0.125)
        np.testing.assert_allclose(r["O"][0, h], ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("N,bq,bk,per_head", [(512, 64, 64, False), (150, 64, 64, True), (300, 128, 64, True)])
def test_all_marginal_equals_linear_attention(oracle, N, bq, bk, per_head):
    rng = np.random.default_rng(2)
    Q, K, V, W = _small(rng, N=N, per_head=per_head)
    p = oracle.make_params(1, 2, N, bq, bk, 0, 0, proj_per_head=per_head)
    r = oracle.forward(p, Q, K, V, W, want_parts=True)
    assert (r["labels"] == 1).all()
    for h in range(2):
        Wd = bf.bf16_bits_to_f64(W[h] if per_head else W)
        ref = bf.linear_attention(*(bf.bf16_bits_to_f64(x[0, h]) for x in (Q, K, V)), Wd)
        np.testing.assert_allclose(r["O"][0, h], ref, rtol=0, atol=1e-12)
        assert np.abs(r["O_sparse"][0, h]).max() == 0.0


def test_linear_attention_with_identity_projection_is_textbook(oracle):
    rng = np.random.default_rng(3)
    Q, K, V, _ = _small(rng, N=200)
    W = synth.to_bf16_bits(np.eye(64))
    p = oracle.make_params(1, 2, 200, 64, 64, 0, 0)
    r = oracle.forward(p, Q, K, V, W)
    fq = bf.phi_softmax(bf.bf16_bits_to_f64(Q[0, 1])); fk = bf.phi_softmax(bf.bf16_bits_to_f64(K[0, 1]))
    A = fq @ fk.T                                       # pairwise kernel form
    ref = (A / A.sum(1, keepdims=True)) @ bf.bf16_bits_to_f64(V[0, 1])
    np.testing.assert_allclose(r["O"][0, 1], ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("N,bq,bk,kc,kn", [(512, 64, 64, 1, 4), (700, 128, 64, 2, 5), (333, 64, 64, 3, 0), (333, 64, 64, 0, 3)])
def test_general_labels_match_tokenlevel_masked_form(oracle, N, bq, bk, kc, kn):
    """Mixed critical/marginal/negligible rows against a dense-mask token-level formulation."""
    rng = np.random.default_rng(4)
    Q, K, V, W = _small(rng, N=N)
    p = oracle.make_params(1, 2, N, bq, bk, kc, kn, proj_per_head=True)
    r = oracle.forward(p, Q, K, V, W, want_parts=True)
    for h in range(2):
        O, Osp, Olin = bf.sla_tokenlevel(*(bf.bf16_bits_to_f64(x[0, h]) for x in (Q, K, V)),
                                         bf.bf16_bits_to_f64(W[h]), r["labels"][0, h], bq, bk, 0.125)
        np.testing.assert_allclose(r["O_sparse"][0, h], Osp, rtol=0, atol=1e-12)
        np.testing.assert_allclose(r["O_lin"][0, h], Olin, rtol=0, atol=1e-12)
        np.testing.assert_allclose(r["O"][0, h], O, rtol=0, atol=1e-12)


def test_v_ones_closed_form(oracle):
    """V == 1: both branches return 1, so O[t,:] = 1 + 1^T W for every row (eq. 1)."""
    cfg = synth.CONFIGS[0]
    d = synth.make_inputs(cfg)
    V = np.full_like(d["V"], 0x3F80)
    kc, kn = oracle.counts(cfg.crit_frac, cfg.neg_frac, 8)
    p = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, kc, kn)
    r = oracle.forward(p, d["Q"], d["K"], V, d["W"])
    expect = 1.0 + bf.bf16_bits_to_f64(d["W"]).sum(axis=0)
    np.testing.assert_allclose(r["O"], np.broadcast_to(expect, r["O"].shape), rtol=0, atol=1e-12)


def test_constant_key_closed_form(oracle):
    """All K rows equal: O_sparse = mean of V over critical tokens, O_lin = mean over marginal tokens."""
    rng = np.random.default_rng(5)
    N, bq, bk = 300, 64, 64
    Q, K, V, W = _small(rng, H=1, N=N, per_head=False)
    K[:] = K[0, 0, 0]
    p = oracle.make_params(1, 1, N, bq, bk, 2, 1)
    r = oracle.forward(p, Q, K, V, W, want_parts=True)
    # every score ties -> critical = blocks 0,1; negligible = last block (tail of 44 tokens); marginal = 2,3
    assert (r["labels"][0, 0] == np.array([2, 2, 1, 1, 0], dtype=np.int8)).all()
    Vd = bf.bf16_bits_to_f64(V[0, 0])
    np.testing.assert_allclose(r["O_sparse"][0, 0], np.broadcast_to(Vd[:128].mean(0), (N, 64)), atol=1e-12)
    np.testing.assert_allclose(r["O_lin"][0, 0], np.broadcast_to(Vd[128:256].mean(0), (N, 64)), atol=1e-12)
    np.testing.assert_allclose(r["O"][0, 0], r["O_sparse"][0, 0] + r["O_lin"][0, 0] @ bf.bf16_bits_to_f64(W), atol=1e-12)


def test_sparse_rows_are_convex_combinations(oracle):
    """W = 0: every output row lies in the coordinate-wise hull of its critical V rows."""
    cfg = synth.CONFIGS[0]
    d = synth.make_inputs(cfg)
    p = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, 1, 4)
    r = oracle.forward(p, d["Q"], d["K"], d["V"], np.zeros_like(d["W"]))
    for h in range(cfg.H):
        Vd = bf.bf16_bits_to_f64(d["V"][0, h]).reshape(8, 64, 64)
        for i in range(8):
            j = int(np.nonzero(r["labels"][0, h, i] == 2)[0][0])
            blk = r["O"][0, h, i * 64:(i + 1) * 64]
            assert (blk <= Vd[j].max(0) + 1e-12).all() and (blk >= Vd[j].min(0) - 1e-12).all()


# ------------------------------------------------------------------------------ classifier
def test_counts_table():
    """k = floor(f*Nkb + 0.5), k_c >= 1 when f_c > 0; the five benchmark configurations."""
    from oracle import sla_oracle as o
    rows = [l.split() for l in open(__file__.rsplit("/", 1)[0] + "/golden/block_counts.txt") if l[0] != "#"]
    assert len(rows) == 5
    for name, nkb, fc, fn, kc, kn, km in rows:
        got = o.counts(float(fc), float(fn), int(nkb))
        assert got == (int(kc), int(kn)), (name, got)
        assert int(nkb) - got[0] - got[1] == int(km)
    assert o.counts(0.0, 1.0, 10) == (0, 10)
    assert o.counts(0.001, 0.999, 10) == (1, 9)       # at least one critical block, negligible clipped
    assert o.counts(1.0, 0.0, 7) == (7, 0)


def test_labels_follow_rank_definition(oracle):
    rng = np.random.default_rng(6)
    N, bq, bk = 1374, 64, 64
    Q, K, _, _ = _small(rng, N=N)
    # force exact ties between pooled logits: duplicate key blocks 3 and 7, 4 and 20
    K[:, :, 7 * 64:8 * 64] = K[:, :, 3 * 64:4 * 64]
    K[:, :, 20 * 64:21 * 64] = K[:, :, 4 * 64:5 * 64]
    for kc, kn in [(2, 13), (1, 0), (0, 22), (22, 0), (5, 17)]:
        p = oracle.make_params(1, 2, N, bq, bk, kc, kn)
        c = oracle.classify(p, Q, K, want_scores=True)
        for h in range(2):
            for i in range(22):
                assert (c["labels"][0, h, i] == bf.rank_labels(c["scores"][0, h, i], kc, kn)).all()
                assert c["scores"][0, h, i, 3] == c["scores"][0, h, i, 7]
        assert ((c["labels"] == 2).sum(-1) == kc).all() and ((c["labels"] == 0).sum(-1) == kn).all()


def test_all_tied_scores_break_by_lowest_index(oracle):
    rng = np.random.default_rng(7)
    Q, K, _, _ = _small(rng, N=640)
    Q[:] = 0
    p = oracle.make_params(1, 2, 640, 64, 64, 3, 4)
    lab = oracle.classify(p, Q, K)["labels"]
    assert (lab == np.array([2, 2, 2, 1, 1, 1, 0, 0, 0, 0], dtype=np.int8)).all()


def test_known_score_order(oracle):
    """K block j = j*e0, Q = e0  =>  pooled logit of block j is j: critical = highest j."""
    N = 10 * 64
    Q = np.zeros((1, 1, N, 64), np.uint16); K = np.zeros_like(Q)
    Q[..., 0] = synth.to_bf16_bits(np.array([1.0]))[0]
    K[0, 0, :, 0] = synth.to_bf16_bits(np.repeat(np.arange(10.0), 64))
    p = oracle.make_params(1, 1, N, 64, 64, 2, 5)
    c = oracle.classify(p, Q, K, want_scores=True, want_pc=True)
    assert (c["scores"][0, 0] == np.arange(10.0)).all()
    assert (c["labels"][0, 0] == np.array([0, 0, 0, 0, 0, 1, 1, 1, 2, 2], dtype=np.int8)).all()
    e = np.exp(np.arange(10.0) * 0.125); e /= e.sum()
    np.testing.assert_allclose(c["Pc"][0, 0, 0], e, rtol=1e-14)


def test_pooled_means_and_logit_chain_are_exact(oracle):
    """Means = exact block sum * (1/count); logits = correctly rounded fma chain (rational arithmetic)."""
    cfg = synth.CONFIGS[0].with_(N=150)
    d = synth.make_inputs(cfg)
    p = oracle.make_params(1, 2, 150, 64, 64, 1, 1)
    c = oracle.classify(p, d["Q"], d["K"], want_scores=True, want_means=True, want_pc=True)
    Kd = bf.bf16_bits_to_f64(d["K"][0, 1]); Qd = bf.bf16_bits_to_f64(d["Q"][0, 1])
    for j, (t0, t1) in enumerate([(0, 64), (64, 128), (128, 150)]):
        for X, m in ((Kd, c["kbar"]), (Qd, c["qbar"])):
            exact = [float(sum(Fraction(v) for v in X[t0:t1, dd])) * (1.0 / (t1 - t0)) for dd in range(64)]
            assert (m[0, 1, j] == np.array(exact)).all()
    for i in range(3):
        for j in range(3):
            s = 0.0
            for dd in range(64):
                s = float(Fraction(c["qbar"][0, 1, i, dd]) * Fraction(c["kbar"][0, 1, j, dd]) + Fraction(s))
            assert s == c["scores"][0, 1, i, j]
    np.testing.assert_allclose(c["Pc"].sum(-1), 1.0, rtol=1e-14)
    x = c["scores"][0, 1] * 0.125
    ref = np.exp(x - x.max(1, keepdims=True)); ref /= ref.sum(1, keepdims=True)
    np.testing.assert_allclose(c["Pc"][0, 1], ref, rtol=1e-13)


def test_permutation_within_key_block_is_invariant(oracle):
    cfg = synth.CONFIGS[0]
    d = synth.make_inputs(cfg)
    p = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, 2, 3)
    r0 = oracle.forward(p, d["Q"], d["K"], d["V"], d["W"])
    perm = np.arange(cfg.N)
    rng = np.random.default_rng(8)
    for j in range(8):
        perm[j * 64:(j + 1) * 64] = j * 64 + rng.permutation(64)
    r1 = oracle.forward(p, d["Q"], np.ascontiguousarray(d["K"][:, :, perm]), np.ascontiguousarray(d["V"][:, :, perm]), d["W"])
    assert (r0["labels"] == r1["labels"]).all()
    np.testing.assert_allclose(r0["O"], r1["O"], rtol=0, atol=1e-12)


def test_batch_items_are_independent_and_selection_matches_full(oracle):
    cfg = synth.CONFIGS[3].with_(B=3, H=2)
    d = synth.make_inputs(cfg)
    kc, kn = oracle.counts(cfg.crit_frac, cfg.neg_frac, 22)
    p = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, kc, kn, proj_per_head=True)
    full = oracle.forward(p, d["Q"], d["K"], d["V"], d["W"])
    p1 = oracle.make_params(1, cfg.H, cfg.N, cfg.bq, cfg.bk, kc, kn, proj_per_head=True)
    one = oracle.forward(p1, *(np.ascontiguousarray(d[k][2:3]) for k in "QKV"), d["W"])
    assert (full["labels"][2] == one["labels"][0]).all()
    assert (full["O"][2] == one["O"][0]).all()
    sel = [(5, 21), (0, 3), (5, 0)]
    part = oracle.forward(p, d["Q"], d["K"], d["V"], d["W"], sel=sel)
    for s, (bh, i) in enumerate(sel):
        rows = min(cfg.N, (i + 1) * 64) - i * 64
        assert (part["O"][s, :rows] == full["O"][bh // 2, bh % 2, i * 64:i * 64 + rows]).all()
        assert (part["O"][s, rows:] == 0).all()


# ------------------------------------------------------------------------------ number formats
def test_e4m3_table_matches_format_definition(oracle):
    """App. B.1: 1-4-3 bits, max 448; every code against torch's float8_e4m3fn and the golden facts."""
    import ctypes
    import torch
    f = oracle.lib().sla_oracle_decode_e4m3
    f.restype = ctypes.c_double
    f.argtypes = [ctypes.c_uint8]
    mine = np.array([f(c) for c in range(256)])
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    assert np.array_equal(np.isnan(mine), np.isnan(ref)) and np.isnan(mine).sum() == 2
    ok = ~np.isnan(ref)
    assert (mine[ok] == ref[ok]).all()
    for line in open(__file__.rsplit("/", 1)[0] + "/golden/e4m3_facts.txt"):
        if line[0] == "#":
            continue
        code, val = line.split()
        assert mine[int(code, 16)] == float(val)
    assert np.nanmax(mine) == 448.0


def test_generator_quantiser_round_trips(oracle):
    """Scaled quantiser of App. B.2 as used by the input generator: amax -> +-448, error <= 2^-4 relative."""
    vals = synth.e4m3_code_values()
    ok = ~np.isnan(vals)
    assert (synth.e4m3_encode(vals[ok].astype(np.float32)) == np.arange(256, dtype=np.uint8)[ok]).all()
    rng = np.random.default_rng(9)
    bits = _rand_bits(rng, (1, 2, 300, 64))
    codes, scales = synth.quantise_e4m3_blocks(bits, 128)
    assert scales.shape == (1, 2, 3) and ((codes & 0x7F) != 0x7F).all()
    x = synth.bf16_bits_to_f32(bits).astype(np.float64)
    deq = vals[codes] * np.repeat(scales.astype(np.float64), 128, axis=-1)[..., :300, None]
    for j in range(3):
        sl = slice(j * 128, min(300, (j + 1) * 128))
        assert np.abs(vals[codes[..., sl, :]]).max(axis=(-1, -2)).tolist() == [[448.0, 448.0]]
    normal = np.abs(x) >= scales.astype(np.float64).max() * 2.0 ** -6
    assert (np.abs(deq - x)[normal] <= np.abs(x)[normal] * 2.0 ** -4).all()


def test_fp8_inputs_all_critical_equals_dense_on_dequantised(oracle):
    cfg = synth.CONFIGS[4].with_(N=300, H=2)
    d = synth.make_inputs(cfg)
    vals = synth.e4m3_code_values()
    p = oracle.make_params(1, 2, 300, 128, 64, 5, 0, dtype="fp8", proj_per_head=True)
    r = oracle.forward(p, d["Q"], d["K"], d["V"], d["W"], d["sQ"], d["sK"], d["sV"])
    for h in range(2):
        deq = [vals[d[k][0, h]] * np.repeat(d["s" + k][0, h].astype(np.float64), b)[:300, None]
               for k, b in (("Q", 128), ("K", 64), ("V", 64))]
        np.testing.assert_allclose(r["O"][0, h], bf.dense_attention(*deq, 0.125), rtol=0, atol=1e-12)


def test_wproj_gradient_matches_difference_quotient_of_the_forward(oracle):
    """O is linear in W_O (Alg. 1 step 10), so the difference quotient of L = sum(O * G) between two projections
    that differ in one entry IS dL/dW for that entry; this fixes the orientation ([D_in, D_out], right-multiplied),
    the use of the normalised O_lin, and the sum over heads of a shared projection."""
    for per_head in (False, True):
        cfg = synth.CONFIGS[0].with_(N=200, proj_per_head=per_head)
        d = synth.make_inputs(cfg)
        po = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, 1, 1, cfg.dtype, cfg.proj_per_head)
        labels = oracle.classify(po, d["Q"], d["K"])["labels"]
        rng = np.random.default_rng(5)
        G = rng.standard_normal((cfg.B, cfg.H, cfg.N, 64))
        dW = oracle.grad_wproj(po, d["Q"], d["K"], d["V"], labels, G)
        assert dW.shape == ((cfg.H if per_head else 1), 64, 64)
        base = oracle.forward(po, d["Q"], d["K"], d["V"], d["W"])["O"]
        L0 = float((base * G).sum())
        W = d["W"].reshape(-1, 64, 64)
        for (w, e_in, e_out) in [(0, 3, 17), (W.shape[0] - 1, 63, 0), (0, 40, 40)]:
            W2 = W.copy()
            bf = lambda bits: float((np.array([bits], np.uint32) << 16).view(np.float32)[0])     # bf16 bits -> value
            old = bf(int(W2[w, e_in, e_out]))
            W2[w, e_in, e_out] = synth.to_bf16_bits(np.array([old + 0.5], np.float32))[0]      # another bf16 value
            delta = bf(int(W2[w, e_in, e_out])) - old
            assert delta != 0.0
            O2 = oracle.forward(po, d["Q"], d["K"], d["V"], W2.reshape(d["W"].shape))["O"]
            quotient = (float((O2 * G).sum()) - L0) / delta
            assert abs(quotient - dW[w, e_in, e_out]) <= 1e-9 * max(1.0, abs(dW[w, e_in, e_out])), (per_head, w, e_in, e_out)


def test_wproj_gradient_closed_form_for_constant_values(oracle):
    """V == 1 makes O_lin the all-ones row for every token whose query block has a marginal block (a weighted
    mean of ones), so every row of dL/dW_O is the column sum of dO over those tokens."""
    cfg = synth.CONFIGS[0]
    d = dict(synth.make_inputs(cfg))
    d["V"] = np.full_like(d["V"], 0x3F80)
    po = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, 1, 4, cfg.dtype, cfg.proj_per_head)
    labels = oracle.classify(po, d["Q"], d["K"])["labels"]
    assert (labels == 1).any(axis=-1).all()                      # every query block has marginal blocks here
    G = np.random.default_rng(6).standard_normal((cfg.B, cfg.H, cfg.N, 64))
    dW = oracle.grad_wproj(po, d["Q"], d["K"], d["V"], labels, G)
    expect = np.broadcast_to(G.sum(axis=(0, 1, 2)), (64, 64))
    np.testing.assert_allclose(dW[0], expect, rtol=1e-12, atol=1e-10)
    # and no marginal block at all: no gradient
    po0 = oracle.make_params(cfg.B, cfg.H, cfg.N, cfg.bq, cfg.bk, 4, 4, cfg.dtype, cfg.proj_per_head)
    lab0 = oracle.classify(po0, d["Q"], d["K"])["labels"]
    assert not (lab0 == 1).any()
    assert np.all(oracle.grad_wproj(po0, d["Q"], d["K"], d["V"], lab0, G) == 0.0)


@pytest.mark.parametrize("N,bq,bk,kc,kn", [(512, 64, 64, 0, 0), (700, 128, 64, 2, 5), (333, 64, 64, 3, 0)])
def test_elu_feature_map_matches_tokenlevel_form(oracle, N, bq, bk, kc, kn):
    """phi = ELU(x)+1 as Alg. 1 step 6 prints it: all-marginal equals token-level linear attention (steps 6-10),
    mixed labels equal the dense-mask token-level form; the sparse branch does not depend on phi."""
    rng = np.random.default_rng(7)
    Q, K, V, W = _small(rng, N=N)
    p = oracle.make_params(1, 2, N, bq, bk, kc, kn, proj_per_head=True, phi="elu1")
    ps = oracle.make_params(1, 2, N, bq, bk, kc, kn, proj_per_head=True)
    r = oracle.forward(p, Q, K, V, W, want_parts=True)
    rs = oracle.forward(ps, Q, K, V, W, want_parts=True)
    assert np.array_equal(r["labels"], rs["labels"]) and np.array_equal(r["O_sparse"], rs["O_sparse"])
    if kc == 0 and kn == 0:
        assert np.abs(r["O_lin"] - rs["O_lin"]).max() > 1e-3          # the two feature maps do differ
    for h in range(2):
        q, k, v = (bf.bf16_bits_to_f64(x[0, h]) for x in (Q, K, V))
        Wd = bf.bf16_bits_to_f64(W[h])
        O, Osp, Olin = bf.sla_tokenlevel(q, k, v, Wd, r["labels"][0, h], bq, bk, 0.125, phi="elu1")
        np.testing.assert_allclose(r["O_lin"][0, h], Olin, rtol=0, atol=1e-11)
        np.testing.assert_allclose(r["O"][0, h], O, rtol=0, atol=1e-11)
        if kc == 0 and kn == 0:
            np.testing.assert_allclose(r["O"][0, h], bf.linear_attention(q, k, v, Wd, phi="elu1"), rtol=0, atol=1e-11)


def test_elu_feature_map_values():
    """ELU(x)+1: 1 at 0, x+1 above, exp(x) below (continuous, positive)."""
    x = np.array([-30.0, -1.0, -0.0, 0.0, 0.5, 3.0])
    np.testing.assert_allclose(bf.phi_elu1(x), [np.exp(-30.0), np.exp(-1.0), 1.0, 1.0, 1.5, 4.0], rtol=1e-15)


def test_block_quantiser_matches_library_cast_and_host_generator(oracle):
    """The oracle's quantiser (App. B.2 per token block) against two independent casts: torch's float8_e4m3fn
    conversion of the same clamped fp32 quotients, and the benchmark generator's own quantiser."""
    import torch
    rng = np.random.default_rng(8)
    x = rng.standard_normal((2, 3, 333, 64)).astype(np.float32) * np.exp(rng.uniform(-12, 6, (2, 3, 333, 1))).astype(np.float32)
    x[0, 0, :64] = 0.0                                              # an all-zero block: scale = 1e-8/448, codes 0
    x[0, 1, 5, 7] = 3.0e4                                           # a block whose amax is a single outlier
    bits = synth.to_bf16_bits(x)
    codes, scales = oracle.quantise_e4m3_blocks(bits, 64)
    xb = (bits.astype(np.uint32) << 16).view(np.float32)
    for j in range(6):
        sl = slice(64 * j, min(333, 64 * j + 64))
        amax = np.abs(xb[..., sl, :]).max(axis=(-2, -1))
        sc = np.maximum(amax, np.float32(1e-8)) / np.float32(448.0)
        assert np.array_equal(scales[..., j], sc.astype(np.float32))
        y = np.clip(xb[..., sl, :] / sc[..., None, None].astype(np.float32), -448.0, 448.0).astype(np.float32)
        t = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        got = codes[..., sl, :]
        same = (got == t) | ((got & 0x7F == 0) & (t & 0x7F == 0))   # +0 / -0 may differ in sign conventions only
        assert same.all()
    c2, s2 = synth.quantise_e4m3_blocks(bits, 64)
    assert np.array_equal(s2, scales) and np.array_equal(c2, codes)
    assert np.all(codes[0, 0, :64] == 0) and scales[0, 0, 0] == np.float32(1e-8) / np.float32(448.0)
    # exact half-way cases go to the even code: 1.0625 = midpoint of 1.0 (0x38) and 1.125 (0x39) at scale 1
    tie = np.zeros((1, 1, 64, 64), np.float32); tie[0, 0, 0, 0] = 448.0; tie[0, 0, 0, 1] = 1.0625; tie[0, 0, 0, 2] = 1.1875
    ct, st = oracle.quantise_e4m3_blocks(synth.to_bf16_bits(tie), 64)
    assert st[0, 0, 0] == 1.0 and ct[0, 0, 0, 0] == 0x7E and ct[0, 0, 0, 1] == 0x38 and ct[0, 0, 0, 2] == 0x3A


def test_fp8_linear_matches_torch_fake_quant(oracle):
    """Alg. 2 forward (per-token activation scales, per-output-channel weight scales) against the same steps written
    with torch tensor ops and torch's float8_e4m3fn cast; plus: a power-of-two rescaling of a token leaves its codes
    unchanged (the scale absorbs it) and scales y by the same factor."""
    import torch
    rng = np.random.default_rng(9)
    x = (rng.standard_normal((37, 192)) * np.exp(rng.uniform(-3, 3, (37, 1)))).astype(np.float32)
    W = (rng.standard_normal((70, 192)) * 0.05).astype(np.float32)
    b = rng.standard_normal(70).astype(np.float32)
    xb, Wb, bb = synth.to_bf16_bits(x), synth.to_bf16_bits(W), synth.to_bf16_bits(b)
    y = oracle.fp8_linear(xb, Wb, bb)
    f = lambda bits: torch.from_numpy((bits.astype(np.uint32) << 16).view(np.float32).copy())

    def fq(t):
        scale = torch.clamp(t.abs().amax(dim=-1, keepdim=True), min=1e-8) / 448.0
        q = torch.clamp(t / scale, -448.0, 448.0).to(torch.float8_e4m3fn).to(torch.float64)
        return q * scale.to(torch.float64)
    ref = fq(f(xb)) @ fq(f(Wb)).T + f(bb).to(torch.float64)
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)
    x2 = x.copy(); x2[5] *= 8.0
    c1, s1 = oracle.quantise_e4m3_rows(xb)
    c2, s2 = oracle.quantise_e4m3_rows(synth.to_bf16_bits(x2))
    assert np.array_equal(c1, c2) and s2[5] == s1[5] * 8 and np.array_equal(np.delete(s1, 5), np.delete(s2, 5))
    y2 = oracle.fp8_linear(synth.to_bf16_bits(x2), Wb, None)
    np.testing.assert_allclose(y2[5], 8.0 * (y[5] - (bb.astype(np.uint32) << 16).view(np.float32)), rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ Alg. 1 as printed (token-level mask, global linear branch)
def _alg1_inputs(N, seed=4):
    rng = np.random.default_rng(seed)
    f = lambda s: bf.bf16_bits_to_f64(synth.to_bf16_bits(rng.standard_normal((N, 64)) * s))
    return f(1.0), f(1.0), f(1.0), bf.bf16_bits_to_f64(synth.to_bf16_bits(rng.standard_normal((64, 64)) / 8.0))


@pytest.mark.parametrize("phi", ["elu1", "softmax"])
def test_alg1_with_keep_ratio_one_is_dense_plus_global_linear_attention(oracle, phi):
    """lambda = 1 keeps every key: O = Softmax(Q K^T / sqrt(d)) V + LinearAttention(Q, K, V) W_O, both textbook operators."""
    Q, K, V, W = _alg1_inputs(150)
    r = oracle.alg1_token_level(Q, K, V, W, 1.0, phi=phi)
    assert r["M"].all()
    np.testing.assert_allclose(r["O_sparse"], bf.dense_attention(Q, K, V, 0.125), rtol=0, atol=1e-12)
    np.testing.assert_allclose(r["O"], bf.dense_attention(Q, K, V, 0.125) + bf.linear_attention(Q, K, V, W, phi), rtol=0, atol=1e-12)


def test_alg1_mask_on_a_hand_built_score_order(oracle):
    """Scores with a known order: Q = one-hot rows, K = columns of a table, so S = table / 8 entry for entry.  The mask
    keeps ceil(lambda N) keys per row, the largest first, equal scores by lowest key index; the sparse output is then the
    softmax-weighted mean of the kept V rows, and the linear branch does not depend on lambda."""
    N = 8
    table = np.array([[7, 6, 5, 4, 3, 2, 1, 0],            # descending: keeps 0, 1, 2
                      [0, 1, 2, 3, 4, 5, 6, 7],            # ascending: keeps 7, 6, 5
                      [5, 5, 5, 5, 5, 5, 5, 5],            # all tied: keeps 0, 1, 2
                      [1, 9, 1, 9, 1, 9, 1, 9],            # ties at the top: 1, 3, 5
                      [2, 0, 2, 0, 2, 0, 2, 0],            # ties at the threshold: 0, 2, 4
                      [0, 0, 0, 8, 0, 0, 0, 0],            # one peak, then ties by index: 3, 0, 1
                      [-1, -2, -3, -4, -5, -6, -7, -8],    # negative scores: 0, 1, 2
                      [3, 1, 4, 1, 5, 9, 2, 6]], float)    # 5, 7, 4
    Q = np.zeros((N, 64)); Q[np.arange(N), np.arange(N)] = 1.0
    K = np.zeros((N, 64)); K[:, :N] = table.T
    rng = np.random.default_rng(6)
    V = rng.standard_normal((N, 64)); W = rng.standard_normal((64, 64)) / 8.0
    r = oracle.alg1_token_level(Q, K, V, W, 3.0 / 8.0)
    want = [[0, 1, 2], [7, 6, 5], [0, 1, 2], [1, 3, 5], [0, 2, 4], [3, 0, 1], [0, 1, 2], [5, 7, 4]]
    for i in range(N):
        assert sorted(np.nonzero(r["M"][i])[0].tolist()) == sorted(want[i]), i
        w = np.exp(table[i, want[i]] / 8.0); w /= w.sum()
        np.testing.assert_allclose(r["O_sparse"][i], w @ V[want[i]], rtol=0, atol=1e-13)
    np.testing.assert_allclose(r["O_lin"] @ W, bf.linear_attention(Q, K, V, W, "elu1"), rtol=0, atol=1e-12)
    assert oracle.alg1_token_level(Q, K, V, W, 0.3)["M"].sum(axis=1).tolist() == [3] * N      # ceil(0.3 * 8) = 3
    r0 = oracle.alg1_token_level(Q, K, V, W, 0.0)
    assert not r0["M"].any() and np.abs(r0["O_sparse"]).max() == 0.0


def test_alg1_agrees_with_the_block_level_module_at_its_two_limits(oracle):
    """Where the two granularities coincide: everything kept (lambda = 1 / all blocks critical) and nothing kept
    (lambda = 0 / all blocks marginal): the block-level oracle and Alg. 1 as printed give the same output."""
    rng = np.random.default_rng(9)
    Qb, Kb, Vb, Wb = _small(rng, N=200, per_head=False)
    Q, K, V, W = (bf.bf16_bits_to_f64(x) for x in (Qb[0, 0], Kb[0, 0], Vb[0, 0], Wb))
    p = oracle.make_params(1, 2, 200, 64, 64, 4, 0, phi="elu1")
    np.testing.assert_allclose(oracle.forward(p, Qb, Kb, Vb, Wb, want_parts=True)["O_sparse"][0, 0],
                               oracle.alg1_token_level(Q, K, V, W, 1.0)["O_sparse"], rtol=0, atol=1e-12)
    p = oracle.make_params(1, 2, 200, 64, 64, 0, 0, phi="elu1")
    np.testing.assert_allclose(oracle.forward(p, Qb, Kb, Vb, Wb)["O"][0, 0], oracle.alg1_token_level(Q, K, V, W, 0.0)["O"], rtol=0, atol=1e-12)
