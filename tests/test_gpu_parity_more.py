"""GPU parity, second part: the tolerance as stated (on the fp32 result), shapes and paths the first part
does not reach (odd head counts, E4M3 with batch > 1 and with 64-row query blocks, all-zero blocks, short and long
critical lists, V blocks of very different magnitude, a running maximum that has to be raised in mid-list) and
whole-tensor invariants at full size."""
import numpy as np
import pytest
import torch

from paper_2605_11354_amd import binding as B
from paper_2605_11354_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

C0, C1, C2, C3, C4 = synth.CONFIGS

CASES = {
    "c0": (C0, -1, -1),
    "c0_tail150": (C0.with_(N=150), 1, 1),
    "c0_bq128_tail": (C0.with_(N=700, bq=128, proj_per_head=True), 2, 5),
    "c1_small": (C1.with_(H=2, N=2 * 1374), -1, -1),
    "c2_small": (C2.with_(H=2, N=3 * 1374), -1, -1),
    "c3_small": (C3.with_(B=3, H=2), -1, -1),
    "c4_small": (C4.with_(H=2, N=3 * 1374), -1, -1),
    "h3_per_head": (C0.with_(H=3, N=700, proj_per_head=True), 2, 5),
    "h3_per_head_bq128": (C0.with_(B=2, H=3, N=900, bq=128, proj_per_head=True), 3, 6),
    "c4_batch2": (C4.with_(B=2, H=2, N=1374), 2, 12),
    "c4_bq64_kc6": (C4.with_(H=2, N=1000, bq=64), 6, 5),          # E4M3, 64-row query blocks
    "c4_batch2_bq64": (C4.with_(B=2, H=3, N=900, bq=64), 5, 4),
    # 64-row query blocks with at most two critical blocks: the attention kernel for short lists
    "c4_bq64_kc2": (C4.with_(H=2, N=1000, bq=64), 2, 5),
    "c4_batch2_bq64_kc1": (C4.with_(B=2, H=3, N=650, bq=64, proj_per_head=True), 1, 3),
    "c0_batch2_kc1_tail": (C0.with_(B=2, H=3, N=330), 1, 2),
}


def _case(name, **kw):
    cfg, kc, kn = CASES[name]
    return G.Case(cfg, k_crit=kc, k_neg=kn, **kw)


def _f32_forward(case, labels_np):
    """The staged path up to the fp32 result: states -> aggregate -> sparse + linear + projection, fp32 store."""
    lab = torch.from_numpy(labels_np).cuda()
    Hq = case.aggregate(lab, case.states())
    c = case.cfg
    O32 = torch.full((c.B, c.H, c.N, 64), float("nan"), dtype=torch.float32, device="cuda")
    B.sla_sparse_combine_f32(case.p, case.Q, case.K, case.V, case.W, lab, Hq, O32, case.sQ, case.sK, case.sV, case.ws)
    O16 = case.sparse_combine(lab, Hq)
    torch.cuda.synchronize()
    return O32, O16


@pytest.mark.parametrize("name", ["c0", "c0_tail150", "c0_bq128_tail", "c1_small", "c2_small", "c3_small", "c4_small",
                                  "h3_per_head", "c4_bq64_kc6", "c4_bq64_kc2", "c4_batch2_bq64_kc1"])
def test_stated_tolerance_on_the_fp32_result(oracle, name):
    """max |O - oracle| <= tau * RMS(oracle), tau = 2e-2 (bf16 inputs) / 6e-2 (E4M3 inputs), asserted as stated on the
    kernel's fp32 result, and the bf16 output is that result rounded to nearest even, bit for bit: together they bound
    the kernel's arithmetic without the allowance for the output format that the bf16 comparisons take."""
    case = _case(name)
    refc = case.oracle_classify(oracle)
    ref = case.oracle_attend(oracle, refc["labels"])
    O32, O16 = _f32_forward(case, refc["labels"])
    assert torch.equal(O32.to(torch.bfloat16).view(torch.int16), O16.view(torch.int16)), "bf16 output is not RNE(fp32 result)"
    got = G.gather_blocks(O32.cpu().numpy().astype(np.float64), ref["sel"], case.cfg.bq, case.cfg.H)
    err = G.rel_err(got, ref["O"])
    print(f"[parity] {name}: fp32 result, max-abs/RMS = {err:.4e} (bar {G.TOL[case.cfg.dtype]:.0e})")
    assert err <= G.TOL[case.cfg.dtype]


@pytest.mark.timeout(600)
def test_stated_tolerance_on_the_fp32_result_full_size_c1(oracle):
    """Configuration 1 at its real shape, every element of the output."""
    case = G.Case(C1)
    refc = case.oracle_classify(oracle)
    ref = case.oracle_attend(oracle, refc["labels"])
    O32, O16 = _f32_forward(case, refc["labels"])
    assert torch.equal(O32.to(torch.bfloat16).view(torch.int16), O16.view(torch.int16))
    got = G.gather_blocks(O32.cpu().numpy().astype(np.float64), ref["sel"], C1.bq, C1.H)
    err = G.rel_err(got, ref["O"])
    print(f"[parity] c1 full size: fp32 result, max-abs/RMS = {err:.4e}")
    assert err <= G.TOL["bf16"]


@pytest.mark.parametrize("name", ["h3_per_head", "h3_per_head_bq128", "c4_batch2", "c4_bq64_kc6", "c4_batch2_bq64", "c4_bq64_kc2",
                                  "c4_batch2_bq64_kc1", "c0_batch2_kc1_tail"])
@pytest.mark.parametrize("phi", ["softmax", "elu1"])
def test_forward_more_shapes(oracle, name, phi):
    case = _case(name, phi=phi)
    c = case.cfg
    O, lab = case.forward()
    refc = case.oracle_classify(oracle)
    assert np.array_equal(lab.cpu().numpy(), refc["labels"])
    ref = case.oracle_attend(oracle, refc["labels"], want_parts=True)
    got = G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], c.bq, c.H)
    G.assert_output(got, ref["O"], c.dtype, f"{name} phi={phi}")
    # the sparse branch alone (Hq = NULL), and the token-major layout of the same problem
    Osp = case.sparse_combine(torch.from_numpy(refc["labels"]).cuda(), None)
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(Osp), ref["sel"], c.bq, c.H), ref["O_sparse"], c.dtype, f"{name} sparse branch")
    tm = lambda x: x.permute(0, 2, 1, 3).contiguous()
    pt = B.make_params(c.B, c.H, c.N, c.bq, c.bk, c.crit_frac, c.neg_frac, case.k_c, case.k_n, c.dtype, c.proj_per_head,
                       phi=phi, layout="bnhd")
    Ot = torch.zeros((c.B, c.N, c.H, 64), dtype=torch.bfloat16, device="cuda")
    B.sla_forward(pt, tm(case.Q), tm(case.K), tm(case.V), case.W, Ot, None, case.sQ, case.sK, case.sV, B.alloc_workspace(pt))
    torch.cuda.synchronize()
    assert torch.equal(tm(O).view(torch.int16), Ot.view(torch.int16))


def _requantise(cfg, d16):
    out = dict(d16)
    out["Q"], out["sQ"] = synth.quantise_e4m3_blocks(d16["Q"], cfg.bq)
    out["K"], out["sK"] = synth.quantise_e4m3_blocks(d16["K"], cfg.bk)
    out["V"], out["sV"] = synth.quantise_e4m3_blocks(d16["V"], cfg.bk)
    return out


@pytest.mark.parametrize("bq", [64, 128])
def test_e4m3_forward_with_all_zero_blocks(oracle, bq):
    """An all-zero K / V key block (its block scale is the quantiser's epsilon / 448: 29 binades below the others) and
    an all-zero Q block, attended as critical blocks by every row: the zero-V block must still take its share of the
    softmax mass (row sums formed apart from the scaled weights), and nothing may turn into inf or nan."""
    cfg = C4.with_(H=2, N=1000, bq=bq)
    d16 = dict(synth.make_inputs(cfg.with_(dtype="bf16")))
    for k in ("Q", "K", "V"):
        d16[k] = d16[k].copy()
    d16["K"][:, :, 2 * 64:3 * 64] = 0
    d16["V"][:, :, 2 * 64:3 * 64] = 0
    d16["V"][:, 1, 5 * 64:6 * 64] = 0                       # zero V under live keys: pure dilution of the row
    d16["Q"][:, :, bq:2 * bq] = 0
    d = _requantise(cfg, d16)
    assert d["sV"][0, 0, 2] < 1e-9 and d["sK"][0, 0, 2] < 1e-9
    case = G.Case(cfg, d, k_crit=6, k_neg=4)
    Nqb, Nkb = case.Nqb, case.Nkb
    lab = np.ones((1, 2, Nqb, Nkb), np.int8)
    lab[..., [0, 2, 5, 7, 9, Nkb - 1]] = 2                  # the zero blocks first and in mid-list, the ragged one last
    lab[..., [1, 3, 4, 6]] = 0
    O = torch.full((1, 2, cfg.N, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.sla_forward_with_labels(case.p, case.Q, case.K, case.V, case.W, torch.from_numpy(lab).cuda(), O, case.sQ, case.sK, case.sV, case.ws)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all()
    ref = case.oracle_attend(oracle, lab)
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], bq, 2), ref["O"], "fp8", f"zero blocks bq={bq}")
    lab2 = lab.copy()                                       # the zero block as the FIRST critical block of every row
    lab2[..., 0] = 1
    B.sla_forward_with_labels(case.p, case.Q, case.K, case.V, case.W, torch.from_numpy(lab2).cuda(), O, case.sQ, case.sK, case.sV, case.ws)
    torch.cuda.synchronize()
    ref = case.oracle_attend(oracle, lab2)
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], bq, 2), ref["O"], "fp8", f"zero block first bq={bq}")
    O2, lab_dev = case.forward()                            # and through the classifier
    refc = case.oracle_classify(oracle)
    assert np.array_equal(lab_dev.cpu().numpy(), refc["labels"])
    ref = case.oracle_attend(oracle, refc["labels"])
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O2), ref["sel"], bq, 2), ref["O"], "fp8", f"zero blocks, classified, bq={bq}")


@pytest.mark.parametrize("name", ["c0_bq128_tail", "h3_per_head", "c4_bq64_kc6", "c4_small", "c4_bq64_kc2", "c0_batch2_kc1_tail"])
def test_given_labels_with_short_critical_lists(oracle, name):
    """Labels whose rows hold fewer critical blocks than k_crit (their lists end in unfilled entries), none at all, or
    only the ragged last block."""
    case = _case(name)
    c = case.cfg
    rng = np.random.default_rng(5)
    lab = rng.integers(0, 2, size=(c.B, c.H, case.Nqb, case.Nkb)).astype(np.int8)          # marginal / negligible
    for idx in np.ndindex(c.B, c.H, case.Nqb):
        n = int(rng.integers(0, case.k_c + 1))
        if idx[2] == 0:
            n = 0
        lab[idx][rng.choice(case.Nkb, n, replace=False)] = 2
        if idx[2] == 1:
            lab[idx] = 1
            lab[idx][case.Nkb - 1] = 2
    O = torch.full((c.B, c.H, c.N, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.sla_forward_with_labels(case.p, case.Q, case.K, case.V, case.W, torch.from_numpy(lab).cuda(), O, case.sQ, case.sK, case.sV, case.ws)
    torch.cuda.synchronize()
    ref = case.oracle_attend(oracle, lab)
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], c.bq, c.H), ref["O"], c.dtype, f"{name} short lists")


@pytest.mark.parametrize("bq,dtype", [(64, "bf16"), (128, "bf16"), (128, "fp8"), (64, "fp8")])
def test_critical_lists_longer_than_a_window(oracle, bq, dtype):
    """More than 64 critical blocks per row: the list window of the attention kernel moves (every 32 tiles)."""
    cfg = (C4 if dtype == "fp8" else C1).with_(H=1, N=140 * 64 - 9, bq=bq)
    case = G.Case(cfg, k_crit=131, k_neg=3)
    O, lab = case.forward()
    refc = case.oracle_classify(oracle)
    assert np.array_equal(lab.cpu().numpy(), refc["labels"])
    sel = [(0, i) for i in (0, 1, case.Nqb // 2, case.Nqb - 1)]
    ref = case.oracle_attend(oracle, refc["labels"], sel)
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], bq, 1), ref["O"], dtype, f"131 critical blocks bq={bq} {dtype}")


@pytest.mark.parametrize("bq", [64, 128])
def test_v_blocks_of_very_different_magnitude(oracle, bq):
    """bf16 V whose key blocks differ by up to 2^32 in magnitude: the fp16 copy of V carries one power of two per
    block and the weights its exponent; blocks far below / above the row's first block take the careful step."""
    cfg = C0.with_(N=900, bq=bq, proj_per_head=True)
    d = dict(synth.make_inputs(cfg))
    f = lambda bits: (bits.astype(np.uint32) << 16).view(np.float32)
    v = f(d["V"]).copy()
    gains = {1: 2.0 ** -20, 3: 2.0 ** 12, 4: 2.0 ** -9, 6: 2.0 ** 9, 8: 0.0, 10: 2.0 ** -3}
    for j, gn in gains.items():
        v[:, :, j * 64:(j + 1) * 64] *= np.float32(gn)
    d["V"] = synth.to_bf16_bits(v)
    case = G.Case(cfg, d, k_crit=case_kc(cfg), k_neg=0)
    lab = np.full((1, 2, case.Nqb, case.Nkb), 2, np.int8)      # every block critical: dense attention over mixed scales
    for order in ("all", "small_first"):
        if order == "small_first":
            lab[..., 0] = 0                                     # the 2^-20 block opens the list
        O = torch.full((1, 2, cfg.N, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.sla_forward_with_labels(case.p, case.Q, case.K, case.V, case.W, torch.from_numpy(lab).cuda(), O, None, None, None, case.ws)
        torch.cuda.synchronize()
        assert torch.isfinite(O.float()).all()
        ref = case.oracle_attend(oracle, lab)
        G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], bq, 2), ref["O"], "bf16", f"mixed V scales bq={bq} {order}")


def case_kc(cfg):
    return -(-cfg.N // cfg.bk)


@pytest.mark.parametrize("bq", [64, 128])
@pytest.mark.parametrize("where", ["late", "middle", "staircase"])
def test_running_maximum_raised_in_mid_list(oracle, bq, where):
    """Keys of one block scaled so that their logits tower over everything seen before: the attention kernel's
    running maximum, set by the first block, has to be raised when the list reaches that block (staircase: every
    block from the fourth to the twelfth towers over the one before, so the maximum is raised again and again in the
    middle of the list, where the kernel runs its iterations without per-tile checks)."""
    cfg = C0.with_(N=1100, bq=bq)
    d = dict(synth.make_inputs(cfg))
    f = lambda bits: (bits.astype(np.uint32) << 16).view(np.float32)
    kk = f(d["K"]).copy()
    if where == "staircase":
        for j in range(3, 12):
            kk[:, :, j * 64 + (j % 3) * 16:(j + 1) * 64] *= np.float32(1.9 ** (j - 2))
    else:
        j = 14 if where == "late" else 7
        kk[:, :, j * 64:(j + 1) * 64] *= np.float32(24.0)
        kk[:, :, (j + 1) * 64:(j + 1) * 64 + 32] *= np.float32(6.0)
    d["K"] = synth.to_bf16_bits(kk)
    case = G.Case(cfg, d, k_crit=case_kc(cfg), k_neg=0)
    O, lab = case.forward()
    assert (lab == 2).all()
    ref = case.oracle_attend(oracle, lab.cpu().numpy())
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], bq, cfg.H), ref["O"], "bf16", f"raised maximum bq={bq} {where}")


@pytest.mark.timeout(900)
@pytest.mark.parametrize("idx", [2, 4])
def test_full_size_outputs_over_all_heads_and_the_value_hull(oracle, idx):
    """Configurations 2 and 4 at full size: 512 query blocks spread over all 16 heads (always with both ends of the
    first and the last head) against the oracle, and, on the whole tensor, the sparse branch alone stays inside the
    per-channel range of the head's V rows (a row of it is a convex combination of V rows)."""
    from bench import sample_blocks
    cfg = synth.CONFIGS[idx]
    case = G.Case(cfg)
    O, lab = case.forward()
    refc = case.oracle_classify(oracle)
    assert np.array_equal(lab.cpu().numpy(), refc["labels"])
    sel = sample_blocks(cfg.B * cfg.H, case.Nqb, 512, np.random.default_rng(3))
    assert {bh for bh, _ in sel} == set(range(cfg.B * cfg.H))
    ref = case.oracle_attend(oracle, refc["labels"], sel)
    G.assert_output(G.gather_blocks(G.bf16_tensor_to_f64(O), ref["sel"], cfg.bq, cfg.H), ref["O"], cfg.dtype,
                    f"{cfg.name} ({len(sel)} query blocks over all heads)")
    del O
    Osp = case.sparse_combine(lab, None).float()
    if case.fp8:
        Vf = case.V.view(torch.float8_e4m3fn).float() * case.sV.repeat_interleave(cfg.bk, dim=2)[:, :, :cfg.N, None]
    else:
        Vf = case.V.float()
    lo, hi = Vf.amin(dim=2, keepdim=True), Vf.amax(dim=2, keepdim=True)
    slack = 2.0 ** -7 * torch.maximum(lo.abs(), hi.abs())          # the bf16 store of a value at the edge
    assert bool(((Osp >= lo - slack) & (Osp <= hi + slack)).all())


def test_frame_then_global_attention_on_the_same_activations(oracle):
    """Section 3.3: SLA replaces both the frame attention and the global attention of the backbone.  The same
    token-major activations [S, 1374, H, 64] are consumed as B = S frames of 1374 tokens (frame attention) and then as
    B = 1 with S x 1374 tokens (global attention), back to back on one stream with one workspace; both results are
    checked against the oracle evaluated on the corresponding head-major views."""
    S, Nf, H = 3, 1374, 2
    cg = C1.with_(H=H, N=S * Nf)                                  # global view: [1, H, S*Nf, 64]
    cf = C3.with_(B=S, H=H, N=Nf)                                 # frame view:  [S, H, Nf, 64]
    d = synth.make_inputs(cg)
    tm = lambda a: np.ascontiguousarray(a.transpose(0, 2, 1, 3))  # head-major -> token-major
    Q, K, V = (G.dev_bf16(tm(d[k])) for k in ("Q", "K", "V"))     # [1, S*Nf, H, 64] == [S, Nf, H, 64] in memory
    W = G.dev_bf16(d["W"])
    pg = B.make_params(1, H, S * Nf, cg.bq, cg.bk, cg.crit_frac, cg.neg_frac, -1, -1, "bf16", True, layout="bnhd")
    pf = B.make_params(S, H, Nf, cf.bq, cf.bk, cf.crit_frac, cf.neg_frac, -1, -1, "bf16", True, layout="bnhd")
    ws = torch.empty(max(B.sla_workspace_bytes(pg), B.sla_workspace_bytes(pf)), dtype=torch.uint8, device="cuda")
    Of, Og = torch.empty_like(Q), torch.empty_like(Q)
    labf = torch.empty((S, H, -(-Nf // cf.bq), -(-Nf // cf.bk)), dtype=torch.int8, device="cuda")
    labg = torch.empty((1, H, -(-S * Nf // cg.bq), -(-S * Nf // cg.bk)), dtype=torch.int8, device="cuda")
    for _ in range(2):                                            # twice: the second pair runs on a used workspace
        B.sla_forward(pf, Q, K, V, W, Of, labf, None, None, None, ws)
        B.sla_forward(pg, Q, K, V, W, Og, labg, None, None, None, ws)
    torch.cuda.synchronize()
    # global view against the oracle
    kc, kn = B.sla_resolve_counts(pg)
    po = oracle.make_params(1, H, S * Nf, cg.bq, cg.bk, kc, kn, "bf16", True)
    r = oracle.forward(po, d["Q"], d["K"], d["V"], d["W"])
    assert np.array_equal(labg.cpu().numpy(), r["labels"])
    got = G.bf16_tensor_to_f64(Og).reshape(1, S * Nf, H, 64).transpose(0, 2, 1, 3)
    G.assert_output(got, r["O"], "bf16", "global attention on token-major activations")
    # frame view: frame s is tokens s*Nf .. (s+1)*Nf of every head
    fv = lambda a: np.ascontiguousarray(a[0].reshape(H, S, Nf, 64).transpose(1, 0, 2, 3))
    kc, kn = B.sla_resolve_counts(pf)
    po = oracle.make_params(S, H, Nf, cf.bq, cf.bk, kc, kn, "bf16", True)
    r = oracle.forward(po, fv(d["Q"]), fv(d["K"]), fv(d["V"]), d["W"])
    assert np.array_equal(labf.cpu().numpy(), r["labels"])
    got = G.bf16_tensor_to_f64(Of).reshape(S, Nf, H, 64).transpose(0, 2, 1, 3)
    G.assert_output(got, r["O"], "bf16", "frame attention on the same activations")


@pytest.mark.parametrize("dtype,heads", [("bf16", 32), ("bf16", 64), ("fp8", 64)])
def test_block_means_of_launches_with_many_blocks(oracle, dtype, heads):
    """pool_kernel gives a thread eight, four or two channels by the number of token blocks in the launch (16384 and 32768
    are the steps); the other tests stay below the first step.  Block means (Alg. 1 step 2, fp64 sums in token order) and
    labels against the oracle on cheap random inputs: random sign, exponent within fifteen binades, random mantissa."""
    N = 512 * 64 - 17
    rng = np.random.default_rng(11)
    cfg = synth.CONFIGS[0].with_(B=1, H=heads, N=N, bq=64, bk=64, dtype=dtype)
    shape = (1, heads, N, 64)
    if dtype == "bf16":
        def draw():
            r = rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
            return (r & np.uint16(0x807F)) | ((np.uint16(118) + ((r >> 7) & np.uint16(15))) << np.uint16(7))
        d = {"Q": draw(), "K": draw(), "sQ": None, "sK": None, "sV": None}
    else:
        def draw():
            r = rng.integers(0, 1 << 8, size=shape, dtype=np.uint8)
            return np.where((r & 0x7F) == 0x7F, r & 0xFE, r).astype(np.uint8)          # no NaN codes
        nb = -(-N // 64)
        d = {"Q": draw(), "K": draw(), "sQ": rng.uniform(0.01, 0.1, (1, heads, nb)).astype(np.float32),
             "sK": rng.uniform(0.01, 0.1, (1, heads, nb)).astype(np.float32)}
        d["sV"] = d["sK"]
    d["V"] = d["K"]
    d["W"] = synth.to_bf16_bits(np.eye(64, dtype=np.float32))
    case = G.Case(cfg, d, k_crit=20, k_neg=300)
    got = case.classify(want=("qbar", "kbar"))
    ref = case.oracle_classify(oracle, want_means=True)
    assert np.array_equal(got["qbar"], ref["qbar"]), "query block means differ"
    assert np.array_equal(got["kbar"], ref["kbar"]), "key block means differ"
    assert np.array_equal(got["labels"], ref["labels"]), "labels differ"
