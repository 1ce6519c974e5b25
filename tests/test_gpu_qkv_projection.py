"""The qkv projection with the E4M3 block quantiser in the GEMM's epilogue (Alg. 2 with the attention's input format of
App. B.2), on the device: against the unfused device path bit for bit, against the oracle's layer followed by the
oracle's quantiser, and as the producer of an E4M3 forward's inputs."""
import numpy as np
import pytest
import torch

from paper_2605_11354_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _inputs(B_, N, H, d_in, seed, with_bias=True):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((B_ * N, d_in)) * np.exp(rng.uniform(-2, 2, (B_ * N, 1)))).astype(np.float32)
    W = (rng.standard_normal((3 * H * 64, d_in)) / np.sqrt(d_in)).astype(np.float32)
    b = rng.standard_normal(3 * H * 64).astype(np.float32)
    return synth.to_bf16_bits(x), synth.to_bf16_bits(W), (synth.to_bf16_bits(b) if with_bias else None)


def _fused(B_, N, H, bq, xb, Wb, bb):
    from paper_2605_11354_amd import binding as B
    codes = [torch.full((B_, N, H, 64), 0xAA, dtype=torch.uint8, device="cuda") for _ in range(3)]
    scales = [torch.full((B_, H, -(-N // blk)), -1.0, dtype=torch.float32, device="cuda") for blk in (bq, 64, 64)]
    B.sla_fp8_linear_qkv(G.dev_bf16(xb), G.dev_bf16(Wb), G.dev_bf16(bb) if bb is not None else None, B_, N, H, bq,
                         codes[0], codes[1], codes[2], scales[0], scales[1], scales[2])
    torch.cuda.synchronize()
    return codes, scales


# (B, N, H, d_in, bq): ragged last blocks, one head more than a 128-channel tile holds evenly (H = 3: a tile spans the
# last head of q and the first of k), B > 1 on whole tiles, a problem large enough for the 256-token tiles, one token
CASES = [(1, 300, 2, 256, 64), (1, 333, 3, 128, 128), (2, 256, 2, 384, 128), (1, 1374, 16, 1024, 128),
         (1, 8000, 16, 128, 128), (2, 512, 3, 128, 64), (1, 1, 1, 128, 64), (1, 65, 1, 128, 128),
         (1, 11000, 16, 256, 128), (1, 11100, 16, 384, 64), (43, 256, 16, 128, 128)]     # the last three take the 256 x 256 tiles


@pytest.mark.parametrize("B_,N,H,d_in,bq", CASES)
def test_fused_epilogue_equals_layer_then_quantiser(B_, N, H, d_in, bq):
    """Same bits as sla_fp8_linear followed by sla_quantise_e4m3 on the q, k and v slices of its output."""
    from paper_2605_11354_amd import binding as B
    xb, Wb, bb = _inputs(B_, N, H, d_in, 41 + N)
    codes, scales = _fused(B_, N, H, bq, xb, Wb, bb)
    y = torch.empty((B_ * N, 3 * H * 64), dtype=torch.bfloat16, device="cuda")
    B.sla_fp8_linear(G.dev_bf16(xb), G.dev_bf16(Wb), G.dev_bf16(bb), y)
    y = y.view(B_, N, 3, H, 64)
    for w, blk in enumerate((bq, 64, 64)):
        part = y[:, :, w].contiguous()
        c = torch.empty((B_, N, H, 64), dtype=torch.uint8, device="cuda")
        s = torch.empty((B_, H, -(-N // blk)), dtype=torch.float32, device="cuda")
        B.sla_quantise_e4m3(part, blk, c, s, layout="bnhd")
        torch.cuda.synchronize()
        assert torch.equal(s, scales[w]), ("scales", w)
        assert torch.equal(c, codes[w]), ("codes", w, (c != codes[w]).nonzero()[:4])


@pytest.mark.parametrize("B_,N,H,d_in,bq", [(1, 300, 2, 256, 64), (1, 333, 3, 128, 128), (2, 256, 2, 384, 128)])
def test_fused_epilogue_against_the_oracle(oracle, B_, N, H, d_in, bq):
    """Against the oracle's FP8 layer (Alg. 2) followed by the oracle's block quantiser (App. B.2).  The layer's result
    agrees with the oracle's up to fp32 accumulation order before the bf16 store, so a few elements may land on the
    neighbouring bf16 value and, from there, on a neighbouring code; what is asserted: every scale within one bf16 step
    (2^-8 relative), and the dequantised tensors within half an E4M3 step of the block (scale * 2^5 at the top binade)
    plus one bf16 step of the value."""
    xb, Wb, bb = _inputs(B_, N, H, d_in, 43)
    codes, scales = _fused(B_, N, H, bq, xb, Wb, bb)
    y = oracle.fp8_linear(xb, Wb, bb)                                   # fp64, [B*N, 3*H*64], before the bf16 store
    ybits = synth.to_bf16_bits(y.astype(np.float32)).reshape(B_, N, 3, H, 64)
    for w, blk in enumerate((bq, 64, 64)):
        part = np.ascontiguousarray(ybits[:, :, w].transpose(0, 2, 1, 3))   # [B,H,N,64]
        rc, rs = oracle.quantise_e4m3_blocks(part, blk)
        gs = scales[w].cpu().numpy()
        assert np.all(np.abs(gs - rs) <= rs * 2.0 ** -7), ("scales", w)
        gc = codes[w].permute(0, 2, 1, 3).contiguous().cpu().numpy()
        same = float(np.mean(gc == rc))
        deq = lambda c, s: synth.e4m3_code_values()[c].astype(np.float64) * np.repeat(s, blk, axis=2)[:, :, :N, None]
        got, ref = deq(gc, gs), deq(rc, rs)
        step = np.repeat(rs, blk, axis=2)[:, :, :N, None] * 32.0
        val = synth.bf16_bits_to_f32(part).astype(np.float64)
        assert np.all(np.abs(got - ref) <= step + np.abs(val) * 2.0 ** -7), ("values", w)
        print(f"tensor {w}: {same:.4%} of the codes identical to the oracle's")
        assert same >= 0.98


def test_forward_on_the_fused_projection_output():
    """The E4M3 forward run on what the fused projection wrote equals the forward run on the unfused path's tensors."""
    from paper_2605_11354_amd import binding as B
    B_, N, H, d_in, bq = 1, 1374, 4, 256, 128
    xb, Wb, bb = _inputs(B_, N, H, d_in, 47)
    codes, scales = _fused(B_, N, H, bq, xb, Wb, bb)
    y = torch.empty((B_ * N, 3 * H * 64), dtype=torch.bfloat16, device="cuda")
    B.sla_fp8_linear(G.dev_bf16(xb), G.dev_bf16(Wb), G.dev_bf16(bb), y)
    y = y.view(B_, N, 3, H, 64)
    ref_c, ref_s = [], []
    for w, blk in enumerate((bq, 64, 64)):
        c = torch.empty((B_, N, H, 64), dtype=torch.uint8, device="cuda")
        s = torch.empty((B_, H, -(-N // blk)), dtype=torch.float32, device="cuda")
        B.sla_quantise_e4m3(y[:, :, w].contiguous(), blk, c, s, layout="bnhd")
        ref_c.append(c); ref_s.append(s)
    Nkb = -(-N // 64)
    p = B.make_params(B_, H, N, bq, 64, 0.05, 0.10, max(1, round(0.05 * Nkb)), round(0.10 * Nkb), "fp8_e4m3", False, layout="bnhd")
    Wp = (torch.randn((1, 64, 64), device="cuda") * 0.05).to(torch.bfloat16)
    outs = []
    for cs, ss in ((codes, scales), (ref_c, ref_s)):
        O = torch.zeros((B_, N, H, 64), dtype=torch.bfloat16, device="cuda")
        lab = torch.zeros((B_, H, -(-N // bq), Nkb), dtype=torch.int8, device="cuda")
        B.sla_forward(p, cs[0], cs[1], cs[2], Wp, O, lab, ss[0], ss[1], ss[2])
        torch.cuda.synchronize()
        outs.append((O, lab))
    assert torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][0].view(torch.int16), outs[1][0].view(torch.int16))
    assert torch.isfinite(outs[0][0].float()).all()


def test_unsupported_shapes_are_refused():
    from paper_2605_11354_amd import binding as B
    xb, Wb, bb = _inputs(2, 300, 2, 128, 49)
    with pytest.raises(B.SlaError) as e:
        _fused(2, 300, 2, 64, xb, Wb, bb)                               # B > 1 and N not a multiple of the token tile
    assert e.value.status == B.SLA_ERR_UNSUPPORTED
