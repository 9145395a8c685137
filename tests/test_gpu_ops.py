"""GPU parity one level below the stage: the operator entry points of the C ABI (the kernels the
stage and the encoder launch, one at a time) against the fp64 oracle of the same operation.

The GEMM cases force every tile configuration of the bf16 MFMA kernels on every operand layout the
stage uses (y = x W^T, dx = dy W, dW = dy^T x), at sizes that span several tiles and leave ragged
tails in both output dimensions, and the two split-K paths (fp32 output, storage-dtype output with
the epilogue applied by the reduction pass)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import ops

pytestmark = pytest.mark.gpu

TOL_BF16, TOL_F32OUT = 2e-2, 1e-4

# tile_cfg value -> contraction multiple it needs (0 = chosen from the shape; 1..6 register-staged
# tiles; 7..17 direct-to-LDS tiles, 12 being the 16x16-MFMA tile for y = x W^T only, 16 and 17 the 64-row tiles)
K_MULTIPLE = {0: 8, 1: 8, 2: 8, 3: 8, 4: 8, 5: 8, 6: 8, 7: 32, 8: 32, 9: 32, 10: 64, 11: 64, 12: 64, 13: 32, 14: 64, 15: 32, 16: 64, 17: 64}
LAYOUTS = {"nt": (0, 0), "nn": (0, 1), "tn": (1, 1)}


def _gemm_case(layout, M, N, K, tile_cfg, seed, bias=True, accumulate=False):
    import torch
    from paper_2405_01248_amd import binding as B
    from paper_2405_01248_amd.harness import _np_to_dev, _dev_to_np, rel_err
    a_k, b_k = LAYOUTS[layout]
    rng = np.random.default_rng(seed)
    A = si.round_bf16(rng.standard_normal((M, K)))           # A_eff [M, K]
    Bm = si.round_bf16(rng.standard_normal((K, N)) * 0.05)    # B_eff [K, N]
    bv = si.round_bf16(rng.standard_normal(N)) if bias else None
    f32 = layout == "tn"                                       # the weight-gradient product has an fp32 output
    dA = _np_to_dev(A.T if a_k else A, "bf16")
    dB = _np_to_dev(Bm if b_k else Bm.T, "bf16")
    dbias = _np_to_dev(bv, "bf16") if (bias and not f32) else None
    ref = ops.linear_fwd(A, Bm.T, bv if (bias and not f32) else None)
    if f32:
        C0 = rng.standard_normal((M, N)) if accumulate else np.zeros((M, N))
        C0 = C0.astype(np.float32).astype(np.float64)
        dC = torch.from_numpy(C0.astype(np.float32)).to("cuda:0")
        ref = ref + C0
    else:
        dC = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda:0")
    ws = torch.empty(max(B.op_gemm_workspace_bytes(M, N, K), 256), dtype=torch.uint8, device="cuda:0")
    B.op_gemm(B.DP_BF16, dA, dA.shape[1], a_k, dB, dB.shape[1], b_k, M, N, K, dbias, dC, N, f32, accumulate, ws, tile_cfg)
    torch.cuda.synchronize()
    return rel_err(_dev_to_np(dC), ref)


@pytest.mark.parametrize("layout", list(LAYOUTS))
def test_gemm_every_tile_configuration_ragged(layout):
    # 333 x 392 output: 2-3 tiles of 128 / 256 per side with ragged tails (tn needs M % 8 == 0: 328)
    M, N = (328 if layout == "tn" else 333), 392
    for tile_cfg, mult in K_MULTIPLE.items():
        if tile_cfg in (12, 16, 17) and layout != "nt":
            continue
        for K in (448, 200):
            if K % mult:
                continue
            e = _gemm_case(layout, M, N, K, tile_cfg, seed=tile_cfg * 7 + K)
            print(f"\n[gemm {layout} cfg {tile_cfg} {M}x{N}x{K}] rel err {e:.2e}", flush=True)
            assert e <= (TOL_F32OUT if layout == "tn" else TOL_BF16)


def test_gemm_unsupported_forced_configuration_is_an_error_not_a_launch():
    from paper_2405_01248_amd import binding as B
    for layout, tile_cfg, K in (("nt", 10, 96), ("nn", 12, 448), ("nt", 7, 200)):
        with pytest.raises(B.DpipeError) as ei:
            _gemm_case(layout, 136, 136, K, tile_cfg, seed=1)
        assert ei.value.code == -2


@pytest.mark.parametrize("M,N,K", [(77, 768, 3072), (308, 768, 768), (1232, 768, 3072), (77, 2304, 768), (40, 2304, 1152)])
def test_gemm_split_k_with_epilogue_in_the_reduction(M, N, K):
    # few tiles and a long contraction: the storage-dtype GEMM is split along K (encoder projections
    # on a partial batch, the adaLN modulation GEMM); bias is applied by the reduction pass
    e = _gemm_case("nt", M, N, K, 0, seed=M)
    print(f"\n[gemm nt split-K {M}x{N}x{K}] rel err {e:.2e}", flush=True)
    assert e <= TOL_BF16


@pytest.mark.parametrize("M,N,K,acc", [(640, 640, 8192, False), (1152, 4608, 2048, True), (320, 328, 4104, True)])
def test_gemm_weight_gradient_split_k(M, N, K, acc):
    e = _gemm_case("tn", M, N, K, 0, seed=N, accumulate=acc)
    print(f"\n[gemm tn split-K {M}x{N}x{K} acc={acc}] rel err {e:.2e}", flush=True)
    assert e <= TOL_F32OUT


ATTN_CASES = [
    # B, H, Nq, Nk, dh, causal, gain, row_shift
    (2, 3, 200, 200, 64, False, 1.0, 0.0),      # self-attention, ragged query and key tiles
    (2, 3, 200, 77, 64, False, 1.0, 0.0),       # cross-attention to the 77-token context
    (2, 2, 256, 256, 72, False, 1.0, 0.0),      # DiT head width (not a multiple of the MFMA depth)
    (1, 2, 130, 130, 32, False, 1.0, 0.0),
    (2, 1, 70, 200, 40, False, 1.0, 0.0),        # head widths that leave part of a tile row empty
    (1, 2, 150, 90, 96, False, 1.0, 0.0),
    (1, 3, 90, 150, 88, True, 1.0, 0.0),
    (3, 4, 77, 77, 64, True, 1.0, 0.0),         # text encoder: causal, forward only
    (2, 2, 200, 200, 64, True, 1.0, 0.0),       # causal over several key tiles: the diagonal mask meets full tiles
    # sharp softmax: logits spread over tens of log2 units, a per-row shift of up to +-80, row maxima
    # arriving in late key tiles -- the running reference of the online softmax has to move after the
    # first tile (gain 16: at almost every tile; gain 4: at some tiles and not at others)
    (2, 3, 200, 200, 64, False, 16.0, 80.0),
    (2, 3, 200, 200, 64, False, 4.0, 80.0),
    (2, 3, 200, 77, 64, False, 16.0, 80.0),
    (2, 2, 256, 256, 72, False, 16.0, 80.0),
    (2, 2, 256, 256, 72, False, 4.0, 30.0),
    (3, 4, 77, 77, 64, True, 16.0, 80.0),
    (2, 2, 200, 200, 64, True, 8.0, 80.0),      # the causal edge mask and the moving reference together
]


def _attn_id(c):
    return "B{}H{}q{}k{}d{}{}{}".format(*c[:5], "c" if c[5] else "", f"_gain{c[6]:g}_shift{c[7]:g}" if c[6] != 1.0 else "")


@pytest.mark.parametrize("case", ATTN_CASES, ids=_attn_id)
def test_attention_forward_and_backward(case):
    import torch
    from paper_2405_01248_amd import binding as B
    from paper_2405_01248_amd.harness import _np_to_dev, _dev_to_np, rel_err, rel_l2
    from softmax_schedule import head_logits, rescale_stats
    Bt, H, Nq, Nk, dh, causal, gain, row_shift = case
    d = H * dh
    q, k, v, do = si.make_attention_inputs(Bt, H, Nq, Nk, dh, seed=Nq * 31 + Nk, gain=gain, row_shift=row_shift)
    s = head_logits(q, k, H, causal)
    if gain != 1.0:
        # the stress must really be a stress: replay the kernel's rule for moving the softmax reference on
        # the oracle's logits and require that it fires after the first key tile, on peaked rows
        st = rescale_stats(s)
        print(f"\n[attention stress {_attn_id(case)}] {st}", flush=True)
        assert st["moves_late"] > 0 and st["max_rise_log2"] > 8.0 and st["mean_max_prob"] > 0.5, st
        if gain <= 4.0:
            assert st["moves_late"] < st["steps_late"], st          # ... and also does not fire at some tiles
    dq_, dk_, dv_, ddo = (_np_to_dev(t, "bf16") for t in (q, k, v, do))
    o = torch.zeros((Bt, Nq, d), dtype=torch.bfloat16, device="cuda:0")
    lse = torch.zeros((Bt, H, Nq), dtype=torch.float32, device="cuda:0")
    scale = 1.0 / np.sqrt(dh)
    B.op_attention_fwd(B.DP_BF16, Bt, H, Nq, Nk, dh, causal, scale, dq_, d, dk_, d, dv_, d, o, d, lse)
    torch.cuda.synchronize()
    ref_o = ops.attention_fwd(q, k, v, H, causal)
    e = rel_err(_dev_to_np(o), ref_o)
    print(f"\n[attention fwd {_attn_id(case)}] rel err {e:.2e}, rel L2 {rel_l2(_dev_to_np(o), ref_o):.2e}", flush=True)
    assert e <= TOL_BF16
    # the log-sum-exp the backward re-derives the probabilities from
    m = s.max(axis=-1)
    ref_lse = m + np.log(np.exp(s - m[..., None]).sum(axis=-1))
    e_lse = float(np.max(np.abs(_dev_to_np(lse) - ref_lse)))
    assert e_lse <= 1e-3 * max(1.0, float(np.max(np.abs(ref_lse)))), e_lse
    if causal:
        return                      # the frozen encoder has no backward
    gq, gk, gv = (torch.zeros_like(t) for t in (dq_, dk_, dv_))
    delta = torch.zeros((Bt, H, Nq), dtype=torch.float32, device="cuda:0")
    B.op_attention_bwd(B.DP_BF16, Bt, H, Nq, Nk, dh, scale, dq_, d, dk_, d, dv_, d, o, d, lse, ddo, d, delta, gq, d, gk, d, gv, d)
    torch.cuda.synchronize()
    rq, rk, rv = ops.attention_bwd(do, q, k, v, H, False)
    errs = {"dq": rel_err(_dev_to_np(gq), rq), "dk": rel_err(_dev_to_np(gk), rk), "dv": rel_err(_dev_to_np(gv), rv)}
    print(f"[attention bwd {_attn_id(case)}] {errs}", flush=True)
    assert max(errs.values()) <= TOL_BF16, errs


# ------------------------------------------------------------------ FP8 (OCP E4M3) projection GEMM
def test_fp8_quantisation_is_bit_exact():
    """The 8-bit codes are integers decided by floating point: both sides take the decision in fp32 (bf16 input times
    the fp32 reciprocal of the scale), so the codes must agree bit for bit -- normal and subnormal range, ties,
    saturation, both signs."""
    import torch
    from oracle import fp8
    from paper_2405_01248_amd import binding as B
    from paper_2405_01248_amd.harness import _np_to_dev
    rng = np.random.default_rng(0)
    rows, cols = 67, 136
    x = rng.standard_normal((rows, cols)) * np.exp(rng.uniform(-9, 7, size=(rows, cols)))       # 2^-13 .. 2^10 in magnitude
    table = fp8.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    mids = 0.5 * (table[1:] + table[:-1])
    x[0, :len(mids)] = mids                       # exact ties (the midpoints are bf16-representable: 5 significant bits)
    x[1, :len(mids)] = -mids
    x = si.round_bf16(x)
    for scale in (1.0, 0.3, 7.25):
        dx = _np_to_dev(x, "bf16")
        q = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda:0")
        B.op_quantize_fp8(dx, cols, q, cols, rows, cols, scale)
        torch.cuda.synchronize()
        _, want = fp8.quantize(x, scale)
        got = q.cpu().numpy()
        bad = np.argwhere(got != want)
        assert bad.size == 0, (scale, bad[:5], got[tuple(bad[0])], want[tuple(bad[0])], x[tuple(bad[0])])


@pytest.mark.parametrize("M,N,K", [(333, 392, 384), (77, 768, 3072), (1300, 136, 128), (2048, 1152, 1152)])
def test_fp8_gemm_matches_oracle(M, N, K):
    import torch
    from oracle import fp8
    from paper_2405_01248_amd import binding as B
    from paper_2405_01248_amd.harness import _np_to_dev, _dev_to_np, rel_err
    rng = np.random.default_rng(M + K)
    x = si.round_bf16(rng.standard_normal((M, K)))
    w = si.round_bf16(rng.standard_normal((N, K)) * 0.05)
    bias = si.round_bf16(rng.standard_normal(N))
    sx, sw = float(np.abs(x).max()) / 448.0, float(np.abs(w).max()) / 448.0          # per-tensor scales: the largest value maps to 448
    qx = torch.zeros((M, K), dtype=torch.uint8, device="cuda:0")
    qw = torch.zeros((N, K), dtype=torch.uint8, device="cuda:0")
    B.op_quantize_fp8(_np_to_dev(x, "bf16"), K, qx, K, M, K, sx)
    B.op_quantize_fp8(_np_to_dev(w, "bf16"), K, qw, K, N, K, sw)
    out = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda:0")
    out_scale = float(np.float32(sx) * np.float32(sw))
    B.op_gemm_fp8(qx, K, qw, K, M, N, K, out_scale, _np_to_dev(bias, "bf16"), out, N)
    torch.cuda.synchronize()
    (ax, cx), (aw, cw) = fp8.quantize(x, sx), fp8.quantize(w, sw)
    assert np.array_equal(qx.cpu().numpy(), cx) and np.array_equal(qw.cpu().numpy(), cw)
    ref = fp8.gemm(ax, aw, out_scale, bias)
    e = rel_err(_dev_to_np(out), ref)
    # what the 8-bit operands cost against the unquantised product (reported, not a bar: it is the format's error)
    e_fmt = rel_err(ref, x @ w.T + bias)
    print(f"\n[gemm fp8 {M}x{N}x{K}] rel err vs fp8 oracle {e:.2e}; quantisation error of the product itself {e_fmt:.2e}", flush=True)
    assert e <= TOL_BF16


def test_fp8_unsupported_shapes_are_errors():
    import torch
    from paper_2405_01248_amd import binding as B
    a = torch.zeros((64, 192), dtype=torch.uint8, device="cuda:0")
    o = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(B.DpipeError) as ei:
        B.op_gemm_fp8(a, 192, a, 192, 64, 64, 192, 1.0, None, o, 64)         # K not a multiple of 128
    assert ei.value.code == -2
    with pytest.raises(B.DpipeError) as ei:
        B.op_gemm_fp8(a, 192, a, 192, 64, 64, 128, 0.0, None, o, 64)
    assert ei.value.code == -1
