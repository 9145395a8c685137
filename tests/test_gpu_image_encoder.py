"""GPU parity of the frozen image encoder (3x3 convolutions as implicit GEMMs, GroupNorm, residual and
attention blocks; partial batches and layer ranges, Sec. 5) against the fp64 oracle, through the C ABI.
Metric per tensor: max|gpu - oracle| / max|oracle| <= 2e-2 (bf16 storage)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import image_encoder as ie

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _oracle(cfg, inp, lb=0, le=None, x=None):
    L = cfg.layer_dicts()
    return ie.encoder_fwd_partial(inp["params"], L, inp["x"] if x is None else x, lb, len(L) if le is None else le, 0, cfg.global_batch,
                                  cfg.groups, cfg.gn_eps)


def _one_layer(kind, ci, co, stride, hw, batch=2, groups=4):
    return si.ImageEncoderConfig(f"one_{kind}_{ci}_{co}_s{stride}_{hw[0]}x{hw[1]}", "bf16", hw[0], hw[1], ci, groups, ((kind, ci, co, stride),), batch)


SINGLE_LAYERS = [
    _one_layer("conv", 8, 128, 1, (20, 17), batch=3),       # the input convolution: 8 padded channels, K = 72 (ragged k-tile), ragged pixel tiles
    _one_layer("conv", 64, 64, 1, (9, 13)),                  # k-tiles inside one tap; narrow output tile
    _one_layer("conv", 64, 136, 2, (11, 14)),                # stride 2 on odd and even sizes; ragged output-channel tile
    _one_layer("conv", 24, 8, 1, (5, 5)),                    # taps not aligned with k-tiles; the 8-channel output head width
    _one_layer("conv", 128, 128, 2, (34, 33), batch=1),
    _one_layer("conv", 16, 16, 1, (1, 1)),                   # a single pixel: only the centre tap is inside
    # large enough for the direct-to-LDS kernel (C_in a multiple of 64, at least 1024 output pixels per sample): padding taps
    # answered by out-of-range copies, ragged pixel and channel tiles, stride 2, a half-empty channel tile
    _one_layer("conv", 64, 128, 1, (48, 50)),
    _one_layer("conv", 64, 192, 2, (65, 70)),
    _one_layer("conv", 128, 64, 1, (33, 32)),
    _one_layer("conv", 192, 72, 1, (47, 45), batch=1),
    _one_layer("resnet", 64, 128, 1, (40, 40)),
    _one_layer("resnet", 32, 32, 1, (12, 10)),
    _one_layer("resnet", 32, 72, 1, (7, 9), groups=8),       # with the 1x1 skip convolution
    _one_layer("attn", 64, 64, 1, (8, 9), batch=3),          # 72 pixels: ragged tiles of the score and value products
    _one_layer("norm_conv", 64, 8, 1, (10, 6)),
    # pixel counts per sample that are multiples of 256 on the direct-to-LDS convolution: its epilogue also produces the
    # statistics pass of the GroupNorm that follows (inside the residual block: the second norm reads them)
    _one_layer("resnet", 64, 128, 1, (32, 48)),              # 64-deep k-tiles; with the 1x1 skip convolution
    _one_layer("resnet", 128, 128, 1, (32, 32), batch=2, groups=32),   # 32-deep k-tiles, two workgroups per CU
    _one_layer("resnet", 64, 192, 1, (32, 32), batch=3, groups=8),     # a half-empty output-channel tile; odd sample count
    _one_layer("resnet", 256, 256, 1, (32, 32), batch=2, groups=32),   # 256 output channels: the 256-wide tile, two samples in one tile row
    _one_layer("resnet", 256, 512, 1, (32, 40), batch=1, groups=32),   # ... two tiles across, ragged pixel count, 1x1 skip
]

# The statistics handed from one layer to the next: a stride-2 convolution (the norm of the residual block that follows
# reads the sums its epilogue wrote, at the halved resolution), then a block whose last convolution feeds the output head's norm.
CHAIN = si.ImageEncoderConfig("chain_conv_resnet_head", "bf16", 64, 64, 64, 8,
                              (("conv", 64, 64, 2), ("resnet", 64, 128, 1), ("norm_conv", 128, 8, 1)), 3)


@pytest.mark.parametrize("cfg", SINGLE_LAYERS, ids=lambda c: c.name)
def test_single_layers_match_oracle(cfg):
    import torch
    from paper_2405_01248_amd.harness import DeviceImageEncoder, rel_err, rel_l2
    inp = si.make_image_encoder_inputs(cfg, seed=len(cfg.name), randomize_norm=True, weight_std=0.0)
    de = DeviceImageEncoder(cfg, inp)
    de.run_slices(cfg.global_batch)
    torch.cuda.synchronize()
    got, ref = de.output(), _oracle(cfg, inp)
    assert got.shape == ref.shape
    e = rel_err(got, ref)
    print(f"\n[{cfg.name}] rel err {e:.2e}, rel L2 {rel_l2(got, ref):.2e}", flush=True)
    assert np.isfinite(got).all() and e <= TOL


def test_statistics_pass_from_layer_to_layer():
    import torch
    from paper_2405_01248_amd.harness import DeviceImageEncoder, rel_err, rel_l2
    inp = si.make_image_encoder_inputs(CHAIN, seed=11, randomize_norm=True, weight_std=0.0)
    de = DeviceImageEncoder(CHAIN, inp)
    de.run_slices(CHAIN.global_batch)
    torch.cuda.synchronize()
    whole = de.output()
    ref = _oracle(CHAIN, inp)
    e = rel_err(whole, ref)
    print(f"\n[{CHAIN.name}] rel err {e:.2e}, rel L2 {rel_l2(whole, ref):.2e}", flush=True)
    assert np.isfinite(whole).all() and e <= TOL
    # one sample at a time gives the same bits: the sums are taken per sample and per tile, in a fixed order
    de.run_slices(1)
    torch.cuda.synchronize()
    assert np.array_equal(de.output(), whole)


def test_both_convolution_tile_shapes_give_the_same_bits():
    """With 256 output channels the convolution takes 256 x 256 tiles when they load the CUs at least as well as 256 x 128
    ones, which depends on how many samples a call covers: 16 samples of 64 x 64 pixels make 256 wide tiles (taken), 4 make
    64 and 1 makes 16 (not taken).  Both shapes accumulate in the same order and form the GroupNorm sums per 64-row band,
    so every slicing of the batch has to give the same bits (the second norm of the block reads the sums)."""
    import torch
    from paper_2405_01248_amd.harness import DeviceImageEncoder
    cfg = si.ImageEncoderConfig("wide_and_narrow_tiles", "bf16", 64, 64, 256, 32, (("resnet", 256, 256, 1), ("resnet", 256, 512, 1)), 16)
    inp = si.make_image_encoder_inputs(cfg, seed=5, randomize_norm=True, weight_std=0.0)
    de = DeviceImageEncoder(cfg, inp)
    de.run_slices(16)
    torch.cuda.synchronize()
    whole = de.output()
    assert np.isfinite(whole).all() and float(np.abs(whole).max()) > 0.0
    for b in (4, 1):
        de.out.zero_()
        de.run_slices(b)
        torch.cuda.synchronize()
        assert np.array_equal(de.output(), whole), b


SMALL = si.ImageEncoderConfig("small_img_enc_bf16", "bf16", 24, 16, 8, 4, si.vae_encoder_layers(16, (1, 2, 2), 8, 8), 5)


def test_encoder_partial_batches_and_layer_ranges():
    """Sec. 5: layers run on part of the batch, the rest in a later call; layer ranges continue from the
    previous call's output buffer; disjoint sample ranges in any order."""
    import torch
    from paper_2405_01248_amd.harness import DeviceImageEncoder, _dev_to_np, rel_err
    cfg = SMALL
    inp = si.make_image_encoder_inputs(cfg, seed=1, randomize_norm=True, weight_std=0.0)
    ref = _oracle(cfg, inp)
    de = DeviceImageEncoder(cfg, inp)
    outs = {}
    for b in (cfg.global_batch, 1, 2):               # 2 leaves a ragged last slice
        de.out.zero_()
        de.run_slices(b)
        torch.cuda.synchronize()
        outs[b] = de.output()
        e = rel_err(outs[b], ref)
        print(f"\n[{cfg.name}] slice {b}: rel err {e:.2e}", flush=True)
        assert e <= TOL
    # every kernel treats samples independently and none splits a sum by the number of rows: slices
    # reproduce the full batch bit for bit (the batch invariance Sec. 5 relies on when it concatenates outputs)
    for b in (1, 2):
        assert np.array_equal(outs[b], outs[cfg.global_batch]), b
    # layer ranges through an intermediate global-batch buffer, sample ranges out of order
    mid_l = 5
    mid = de.buffer(mid_l)
    for off, n in ((3, 2), (0, 3)):
        de.enc.fwd_partial(de.params, de.x, mid, cfg.global_batch, 0, mid_l, off, n, de.ws)
    torch.cuda.synchronize()
    e_mid = rel_err(_dev_to_np(mid), _oracle(cfg, inp, 0, mid_l))
    assert e_mid <= TOL, e_mid
    de.out.zero_()
    for off, n in ((1, 4), (0, 1)):
        de.enc.fwd_partial(de.params, mid, de.out, cfg.global_batch, mid_l, len(cfg.layers), off, n, de.ws)
    torch.cuda.synchronize()
    assert np.array_equal(de.output(), outs[cfg.global_batch])     # the state between calls is the layer's own bf16 output
    # untouched rows stay untouched; an empty slice is valid
    de.out.fill_(7.0)
    de.enc.fwd_partial(de.params, de.x, de.out, cfg.global_batch, 0, len(cfg.layers), 2, 1, de.ws)
    de.enc.fwd_partial(de.params, de.x, de.out, cfg.global_batch, 0, len(cfg.layers), 4, 0, de.ws)
    torch.cuda.synchronize()
    o = de.output()
    assert np.all(o[[0, 1, 3, 4]] == 7.0) and np.array_equal(o[2], outs[cfg.global_batch][2])
    # run-to-run identical
    de.run_slices(2); torch.cuda.synchronize()
    assert np.array_equal(de.output(), outs[2])


def test_image_encoder_cost_profile_rows():
    import torch
    from paper_2405_01248_amd.harness import DeviceImageEncoder
    cfg = SMALL
    de = DeviceImageEncoder(cfg, si.make_image_encoder_inputs(cfg, seed=2, weight_std=0.0))
    batches = [1, 4]
    rows = de.enc.profile(de.params, de.x, de.out, de.gb, batches, de.ws, reps=2)
    torch.cuda.synchronize()
    nl = len(cfg.layers)
    assert len(rows) == nl * len(batches)
    for j, b in enumerate(batches):
        for l in range(nl):
            r = rows[j * nl + l]
            h, w, c = cfg.out_shape(l + 1)
            assert (r["component"], r["layer"], r["batch"]) == (2, l, b)
            assert 0.0 < r["fwd_ms"] < 1e3 and r["bwd_ms"] == 0.0 and r["grad_bytes"] == 0 and r["cb_bytes"] == 0
            assert r["out_bytes"] == b * h * w * c * 2 == r["cf_bytes"]


def test_bad_calls_are_rejected_before_any_launch():
    import torch
    from paper_2405_01248_amd import binding as B
    from paper_2405_01248_amd.harness import DeviceImageEncoder
    cfg = SMALL
    de = DeviceImageEncoder(cfg, si.make_image_encoder_inputs(cfg, seed=3, weight_std=0.0))
    nl = len(cfg.layers)
    de.out.fill_(5.0)
    small_ws = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    for args, code in (((de.x, de.out, cfg.global_batch, 0, nl, 4, 2, de.ws), -1),            # samples beyond the batch
                       ((de.x, de.out, cfg.global_batch, 3, 3, 0, 1, de.ws), -1),             # empty layer range
                       ((de.x, de.out, cfg.global_batch, 0, nl + 1, 0, 1, de.ws), -1),
                       ((de.x, de.x, cfg.global_batch, 0, nl, 0, 1, de.ws), -1),              # in place
                       ((de.x, de.out, cfg.global_batch, 0, nl, 0, 1, small_ws), -3)):
        with pytest.raises(B.DpipeError) as ei:
            de.enc.fwd_partial(de.params, *args)
        assert ei.value.code == code
    torch.cuda.synchronize()
    assert float(de.out.min()) == 5.0 and float(de.out.max()) == 5.0


def test_full_size_encoder_first_sample_against_oracle():
    """The 16-layer encoder at the 512 x 512 training resolution (Sec. "Evaluation"): a global batch of 2 run
    as two partial-batch calls; the oracle computes sample 0 (a 512 x 512 sample takes it about half a
    minute), sample 1 is checked for independence of the slicing."""
    import torch
    from paper_2405_01248_amd.harness import DeviceImageEncoder, rel_err, rel_l2
    cfg = si.CONFIG6.replace(global_batch=2)
    inp = si.make_image_encoder_inputs(cfg, seed=0, weight_std=0.0)
    de = DeviceImageEncoder(cfg, inp)
    de.run_slices(1)
    torch.cuda.synchronize()
    sliced = de.output()
    de.out.zero_()
    de.run_slices(2)
    torch.cuda.synchronize()
    full = de.output()
    del de
    one = cfg.replace(global_batch=1)
    ref0 = ie.encoder_fwd(inp["params"], one.layer_dicts(), inp["x"][:1], one.groups, one.gn_eps)
    e = rel_err(full[:1], ref0)
    print(f"\n[{cfg.name}] sample 0: rel err {e:.2e}, rel L2 {rel_l2(full[:1], ref0):.2e}; "
          f"slices of 1 vs one call of 2: max {rel_err(sliced, full):.2e}", flush=True)
    assert e <= TOL
    assert np.array_equal(sliced, full)
