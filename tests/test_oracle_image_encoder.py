"""Pins of the image-encoder oracle (oracle/image_encoder.py) to what the mathematics fixes: brute
force from the scalar definition, impulse responses, constant inputs, hand-worked group statistics,
closed forms of degenerate blocks, and torch CPU fp64 as a second opinion.  The paper prints no worked
example of these layers (it treats them as black boxes): absolute values are pinned by these alone."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import image_encoder as ie
from oracle import ops


def _rng(seed=0):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ convolution
def _conv_scalar(x, w, b, stride):
    """The definition, one multiply-add at a time."""
    B, H, W, Ci = x.shape
    Co = w.shape[0]
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    y = np.zeros((B, Ho, Wo, Co))
    for n in range(B):
        for i in range(Ho):
            for j in range(Wo):
                for o in range(Co):
                    acc = b[o]
                    for u in range(3):
                        for v in range(3):
                            r, c = i * stride + u - 1, j * stride + v - 1
                            if 0 <= r < H and 0 <= c < W:
                                for ch in range(Ci):
                                    acc += x[n, r, c, ch] * w[o, u, v, ch]
                    y[n, i, j, o] = acc
    return y


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("hw", [(5, 4), (6, 7), (1, 1)])
def test_conv_matches_the_scalar_definition(stride, hw):
    r = _rng(stride + hw[0])
    x, w, b = r.normal(size=(2, hw[0], hw[1], 3)), r.normal(size=(4, 3, 3, 3)), r.normal(size=4)
    want = _conv_scalar(x, w, b, stride)
    assert np.allclose(ie.conv3x3(x, w, b, stride), want, rtol=0, atol=1e-12)
    assert np.allclose(ie.conv3x3(x, w.reshape(4, 27), b, stride), want, rtol=0, atol=1e-12)     # flat weight form


def test_conv_impulse_response_is_the_flipped_kernel():
    # a unit impulse in channel c at the centre: output channel o around it reads w[o, :, :, c] mirrored in both axes
    r = _rng(1)
    w = r.normal(size=(3, 3, 3, 2))
    x = np.zeros((1, 5, 5, 2))
    x[0, 2, 2, 1] = 1.0
    y = ie.conv3x3(x, w)
    for o in range(3):
        assert np.allclose(y[0, 1:4, 1:4, o], w[o, ::-1, ::-1, 1], rtol=0, atol=1e-15)
    assert np.all(y[0, 0, :, :] == 0) and np.all(y[0, :, 0, :] == 0)


def test_conv_constant_input_sums_the_taps_inside_the_padding():
    r = _rng(2)
    w, b = r.normal(size=(2, 3, 3, 3)), r.normal(size=2)
    y = ie.conv3x3(np.ones((1, 4, 4, 3)), w, b)
    assert np.allclose(y[0, 1, 1], w.sum(axis=(1, 2, 3)) + b)                       # interior: all nine taps
    assert np.allclose(y[0, 0, 0], w[:, 1:, 1:, :].sum(axis=(1, 2, 3)) + b)          # corner: the four taps inside
    assert np.allclose(y[0, 0, 2], w[:, 1:, :, :].sum(axis=(1, 2, 3)) + b)           # top edge: six taps


def test_conv_stride_two_subsamples_stride_one_and_is_linear():
    r = _rng(3)
    x, x2, w, b = r.normal(size=(2, 7, 6, 3)), r.normal(size=(2, 7, 6, 3)), r.normal(size=(4, 3, 3, 3)), r.normal(size=4)
    assert np.allclose(ie.conv3x3(x, w, b, 2), ie.conv3x3(x, w, b, 1)[:, ::2, ::2, :], rtol=0, atol=1e-13)
    assert np.allclose(ie.conv3x3(2 * x - 3 * x2, w), 2 * ie.conv3x3(x, w) - 3 * ie.conv3x3(x2, w), rtol=0, atol=1e-12)


def test_conv_and_groupnorm_against_torch_fp64():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    r = _rng(4)
    x, w, b = r.normal(size=(2, 9, 8, 6)), r.normal(size=(5, 3, 3, 6)), r.normal(size=5)
    for stride in (1, 2):
        t = F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w).permute(0, 3, 1, 2), torch.from_numpy(b), stride=stride, padding=1)
        assert np.allclose(ie.conv3x3(x, w, b, stride), t.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)
    g, be = r.normal(size=6), r.normal(size=6)
    t = F.group_norm(torch.from_numpy(x).permute(0, 3, 1, 2), 3, torch.from_numpy(g), torch.from_numpy(be), eps=1e-6)
    assert np.allclose(ie.groupnorm(x, g, be, 3, 1e-6), t.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-12)


# ------------------------------------------------------------------ GroupNorm
def test_groupnorm_hand_worked_statistics():
    # one sample, 1 x 2 pixels, 4 channels in 2 groups: group 0 holds {1, 3, 5, 7}, group 1 holds {2, 2, 2, 2}
    x = np.array([[[[1.0, 3.0, 2.0, 2.0], [5.0, 7.0, 2.0, 2.0]]]])
    y = ie.groupnorm(x, np.ones(4), np.zeros(4), 2, eps=0.0 + 1e-30)
    # group 0: mean 4, biased variance (9 + 1 + 1 + 9) / 4 = 5
    want0 = (np.array([1.0, 3.0, 5.0, 7.0]) - 4.0) / math.sqrt(5.0)
    assert np.allclose([y[0, 0, 0, 0], y[0, 0, 0, 1], y[0, 0, 1, 0], y[0, 0, 1, 1]], want0, rtol=1e-12)
    assert np.all(y[..., 2:] == 0.0)                       # a constant group normalises to zero


def test_groupnorm_invariants():
    r = _rng(5)
    x = r.normal(size=(3, 4, 5, 12)) * 3.0 + 1.5
    g, b = r.normal(size=12), r.normal(size=12)
    y = ie.groupnorm(x, np.ones(12), np.zeros(12), 4, 1e-6).reshape(3, 20, 4, 3)
    assert np.allclose(y.mean(axis=(1, 3)), 0.0, atol=1e-12)
    var = x.reshape(3, 20, 4, 3).var(axis=(1, 3))
    assert np.allclose(y.var(axis=(1, 3)), var / (var + 1e-6), rtol=1e-10)
    assert np.allclose(ie.groupnorm(np.full((1, 2, 2, 12), 7.0), g, b, 4), b)            # constant input -> beta
    # a per-(sample, group) affine change of the input does not change the output (up to eps)
    scale = r.uniform(0.5, 2.0, size=(3, 1, 1, 4, 1)); shift = r.normal(size=(3, 1, 1, 4, 1))
    x2 = (x.reshape(3, 4, 5, 4, 3) * scale + shift).reshape(x.shape)
    assert np.allclose(ie.groupnorm(x2, g, b, 4, 1e-12), ie.groupnorm(x, g, b, 4, 1e-12), atol=1e-8)
    # one group = LayerNorm over all of (H, W, C); one channel per group = per-channel instance norm
    ln, _, _ = ops.layernorm_fwd(x.reshape(3, -1), None, None, 1e-6)
    assert np.allclose(ie.groupnorm(x, np.ones(12), np.zeros(12), 1, 1e-6), ln.reshape(x.shape), atol=1e-12)
    inorm = (x - x.mean(axis=(1, 2), keepdims=True)) / np.sqrt(x.var(axis=(1, 2), keepdims=True) + 1e-6)
    assert np.allclose(ie.groupnorm(x, np.ones(12), np.zeros(12), 12, 1e-6), inorm, atol=1e-12)


# ------------------------------------------------------------------ blocks
def _block_cfg(kind, ci, co, hw=(4, 5), groups=2, stride=1):
    return si.ImageEncoderConfig("t", "f32", hw[0], hw[1], ci, groups, ((kind, ci, co, stride),), 2)


def test_resnet_block_with_zero_convolutions_is_its_skip_path():
    for ci, co in ((4, 4), (4, 6)):
        c = _block_cfg("resnet", ci, co)
        inp = si.make_image_encoder_inputs(c, 1, True, weight_std=0.3)
        p = dict(inp["params"])
        for n in ("conv2_w", "conv2_b"):
            p["layer0." + n] = np.zeros_like(p["layer0." + n])
        y = ie.encoder_fwd(p, c.layer_dicts(), inp["x"], c.groups)
        want = inp["x"] if ci == co else inp["x"] @ p["layer0.skip_w"].T + p["layer0.skip_b"]
        assert np.allclose(y, want, atol=1e-14)


def test_resnet_block_written_out_independently():
    c = _block_cfg("resnet", 4, 6)
    inp = si.make_image_encoder_inputs(c, 2, True, weight_std=0.3)
    p, x = inp["params"], inp["x"]
    sw = lambda t: t / (1.0 + np.exp(-t))
    h = _conv_scalar(sw(ie.groupnorm(x, p["layer0.norm1_g"], p["layer0.norm1_b"], 2)), p["layer0.conv1_w"].reshape(6, 3, 3, 4), p["layer0.conv1_b"], 1)
    h = _conv_scalar(sw(ie.groupnorm(h, p["layer0.norm2_g"], p["layer0.norm2_b"], 2)), p["layer0.conv2_w"].reshape(6, 3, 3, 6), p["layer0.conv2_b"], 1)
    want = x @ p["layer0.skip_w"].T + p["layer0.skip_b"] + h
    assert np.allclose(ie.encoder_fwd(p, c.layer_dicts(), x, 2), want, atol=1e-12)


def test_attention_block_closed_forms():
    c = _block_cfg("attn", 4, 4, hw=(3, 3))
    inp = si.make_image_encoder_inputs(c, 3, True, weight_std=0.5)
    p, x = dict(inp["params"]), inp["x"]
    L = c.layer_dicts()
    # zero query weights and bias: uniform attention, every pixel receives the mean value vector of its sample
    p0 = dict(p); p0["layer0.q_w"] = np.zeros((4, 4)); p0["layer0.q_b"] = np.zeros(4)
    h = ie.groupnorm(x, p["layer0.norm_g"], p["layer0.norm_b"], 2).reshape(2, 9, 4)
    v = h @ p["layer0.v_w"].T + p["layer0.v_b"]
    want = x + (np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape) @ p["layer0.proj_w"].T + p["layer0.proj_b"]).reshape(x.shape)
    assert np.allclose(ie.encoder_fwd(p0, L, x, 2), want, atol=1e-13)
    # a single pixel attends to itself with probability one
    c1 = _block_cfg("attn", 4, 4, hw=(1, 1))
    x1 = x[:, :1, :1, :]
    h1 = ie.groupnorm(x1, p["layer0.norm_g"], p["layer0.norm_b"], 2)
    want1 = x1 + ((h1 @ p["layer0.v_w"].T + p["layer0.v_b"]) @ p["layer0.proj_w"].T + p["layer0.proj_b"])
    assert np.allclose(ie.encoder_fwd(p, c1.layer_dicts(), x1, 2), want1, atol=1e-13)
    # pixels carry no position: permuting them permutes the output
    perm = _rng(9).permutation(9)
    xp = x.reshape(2, 9, 4)[:, perm, :].reshape(2, 3, 3, 4)
    y, yp = ie.encoder_fwd(p, L, x, 2), ie.encoder_fwd(p, L, xp, 2)
    assert np.allclose(yp.reshape(2, 9, 4), y.reshape(2, 9, 4)[:, perm, :], atol=1e-13)


def test_attention_block_against_torch_fp64():
    torch = pytest.importorskip("torch")
    c = _block_cfg("attn", 6, 6, hw=(4, 3), groups=3)
    inp = si.make_image_encoder_inputs(c, 4, True, weight_std=0.4)
    p, x = inp["params"], inp["x"]
    t = lambda a: torch.from_numpy(np.asarray(a))
    xt = t(x).permute(0, 3, 1, 2)
    h = torch.nn.functional.group_norm(xt, 3, t(p["layer0.norm_g"]), t(p["layer0.norm_b"]), eps=1e-6).permute(0, 2, 3, 1).reshape(2, 12, 6)
    q, k, v = (h @ t(p[f"layer0.{n}_w"]).T + t(p[f"layer0.{n}_b"]) for n in ("q", "k", "v"))
    a = torch.softmax(q @ k.transpose(1, 2) / math.sqrt(6.0), dim=-1) @ v
    want = t(x) + (a @ t(p["layer0.proj_w"]).T + t(p["layer0.proj_b"])).reshape(2, 4, 3, 6)
    assert np.allclose(ie.encoder_fwd(p, c.layer_dicts(), x, 3), want.numpy(), atol=1e-12)


# ------------------------------------------------------------------ encoder, partial batches
SMALL = si.ImageEncoderConfig("small_img_enc", "f32", 12, 10, 8, 4, si.vae_encoder_layers(8, (1, 2), 8, 8), 5)


def test_partial_batches_and_layer_ranges_compose():
    """Sec. 5: a layer run on part of the batch, the rest later; outputs concatenated.  Samples are
    independent and layer ranges compose."""
    inp = si.make_image_encoder_inputs(SMALL, 5, True, weight_std=0.0)
    p, x, L = inp["params"], inp["x"], SMALL.layer_dicts()
    full = ie.encoder_fwd(p, L, x, SMALL.groups)
    assert full.shape == (5,) + SMALL.out_shape()
    parts = [ie.encoder_fwd_partial(p, L, x, 0, len(L), off, n, SMALL.groups) for off, n in ((0, 2), (2, 1), (3, 2))]
    assert np.allclose(np.concatenate(parts), full, atol=1e-12)
    mid = ie.encoder_fwd_partial(p, L, x, 0, 4, 0, 5, SMALL.groups)
    assert mid.shape == (5,) + SMALL.out_shape(4)
    assert np.allclose(ie.encoder_fwd_partial(p, L, mid, 4, len(L), 0, 5, SMALL.groups), full, atol=1e-12)
    x2 = x.copy(); x2[3] += 1.0
    assert np.allclose(ie.encoder_fwd(p, L, x2, SMALL.groups)[:3], full[:3], atol=0)        # sample 3 touches only itself


def test_config_tables():
    c = si.CONFIG6
    assert len(c.layers) == 16 and c.out_shape() == (64, 64, 8) and c.out_shape(0) == (512, 512, 8)
    assert [k for k, *_ in c.layers].count("attn") == 1 and [st for *_, st in c.layers].count(2) == 3
    names = [n for n, _, _ in si.image_encoder_param_specs(c)]
    assert len(names) == len(set(names))
    assert ("layer4.skip_w" in names) and ("layer1.skip_w" not in names)     # 128 -> 256 changes width, 128 -> 128 does not
