"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, validates descriptors / pointers / workspaces on the host before any launch,
and agrees with the input generator's parameter tables."""
import ctypes as C
import os
import re

import pytest

import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dp():
    import paper_2405_01248_amd as dp
    if not os.path.exists(dp.library_path()):
        from paper_2405_01248_amd import build
        build.build(verbose=False)
    dp.load_library()
    return dp


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dpipe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{]*\)\s*;", text)))


def test_every_declared_symbol_is_exported(dp):
    names = _declared_functions()
    assert {"stage_fwd", "stage_bwd", "encoder_fwd_partial", "dp_stage_profile", "dp_encoder_profile"} <= set(names)
    lib = dp.load_library()
    for n in names:
        assert hasattr(lib, n), n
    from paper_2405_01248_amd.binding import EXPORTS
    assert sorted(EXPORTS) == names


def test_param_tables_agree_with_input_generator(dp):
    for cfg in (si.CONFIG1, si.CONFIG2, si.CONFIG3, si.CONFIG4):
        kind = dp.KIND_UNET if cfg.kind == si.UNET else dp.KIND_DIT
        st = dp.Stage(kind, dp.DP_BF16 if cfg.dtype == "bf16" else dp.DP_F32, cfg.n_blocks, cfg.batch, cfg.tokens, cfg.d_model,
                      cfg.n_heads, cfg.d_head, cfg.ctx_tokens, cfg.ctx_dim, cfg.ff_inner, cfg.ln_eps, cfg.gelu_tanh)
        assert st.param_specs() == [(n, tuple(s)) for n, s, _ in si.stage_param_specs(cfg)]
        assert st.workspace_bytes(True) > st.workspace_bytes(False) > 0
    c = si.CONFIG5
    enc = dp.Encoder(dp.DP_BF16, c.n_layers, c.d_model, c.n_heads, c.d_head, c.seq, c.vocab, c.ff_inner, c.causal, c.ln_eps)
    assert enc.param_specs() == [(n, tuple(s)) for n, s, _ in si.encoder_param_specs(c)]
    assert enc.workspace_bytes(64) > enc.workspace_bytes(1) > 0


@pytest.mark.parametrize("bad, code", [
    (dict(n_heads=9), -1),            # d_model != n_heads * d_head
    (dict(batch=0), -1),
    (dict(kind=7), -1),
    (dict(dtype=5), -1),
    (dict(ln_eps=0.0), -1),
    (dict(ctx_tokens=0), -1),
    (dict(ff_inner=2564), -2),        # not a multiple of 8 in bf16
    (dict(d_model=1280, n_heads=10, d_head=128), -2),   # head dim beyond the MFMA attention kernels
])
def test_bad_descriptors_are_rejected(dp, bad, code):
    base = dict(kind=0, dtype=1, n_blocks=2, batch=8, tokens=1024, d_model=640, n_heads=10, d_head=64, ctx_tokens=77,
                ctx_dim=768, ff_inner=2560, ln_eps=1e-5, gelu_tanh=0)
    base.update(bad)
    with pytest.raises(dp.DpipeError) as ei:
        dp.Stage(**base)
    assert ei.value.code == code and str(ei.value)


def test_null_misaligned_and_small_workspace_are_rejected_before_launch(dp):
    lib = dp.load_library()
    st = dp.Stage(0, 1, 1, 1, 64, 64, 1, 64, 8, 64, 64)
    n = len(st.param_specs())
    good = (C.c_void_p * n)(*([0x10000] * n))
    x = C.c_void_p(0x20000)
    ws_bytes = st.workspace_bytes(True)
    assert lib.stage_fwd(st._h, None, x, x, x, x, ws_bytes, 1, None) == -1
    assert lib.stage_fwd(None, good, x, x, x, x, ws_bytes, 1, None) == -1
    assert lib.stage_fwd(st._h, good, None, x, x, x, ws_bytes, 1, None) == -1
    assert b"NULL" in lib.dp_last_error()
    assert lib.stage_fwd(st._h, good, C.c_void_p(0x20008), x, x, x, ws_bytes, 1, None) == -4
    assert lib.stage_fwd(st._h, good, x, x, x, C.c_void_p(0x20010), ws_bytes, 1, None) == -4      # workspace needs 256
    assert lib.stage_fwd(st._h, good, x, x, x, C.c_void_p(0x20100), ws_bytes - 1, 1, None) == -3
    assert b"workspace too small" in lib.dp_last_error()
    bad = (C.c_void_p * n)(*([0x10000] * (n - 1) + [0]))
    assert lib.stage_fwd(st._h, bad, x, x, x, C.c_void_p(0x20100), ws_bytes, 1, None) == -1
    assert lib.stage_bwd(st._h, good, x, x, x, None, None, 0, C.c_void_p(0x20100), ws_bytes, None) == -1

    enc = dp.Encoder(1, 2, 64, 1, 64, 16, 100, 128)
    m = len(enc.param_specs())
    eg = (C.c_void_p * m)(*([0x10000] * m))
    ws = C.c_void_p(0x20100)
    wsb = enc.workspace_bytes(4)
    call = lambda **k: lib.encoder_fwd_partial(enc._h, eg, x, x, k.get("gb", 8), k.get("lb", 0), k.get("le", 4), k.get("off", 0),
                                               k.get("n", 4), ws, k.get("wsb", wsb), None)
    assert call(off=6) == -1            # range leaves the global batch
    # batch-invariant modes: 0..2 accepted, anything else refused; mode 1 asks for a larger workspace (its split-K
    # factors come from one sample's rows) and a call with the smaller one is refused before any launch
    assert lib.dp_encoder_set_batch_invariant(enc._h, 3) == -1 and lib.dp_encoder_set_batch_invariant(None, 1) == -1
    big = dp.Encoder(1, 2, 768, 12, 64, 77, 1000, 3072)
    w0 = big.workspace_bytes(64)
    big.set_batch_invariant(1)
    w1 = big.workspace_bytes(64)
    big.set_batch_invariant(2)
    assert w1 > w0 and big.workspace_bytes(64) == w0
    assert call(n=0) == 0               # an empty slice is valid: checked, then nothing is launched (no GPU needed)
    assert call(n=0, off=8) == 0        # ... also at the very end of the batch
    assert call(n=0, off=9) == -1
    assert call(n=-1) == -1
    assert call(le=5) == -1             # only layers 0..n_layers+1 exist
    assert call(lb=3, le=3) == -1
    assert call(wsb=wsb - 1) == -3
    assert call(n=8, wsb=wsb) == -3     # workspace sized for 4 samples


def test_attention_arguments_are_checked_before_launch(dp):
    """The bf16 attention kernels address one batch element's rows with 32-bit byte offsets: a slice of 2 GiB
    or more, a head width they do not cover, a leading dimension or pointer off the 16-byte grid are all
    refused by the host check (no GPU needed: nothing is launched)."""
    lib = dp.load_library()
    p = C.c_void_p(0x10000)
    lse = C.c_void_p(0x20000)
    fwd = lambda **k: lib.dp_op_attention_fwd(dp.DP_BF16, 1, k.get("H", 2), k.get("Nq", 128), k.get("Nk", 128), k.get("dh", 64), 0, C.c_float(0.125),
                                              k.get("q", p), k.get("ld", 128), p, k.get("ld", 128), p, k.get("ld", 128), p, k.get("ld", 128), lse, None)
    assert fwd(dh=104, ld=208) == -2 and fwd(dh=60, ld=120) == -2          # head width
    assert fwd(ld=132) == -2                                                # leading dimension not a multiple of 8
    assert fwd(ld=120) == -1                                                # ... or smaller than heads * d_head
    assert fwd(q=C.c_void_p(0x10008)) == -4                                 # alignment
    assert fwd(Nk=1 << 22, ld=256) == -2                                    # 2^22 rows * 256 * 2 bytes = 2 GiB
    assert b"2 GiB" in lib.dp_last_error()
    assert fwd(Nq=0) == -1


def test_fusion_mask_range(dp):
    st = dp.Stage(0, 1, 1, 1, 64, 64, 1, 64, 8, 64, 64)
    for m in (0, 1, 2, 3):
        st.set_fusion(m)
    for m in (-1, 4):
        with pytest.raises(dp.DpipeError):
            st.set_fusion(m)


def test_last_error_is_never_null(dp):
    assert dp.load_library().dp_last_error() is not None


# ------------------------------------------------------------------ image encoder (host side)
def test_image_encoder_tables_and_shapes_agree_with_input_generator(dp):
    from paper_2405_01248_amd import binding as B
    for c in (si.CONFIG6, si.ImageEncoderConfig("t", "bf16", 16, 12, 8, 4, si.vae_encoder_layers(16, (1, 2), 8, 8), 3)):
        enc = B.ImageEncoder(B.DP_BF16, c.height, c.width, c.in_ch, c.groups, c.layers, c.gn_eps)
        assert enc.param_specs() == [(n, tuple(s)) for n, s, _ in si.image_encoder_param_specs(c)]
        assert enc.layer_shape(-1) == (c.height, c.width, c.in_ch)
        for l in range(len(c.layers)):
            assert enc.layer_shape(l) == c.out_shape(l + 1)
        nl = len(c.layers)
        assert enc.workspace_bytes(0, nl, 4) > enc.workspace_bytes(0, nl, 1) > 0
        assert enc.workspace_bytes(nl - 1, nl, 1) < enc.workspace_bytes(0, nl, 1)
        assert enc.workspace_bytes(0, nl + 1, 1) == 0 and enc.workspace_bytes(2, 2, 1) == 0


@pytest.mark.parametrize("layers, kw, code", [
    ((("conv", 8, 16, 3),), {}, -1),                         # stride 3
    ((("resnet", 8, 16, 2),), {}, -1),                       # only a plain convolution may stride
    ((("conv", 16, 16, 1),), {}, -1),                        # c_in does not match the 8 input channels
    ((("conv", 8, 12, 1),), {}, -2),                         # c_out not a multiple of 8
    ((("conv", 8, 16, 1), ("attn", 16, 24, 1)), {}, -1),     # attention changes the width
    ((("conv", 8, 24, 1), ("resnet", 24, 24, 1)), {"groups": 16}, -1),
    ((("conv", 8, 16, 1),), {"in_ch": 3}, -2),               # unpadded RGB
    ((("conv", 8, 16, 1),), {"dtype": 0}, -2),               # fp32 storage
    ((("conv", 8, 16, 1),), {"gn_eps": 0.0}, -1),
    ((("conv", 8, 16, 1), ("attn", 16, 16, 1)), {"height": 3, "width": 3}, -2),   # 9 pixels: not a multiple of 8
])
def test_bad_image_encoder_descriptors_are_rejected(dp, layers, kw, code):
    from paper_2405_01248_amd import binding as B
    a = dict(dtype=B.DP_BF16, height=8, width=8, in_ch=8, groups=4, gn_eps=1e-6)
    a.update(kw)
    with pytest.raises(B.DpipeError) as ei:
        B.ImageEncoder(a["dtype"], a["height"], a["width"], a["in_ch"], a["groups"], layers, a["gn_eps"])
    assert ei.value.code == code
