"""Device-memory plumbing around the C ABI for tests, smoke and bench.

PyTorch is used for device allocations, host<->device copies and streams only;
all compute goes through ``Stage`` / ``Encoder`` (libdpipe.so).  Nothing here
imports the CPU oracle.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _np_to_dev(a: np.ndarray, dtype: str, device="cuda:0"):
    """float64 host array holding storage-representable values -> device tensor of the storage dtype."""
    if dtype == "bf16":
        f = np.ascontiguousarray(a, dtype=np.float32)
        bits = (f.view(np.uint32) >> 16).astype(np.uint16)          # exact: values are bf16-representable
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def _dev_to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def _torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def _dp_dtype(dtype: str):
    return B.DP_BF16 if dtype == "bf16" else B.DP_F32


class DeviceStage:
    """One stage with its parameters, gradients, activations and workspaces resident on the GPU."""

    def __init__(self, cfg, inputs, device="cuda:0"):
        self.cfg, self.device = cfg, device
        kind = B.KIND_UNET if cfg.kind == "unet_xattn_geglu" else B.KIND_DIT
        self.stage = B.Stage(kind, _dp_dtype(cfg.dtype), cfg.n_blocks, cfg.batch, cfg.tokens, cfg.d_model, cfg.n_heads,
                             cfg.d_head, cfg.ctx_tokens, cfg.ctx_dim, cfg.ff_inner, cfg.ln_eps, cfg.gelu_tanh)
        self.specs = self.stage.param_specs()
        td = _torch_dtype(cfg.dtype)
        self.params = [_np_to_dev(inputs["params"][name], cfg.dtype, device) for name, _ in self.specs]
        for (name, shape), p in zip(self.specs, self.params):
            assert tuple(p.shape) == tuple(shape), (name, p.shape, shape)
        self.dparams = [torch.zeros(shape, dtype=torch.float32, device=device) for _, shape in self.specs]
        self.x = _np_to_dev(inputs["x"], cfg.dtype, device)
        self.x_sc = _np_to_dev(inputs["x_sc"], cfg.dtype, device)
        self.dy = _np_to_dev(inputs["dy"], cfg.dtype, device)
        self.cc = _np_to_dev(inputs["ctx"] if "ctx" in inputs else inputs["cond"], cfg.dtype, device)
        self.y = torch.empty_like(self.x)
        self.y_sc = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        self.d_cond = torch.zeros((cfg.batch, cfg.d_model), dtype=torch.float32, device=device) if kind == B.KIND_DIT else None
        self.ws = torch.empty(self.stage.workspace_bytes(True), dtype=torch.uint8, device=device)
        self.ws_nograd = torch.empty(self.stage.workspace_bytes(False), dtype=torch.uint8, device=device)
        assert td == self.x.dtype

    # one pass of the hot path: [extra no-grad forward] + forward + backward
    def step(self, self_cond=None, accumulate=False):
        if self.cfg.self_cond if self_cond is None else self_cond:
            self.stage.fwd(self.params, self.x_sc, self.cc, self.y_sc, self.ws_nograd, False)
        self.stage.fwd(self.params, self.x, self.cc, self.y, self.ws, True)
        self.stage.bwd(self.params, self.dy, self.cc, self.dx, self.d_cond, self.dparams, accumulate, self.ws)

    def results(self):
        out = {"y": _dev_to_np(self.y), "dx": _dev_to_np(self.dx)}
        if self.d_cond is not None:
            out["dcond"] = _dev_to_np(self.d_cond)
        out["grads"] = {name: _dev_to_np(g) for (name, _), g in zip(self.specs, self.dparams)}
        out["y_sc"] = _dev_to_np(self.y_sc)
        return out


class DeviceEncoder:
    def __init__(self, cfg, inputs, device="cuda:0"):
        self.cfg, self.device = cfg, device
        self.enc = B.Encoder(_dp_dtype(cfg.dtype), cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.d_head, cfg.seq, cfg.vocab,
                             cfg.ff_inner, cfg.causal, cfg.ln_eps)
        self.specs = self.enc.param_specs()
        self.params = [_np_to_dev(inputs["params"][name], cfg.dtype, device) for name, _ in self.specs]
        for (name, shape), p in zip(self.specs, self.params):
            assert tuple(p.shape) == tuple(shape), (name, p.shape, shape)
        self.ids = torch.from_numpy(inputs["ids"].astype(np.int32)).to(device)
        self.gb = cfg.global_batch
        self.hidden = torch.zeros((self.gb, cfg.seq, cfg.d_model), dtype=_torch_dtype(cfg.dtype), device=device)
        self.ws = torch.empty(self.enc.workspace_bytes(self.gb), dtype=torch.uint8, device=device)
        self.n_layer_slots = cfg.n_layers + 2

    def run_slices(self, b, layer_begin=0, layer_end=None):
        """Cover the global batch with consecutive partial-batch calls of b samples."""
        le = self.n_layer_slots if layer_end is None else layer_end
        for off in range(0, self.gb, b):
            self.enc.fwd_partial(self.params, self.ids, self.hidden, self.gb, layer_begin, le, off, min(b, self.gb - off), self.ws)

    def output(self):
        return _dev_to_np(self.hidden)


class DeviceImageEncoder:
    """The frozen image encoder with its parameters, the image batch and the output buffer on the GPU."""

    def __init__(self, cfg, inputs, device="cuda:0"):
        self.cfg, self.device = cfg, device
        self.enc = B.ImageEncoder(_dp_dtype(cfg.dtype), cfg.height, cfg.width, cfg.in_ch, cfg.groups, cfg.layers, cfg.gn_eps)
        self.specs = self.enc.param_specs()
        self.params = [_np_to_dev(inputs["params"][name], cfg.dtype, device) for name, _ in self.specs]
        for (name, shape), p in zip(self.specs, self.params):
            assert tuple(p.shape) == tuple(shape), (name, p.shape, shape)
        self.gb, self.nl = cfg.global_batch, len(cfg.layers)
        self.x = _np_to_dev(inputs["x"], cfg.dtype, device)
        self.out = torch.zeros((self.gb,) + self.enc.layer_shape(self.nl - 1), dtype=_torch_dtype(cfg.dtype), device=device)
        self.ws = torch.empty(max(self.enc.workspace_bytes(0, self.nl, self.gb), 256), dtype=torch.uint8, device=device)

    def buffer(self, layer_end):
        """A zeroed global-batch buffer for the output of layer layer_end - 1."""
        return torch.zeros((self.gb,) + self.enc.layer_shape(layer_end - 1), dtype=self.out.dtype, device=self.device)

    def run_slices(self, b, layer_begin=0, layer_end=None, src=None, dst=None):
        """Cover the global batch with consecutive partial-batch calls of b samples."""
        le = self.nl if layer_end is None else layer_end
        src = self.x if src is None else src
        dst = self.out if dst is None else dst
        for off in range(0, self.gb, b):
            self.enc.fwd_partial(self.params, src, dst, self.gb, layer_begin, le, off, min(b, self.gb - off), self.ws)
        return dst

    def output(self):
        return _dev_to_np(self.out)


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max |gpu - ref| / max |ref| over one tensor (the tolerance metric of the parity tests)."""
    den = float(np.max(np.abs(ref)))
    num = float(np.max(np.abs(gpu - ref)))
    return num / den if den > 0 else num


def rel_l2(gpu: np.ndarray, ref: np.ndarray) -> float:
    """||gpu - ref||_2 / ||ref||_2 over one tensor (reported beside rel_err; not a pass criterion)."""
    den = float(np.sqrt(np.sum(np.square(ref))))
    num = float(np.sqrt(np.sum(np.square(gpu - ref))))
    return num / den if den > 0 else num
