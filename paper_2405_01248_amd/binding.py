"""ctypes binding of libdpipe.so -- same names and arguments as include/dpipe.h.

Argument marshalling only: tensors are passed as raw device pointers
(``tensor.data_ptr()``), the stream as ``torch.cuda.current_stream().cuda_stream``.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

DP_F32, DP_BF16 = 0, 1
KIND_UNET, KIND_DIT = 0, 1


class DpipeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"dpipe error {code}: {msg}")
        self.code = code


class StageDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("kind", "dtype", "n_blocks", "batch", "tokens", "d_model", "n_heads", "d_head",
                                       "ctx_tokens", "ctx_dim", "ff_inner")] + [("ln_eps", C.c_float), ("gelu_tanh", C.c_int)]


class EncoderDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("dtype", "n_layers", "d_model", "n_heads", "d_head", "seq", "vocab", "ff_inner",
                                       "causal")] + [("ln_eps", C.c_float)]


class ImageLayer(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("kind", "c_in", "c_out", "stride")]


class ImageEncoderDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("dtype", "height", "width", "in_ch", "groups", "n_layers")] + [("gn_eps", C.c_float)]


IMG_KINDS = {"conv": 0, "resnet": 1, "attn": 2, "norm_conv": 3}


class LayerCost(C.Structure):
    _fields_ = [("component", C.c_int), ("layer", C.c_int), ("batch", C.c_int), ("fwd_ms", C.c_float), ("bwd_ms", C.c_float),
                ("out_bytes", C.c_int64), ("cf_bytes", C.c_int64), ("cb_bytes", C.c_int64), ("grad_bytes", C.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


DP_MAX_STAGES = 64


class PartitionOpts(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("micro_batch", "n_micro_batches", "n_devices", "max_stages", "uniform_replication")] + \
               [(n, C.c_double) for n in ("p2p_gbps", "p2p_latency_ms", "ar_gbps", "ar_latency_ms", "self_cond_prob")] + [("exact_stages", C.c_int)]


class PartitionPlan(C.Structure):
    _fields_ = [("n_stages", C.c_int), ("first_layer", C.c_int * DP_MAX_STAGES), ("n_layers", C.c_int * DP_MAX_STAGES),
                ("replicas", C.c_int * DP_MAX_STAGES)] + \
               [(n, C.c_double) for n in ("t0_ms", "t0_sc_ms", "gap_ms", "tf_ms", "t_max_ms")]


class BidirPlan(C.Structure):
    _fields_ = [("n_stages", C.c_int)] + [(n, C.c_int * DP_MAX_STAGES) for n in ("first_layer_down", "n_layers_down", "first_layer_up",
                                                                                   "n_layers_up", "replicas")] + \
               [(n, C.c_double) for n in ("t0_ms", "gap_ms", "t_max_ms")]


class SearchOpts(C.Structure):
    _fields_ = [("world_size", C.c_int), ("training_batch", C.c_int), ("group_sizes", C.POINTER(C.c_int)), ("n_group_sizes", C.c_int),
                ("micro_batch_counts", C.POINTER(C.c_int)), ("n_micro_batch_counts", C.c_int), ("max_stages", C.c_int),
                ("uniform_replication", C.c_int)] + \
               [(n, C.c_double) for n in ("p2p_gbps", "p2p_latency_ms", "ar_gbps", "ar_latency_ms", "self_cond_prob", "min_bubble_ms")] + \
               [("dep_pairs", C.POINTER(C.c_int)), ("n_dep_pairs", C.c_int)]


class SearchCandidate(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_stages", "n_micro_batches", "group_size", "micro_batch")] + \
               [(n, C.c_double) for n in ("pipeline_ms", "leftover_ms", "iteration_ms", "bubble_ratio", "bubble_ratio_filled")] + \
               [("plan", PartitionPlan)]


class Bubble(C.Structure):
    _fields_ = [("start_ms", C.c_double), ("end_ms", C.c_double), ("n_devices", C.c_int), ("stage_mask", C.c_uint64)]


class FillRow(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("bubble", "component", "first_layer", "n_layers", "samples", "partial")] + [("fill_ms", C.c_double)]


class FillSummary(C.Structure):
    _fields_ = [("bubble_device_ms", C.c_double), ("filled_device_ms", C.c_double), ("leftover_ms", C.c_double), ("n_fills", C.c_int)]


class KernelTime(C.Structure):
    _fields_ = [("kind", C.c_int), ("m", C.c_int), ("n", C.c_int), ("k", C.c_int), ("ms", C.c_float), ("flops", C.c_double),
                ("bytes", C.c_double)]


KERNEL_KINDS = {0: "gemm_nt", 1: "gemm_nn", 2: "gemm_tn", 3: "attn_fwd", 4: "attn_bwd_dq", 5: "attn_bwd_dkv", 6: "ln_fwd",
                7: "ln_bwd", 8: "geglu_fwd", 9: "geglu_bwd", 10: "reduce", 11: "other", 12: "gemm_f32", 13: "attn_f32", 14: "conv3x3", 15: "groupnorm", 16: "softmax_rows", 17: "gemm_fp8"}

EXPORTS = ["dp_stage_create", "dp_stage_destroy", "dp_stage_set_overlap", "dp_stage_set_fusion", "dp_encoder_set_batch_invariant", "dp_stage_param_count", "dp_stage_param_shape", "dp_stage_workspace_bytes",
           "stage_fwd", "stage_bwd", "dp_encoder_create", "dp_encoder_destroy", "dp_encoder_param_count",
           "dp_encoder_param_shape", "dp_encoder_workspace_bytes", "encoder_fwd_partial", "dp_stage_profile",
           "dp_encoder_profile", "dp_image_encoder_create", "dp_image_encoder_destroy", "dp_image_encoder_param_count",
           "dp_image_encoder_param_shape", "dp_image_encoder_layer_shape", "dp_image_encoder_workspace_bytes", "image_encoder_fwd_partial",
           "dp_image_encoder_profile", "dp_ktime_begin", "dp_ktime_end", "dp_ktime_event_overhead_ms", "dp_last_error", "dp_op_gemm", "dp_op_gemm_fp8", "dp_op_quantize_fp8", "dp_op_gemm_static", "dp_op_gemm_workspace_bytes",
           "dp_op_attention_fwd", "dp_op_attention_bwd", "dp_partition_solve", "dp_partition_solve_bidirectional", "dp_bubbles_1f1b", "dp_bubbles_fill", "dp_schedule_search"]


def library_path() -> str:
    return os.path.join(_HERE, "libdpipe.so")


def load_library():
    """Loads libdpipe.so (built by paper_2405_01248_amd/build.py).  Raises if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_2405_01248_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(path)
    vp, pp, i, sz = C.c_void_p, C.POINTER(C.c_void_p), C.c_int, C.c_size_t
    lib.dp_last_error.restype = C.c_char_p
    lib.dp_stage_create.argtypes = [C.POINTER(StageDesc), pp]
    lib.dp_stage_destroy.argtypes = [vp]; lib.dp_stage_destroy.restype = None
    lib.dp_stage_set_overlap.argtypes = [vp, i]
    lib.dp_stage_set_fusion.argtypes = [vp, i]
    lib.dp_encoder_set_batch_invariant.argtypes = [vp, i]
    lib.dp_stage_param_count.argtypes = [vp]
    lib.dp_stage_param_shape.argtypes = [vp, i, C.POINTER(C.c_int64), C.POINTER(C.c_char_p)]
    lib.dp_stage_workspace_bytes.argtypes = [vp, i]; lib.dp_stage_workspace_bytes.restype = sz
    lib.stage_fwd.argtypes = [vp, pp, vp, vp, vp, vp, sz, i, vp]
    lib.stage_bwd.argtypes = [vp, pp, vp, vp, vp, vp, pp, i, vp, sz, vp]
    lib.dp_encoder_create.argtypes = [C.POINTER(EncoderDesc), pp]
    lib.dp_encoder_destroy.argtypes = [vp]; lib.dp_encoder_destroy.restype = None
    lib.dp_encoder_param_count.argtypes = [vp]
    lib.dp_encoder_param_shape.argtypes = [vp, i, C.POINTER(C.c_int64), C.POINTER(C.c_char_p)]
    lib.dp_encoder_workspace_bytes.argtypes = [vp, i]; lib.dp_encoder_workspace_bytes.restype = sz
    lib.encoder_fwd_partial.argtypes = [vp, pp, vp, vp, i, i, i, i, i, vp, sz, vp]
    lib.dp_stage_profile.argtypes = [vp, pp, vp, vp, vp, vp, vp, vp, pp, vp, sz, i, C.POINTER(LayerCost), i, C.POINTER(i), vp]
    lib.dp_encoder_profile.argtypes = [vp, pp, vp, vp, i, C.POINTER(i), i, i, vp, sz, C.POINTER(LayerCost), i, C.POINTER(i), vp]
    lib.dp_image_encoder_create.argtypes = [C.POINTER(ImageEncoderDesc), C.POINTER(ImageLayer), pp]
    lib.dp_image_encoder_destroy.argtypes = [vp]; lib.dp_image_encoder_destroy.restype = None
    lib.dp_image_encoder_param_count.argtypes = [vp]
    lib.dp_image_encoder_param_shape.argtypes = [vp, i, C.POINTER(C.c_int64), C.POINTER(C.c_char_p)]
    lib.dp_image_encoder_layer_shape.argtypes = [vp, i, C.POINTER(C.c_int64)]
    lib.dp_image_encoder_workspace_bytes.argtypes = [vp, i, i, i]; lib.dp_image_encoder_workspace_bytes.restype = sz
    lib.image_encoder_fwd_partial.argtypes = [vp, pp, vp, vp, i, i, i, i, i, vp, sz, vp]
    lib.dp_image_encoder_profile.argtypes = [vp, pp, vp, vp, i, C.POINTER(i), i, i, vp, sz, C.POINTER(LayerCost), i, C.POINTER(i), vp]
    f = C.c_float
    lib.dp_op_gemm_workspace_bytes.argtypes = [i, i, i]; lib.dp_op_gemm_workspace_bytes.restype = sz
    lib.dp_op_gemm.argtypes = [i, vp, i, i, vp, i, i, i, i, i, vp, vp, i, i, i, vp, sz, i, vp]
    lib.dp_op_quantize_fp8.argtypes = [vp, i, vp, i, i, i, f, vp]
    lib.dp_op_gemm_fp8.argtypes = [vp, i, vp, i, i, i, i, f, vp, vp, i, vp]
    lib.dp_op_gemm_static.argtypes = [i, vp, i, i, vp, i, i, i, i, i, vp, vp, i, i, i, i, vp]
    lib.dp_op_attention_fwd.argtypes = [i, i, i, i, i, i, i, f, vp, i, vp, i, vp, i, vp, i, vp, vp]
    lib.dp_op_attention_bwd.argtypes = [i, i, i, i, i, i, f, vp, i, vp, i, vp, i, vp, i, vp, vp, i, vp, vp, i, vp, i, vp, i, vp]
    lib.dp_partition_solve.argtypes = [C.POINTER(LayerCost), i, C.POINTER(PartitionOpts), C.POINTER(PartitionPlan)]
    dptr = C.POINTER(C.c_double)
    lib.dp_bubbles_1f1b.argtypes = [i, dptr, dptr, C.POINTER(i), i, dptr, dptr, dptr, C.c_double, C.POINTER(Bubble), i, C.POINTER(i), dptr]
    lib.dp_bubbles_fill.argtypes = [C.POINTER(Bubble), i, C.POINTER(LayerCost), i, C.POINTER(i), i, i, i, C.POINTER(FillRow), i, C.POINTER(FillSummary)]
    lib.dp_partition_solve_bidirectional.argtypes = [C.POINTER(LayerCost), i, C.POINTER(LayerCost), i, C.POINTER(PartitionOpts), C.POINTER(BidirPlan)]
    lib.dp_schedule_search.argtypes = [C.POINTER(LayerCost), i, C.POINTER(SearchOpts), C.POINTER(SearchCandidate), i, C.POINTER(i), C.POINTER(i)]
    lib.dp_ktime_begin.argtypes = [i]
    lib.dp_ktime_event_overhead_ms.restype = C.c_float
    lib.dp_ktime_end.argtypes = [C.POINTER(KernelTime), i, C.POINTER(i)]
    _LIB = lib
    return lib


def _check(code: int):
    if code != 0:
        raise DpipeError(code, load_library().dp_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    return C.c_void_p(t.data_ptr()) if hasattr(t, "data_ptr") else C.c_void_p(int(t))


def _ptr_array(ts: Sequence):
    arr = (C.c_void_p * len(ts))()
    for k, t in enumerate(ts):
        arr[k] = t.data_ptr() if hasattr(t, "data_ptr") else int(t)
    return arr


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(int(stream))


def _nbytes(t):
    return t.numel() * t.element_size() if t is not None else 0


class _Handle:
    _destroy = None

    def __init__(self):
        self._h = C.c_void_p()

    def close(self):
        if self._h:
            getattr(load_library(), self._destroy)(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _specs(self, count_fn, shape_fn):
        lib = load_library()
        n = getattr(lib, count_fn)(self._h)
        out = []
        for k in range(n):
            shape = (C.c_int64 * 2)()
            name = C.c_char_p()
            _check(getattr(lib, shape_fn)(self._h, k, shape, C.byref(name)))
            out.append((name.value.decode(), (shape[0],) if shape[1] == 0 else (shape[0], shape[1])))
        return out


class Stage(_Handle):
    """dp_stage handle: stage_fwd / stage_bwd / dp_stage_profile."""
    _destroy = "dp_stage_destroy"

    def __init__(self, kind, dtype, n_blocks, batch, tokens, d_model, n_heads, d_head, ctx_tokens=0, ctx_dim=0,
                 ff_inner=0, ln_eps=1e-5, gelu_tanh=0):
        super().__init__()
        self.desc = StageDesc(kind, dtype, n_blocks, batch, tokens, d_model, n_heads, d_head, ctx_tokens, ctx_dim, ff_inner,
                              ln_eps, gelu_tanh)
        _check(load_library().dp_stage_create(C.byref(self.desc), C.byref(self._h)))

    def set_overlap(self, enabled: bool):
        _check(load_library().dp_stage_set_overlap(self._h, int(enabled)))

    def set_fusion(self, mask: int):
        _check(load_library().dp_stage_set_fusion(self._h, int(mask)))

    def param_specs(self):
        return self._specs("dp_stage_param_count", "dp_stage_param_shape")

    def workspace_bytes(self, save_for_bwd: bool) -> int:
        return load_library().dp_stage_workspace_bytes(self._h, int(save_for_bwd))

    def fwd(self, params, x, ctx_or_cond, y, workspace, save_for_bwd, stream=None):
        _check(load_library().stage_fwd(self._h, _ptr_array(params), _ptr(x), _ptr(ctx_or_cond), _ptr(y), _ptr(workspace),
                                        _nbytes(workspace), int(save_for_bwd), _stream(stream)))

    def bwd(self, params, dy, ctx_or_cond, dx, d_cond, dparams, accumulate, workspace, stream=None):
        _check(load_library().stage_bwd(self._h, _ptr_array(params), _ptr(dy), _ptr(ctx_or_cond), _ptr(dx), _ptr(d_cond),
                                        _ptr_array(dparams), int(accumulate), _ptr(workspace), _nbytes(workspace),
                                        _stream(stream)))

    def profile(self, params, x, ctx_or_cond, y, dy, dx, d_cond, dparams, workspace, reps=5, stream=None):
        rows = (LayerCost * self.desc.n_blocks)()
        n = C.c_int(0)
        _check(load_library().dp_stage_profile(self._h, _ptr_array(params), _ptr(x), _ptr(ctx_or_cond), _ptr(y), _ptr(dy),
                                               _ptr(dx), _ptr(d_cond), _ptr_array(dparams), _ptr(workspace),
                                               _nbytes(workspace), reps, rows, len(rows), C.byref(n), _stream(stream)))
        return [rows[k].as_dict() for k in range(n.value)]


class Encoder(_Handle):
    """dp_encoder handle: encoder_fwd_partial / dp_encoder_profile."""
    _destroy = "dp_encoder_destroy"

    def __init__(self, dtype, n_layers, d_model, n_heads, d_head, seq, vocab, ff_inner, causal=1, ln_eps=1e-5):
        super().__init__()
        self.desc = EncoderDesc(dtype, n_layers, d_model, n_heads, d_head, seq, vocab, ff_inner, causal, ln_eps)
        _check(load_library().dp_encoder_create(C.byref(self.desc), C.byref(self._h)))

    def param_specs(self):
        return self._specs("dp_encoder_param_count", "dp_encoder_param_shape")

    def set_batch_invariant(self, on):
        _check(load_library().dp_encoder_set_batch_invariant(self._h, int(on)))

    def workspace_bytes(self, max_samples: int) -> int:
        return load_library().dp_encoder_workspace_bytes(self._h, max_samples)

    def fwd_partial(self, params, ids, hidden, global_batch, layer_begin, layer_end, sample_offset, num_samples, workspace,
                    stream=None):
        _check(load_library().encoder_fwd_partial(self._h, _ptr_array(params), _ptr(ids), _ptr(hidden), global_batch,
                                                  layer_begin, layer_end, sample_offset, num_samples, _ptr(workspace),
                                                  _nbytes(workspace), _stream(stream)))

    def profile(self, params, ids, hidden, global_batch, batches, workspace, reps=5, stream=None):
        nl = self.desc.n_layers + 2
        rows = (LayerCost * (nl * len(batches)))()
        n = C.c_int(0)
        arr = (C.c_int * len(batches))(*batches)
        _check(load_library().dp_encoder_profile(self._h, _ptr_array(params), _ptr(ids), _ptr(hidden), global_batch, arr,
                                                 len(batches), reps, _ptr(workspace), _nbytes(workspace), rows, len(rows),
                                                 C.byref(n), _stream(stream)))
        return [rows[k].as_dict() for k in range(n.value)]


class ImageEncoder(_Handle):
    """Frozen image encoder; `layers` is a sequence of (kind, c_in, c_out, stride) with kind a key of IMG_KINDS."""
    _destroy = "dp_image_encoder_destroy"

    def __init__(self, dtype, height, width, in_ch, groups, layers, gn_eps=1e-6):
        super().__init__()
        self.n_layers = len(layers)
        arr = (ImageLayer * len(layers))(*[ImageLayer(IMG_KINDS[k], ci, co, st) for (k, ci, co, st) in layers])
        desc = ImageEncoderDesc(dtype, height, width, in_ch, groups, len(layers), gn_eps)
        _check(load_library().dp_image_encoder_create(C.byref(desc), arr, C.byref(self._h)))

    def param_specs(self):
        return self._specs("dp_image_encoder_param_count", "dp_image_encoder_param_shape")

    def layer_shape(self, layer: int):
        hwc = (C.c_int64 * 3)()
        _check(load_library().dp_image_encoder_layer_shape(self._h, layer, hwc))
        return tuple(int(v) for v in hwc)

    def workspace_bytes(self, layer_begin: int, layer_end: int, max_samples: int) -> int:
        return load_library().dp_image_encoder_workspace_bytes(self._h, layer_begin, layer_end, max_samples)

    def fwd_partial(self, params, x_in, out, global_batch, layer_begin, layer_end, sample_offset, num_samples, workspace, stream=None):
        _check(load_library().image_encoder_fwd_partial(self._h, _ptr_array(params), _ptr(x_in), _ptr(out), global_batch, layer_begin, layer_end,
                                                        sample_offset, num_samples, _ptr(workspace), _nbytes(workspace), _stream(stream)))

    def profile(self, params, x_in, out, global_batch, batches, workspace, reps=5, stream=None):
        n = self.n_layers * len(batches)
        rows = (LayerCost * n)()
        got = C.c_int(0)
        barr = (C.c_int * len(batches))(*batches)
        _check(load_library().dp_image_encoder_profile(self._h, _ptr_array(params), _ptr(x_in), _ptr(out), global_batch, barr, len(batches), reps,
                                                       _ptr(workspace), _nbytes(workspace), rows, n, C.byref(got), _stream(stream)))
        return [rows[k].as_dict() for k in range(got.value)]


def ktime_begin(max_records: int = 65536):
    _check(load_library().dp_ktime_begin(max_records))


def ktime_end(max_records: int = 65536):
    """Returns a list of dicts (kind name, m, n, k, ms, flops, bytes), one per recorded launch."""
    rows = (KernelTime * max_records)()
    n = C.c_int(0)
    _check(load_library().dp_ktime_end(rows, max_records, C.byref(n)))
    return [{"kind": KERNEL_KINDS.get(rows[j].kind, str(rows[j].kind)), "m": rows[j].m, "n": rows[j].n, "k": rows[j].k,
             "ms": rows[j].ms, "flops": rows[j].flops, "bytes": rows[j].bytes} for j in range(n.value)]


def ktime_event_overhead_ms() -> float:
    """What an empty pair of events read in the last ktime_end (for scale; the records are not corrected by it)."""
    return float(load_library().dp_ktime_event_overhead_ms())


def partition_solve(rows, micro_batch, n_micro_batches, n_devices, p2p_gbps, p2p_latency_ms, ar_gbps, ar_latency_ms,
                    self_cond_prob=0.0, max_stages=0, uniform_replication=False, exact_stages=0):
    """rows: sequence of LayerCost or of dicts with its fields (host data).  Returns a dict with the plan."""
    arr = (LayerCost * len(rows))()
    for i, r in enumerate(rows):
        d = r if isinstance(r, dict) else r.as_dict()
        for n, _ in LayerCost._fields_:
            setattr(arr[i], n, d[n])
    opts = PartitionOpts(micro_batch, n_micro_batches, n_devices, max_stages, int(uniform_replication), p2p_gbps, p2p_latency_ms,
                         ar_gbps, ar_latency_ms, self_cond_prob, exact_stages)
    plan = PartitionPlan()
    lib = load_library()
    _check(lib.dp_partition_solve(arr, len(rows), C.byref(opts), C.byref(plan)))
    n = plan.n_stages
    return {"n_stages": n, "first_layer": list(plan.first_layer[:n]), "n_layers": list(plan.n_layers[:n]),
            "replicas": list(plan.replicas[:n]), "t0_ms": plan.t0_ms, "t0_sc_ms": plan.t0_sc_ms, "gap_ms": plan.gap_ms,
            "tf_ms": plan.tf_ms, "t_max_ms": plan.t_max_ms}


def _rows_array(rows):
    arr = (LayerCost * len(rows))()
    for i, r in enumerate(rows):
        d = r if isinstance(r, dict) else r.as_dict()
        for n, _ in LayerCost._fields_:
            setattr(arr[i], n, d[n])
    return arr


def partition_solve_bidirectional(rows_down, rows_up, micro_batch, n_paired_micro_batches, n_devices, p2p_gbps, p2p_latency_ms, ar_gbps,
                                  ar_latency_ms, max_stages=0, uniform_replication=False, exact_stages=0):
    opts = PartitionOpts(micro_batch, n_paired_micro_batches, n_devices, max_stages, int(uniform_replication), p2p_gbps, p2p_latency_ms,
                         ar_gbps, ar_latency_ms, 0.0, exact_stages)
    plan = BidirPlan()
    _check(load_library().dp_partition_solve_bidirectional(_rows_array(rows_down), len(rows_down), _rows_array(rows_up), len(rows_up),
                                                           C.byref(opts), C.byref(plan)))
    n = plan.n_stages
    out = {k: list(getattr(plan, k)[:n]) for k in ("first_layer_down", "n_layers_down", "first_layer_up", "n_layers_up", "replicas")}
    out.update(n_stages=n, t0_ms=plan.t0_ms, gap_ms=plan.gap_ms, t_max_ms=plan.t_max_ms)
    return out


def schedule_search(rows, world_size, training_batch, group_sizes, micro_batch_counts, p2p_gbps, p2p_latency_ms, ar_gbps, ar_latency_ms,
                    self_cond_prob=0.0, max_stages=0, uniform_replication=True, min_bubble_ms=0.0, deps=(), max_cands=4096):
    """Returns (list of candidate dicts in walking order, index of the best)."""
    gs = (C.c_int * len(group_sizes))(*group_sizes)
    ms = (C.c_int * len(micro_batch_counts))(*micro_batch_counts)
    flat = [x for pair in deps for x in pair]
    dp = (C.c_int * max(len(flat), 1))(*flat)
    opts = SearchOpts(world_size, training_batch, gs, len(group_sizes), ms, len(micro_batch_counts), max_stages, int(uniform_replication),
                      p2p_gbps, p2p_latency_ms, ar_gbps, ar_latency_ms, self_cond_prob, min_bubble_ms, dp, len(deps))
    cands = (SearchCandidate * max_cands)()
    n, best = C.c_int(0), C.c_int(-1)
    _check(load_library().dp_schedule_search(_rows_array(rows), len(rows), C.byref(opts), cands, max_cands, C.byref(n), C.byref(best)))
    out = []
    for k in range(n.value):
        c = cands[k]
        ns = c.plan.n_stages
        out.append({"n_stages": c.n_stages, "n_micro_batches": c.n_micro_batches, "group_size": c.group_size, "micro_batch": c.micro_batch,
                    "pipeline_ms": c.pipeline_ms, "leftover_ms": c.leftover_ms, "iteration_ms": c.iteration_ms, "bubble_ratio": c.bubble_ratio,
                    "bubble_ratio_filled": c.bubble_ratio_filled, "first_layer": list(c.plan.first_layer[:ns]),
                    "n_layers": list(c.plan.n_layers[:ns]), "replicas": list(c.plan.replicas[:ns]), "t_max_ms": c.plan.t_max_ms})
    return out, best.value


def _darr(v):
    return None if v is None else (C.c_double * len(v))(*v)


def bubbles_1f1b(fwd_ms, bwd_ms, replicas, n_micro_batches, comm_fwd_ms=None, comm_bwd_ms=None, tail_ms=None, min_ms=0.0,
                 max_out=4096):
    """Returns (list of bubble dicts, iteration_ms)."""
    S = len(fwd_ms)
    out = (Bubble * max_out)()
    n, t = C.c_int(0), C.c_double(0.0)
    _check(load_library().dp_bubbles_1f1b(S, _darr(fwd_ms), _darr(bwd_ms), (C.c_int * S)(*replicas), n_micro_batches,
                                          _darr(comm_fwd_ms), _darr(comm_bwd_ms), _darr(tail_ms), min_ms, out, max_out,
                                          C.byref(n), C.byref(t)))
    return [{"start_ms": out[i].start_ms, "end_ms": out[i].end_ms, "n_devices": out[i].n_devices,
             "stages": tuple(s for s in range(S) if out[i].stage_mask >> s & 1)} for i in range(n.value)], t.value


def bubbles_fill(bubbles, rows, batch, n_devices, deps=(), max_fills=4096):
    """bubbles: dicts as returned by bubbles_1f1b (start_ms, end_ms, n_devices); rows: LayerCost dicts of the
    non-trainable components; deps: (component, depends_on) pairs.  Returns (fill row dicts, summary dict)."""
    barr = (Bubble * max(len(bubbles), 1))()
    for i, b in enumerate(bubbles):
        barr[i].start_ms, barr[i].end_ms, barr[i].n_devices = b["start_ms"], b["end_ms"], b["n_devices"]
        barr[i].stage_mask = sum(1 << s for s in b.get("stages", ()))
    arr = (LayerCost * len(rows))()
    for i, r in enumerate(rows):
        for n, _ in LayerCost._fields_:
            setattr(arr[i], n, r[n])
    flat = [x for pair in deps for x in pair]
    darr = (C.c_int * max(len(flat), 1))(*flat)
    fills = (FillRow * max_fills)()
    summ = FillSummary()
    _check(load_library().dp_bubbles_fill(barr, len(bubbles), arr, len(rows), darr, len(deps), batch, n_devices, fills, max_fills,
                                          C.byref(summ)))
    names = [n for n, _ in FillRow._fields_]
    return ([{n: getattr(fills[i], n) for n in names} for i in range(summ.n_fills)],
            {"bubble_device_ms": summ.bubble_device_ms, "filled_device_ms": summ.filled_device_ms, "leftover_ms": summ.leftover_ms})


def op_gemm(dtype, A, lda, a_kmajor, B, ldb, b_kmajor, M, N, K, bias, Cout, ldc, out_is_f32=False, accumulate=False,
            workspace=None, tile_cfg=0, stream=None):
    _check(load_library().dp_op_gemm(dtype, _ptr(A), lda, int(a_kmajor), _ptr(B), ldb, int(b_kmajor), M, N, K, _ptr(bias),
                                     _ptr(Cout), ldc, int(out_is_f32), int(accumulate), _ptr(workspace), _nbytes(workspace),
                                     tile_cfg, _stream(stream)))


STATIC_SCRATCH_BYTES = 64 << 20


def op_gemm_static(dtype, A, lda, a_kmajor, B, ldb, b_kmajor, M, N, K, bias, Cout, ldc, out_is_f32=False, accumulate=False,
                   tile_cfg=0, stream=None):
    _check(load_library().dp_op_gemm_static(dtype, _ptr(A), lda, int(a_kmajor), _ptr(B), ldb, int(b_kmajor), M, N, K, _ptr(bias),
                                            _ptr(Cout), ldc, int(out_is_f32), int(accumulate), tile_cfg, _stream(stream)))


def op_quantize_fp8(x, ldx, q, ldq, rows, cols, scale, stream=None):
    _check(load_library().dp_op_quantize_fp8(_ptr(x), ldx, _ptr(q), ldq, rows, cols, scale, _stream(stream)))


def op_gemm_fp8(A, lda, B, ldb, M, N, K, out_scale, bias, Cout, ldc, stream=None):
    _check(load_library().dp_op_gemm_fp8(_ptr(A), lda, _ptr(B), ldb, M, N, K, out_scale, _ptr(bias), _ptr(Cout), ldc, _stream(stream)))


def op_gemm_workspace_bytes(M, N, K):
    return load_library().dp_op_gemm_workspace_bytes(M, N, K)


def op_attention_fwd(dtype, B, H, Nq, Nk, d_head, causal, scale, q, ldq, k, ldk, v, ldv, o, ldo, lse, stream=None):
    _check(load_library().dp_op_attention_fwd(dtype, B, H, Nq, Nk, d_head, int(causal), scale, _ptr(q), ldq, _ptr(k), ldk,
                                              _ptr(v), ldv, _ptr(o), ldo, _ptr(lse), _stream(stream)))


def op_attention_bwd(dtype, B, H, Nq, Nk, d_head, scale, q, ldq, k, ldk, v, ldv, o, ldo, lse, d_o, lddo, delta, dq, lddq, dk,
                     lddk, dv, lddv, stream=None):
    _check(load_library().dp_op_attention_bwd(dtype, B, H, Nq, Nk, d_head, scale, _ptr(q), ldq, _ptr(k), ldk, _ptr(v), ldv,
                                              _ptr(o), ldo, _ptr(lse), _ptr(d_o), lddo, _ptr(delta), _ptr(dq), lddq,
                                              _ptr(dk), lddk, _ptr(dv), lddv, _stream(stream)))
