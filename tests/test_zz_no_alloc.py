"""dp_op_gemm_static, the GEMM entry point that allocates nothing (its split-K partial sums live in a
device array inside the library), against dp_op_gemm with a caller-provided workspace: the same
kernels on the same splits, so the results must agree bit for bit -- on two calls in a row, the
second on a smaller problem (the array keeps the first call's contents), for both split-K paths
(fp32 weight-gradient output; storage-dtype output with the epilogue in the reduction pass).
The calls go through the C ABI with raw ctypes."""
import ctypes as C

import numpy as np
import pytest

import synth_inputs as si
from oracle import ops

pytestmark = pytest.mark.gpu


def _raw_pair(layout, M, N, K, seed, accumulate):
    """Runs dp_op_gemm (workspace from torch) and dp_op_gemm_static on the same operands; returns
    (result with workspace, result with the static scratch, oracle)."""
    import torch
    from paper_2405_01248_amd import binding as B
    from paper_2405_01248_amd.harness import _np_to_dev, _dev_to_np
    lib = B.load_library()
    a_k, b_k = {"nt": (0, 0), "tn": (1, 1)}[layout]
    rng = np.random.default_rng(seed)
    A = si.round_bf16(rng.standard_normal((M, K)))
    Bm = si.round_bf16(rng.standard_normal((K, N)) * 0.05)
    f32 = layout == "tn"
    bias = None if f32 else si.round_bf16(rng.standard_normal(N))
    dA = _np_to_dev(A.T if a_k else A, "bf16")
    dB = _np_to_dev(Bm if b_k else Bm.T, "bf16")
    dbias = None if f32 else _np_to_dev(bias, "bf16")
    C0 = (rng.standard_normal((M, N)) if accumulate else np.zeros((M, N))).astype(np.float32)
    ref = ops.linear_fwd(A, Bm.T, bias) + (C0.astype(np.float64) if f32 else 0.0)
    need = lib.dp_op_gemm_workspace_bytes(M, N, K)
    assert 0 < need <= B.STATIC_SCRATCH_BYTES, need            # the case really is split along K
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    outs = []
    for static in (False, True):
        dC = torch.from_numpy(C0).to("cuda:0") if f32 else torch.zeros((M, N), dtype=torch.bfloat16, device="cuda:0")
        common = (B.DP_BF16, C.c_void_p(dA.data_ptr()), dA.shape[1], a_k, C.c_void_p(dB.data_ptr()), dB.shape[1], b_k, M, N, K,
                  C.c_void_p(dbias.data_ptr()) if dbias is not None else None, C.c_void_p(dC.data_ptr()), N, int(f32), int(accumulate))
        if static:
            rc = lib.dp_op_gemm_static(*common, 0, stream)
        else:
            rc = lib.dp_op_gemm(*common, C.c_void_p(ws.data_ptr()), C.c_size_t(need), 0, stream)
        assert rc == 0, lib.dp_last_error().decode()
        torch.cuda.synchronize()
        outs.append(_dev_to_np(dC))
    return outs[0], outs[1], ref


def test_static_scratch_gemm_matches_workspace_gemm_on_two_calls_in_a_row():
    from paper_2405_01248_amd.harness import rel_err
    # first a large problem, then a smaller one of each kind: the second call of each pair finds the
    # first call's partial sums in the array
    for layout, shapes, tol in (("tn", [(640, 640, 8192, True), (320, 328, 4104, False)], 1e-4),
                                ("nt", [(1232, 768, 3072, False), (77, 768, 3072, False)], 2e-2)):
        for (M, N, K, acc) in shapes:
            print(f"\n[static gemm {layout} {M}x{N}x{K} acc={acc}]", flush=True)
            with_ws, static, ref = _raw_pair(layout, M, N, K, seed=M + K, accumulate=acc)
            assert np.array_equal(with_ws, static)
            e = rel_err(static, ref)
            print(f"[static gemm {layout} {M}x{N}x{K}] rel err vs oracle {e:.2e}", flush=True)
            assert e <= tol


def test_static_scratch_gemm_rejects_what_does_not_fit():
    import torch
    from paper_2405_01248_amd import binding as B
    lib = B.load_library()
    M, N, K = 4608, 1152, 8192                      # its split-K partial sums exceed the static array
    assert lib.dp_op_gemm_workspace_bytes(M, N, K) > B.STATIC_SCRATCH_BYTES
    a = torch.zeros((K, M), dtype=torch.bfloat16, device="cuda:0")
    b = torch.zeros((K, N), dtype=torch.bfloat16, device="cuda:0")
    c = torch.full((M, N), 3.0, dtype=torch.float32, device="cuda:0")
    with pytest.raises(B.DpipeError) as ei:
        B.op_gemm_static(B.DP_BF16, a, M, 1, b, N, 1, M, N, K, None, c, N, True, False)
    assert ei.value.code == -3 and "static scratch" in str(ei.value)
    torch.cuda.synchronize()
    assert float(c.min()) == 3.0 and float(c.max()) == 3.0          # nothing was launched
