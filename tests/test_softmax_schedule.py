"""The host model of the online softmax's moving reference (tests/softmax_schedule.py) on hand-made
logits, and the stress inputs of the GPU attention tests against it -- on the CPU, so that a stress
case that stresses nothing is caught before a GPU run."""
import numpy as np
import pytest

import synth_inputs as si
from softmax_schedule import LOG2E, head_logits, rescale_stats


def _two_tiles(rise_log2):
    s = np.zeros((1, 32, 128))
    s[0, 5, 64 + 3] = rise_log2 / LOG2E        # one query meets a larger score in the second key tile
    return s


def test_reference_moves_only_beyond_the_threshold():
    st = rescale_stats(_two_tiles(10.0))
    assert (st["steps_late"], st["moves_late"]) == (1, 1) and abs(st["max_rise_log2"] - 10.0) < 1e-9
    st = rescale_stats(_two_tiles(7.5))
    assert (st["steps_late"], st["moves_late"], st["max_rise_log2"]) == (1, 0, 0.0)
    # uniform rows: probability 1 / Nk everywhere
    assert abs(rescale_stats(np.zeros((2, 40, 77)))["mean_max_prob"] - 1.0 / 77) < 1e-12


def test_masked_tiles_and_waves_are_counted_as_the_kernel_walks_them():
    # causal 100 x 100: the waves of queries 0..31 and 32..63 never see key tile 1 (keys 64..), the other two do
    s = np.where(np.arange(100)[None, :] > np.arange(100)[:, None], -np.inf, 0.0)[None]
    st = rescale_stats(s)
    assert st["steps_late"] == 2 and st["moves_late"] == 0    # flat logits never move the reference
    # a reference set in tile 0 and a rise of 9 in tile 1 for a late query only
    s[0, 99, 70] = 9.0 / LOG2E
    assert rescale_stats(s)["moves_late"] == 1


def test_attention_stress_inputs_move_the_reference_late():
    from test_gpu_ops import ATTN_CASES
    stressed = [c for c in ATTN_CASES if c[6] != 1.0]
    assert len(stressed) >= 5 and any(c[5] and c[2] > 64 for c in stressed)      # incl. causal over several tiles
    for (B, H, Nq, Nk, dh, causal, gain, shift) in stressed:
        q, k, _, _ = si.make_attention_inputs(B, H, Nq, Nk, dh, seed=Nq * 31 + Nk, gain=gain, row_shift=shift)
        st = rescale_stats(head_logits(q, k, H, causal))
        assert st["moves_late"] > 0 and st["max_rise_log2"] > 8.0 and st["mean_max_prob"] > 0.5, st
        if gain <= 4.0:
            assert st["moves_late"] < st["steps_late"], st
    # the plain N(0,1) cases are the opposite regime: flat rows, (almost) no late move
    q, k, _, _ = si.make_attention_inputs(2, 3, 200, 200, 64, seed=1)
    st = rescale_stats(head_logits(q, k, 3))
    assert st["moves_late"] <= 1 and st["mean_max_prob"] < 0.2


def test_row_shift_is_a_per_row_constant():
    q, k, _, _ = si.make_attention_inputs(1, 2, 40, 50, 64, seed=0, gain=2.0, row_shift=80.0)
    q0 = q.copy()
    q0[:, :, 0::64] = 0.0
    diff = head_logits(q, k, 2) - head_logits(q0, k, 2)
    assert np.allclose(diff, diff[..., :1], rtol=0, atol=1e-9) and np.abs(diff).max() > 40.0
