"""fp64 CPU oracle for the stage-compute hot path (TEST INFRASTRUCTURE ONLY).

Plain, slow numpy float64 implementations of what one pipeline stage computes
per micro-batch (Sec. 4.1: a stage's time is the sum of its layers' forward
and backward times; Sec. 4.3: one extra forward under self-conditioning) and of
the frozen text encoder's forward on a partial batch (Sec. 5, partial-batch
layers).  The paper treats each layer as a black box, so the arithmetic here is
the textbook definition of the named architectures, written out without
blocking, fusion or reordering.

Further modules, each with its own header and pins:
  partition.py      backbone partitioning, single (Sec. 4.1 Eq. 1-9, Sec. 4.3 Eq. 17-18) and bidirectional
                    (Sec. 4.2 Eq. 10-16; the expression for M_CDM is an input: "parity unpinned"), brute force
  bubbles.py        1F1B bubbles and their filling (Sec. 5, Algorithms 1-2)
  search.py         the walk over (S, M, D) (Sec. 3, steps 2-5)
  image_encoder.py  3x3 convolution, GroupNorm, residual and attention blocks of the frozen image encoder
  fp8.py            OCP E4M3 quantisation and the FP8 projection product (an extension beyond the paper)

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with the HIP path and imports nothing from it.

Pins (tests/test_oracle_*.py): central finite differences for every backward,
softmax/LayerNorm invariants, zero-input / identity-weight / adaLN-zero closed
forms, partial-batch concat and layer-range composition, and a second-opinion
check against torch CPU fp64 autograd.  Absolute values have no worked example
in the paper: "parity unpinned" by the paper itself, pinned by the above.
"""
