"""fp64 CPU oracle for the stage-compute hot path (TEST INFRASTRUCTURE ONLY).

Plain, slow numpy float64 implementations of what one pipeline stage computes
per micro-batch (Sec. 4.1: a stage's time is the sum of its layers' forward
and backward times; Sec. 4.3: one extra forward under self-conditioning) and of
the frozen text encoder's forward on a partial batch (Sec. 5, partial-batch
layers).  The paper treats each layer as a black box, so the arithmetic here is
the textbook definition of the named architectures, written out without
blocking, fusion or reordering.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with the HIP path and imports nothing from it.

Pins (tests/test_oracle_*.py): central finite differences for every backward,
softmax/LayerNorm invariants, zero-input / identity-weight / adaLN-zero closed
forms, partial-batch concat and layer-range composition, and a second-opinion
check against torch CPU fp64 autograd.  Absolute values have no worked example
in the paper: "parity unpinned" by the paper itself, pinned by the above.
"""
