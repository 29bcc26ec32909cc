"""MI355X-native hot path of one GLEAM module step (unrolled PGD, greedy local training).

`synth` draws seeded inputs; `binding` marshals arguments into the C-ABI library built from
`csrc/` (hand-written HIP for gfx950).  There is no CPU fallback: calling the binding without the
built library raises.
"""
from . import synth  # noqa: F401
