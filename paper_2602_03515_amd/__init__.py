"""MI355X-native basis-rotation optimizer step (hand-written HIP behind a C ABI).

`paper_2602_03515_amd.binding` wraps the C-ABI library (it raises if the
library has not been built); `paper_2602_03515_amd.synth` makes seeded inputs;
`paper_2602_03515_amd.ring` is the host-side delayed-gradient ring.
"""
__all__ = ["synth"]
