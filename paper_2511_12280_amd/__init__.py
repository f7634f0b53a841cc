"""MI355X-native D3ToM merge layer + bidirectional attention over the shortened sequence.

`binding` wraps the C-ABI library (include/d3tom.h) built from csrc/ by `build`; `workloads`
draws the seeded synthetic inputs.  Nothing here falls back to a CPU implementation.
"""
__all__ = ["binding", "workloads", "build"]
