"""CPU oracle for the selective KV-recompute prefill path (test infrastructure).

A plain, slow numpy implementation of what the path computes, written from the
paper: Section 4.2 (importance scores, top-k candidates), Section 4.3 (sliding
window grouping, recompute-and-overwrite), Section 4.1 (cache concatenation
and position re-numbering, used only to fabricate stale caches).  Floating
point runs in fp64 except where a decision must be reproducible bit for bit
(the column sums that feed top-k are fp32, added in ascending query order).

It shares no code with the HIP library and must never be imported by the
product path: only tests, the smoke check and the benchmark's CPU-baseline
leg may use it.
"""
from . import bf16, select, layer, fixture  # noqa: F401
