"""CPU oracle for the ResIST sub-ResNet hot path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 implementation of what the HIP library computes, written
from the paper: the random layer-wise split into sub-ResNets (Sec. 2.2), one local
SGD iteration of one sub-ResNet (Algorithm 1, inner loop), and the reassembly that
averages the blocks shared between sub-ResNets (Sec. 2.3; Appendix B, definition of
the aggregated weights).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It shares no code with the HIP path and never imports it.

Pin status of each function is listed in each module's header; every function here
is pinned by tests/test_oracle_*.py unless its header says "parity unpinned".
"""
