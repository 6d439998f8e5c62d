"""CPU oracle of the GTree three-party protocols — TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It wraps ``libgtree_oracle.so`` (plain C, built from ``gtree_oracle.c``)
with ctypes; shared vectors are numpy uint64 arrays of shape ``(3, n)`` holding the
three additive components (Section II-B of the paper).
"""
from .orc import Oracle, build_oracle, X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_L, X_SCORE, X_C_PAPER  # noqa: F401
