"""CPU oracle for C2T tree construction: test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It never imports the HIP package and shares no code with it.
"""
from .ref import RefTree, build_oracle, ref_row, ref_entropy_top_m, ref_mlp_logit, ref_logit_of_beta  # noqa: F401
