"""CPU oracle (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It loads oracle/liblotts_oracle.so (plain C, fp64, built by gcc from
lotts_oracle.c) and exposes numpy wrappers with the same three names as the GPU library.
It imports nothing from the HIP package.
"""
from .oracle import (build, verify_attention, spec_accept, majority_vote,  # noqa: F401
                     spec_accept_logits, logit_weights, confidence_vote, skinny_gemm, kv_append, n_threads,
                     set_threads)
