"""MI355X-native speculative verification step across B reasoning branches (gfx950, HIP).

The product is liblotts.so (csrc/, C ABI in include/lotts.h); this package is its thin
binding.  Importing it loads the library and fails loudly if it has not been built.
"""
from .binding import (AttnDesc, LottsError, load, strerror, verify_attention, verify_attention_noalloc, spec_accept,  # noqa: F401
                      spec_accept_logits, majority_vote, confidence_vote, greedy_search, skinny_gemm, kv_append,
                      make_attn_desc, kernel_timer,
                      EXPORTS, LIB_PATH)

load()
