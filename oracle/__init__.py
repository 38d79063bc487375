"""TEST INFRASTRUCTURE -- not the product.  Slow fp64 CPU definitions of the hot path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the GPU library never does and shares no code with it.
"""
from .reference import (attn_oracle, attn_oracle_request, attn_probs, attn_bruteforce,
                        gather_request_kv, kv_append_reference, combine_partials,
                        partial_attention, bf16_to_f64, oracle_threads)
from .fp8 import (e4m3_decode, e4m3_encode_rne, scale_exponent, fp8_append_reference,
                  fp8_dequant_request)
