"""CPU oracle for the batched-verify path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, by-eye-checkable numpy implementation of what the HIP path
computes: a Llama-style decoder forward over offloaded draft chunks against a
paged KV cache, the per-token confidence statistics, and the greedy
accept-prefix rule.  It exists so the tests can compare the GPU results with an
independent implementation.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product package never does, and this
package never imports the product package.  It shares no code with the HIP
path: only the seeded input draws (package `workloads`) serve both.

Precision: every function takes a working dtype, float64 by default, and the
parity runs use float64, the exact arithmetic of the definition.  A float32 run
of the same code is not a usable reference for a deep decoder: bf16 KV-cache
rounding decisions flip where a value sits near a rounding boundary, attention
carries each flip into the next layer, and the distance between the two runs
depends on the requests looked at.  Measured at the 70B shape (width 8192, all
80 layers), max |dlogit| float32 run vs float64 run: 4.2e-3 on one pair of
requests, 1.1e-1 on a sample of six.
Parameters and the KV cache hold bf16 values (the cache format is part of the
method's state), widened exactly.

Pins (tests/test_oracle_*.py): chunked == sequential == full prefill, paging and
batch invariance, accept-rule properties and brute force, softmax/entropy closed
forms, top-k / margin / dispatch-probability closed forms and brute force, attention/RoPE/RMSNorm special cases, an independently written dense
float64 decoder on the tiny config, the capped-geometric expected accept
length, and for the scheduler (Algorithm 1) hand-worked iteration traces, the chunk
count in closed form and conservation invariants on seeded random arrival traces;
for the importance score the harmonic closed form under uniform attention, the row-sum
invariant and a literal recomputation of the first layer's attention matrix; for
speculative sampling the exact output distribution on a tiny vocabulary (it must equal q).
No function here is "parity unpinned".
"""
from .numerics import bf16_round, bf16_bits, bf16_from_bits  # noqa: F401
from .confidence import confidence_row, confidence  # noqa: F401
from .dispatch import softmax_probs, topk_row, topk, margin_row, topp_count, nucleus_row, p_conf, p_imp, chunk_dispatch  # noqa: F401
from .decoder import (  # noqa: F401
    OracleModel, PagedKV, rmsnorm, rope, attention_one_query, decode_token, forward_tokens,
    lm_head,
)
from .verify import accept_prefix, verify_chunks, draft_chain, prefill_context  # noqa: F401
from .scheduler import SchedulerOracle, EngineItem  # noqa: F401
from .sampling import inverse_cdf, compressed_to_dense, speculative_accept  # noqa: F401
from .importance import importance_from_attention, importance_scores, mean_draft_importance  # noqa: F401
