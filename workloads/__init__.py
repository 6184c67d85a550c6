"""Seeded synthetic inputs for the batched-verify path.

This package only *draws* inputs (model shapes, weights, context lengths,
chunk lengths, block tables, cached KV contents, the uniform numbers and random
tokens a draft generator consumes).  It contains none of the method's
arithmetic: no normalisation, attention, softmax, accept rule or page
addressing lives here.  Both the CPU oracle's tests and the HIP path's tests /
benchmark take their inputs from here so that the two sides see identical
bytes.
"""
from .shapes import ModelShape, BatchRecipe, CONFIGS, config, TINY, LLAMA_8B, LLAMA_70B  # noqa: F401
from .gen import (  # noqa: F401
    tensor_seed, draw_normal_bf16, draw_layer_weights, draw_head_weights,
    draw_batch, draw_context_tokens, draw_context_kv, draw_draft_randoms,
    draw_confidence_logits, PAGE_SIZE, MAX_CHUNK,
)
