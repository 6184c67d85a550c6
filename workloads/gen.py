"""Seeded draws of every synthetic input.

Small integer metadata (lengths, chunk sizes, page assignment) is drawn with
numpy's PCG64 on the host.  Large tensors (weights, cached KV, logits) are drawn
with torch's generator on the device they are needed on (CPU in CPU-only tests,
the GPU otherwise) and the CPU oracle is handed a host copy of exactly those
bytes, so both sides always see bit-identical inputs within one process.
"""
import math

import numpy as np
import torch

from .shapes import BatchRecipe, ModelShape

PAGE_SIZE = 16
MAX_CHUNK = 32          # longest chunk (uncached + drafts) one request may carry

_M64 = (1 << 64) - 1


def _mix(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def tensor_seed(seed: int, *ids: int) -> int:
    """A 63-bit seed for one tensor, derived from the workload seed and ids."""
    z = _mix(seed & _M64)
    for i in ids:
        z = _mix(z ^ (int(i) & _M64))
    return z >> 1


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def draw_normal_bf16(shape, std, seed, device="cpu", mean=0.0):
    """N(mean, std^2) drawn in fp32, rounded once (RNE) to bf16."""
    x = torch.randn(shape, generator=_gen(device, seed), device=device, dtype=torch.float32)
    x.mul_(std)
    if mean != 0.0:
        x.add_(mean)
    return x.to(torch.bfloat16)


# tensor ids inside one layer
_LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")


def draw_layer_weights(shape: ModelShape, seed: int, layer: int, device="cpu"):
    """bf16 weights of one decoder layer; matrices are [out_features, in_features]."""
    d, f = shape.d_model, shape.d_ffn
    dims = {
        "attn_norm": (d,), "wq": (shape.q_dim, d), "wk": (shape.kv_dim, d),
        "wv": (shape.kv_dim, d), "wo": (d, shape.q_dim), "mlp_norm": (d,),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }
    out = {}
    for tid, name in enumerate(_LAYER_TENSORS):
        s = tensor_seed(seed, 1, layer, tid)
        if name.endswith("norm"):
            out[name] = draw_normal_bf16(dims[name], 0.02, s, device, mean=1.0)
        else:
            out[name] = draw_normal_bf16(dims[name], 0.02, s, device)
    return out


def draw_head_weights(shape: ModelShape, seed: int, device="cpu"):
    """Embedding table, final norm gain and (untied) LM head, bf16."""
    V, d = shape.vocab, shape.d_model
    return {
        "embed": draw_normal_bf16((V, d), 0.02, tensor_seed(seed, 2, 0), device),
        "final_norm": draw_normal_bf16((d,), 0.02, tensor_seed(seed, 2, 1), device, mean=1.0),
        "lm_head": draw_normal_bf16((V, d), 0.02, tensor_seed(seed, 2, 2), device),
    }


def draw_batch(recipe: BatchRecipe, batch=None, seed=None):
    """Context lengths, chunk lengths and a page assignment for one batch.

    Returns a dict of numpy int32 arrays: ctx_len[B], n_draft[B], n_uncached[B]
    (zeros), block_table[B, max_pages] (-1 where unused), plus n_pages (pool
    size) and max_pages.  Each request owns ceil((L + MAX_CHUNK) / PAGE_SIZE)
    pages, drawn without replacement from a pool with 10 % slack; consecutive
    unless the recipe asks for a permuted pool.
    """
    B = recipe.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64(tensor_seed(recipe.seed if seed is None else seed, 3)))
    lo, hi = recipe.ctx_lo, recipe.ctx_hi
    if recipe.ctx_dist == "uniform":
        L = rng.integers(lo, hi + 1, size=B)
    elif recipe.ctx_dist == "loguniform":
        L = np.rint(np.exp(rng.uniform(math.log(lo), math.log(hi), size=B))).astype(np.int64)
    elif recipe.ctx_dist == "lognormal":
        L = np.rint(np.exp(rng.normal(math.log(recipe.ctx_median), recipe.ctx_sigma, size=B)))
        L = np.clip(L, lo, hi).astype(np.int64)
    else:
        raise ValueError(recipe.ctx_dist)
    L = np.clip(L, lo, hi)
    k = rng.integers(recipe.k_lo, recipe.k_hi + 1, size=B)
    need = (L + MAX_CHUNK + PAGE_SIZE - 1) // PAGE_SIZE
    total = int(need.sum())
    n_pages = int(math.ceil(total * 1.1))
    order = rng.permutation(n_pages) if recipe.permute_pages else np.arange(n_pages)
    max_pages = int(need.max())
    bt = np.full((B, max_pages), -1, dtype=np.int32)
    at = 0
    for i in range(B):
        bt[i, : need[i]] = order[at: at + need[i]]
        at += int(need[i])
    return {
        "ctx_len": L.astype(np.int32), "n_draft": k.astype(np.int32),
        "n_uncached": np.zeros(B, dtype=np.int32), "block_table": bt,
        "n_pages": n_pages, "max_pages": max_pages,
    }


def draw_context_tokens(recipe: BatchRecipe, ctx_len, seed=None):
    """Random token ids for each request's cached context (used when the recipe
    fills the cache by a real prefill)."""
    rng = np.random.Generator(np.random.PCG64(tensor_seed(recipe.seed if seed is None else seed, 4)))
    return [rng.integers(0, recipe.shape.vocab, size=int(n)).astype(np.int32) for n in ctx_len]


def draw_context_kv(shape: ModelShape, seed: int, layer: int, n_tokens: int, device="cpu"):
    """Stand-in cached K and V rows of one layer: N(0,1), bf16, each
    [n_tokens, n_kv_heads, head_dim] (flat over the requests of a batch)."""
    dims = (n_tokens, shape.n_kv_heads, shape.head_dim)
    k = draw_normal_bf16(dims, 1.0, tensor_seed(seed, 5, layer, 0), device)
    v = draw_normal_bf16(dims, 1.0, tensor_seed(seed, 5, layer, 1), device)
    return k, v


def draw_draft_randoms(recipe: BatchRecipe, batch=None, seed=None):
    """Random numbers a draft generator consumes: per (request, position) a
    uniform in [0,1) and a uniformly random token id, and per request one random
    'last context token'."""
    B = recipe.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64(tensor_seed(recipe.seed if seed is None else seed, 6)))
    V = recipe.shape.vocab
    return {
        "u": rng.random(size=(B, MAX_CHUNK)),
        "tok": rng.integers(0, V, size=(B, MAX_CHUNK)).astype(np.int32),
        "last_ctx_tok": rng.integers(0, V, size=B).astype(np.int32),
    }


def draw_confidence_logits(rows, vocab, std, boost_hi, seed, device="cpu", dtype=torch.bfloat16):
    """Logit rows ~ N(0, std^2) with one uniformly chosen entry per row raised by
    U[0, boost_hi]."""
    g = _gen(device, tensor_seed(seed, 7, 0))
    x = torch.randn((rows, vocab), generator=g, device=device, dtype=torch.float32)
    x.mul_(std)
    g2 = _gen(device, tensor_seed(seed, 7, 1))
    col = torch.randint(0, vocab, (rows,), generator=g2, device=device)
    boost = torch.rand((rows,), generator=g2, device=device, dtype=torch.float32) * boost_hi
    x[torch.arange(rows, device=device), col] += boost
    return x.to(dtype)
