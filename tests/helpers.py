"""Glue shared by the tests: turns drawn inputs into what the oracle consumes."""
import numpy as np
import torch

import oracle
import workloads as wl


def to_np(t):
    """torch tensor (any float dtype, any device) -> float32 numpy, exact for bf16."""
    return t.detach().to("cpu", torch.float32).numpy()


def drawn_model(shape, seed, device="cpu"):
    """All weights of a model as torch bf16 tensors: (head dict, list of layer dicts)."""
    head = wl.draw_head_weights(shape, seed, device)
    layers = [wl.draw_layer_weights(shape, seed, l, device) for l in range(shape.n_layers)]
    return head, layers


def oracle_model(shape, head, layers, dtype=np.float64):
    """Build the oracle's model from drawn torch weights (host copies, widened exactly).
    `layers` may be a list of dicts or a callable layer -> dict of torch tensors."""
    if callable(layers):
        lay = lambda l: {k: to_np(v) for k, v in layers(l).items()}   # noqa: E731
    else:
        lay = [{k: to_np(v) for k, v in d.items()} for d in layers]
    return oracle.OracleModel(
        shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
        shape.d_ffn, shape.vocab, to_np(head["embed"]), lay, to_np(head["final_norm"]),
        to_np(head["lm_head"]), rope_base=shape.rope_base, rms_eps=shape.rms_eps, dtype=dtype)


def small_shape(**kw):
    base = dict(name="mini", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16,
                d_ffn=96, vocab=50)
    base.update(kw)
    return wl.ModelShape(**base)
