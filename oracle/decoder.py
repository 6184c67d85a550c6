"""Plain Llama-style decoder over a paged KV cache (CPU oracle, numpy).

What is computed follows the paper's description of the cloud engine: the
tokens of a verification request are forwarded like a prefill, but against an
existing KV-cached prefix ("partial prefill", Section 3.4), the tokens of all
requests being flattened into one batch (Section 4.5).  Attention is
softmax(Q K^T / sqrt(d_k)) V (Section 3.2, the attention definition).  The
architecture details the paper leaves open (RMSNorm, rotary embedding on
adjacent pairs with base 10000, grouped-query attention with contiguous groups,
gated SiLU MLP, untied LM head) are the benchmark spec's.

Two independently written evaluation modes exist on purpose:
  * `decode_token`   - the literal definition: one token, explicit loops over
                       layers and heads, attends to everything cached so far;
  * `forward_tokens` - several tokens of several requests at once, layer by
                       layer, with a causal mask inside each request's chunk.
Their equality is one of the pins.

KV cache layout (an interface the HIP path must reproduce bit-exactly, written
here independently): position t of a request lives in page block_table[t // 16],
slot t % 16.  K pages are [kv_head][slot][dim]; V pages are [kv_head][dim][slot].
Values are stored as bf16.
"""
import math

import numpy as np

from .numerics import bf16_bits, bf16_from_bits

PAGE = 16


class OracleModel:
    """Shape parameters plus weights.

    `layers` is a list of dicts, or a callable layer -> dict (so a 70B model can
    be produced layer by layer); each dict holds float arrays with
    bf16-representable values: attn_norm[d], wq[Hq*h,d], wk[Hkv*h,d], wv[Hkv*h,d],
    wo[d,Hq*h], mlp_norm[d], w_gate[f,d], w_up[f,d], w_down[d,f].
    """

    def __init__(self, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
                 embed, layers, final_norm, lm_head, rope_base=10000.0, rms_eps=1e-5,
                 dtype=np.float64):
        self.n_layers, self.d_model = n_layers, d_model
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.d_ffn, self.vocab = d_ffn, vocab
        self.embed, self._layers, self.final_norm, self.lm_head_w = embed, layers, final_norm, lm_head
        self.rope_base, self.rms_eps = rope_base, rms_eps
        self.dtype = dtype

    def layer(self, l):
        return self._layers(l) if callable(self._layers) else self._layers[l]


class PagedKV:
    """bf16 paged KV pool.  With `pages` given, only those page ids are backed
    (a sparse pool, for oracle runs over a sample of a large batch)."""

    def __init__(self, n_layers, n_pages, n_kv_heads, head_dim, pages=None):
        self.n_layers, self.n_pages = n_layers, n_pages
        self.n_kv_heads, self.head_dim = n_kv_heads, head_dim
        if pages is None:
            self.slot_of = None
            n_backed = n_pages
        else:
            ids = sorted(set(int(p) for p in pages))
            self.slot_of = {p: s for s, p in enumerate(ids)}
            n_backed = len(ids)
        self.k = np.zeros((n_layers, n_backed, n_kv_heads, PAGE, head_dim), np.uint16)
        self.v = np.zeros((n_layers, n_backed, n_kv_heads, head_dim, PAGE), np.uint16)

    def _backing(self, page):
        page = int(page)
        if not 0 <= page < self.n_pages:
            raise IndexError(f"page id {page} outside pool of {self.n_pages}")
        return page if self.slot_of is None else self.slot_of[page]

    def append(self, layer, block_table_row, pos, k_row, v_row):
        """Store K and V of one position ([kv_head, dim] each), rounded to bf16."""
        b = self._backing(block_table_row[pos // PAGE])
        s = pos % PAGE
        self.k[layer, b, :, s, :] = bf16_bits(k_row)
        self.v[layer, b, :, :, s] = bf16_bits(v_row)

    def append_many(self, layer, block_table_row, start, k_rows, v_rows):
        """Store K and V of positions start..start+n-1 ([n, kv_head, dim] each), page by page."""
        n = len(k_rows)
        kb, vb = bf16_bits(k_rows), bf16_bits(v_rows)
        t = start
        while t < start + n:
            b = self._backing(block_table_row[t // PAGE])
            s = t % PAGE
            m = min(PAGE - s, start + n - t)
            self.k[layer, b, :, s:s + m, :] = kb[t - start:t - start + m].transpose(1, 0, 2)
            self.v[layer, b, :, :, s:s + m] = vb[t - start:t - start + m].transpose(1, 2, 0)
            t += m

    def gather(self, layer, block_table_row, n):
        """K and V of positions 0..n-1, widened to float32: [n, kv_head, dim] each."""
        n_pg = (n + PAGE - 1) // PAGE
        b = [self._backing(block_table_row[p]) for p in range(n_pg)]
        # [pages, kv_head, slot, dim] -> [pages*slot, kv_head, dim]; V pages are [kv_head, dim, slot]
        K = bf16_from_bits(self.k[layer, b]).transpose(0, 2, 1, 3).reshape(n_pg * PAGE, self.n_kv_heads, self.head_dim)
        V = bf16_from_bits(self.v[layer, b]).transpose(0, 3, 1, 2).reshape(n_pg * PAGE, self.n_kv_heads, self.head_dim)
        K, V = K[:n], V[:n]
        return K, V


def rmsnorm(x, g, eps, dtype=np.float64):
    """y = x / sqrt(mean(x^2) + eps) * g over the last axis."""
    x = np.asarray(x, dtype)
    ms = np.mean(x * x, axis=-1, keepdims=True, dtype=dtype)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype)


def rope(v, pos, base=10000.0, dtype=np.float64):
    """Rotate adjacent pairs (2i, 2i+1) of the last axis by pos * base^(-2i/h).

    The angle is formed in float64 whatever the working dtype.
    """
    v = np.asarray(v, dtype)
    h = v.shape[-1]
    i = np.arange(h // 2, dtype=np.float64)
    ang = float(pos) * base ** (-2.0 * i / h)
    c, s = np.cos(ang).astype(dtype), np.sin(ang).astype(dtype)
    out = np.empty_like(v)
    a, b = v[..., 0::2], v[..., 1::2]
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


def attention_one_query(q, K, V, dtype=np.float64):
    """softmax(q K^T / sqrt(h)) V for one query position.

    q [Hq, h]; K, V [n, Hkv, h] hold every visible position.  Query head hq uses
    KV head hq // (Hq // Hkv).  Returns [Hq, h].
    """
    Hq, h = q.shape
    G = Hq // K.shape[1]
    out = np.empty((Hq, h), dtype)
    for hq in range(Hq):
        kh = hq // G
        s = (np.asarray(K[:, kh, :], dtype) @ np.asarray(q[hq], dtype)) / math.sqrt(h)
        e = np.exp(s - s.max())
        p = e / e.sum(dtype=dtype)
        out[hq] = p @ np.asarray(V[:, kh, :], dtype)
    return out


def _silu(x):
    return x / (1.0 + np.exp(-x))


def decode_token(model, kv, block_table_row, pos, token):
    """The literal definition: forward ONE token at position `pos`, appending its
    K/V to the cache and attending to positions 0..pos.  Returns the final hidden
    state [d] (before the final norm)."""
    dt = model.dtype
    Hq, Hkv, h = model.n_q_heads, model.n_kv_heads, model.head_dim
    x = np.asarray(model.embed[token], dt).copy()
    for l in range(model.n_layers):
        w = model.layer(l)
        y = rmsnorm(x, w["attn_norm"], model.rms_eps, dt)
        q = (np.asarray(w["wq"], dt) @ y).reshape(Hq, h)
        k = (np.asarray(w["wk"], dt) @ y).reshape(Hkv, h)
        v = (np.asarray(w["wv"], dt) @ y).reshape(Hkv, h)
        q = rope(q, pos, model.rope_base, dt)
        k = rope(k, pos, model.rope_base, dt)
        kv.append(l, block_table_row, pos, k, v)
        K, V = kv.gather(l, block_table_row, pos + 1)
        o = attention_one_query(q, K, V, dt).reshape(Hq * h)
        x = x + np.asarray(w["wo"], dt) @ o
        y = rmsnorm(x, w["mlp_norm"], model.rms_eps, dt)
        a = _silu(np.asarray(w["w_gate"], dt) @ y) * (np.asarray(w["w_up"], dt) @ y)
        x = x + np.asarray(w["w_down"], dt) @ a
    return x


def forward_tokens(model, kv, items, attn_probe=None):
    """Partial prefill of a flattened ragged batch, layer by layer.

    items: list of (block_table_row, start_pos, tokens) - request i forwards
    len(tokens) tokens at positions start_pos.. against its cached prefix
    0..start_pos-1.  Chunk row j sees keys 0..start_pos+j (full prefix, causal
    inside the chunk).  K/V of every forwarded token are appended.  Returns the
    final hidden states [T, d] in flattened order.

    attn_probe: optional (layer, list); the attention matrices softmax(Q K^T / sqrt(h)) of that layer are
    appended to the list, one array [Hq, n, keys] per item (zero where a key is not visible).
    """
    dt = model.dtype
    Hq, Hkv, h = model.n_q_heads, model.n_kv_heads, model.head_dim
    G = Hq // Hkv
    toks = np.concatenate([np.asarray(t, np.int64) for _, _, t in items])
    x = np.asarray(model.embed[toks], dt)
    T = x.shape[0]
    for l in range(model.n_layers):
        w = model.layer(l)
        y = rmsnorm(x, w["attn_norm"], model.rms_eps, dt)
        q = (y @ np.asarray(w["wq"], dt).T).reshape(T, Hq, h)
        k = (y @ np.asarray(w["wk"], dt).T).reshape(T, Hkv, h)
        v = (y @ np.asarray(w["wv"], dt).T).reshape(T, Hkv, h)
        o = np.empty((T, Hq, h), dt)
        r0 = 0
        for bt, start, t in items:
            n = len(t)
            for j in range(n):
                q[r0 + j] = rope(q[r0 + j], start + j, model.rope_base, dt)
                k[r0 + j] = rope(k[r0 + j], start + j, model.rope_base, dt)
                kv.append(l, bt, start + j, k[r0 + j], v[r0 + j])
            K, V = kv.gather(l, bt, start + n)
            K, V = np.asarray(K, dt), np.asarray(V, dt)
            key_pos = np.arange(start + n)
            visible = key_pos[None, :] <= (start + np.arange(n))[:, None]      # [n, keys]
            probed = np.empty((Hq, n, start + n), dt) if attn_probe is not None and attn_probe[0] == l else None
            for hq in range(Hq):
                s = (q[r0:r0 + n, hq, :] @ K[:, hq // G, :].T) / math.sqrt(h)
                s = np.where(visible, s, -np.inf)
                e = np.exp(s - s.max(axis=1, keepdims=True))
                p = e / e.sum(axis=1, keepdims=True, dtype=dt)
                o[r0:r0 + n, hq, :] = p @ V[:, hq // G, :]
                if probed is not None:
                    probed[hq] = p
            if probed is not None:
                attn_probe[1].append(probed)
            r0 += n
        x = x + o.reshape(T, Hq * h) @ np.asarray(w["wo"], dt).T
        y = rmsnorm(x, w["mlp_norm"], model.rms_eps, dt)
        a = _silu(y @ np.asarray(w["w_gate"], dt).T) * (y @ np.asarray(w["w_up"], dt).T)
        x = x + a @ np.asarray(w["w_down"], dt).T
    return x


def lm_head(model, x):
    """logits = rmsnorm(x; final gain) W_lm^T for one row [d] or rows [R, d]."""
    dt = model.dtype
    y = rmsnorm(x, model.final_norm, model.rms_eps, dt)
    return y @ np.asarray(model.lm_head_w, dt).T
