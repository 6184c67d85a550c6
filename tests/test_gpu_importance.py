"""synera_importance against the oracle (Section 3.2: column-wise sum of the attention matrix, last layer,
mean over heads), on ragged requests with uncached tokens, contexts from empty to several key blocks
and permuted pages; plus the mean over the draft positions and P_imp (Section 4.2, second equation)."""
import numpy as np
import pytest
import torch

import gpu_harness as gh
import oracle
import workloads as wl
from helpers import oracle_model

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("shape", [wl.ModelShape("mini_gqa", 3, 128, 4, 2, 64, 256, 256),
                                   wl.ModelShape("mini_h128", 2, 256, 4, 1, 128, 256, 256)])
def test_importance_scores_match_the_oracle(shape):
    import paper_2511_07423_amd as synera
    head = wl.draw_head_weights(shape, 31, DEV)
    layers = [wl.draw_layer_weights(shape, 31, l, DEV) for l in range(shape.n_layers)]
    model = oracle_model(shape, head, layers, np.float64)
    rng = np.random.default_rng(32)
    ctx = np.array([0, 1, 15, 16, 250, 255, 256, 257, 700, 1500, 33], np.int32)
    unc = np.array([1, 0, 3, 0, 31, 0, 5, 16, 0, 2, 0], np.int32)
    k = np.array([4, 1, 2, 32, 1, 7, 9, 16, 3, 8, 11], np.int32)
    B = len(ctx)
    need = (ctx + unc + k + 15) // 16
    n_pages = int(need.sum()) + 5
    perm = rng.permutation(n_pages)
    max_pages = int(need.max()) + 1
    bt = np.full((B, max_pages), -1, np.int32)
    at = 0
    for i in range(B):
        bt[i, :need[i]] = perm[at:at + need[i]]
        at += int(need[i])
    okv = oracle.PagedKV(shape.n_layers, n_pages, shape.n_kv_heads, shape.head_dim)
    toks, items = [], []
    for i in range(B):
        if ctx[i] > 0:
            oracle.prefill_context(model, okv, bt[i], rng.integers(0, shape.vocab, int(ctx[i])))
        t = rng.integers(0, shape.vocab, int(unc[i] + k[i]))
        toks.append(t)
        items.append((bt[i], int(ctx[i]), t))
    kp = gh.nan_pool(shape, n_pages, DEV, False)
    vp = gh.nan_pool(shape, n_pages, DEV, True)
    kd, vd = gh._oracle_pool_to_device(okv, DEV)
    for i in range(B):
        for t0 in range(0, int(ctx[i]), 16):
            m = min(16, int(ctx[i]) - t0)
            kp[:, bt[i, t0 // 16], :, :m, :] = kd[:, bt[i, t0 // 16], :, :m, :]
            vp[:, bt[i, t0 // 16], :, :, :m] = vd[:, bt[i, t0 // 16], :, :, :m]
    want = oracle.importance_scores(model, okv, items)
    ver = synera.Verifier(shape, head, layers, max_batch=B, max_tokens=int((unc + k).sum()), max_pages=max_pages)
    with pytest.raises(synera.SyneraError):
        ver.importance(ctx, unc, k, n_pages, kp)                 # nothing verified yet
    tokens = torch.from_numpy(np.concatenate(toks).astype(np.int32)).to(DEV)
    ver.verify(ctx, unc, k, tokens, torch.zeros(B, dtype=torch.int32, device=DEV), bt, n_pages, kp, vp)
    i_th = 0.2
    out = ver.importance(ctx, unc, k, n_pages, kp, i_th=i_th)
    torch.cuda.synchronize()
    # the KV-head shares of a score are added in a fixed order: a second call returns the same bits
    again = ver.importance(ctx, unc, k, n_pages, kp, i_th=i_th)
    torch.cuda.synchronize()
    assert torch.equal(out["scores"], again["scores"])
    got = out["scores"].cpu().numpy().astype(np.float64)
    off = out["offsets"]
    worst = 0.0
    for i in range(B):
        g, w = got[off[i]:off[i + 1]], want[i]
        assert len(g) == len(w) == ctx[i] + unc[i] + k[i]
        assert abs(g.sum() - (unc[i] + k[i])) < 1e-3 * (unc[i] + k[i])         # every row hands out weight 1
        worst = max(worst, float(np.max(np.abs(g - w) / (w + 1e-3))))
        assert np.all(np.abs(g - w) <= 1e-3 * w + 1e-6), i           # shallow decoders: measured 5e-5
    print(f"\n[importance {shape.name}] worst relative deviation {worst:.3e}", flush=True)
    mean = out["mean"].cpu().numpy()
    p = out["p_imp"].cpu().numpy()
    for i in range(B):
        m = oracle.mean_draft_importance(got[off[i]:off[i + 1]], int(ctx[i]), int(unc[i]), int(k[i]))
        assert abs(mean[i] - m) <= 1e-5 * max(1.0, m)
        assert abs(p[i] - oracle.p_imp(float(mean[i]), i_th, -10.0)) <= 1e-5
    assert 0 < (p > 0).sum() and (p < 1).sum() > 0                 # the threshold splits this batch
    with pytest.raises(synera.SyneraError):
        ver.importance(ctx, unc, k + 1, n_pages, kp)             # not the batch that was verified
    # any later call that re-plans the batch metadata (here a raw K/V append) retires the verify's state
    rows = torch.zeros((1, shape.n_kv_heads, shape.head_dim), dtype=torch.bfloat16, device=DEV)
    ver.kv_append(0, ctx[:1] + unc[:1] + k[:1] - 1, np.ones(1, np.int32), rows, rows, bt[:1], n_pages, kp, vp)
    with pytest.raises(synera.SyneraError) as e:
        ver.importance(ctx, unc, k, n_pages, kp)
    assert e.value.status == synera.EINVAL
    ver.close()
