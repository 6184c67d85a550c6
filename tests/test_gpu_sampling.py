"""synera_stochastic_accept against the speculative-sampling oracle.  The sampling step's inputs are the LLM's
logits rows, so the oracle is fed the HIP path's own logits (a second verify call that presents each request's
last uncached token as a draft returns the row the first distribution comes from); what is compared is the
sampling arithmetic: accept lengths and emitted tokens, exact except where a uniform number falls within
1e-5 of an acceptance ratio or within 1e-5 (relative) of a cumulative-weight boundary."""
import numpy as np
import pytest
import torch

import gpu_harness as gh
import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("vocab,k_list", [(256, 4), (2048, 8), (2048, 1), (2048, 64), (4096, 160), (4096, 256)])
def test_stochastic_accept_matches_the_oracle(vocab, k_list):
    import paper_2511_07423_amd as synera
    shape = wl.ModelShape("mini_sampling", 2, 128, 4, 2, 64, 256, vocab)
    head = wl.draw_head_weights(shape, 41, DEV)
    layers = [wl.draw_layer_weights(shape, 41, l, DEV) for l in range(shape.n_layers)]
    rng = np.random.default_rng(42 + vocab + k_list)
    B = 48
    ctx = rng.integers(0, 90, B).astype(np.int32)
    unc = rng.integers(1, 4, B).astype(np.int32)
    k = rng.integers(1, 9, B).astype(np.int32)
    need = (ctx + unc + k + 15) // 16
    n_pages, max_pages = int(need.sum()), int(need.max())
    bt = np.full((B, max_pages), -1, np.int32)
    at = 0
    for i in range(B):
        bt[i, :need[i]] = np.arange(at, at + need[i])
        at += int(need[i])
    kp = gh.nan_pool(shape, n_pages, DEV, False)
    vp = gh.nan_pool(shape, n_pages, DEV, True)
    ver = synera.Verifier(shape, head, layers, max_batch=B, max_tokens=int((ctx + unc + k).sum()) + B, max_pages=max_pages)
    zeros = np.zeros(B, np.int32)
    anchor = torch.zeros(B, dtype=torch.int32, device=DEV)
    # contexts: forwarded as uncached tokens in chunks of at most 31 (+ one marked row), by the HIP path itself
    ctx_tok = [rng.integers(0, vocab, int(c)) for c in ctx]
    done = np.zeros(B, np.int32)
    while (done < ctx).any():
        live = np.nonzero(done < ctx)[0]
        n = np.minimum(ctx[live] - done[live], 32)
        toks = np.concatenate([ctx_tok[i][done[i]:done[i] + m] for i, m in zip(live, n)]).astype(np.int32)
        ver.verify(done[live], (n - 1).astype(np.int32), np.ones(len(live), np.int32), torch.from_numpy(toks).to(DEV),
                   anchor[:len(live)], bt[live], n_pages, kp, vp, want_logits=False)
        done[live] += n
    chunk = [rng.integers(0, vocab, int(unc[i] + k[i])) for i in range(B)]
    tokens = torch.from_numpy(np.concatenate(chunk).astype(np.int32)).to(DEV)
    # call A: the last uncached token presented as a draft -> logits of the k + 1 rows the rule needs
    a = ver.verify(ctx, unc - 1, k + 1, tokens, anchor, bt, n_pages, kp, vp)
    logits = a["logits"].double().cpu().numpy()
    cu1 = np.concatenate([[0], np.cumsum(k + 1)])
    # the device's lists: its own (random) distribution per draft row, top k_list entries, drafts drawn from them
    R = int(k.sum())
    cu = np.concatenate([[0], np.cumsum(k)])
    p_id = np.zeros((R, k_list), np.int32)
    p_prob = np.zeros((R, k_list), np.float32)
    for i in range(B):
        for j in range(int(k[i])):
            # centred on the LLM's likely tokens so that acceptance ratios spread over (0, 1]
            row = logits[cu1[i] + j] + rng.normal(0, 1.0, vocab)
            ids, pr = oracle.topk_row(row, k_list)
            p_id[cu[i] + j], p_prob[cu[i] + j] = ids, pr
            pick = rng.choice(k_list, p=pr / pr.sum())
            chunk[i][unc[i] + j] = ids[pick] if rng.random() < 0.9 else rng.integers(0, vocab)   # some drafts off-list
    tokens = torch.from_numpy(np.concatenate(chunk).astype(np.int32)).to(DEV)
    # the drafts changed: forward again (call A'), then the real call B and the sampling step
    a = ver.verify(ctx, unc - 1, k + 1, tokens, anchor, bt, n_pages, kp, vp)
    logits = a["logits"].double().cpu().numpy()
    ver.verify(ctx, unc, k, tokens, anchor, bt, n_pages, kp, vp)
    # the small decoder's distributions are flat (q_x ~ 1 / vocab against p_x >= 1 / k_list): most uniforms are
    # drawn small so that acceptance chains of every length occur
    u_acc = (rng.random(R) * np.where(rng.random(R) < 0.7, 4.0 / vocab, 1.0)).astype(np.float32)
    u_smp = rng.random(B).astype(np.float32)
    acc, tok = ver.stochastic_accept(tokens, torch.from_numpy(p_id).to(DEV), torch.from_numpy(p_prob).to(DEV),
                                     torch.from_numpy(u_acc).to(DEV), torch.from_numpy(u_smp).to(DEV))
    torch.cuda.synchronize()
    acc, tok = acc.cpu().numpy(), tok.cpu().numpy()
    checked, lens = 0, []
    for i in range(B):
        rows = logits[cu1[i]:cu1[i + 1]]
        q = np.exp(rows - rows.max(axis=1, keepdims=True))
        q /= q.sum(axis=1, keepdims=True)
        lists = [(p_id[cu[i] + j], p_prob[cu[i] + j].astype(np.float64)) for j in range(int(k[i]))]
        n, t, info = oracle.speculative_accept(q, lists, chunk[i][unc[i]:], u_acc[cu[i]:cu[i + 1]].astype(np.float64),
                                               float(u_smp[i]))
        lens.append(n)
        if info["ratio_gap"] < 1e-5:
            continue
        assert acc[i] == n, i
        if info["cdf_gap"] < 1e-5:
            continue
        assert tok[i] == t, i
        checked += 1
    assert checked >= B * 3 // 4
    assert 0 < np.mean(np.asarray(lens) == k) < 1 and min(lens) == 0      # full accepts and early rejections both occur
    with pytest.raises(synera.SyneraError) as e:               # lists longer than 256 entries are not supported
        ver.stochastic_accept(tokens, torch.zeros((R, 257), dtype=torch.int32, device=DEV),
                              torch.ones((R, 257), dtype=torch.float32, device=DEV), torch.from_numpy(u_acc).to(DEV),
                              torch.from_numpy(u_smp).to(DEV))
    assert e.value.status == synera.EUNSUP
    # a request without an uncached token has no first distribution: refused
    ver.verify(ctx, zeros, k, tokens[:int(k.sum())], anchor, bt, n_pages, kp, vp)
    with pytest.raises(synera.SyneraError) as e:
        ver.stochastic_accept(tokens, torch.from_numpy(p_id).to(DEV), torch.from_numpy(p_prob).to(DEV),
                              torch.from_numpy(u_acc).to(DEV), torch.from_numpy(u_smp).to(DEV))
    assert e.value.status == synera.EUNSUP
    ver.close()
