"""Full-size parity on the 8B-shaped configs, in the launch configuration bench.py times.

The oracle follows a sample of the requests (chosen to include the shortest and longest context
and the shortest and longest chunk) element by element; for the others the HIP path's outputs are
checked through size-independent properties (accept/correction consistent with its own argmax rows,
argmax consistent with the returned logits, probabilities and entropies in range, no NaN although
every unwritten KV slot holds NaN).  The three configs share one set of 8B weights (drawn once) to
bound host time; each config draws its own batch.
"""
import os

import numpy as np
import pytest
import torch

import gpu_harness as gh
import paper_2511_07423_amd as synera
import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def weights_8b():
    w = gh.draw_weights(wl.LLAMA_8B, wl.config(2).seed, DEV)
    yield w
    del w
    torch.cuda.empty_cache()


def _run(n, n_oracle, weights, importance=False):
    case = gh.build_case(wl.config(n), DEV, n_oracle=n_oracle, weights=weights, verbose=True)
    out = gh.run_verify(case)
    rep = gh.compare_with_oracle(case, out)
    kv = gh.compare_kv(case)
    print(f"\n[c{n}] T={int(case.batch['n_draft'].sum())} sampled={case.sampled} rows={rep['rows_checked']} "
          f"max|dlogit|={rep['max_logit_err']:.3e} max rel dH={rep['max_entropy_rel']:.3e} "
          f"max rel dp={rep['max_prob_rel']:.3e} exempt rows/requests={rep['exempt_rows']}/{rep['exempt_requests']} "
          f"max|dKV|={kv['max_kv_err']:.3e} KV roundings differing: {kv['chunk_entries_differing']}/{kv['chunk_entries']} "
          f"(layer 0: {kv['layer0_entries_differing']}/{kv['layer0_entries']}) "
          f"accept_len mean={out['accept_len'].mean():.2f} "
          f"oracle chain {case.timing['oracle_chain_s']:.1f}s", flush=True)
    if importance:
        _check_importance(case)
    case.verifier.close()
    assert rep["ok"], rep["fail"]
    assert kv["ok"], kv["fail"]
    return case, out, rep


def _check_importance(case, n_sample=3):
    """Importance scores of the batch just verified (last layer, mean over heads) against the oracle's, for
    a few of the requests the oracle follows; the row-sum property for all."""
    b = case.batch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    imp = case.verifier.importance(b["ctx_len"], case.n_uncached, b["n_draft"], b["n_pages"], case.k_pool, i_th=0.05)
    e0.record()                                   # timed on a repeat: the first launch also loads the kernel
    imp = case.verifier.importance(b["ctx_len"], case.n_uncached, b["n_draft"], b["n_pages"], case.k_pool, i_th=0.05)
    e1.record()
    torch.cuda.synchronize()
    got, off = imp["scores"].cpu().numpy().astype(np.float64), imp["offsets"]
    assert np.isfinite(got).all() and (got >= 0).all()
    for i in range(len(b["ctx_len"])):
        assert abs(got[off[i]:off[i + 1]].sum() - b["n_draft"][i]) < 2e-3 * b["n_draft"][i]
    sample = case.sampled[:n_sample]
    want = oracle.importance_scores(case.model, case.okv, [(b["block_table"][i], int(b["ctx_len"][i]), case.drafts[i])
                                                           for i in sample])
    worst = 0.0
    for i, w in zip(sample, want):
        g = got[off[i]:off[i + 1]]
        worst = max(worst, float(np.max(np.abs(g - w) / (w + 1e-4))))
        assert np.all(np.abs(g - w) <= 3e-2 * w + 1e-5), i
    print(f"[importance] {e0.elapsed_time(e1) * 1e3:.0f} us for {off[-1]} scores, worst relative deviation "
          f"{worst:.2e} on requests {sample}", flush=True)


def test_config2_8b_batch16(weights_8b):
    case, out, rep = _run(2, 6, weights_8b)
    assert rep["rows_checked"] == 48


def test_config3_8b_ragged_batch64(weights_8b):
    case, out, rep = _run(3, 10, weights_8b, importance=True)
    k = case.batch["n_draft"]
    assert k.min() == 1 and k.max() == 16


def test_config5_8b_batch256_permuted_pool(weights_8b):
    case, out, rep = _run(5, 8, weights_8b)
    assert len(case.batch["ctx_len"]) == 256


def test_config4_70b_shape_cut_to_8_layers_with_a_draft_chain():
    """The 70B shape (d_model 8192, 64 query / 8 KV heads, FFN 28672, batch 32, contexts 1024..4096, k = 8) cut
    to its first 8 layers, so that the oracle can afford its sequential draft chain (nine passes over the
    weights) and accepted prefixes are exercised at this width.  NOT config 4 (that is the next test, at the
    full depth, held to the 2e-2 logits bar).  Ids, accept lengths, corrections, entropies and the cache are
    held to the same bars as everywhere; the logits bar here is the larger of 2e-2 and the distance at which the
    oracle's own float32 run lands from its float64 run on the same rows.  Why: at this width, with the stand-in
    context, chunk keys carry a large share of the attention weight, and one bf16 cache rounding that falls the
    other way (7 % of the chunk's entries do, at ANY working precision: 8 % with 16-bit activation pairs, 7 %
    with 22-bit ones) moves single logits by more than 2e-2; which entries flip is a property of the noise, not
    of the method."""
    import copy
    import dataclasses
    rec = wl.config(4)
    rec = dataclasses.replace(rec, shape=dataclasses.replace(rec.shape, n_layers=8))
    weights = gh.draw_weights(rec.shape, rec.seed, DEV)
    case = gh.build_case(rec, DEV, n_oracle=4, weights=weights, verbose=True)
    out = gh.run_verify(case)
    # the oracle once more in float32, on the same drafts and the same cache
    b, shape, model = case.batch, rec.shape, case.model
    model32 = oracle.OracleModel(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                                 shape.d_ffn, shape.vocab, model.embed, model._layers, model.final_norm, model.lm_head_w,
                                 rope_base=shape.rope_base, rms_eps=shape.rms_eps, dtype=np.float32)
    reqs = [{"block_table": b["block_table"][i], "ctx_len": int(b["ctx_len"][i]), "uncached": [], "drafts": case.drafts[i],
             "anchor": int(case.anchor[i])} for i in case.sampled]
    want32 = oracle.verify_chunks(model32, copy.deepcopy(case.okv), reqs)["logits"].astype(np.float64)
    floor = float(np.abs(want32 - np.concatenate([case.want_rows[i] for i in case.sampled])).max())
    rep = gh.compare_with_oracle(case, out, logit_tol=max(gh.LOGIT_TOL, floor))
    kv = gh.compare_kv(case)
    print(f"\n[70B shape, 8 layers] rows={rep['rows_checked']} max|dlogit|={rep['max_logit_err']:.3e} (float32 oracle vs "
          f"float64 oracle on the same rows: {floor:.3e}) "
          f"max rel dH={rep['max_entropy_rel']:.3e} exempt rows/requests={rep['exempt_rows']}/{rep['exempt_requests']} "
          f"max|dKV|={kv['max_kv_err']:.3e} KV roundings differing: {kv['chunk_entries_differing']}/{kv['chunk_entries']} "
          f"(layer 0: {kv['layer0_entries_differing']}/{kv['layer0_entries']}) "
          f"oracle chain {case.timing['oracle_chain_s']:.1f}s", flush=True)
    case.verifier.close()
    assert rep["ok"], rep["fail"]
    assert kv["ok"], kv["fail"]


def test_config4_70b_all_80_layers():
    """Config 4 at its full depth (140 GB of weights on the GPU).  The oracle widens one layer at a time from the
    device copy, so it can afford one pass over the 80 layers, not the nine of a greedy draft chain: the one-pass
    form of gpu_harness.one_pass_parity on a sample of the requests.  The same oracle run in float32 is printed
    beside it: how far a correct implementation in ordinary single precision lands from the float64 run at this
    depth (bf16 cache roundings flip where a value sits near a rounding boundary, and attention amplifies each
    flip from layer to layer)."""
    rec = wl.config(4)
    weights = gh.draw_weights(rec.shape, rec.seed, DEV, lazy_oracle=True)
    rep, kv = gh.one_pass_parity(rec, weights, DEV, n_requests=int(os.environ.get("SYNERA_C4_REQUESTS", "6")),
                                 float32_too=True, tag="c4 80 layers")
    assert rep["ok"], rep["fail"]
    assert kv["ok"], kv["fail"]
    assert rep["max_logit_err"] <= gh.LOGIT_TOL


@pytest.mark.parametrize("n,n_requests", [(2, None), (3, None), (5, 48)], ids=["c2_all16", "c3_all64", "c5_48of256"])
def test_every_request_element_wise_in_one_pass(weights_8b, n, n_requests):
    """The whole batch against the oracle, element by element, in the one-pass form (no input of the oracle comes
    from the HIP path): all 16 / all 64 requests of configs 2 and 3; of config 5's 256 requests as many as the
    host memory for their contexts and a few minutes of oracle time allow."""
    rec = wl.config(n)
    rep, kv = gh.one_pass_parity(rec, weights_8b, DEV, n_requests=n_requests)
    assert rep["ok"], rep["fail"]
    assert kv["ok"], kv["fail"]
    B = len(wl.draw_batch(rec)["ctx_len"])
    assert rep["requests_checked"] == (B if n_requests is None else n_requests)
    if n_requests is None:
        assert rep["rows_checked"] == int(wl.draw_batch(rec)["n_draft"].sum())


def test_config5b_standalone_confidence_full_size():
    import oracle
    from workloads import shapes
    x = wl.draw_confidence_logits(shapes.C5B_ROWS, shapes.C5B_VOCAB, shapes.C5B_STD, shapes.C5B_BOOST_HI,
                                  wl.config(5).seed, DEV, torch.bfloat16)
    ids, p, H = synera.confidence(x)
    torch.cuda.synchronize()
    ids, p, H = ids.cpu().numpy(), p.cpu().numpy(), H.cpu().numpy()
    rows = np.unique(np.concatenate([[0, shapes.C5B_ROWS - 1], np.random.default_rng(5).integers(0, shapes.C5B_ROWS, 62)]))
    wi, wp, wH, _ = oracle.confidence(x[rows].float().cpu().numpy().astype(np.float64))
    assert np.array_equal(ids[rows], wi)
    assert np.all(np.abs(p[rows] - wp) <= 1e-4 * wp) and np.all(np.abs(H[rows] - wH) <= 1e-3 * wH)
    # every row: the reported id is the row's maximum and p, H are in range
    mx = x.float().max(dim=1)
    assert torch.equal(x.float()[torch.arange(x.shape[0]), torch.from_numpy(ids).long().to(DEV)], mx.values)
    assert np.all(p > 0) and np.all(p <= 1) and np.all(H >= 0) and np.all(H <= np.log(shapes.C5B_VOCAB))
