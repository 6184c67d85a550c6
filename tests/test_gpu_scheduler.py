"""The scheduler module in front of the HIP path: a scripted serving session (tests/sched_script.py, produced
by the oracle alone) is replayed against synera_sched_* + synera_verify on the GPU.  Every engine call must
carry the same requests, lengths and chunks as the oracle scheduler's, and its outputs must match the
oracle's verify of the same tokens: logits within 2e-2, greedy ids where the oracle's top-2 margin is at
least 1e-2, accept length and correction token where no row that decides them is closer than that."""
import numpy as np
import pytest
import torch

import workloads as wl
import gpu_harness as gh
import sched_script as ss

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
KIND = {"prefill": 1, "verify": 2}


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_scripted_session_matches_the_oracle(seed):
    import paper_2511_07423_amd as synera
    shape = wl.ModelShape("mini", 2, 128, 4, 2, 64, 256, 256)
    w = gh.draw_weights(shape, 9, DEV)
    n_pages, max_pages, max_batch, max_tokens = 80, 12, 4, 96
    sc = ss.make_script(w["model"], shape, seed, n_pages=n_pages, max_pages=max_pages, max_batch=max_batch,
                        max_tokens=max_tokens)
    assert len(sc.calls) > 30
    sched = synera.Scheduler(n_pages, max_pages, max_batch, max_tokens)
    ver = synera.Verifier(shape, w["head"], w["layers"], max_batch=max_batch, max_tokens=max_tokens,
                          max_pages=max_pages)
    k_pool = gh.nan_pool(shape, n_pages, DEV, False)
    v_pool = gh.nan_pool(shape, n_pages, DEV, True)
    arrivals = list(sc.arrivals)

    def replay():
        for what, i, a, b in arrivals.pop(0):
            {"prefill": lambda: sched.submit_prefill(i, a), "verify": lambda: sched.submit_verify(i, a, b),
             "finish": lambda: sched.finish(i)}[what]()

    n_call, checked_rows, checked_accepts, worst = 0, 0, 0, 0.0
    for n_calls in sc.iterations:
        replay()                                         # arrivals before the iteration
        if n_calls == 0:
            kind, out = sched.next()
            assert kind == synera.SCHED_IDLE
            continue
        for _ in range(n_calls):
            kind, out = sched.next()
            call = sc.calls[n_call]
            assert kind == KIND[call.kind]
            assert out["request_id"].tolist() == [it.request_id for it in call.items]
            assert out["ctx_len"].tolist() == [it.ctx_len for it in call.items]
            assert out["n_uncached"].tolist() == [it.n_uncached for it in call.items]
            assert out["n_draft"].tolist() == [it.n_draft for it in call.items]
            assert out["token_begin"].tolist() == [it.token_begin for it in call.items]
            assert out["final_verify"].tolist() == [int(it.final_verify) for it in call.items]
            tokens = torch.tensor([t for ts in call.tokens for t in ts], dtype=torch.int32, device=DEV)
            anchor = torch.tensor(call.anchors, dtype=torch.int32, device=DEV)
            res = ver.verify(out["ctx_len"].copy(), out["n_uncached"].copy(), out["n_draft"].copy(), tokens, anchor,
                             out["block_table"].copy(), n_pages, k_pool, v_pool)
            torch.cuda.synchronize()
            worst = max(worst, float(np.abs(res["logits"].double().cpu().numpy() - call.logits).max()))
            argmax = res["argmax"].cpu().numpy()
            acc = res["accept_len"].cpu().numpy()
            corr = res["correction"].cpu().numpy()
            at = 0
            for j, it in enumerate(call.items):
                rows = slice(at, at + it.n_draft)
                at += it.n_draft
                margins = np.asarray(call.margin[j])
                clear = margins >= 1e-2
                assert np.array_equal(argmax[rows][clear], np.asarray(call.argmax[j])[clear])
                checked_rows += int(clear.sum())
                if it.final_verify:
                    a = call.accept_len[j]
                    # rows that decide the result: the one that supplies q(x | prefix) and drafts 0 .. a-1
                    # (the greedy token after draft j decides draft j+1; after draft a-1, the correction)
                    deciding = [call.first_margin[j]] + list(margins[:a])
                    if min(deciding) >= 1e-2:
                        assert (int(acc[j]), int(corr[j])) == (a, call.correction[j])
                        checked_accepts += 1
            n_call += 1
            replay()                                     # arrivals while the call runs
            sched.commit([0 if a is None else a for a in call.accept_len])
    assert n_call == len(sc.calls) and worst <= 2e-2, worst
    assert checked_rows > 100 and checked_accepts > 15
    assert sched.stats()["engine_calls"] == len(sc.calls)
