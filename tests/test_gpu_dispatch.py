"""GPU parity of the richer vocabulary reduction (top-k compressed distribution, margin score) and of the
chunk dispatch probability against the CPU oracle, through the C ABI.  Ids bit-exact; probabilities
1e-4 relative, entropy 1e-3 relative (the standalone confidence tolerances), margin 1e-4 absolute."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import shapes

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _synera():
    import paper_2511_07423_amd as synera
    return synera


def _check_topk(x_t, k, name):
    synera = _synera()
    ids, pr, mg, H = synera.confidence_topk(x_t, k)
    torch.cuda.synchronize()
    x = x_t.detach().to("cpu", torch.float32).numpy().astype(np.float64)
    wi, wp, wm = oracle.topk(x, k)
    _, _, wH, _ = oracle.confidence(x)
    ids, pr, mg, H = ids.cpu().numpy(), pr.cpu().numpy(), mg.cpu().numpy(), H.cpu().numpy()
    assert np.array_equal(ids, wi), f"{name}: ids differ at rows {np.nonzero((ids != wi).any(1))[0][:8]}"
    assert np.all(np.abs(pr - wp) <= 1e-4 * wp + 1e-12), f"{name}: prob rel err {np.max(np.abs(pr - wp) / (wp + 1e-300)):.3e}"
    assert np.all(np.abs(mg - wm) <= 1e-4), f"{name}: margin err {np.max(np.abs(mg - wm)):.3e}"
    assert np.all(np.abs(H - wH) <= 1e-3 * wH + 1e-6), f"{name}: entropy err {np.max(np.abs(H - wH)):.3e}"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("rows,vocab,k", [(1, 8, 8), (3, 40, 3), (5, 1000, 8), (7, 4096, 1), (4, 32000, 4),
                                          (2, 128256, 8), (9, 1037, 5), (6, 2050, 2),
                                          (3, 40, 9), (2, 64, 64), (5, 1000, 64), (4, 32000, 64), (3, 32000, 160),
                                          (2, 128256, 256), (5, 1037, 129), (3, 300, 256), (2, 2050, 65)])
def test_topk_matches_oracle(dtype, rows, vocab, k):
    g = torch.Generator(device=DEV).manual_seed(rows * 100003 + vocab + k)
    wide = (vocab + 7) // 8 * 8                      # rows must start 16-byte aligned; the tail may be ragged
    x = (torch.randn((rows, wide), generator=g, device=DEV) * 3).to(dtype)[:, :vocab]
    _check_topk(x, k, f"{rows}x{vocab} k={k}")


def test_topk_ties_plateaus_and_degenerate_rows():
    V = 4096
    x = torch.zeros((6, V), device=DEV)
    x[1, 5] = 3.0; x[1, 4000] = 3.0; x[1, 17] = 3.0          # three-way tie for the top: lowest ids first
    x[2, :] = torch.arange(V, device=DEV) % 7                 # plateaus of equal values across all threads
    x[3, V - 1] = 50.0                                        # one-hot in the last column
    x[4, :] = -1e4; x[4, 100] = -9e3                          # large negative logits
    x[5, ::2] = 1.0                                           # half the vocabulary tied
    for dt in (torch.float32, torch.bfloat16):
        for k in (8, 64, 200):
            _check_topk(x.to(dt), k, f"degenerate {dt} k={k}")
    # bf16 rounding creates many exact ties among the largest values of a random row
    g = torch.Generator(device=DEV).manual_seed(9)
    y = (torch.randn((8, 32000), generator=g, device=DEV) * 0.05 + 4.0).to(torch.bfloat16)
    for k in (8, 64, 160, 256):
        _check_topk(y, k, f"bf16 ties k={k}")


def test_topk_first_entry_equals_plain_confidence_and_errors():
    synera = _synera()
    x = wl.draw_confidence_logits(64, shapes.C5B_VOCAB, shapes.C5B_STD, shapes.C5B_BOOST_HI, 77, DEV, torch.bfloat16)
    ids, pr, mg, H = synera.confidence_topk(x, 4)
    i1, p1, H1 = synera.confidence(x)
    torch.cuda.synchronize()
    assert torch.equal(ids[:, 0], i1)
    assert torch.allclose(pr[:, 0], p1, rtol=1e-6, atol=0) and torch.allclose(H, H1, rtol=1e-6, atol=1e-7)
    assert torch.all(pr[:, :-1] >= pr[:, 1:]) and torch.all(mg >= 0)
    with pytest.raises(synera.SyneraError) as e:
        synera.confidence_topk(x, 257)
    assert e.value.status == synera.EUNSUP
    big, pbig, _, _ = synera.confidence_topk(x, 160)             # the first entries of a longer list are the shorter list
    assert torch.equal(big[:, :4], ids) and torch.allclose(pbig[:, :4], pr, rtol=1e-6, atol=0)
    with pytest.raises(synera.SyneraError) as e:
        synera.confidence_topk(x[:, :4], 8)
    assert e.value.status in (synera.EUNSUP, synera.EINVAL)


def test_topk_full_size_sampled_rows():
    """The 2048 x 128256 bf16 block of the standalone confidence workload: sampled rows against the oracle,
    every row against properties that hold at any size."""
    synera = _synera()
    x = wl.draw_confidence_logits(shapes.C5B_ROWS, shapes.C5B_VOCAB, shapes.C5B_STD, shapes.C5B_BOOST_HI,
                                  wl.config(5).seed, DEV, torch.bfloat16)
    ids, pr, mg, H = synera.confidence_topk(x, 8)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, shapes.C5B_ROWS - 1], np.random.default_rng(6).integers(0, shapes.C5B_ROWS, 14)]))
    xs = x[torch.from_numpy(rows).to(DEV)].float().cpu().numpy().astype(np.float64)
    wi, wp, wm = oracle.topk(xs, 8)
    assert np.array_equal(ids.cpu().numpy()[rows], wi)
    assert np.all(np.abs(pr.cpu().numpy()[rows] - wp) <= 1e-4 * wp + 1e-12)
    assert np.all(np.abs(mg.cpu().numpy()[rows] - wm) <= 1e-4)
    # the values at the reported ids are the row's 8 largest, in order
    got = torch.gather(x.float(), 1, ids.long())
    top = torch.topk(x.float(), 8, dim=1).values
    assert torch.equal(got, top)
    assert torch.all(pr.sum(1) <= 1 + 1e-5) and torch.all(pr > 0)


def test_chunk_dispatch_matches_oracle():
    synera = _synera()
    rng = np.random.default_rng(11)
    k = rng.integers(0, 17, 300)                                  # empty chunks included
    cu = np.concatenate([[0], np.cumsum(k)]).astype(np.int32)
    p1 = rng.beta(5, 1, int(cu[-1])).astype(np.float32)
    p1[: int(k[0])] = 1.0                                         # a chunk of full confidence: c = 1
    for c_th in (0.7, 0.85, 0.99):
        mean, pc = synera.chunk_dispatch(torch.from_numpy(p1).to(DEV), torch.from_numpy(cu).to(DEV), c_th)
        torch.cuda.synchronize()
        wm, wp = oracle.chunk_dispatch(p1.astype(np.float64), cu, c_th)
        assert np.allclose(mean.cpu().numpy(), wm, rtol=1e-6, atol=1e-7)
        got = pc.cpu().numpy()
        # near the threshold P_conf jumps from 1 to 0.993: compare only where the mean is clear of it
        clear = np.abs(wm - c_th) > 1e-5
        assert np.allclose(got[clear], wp[clear], rtol=2e-4, atol=1e-6)
        assert np.all((got == 1.0) | (got < 0.9934))
    with pytest.raises(synera.SyneraError):
        synera.chunk_dispatch(torch.from_numpy(p1).to(DEV), torch.from_numpy(cu).to(DEV), 1.0)


@pytest.mark.parametrize("top_p", [0.1, 0.5, 0.9, 0.999, 1.0])
def test_topp_count_is_bit_exact_with_the_oracle(top_p):
    """Nucleus size inside the transmitted top-k window: the count is an integer decided by a float32 running
    sum in list order on both sides, so it must agree exactly; the mass to float32 rounding."""
    import paper_2511_07423_amd as synera
    x = wl.draw_confidence_logits(300, 4096, 3.0, 6.0, 77, DEV, torch.float32)
    x[7] = 0.0                                                   # uniform row: the window never reaches top_p
    x[8, 5] = 80.0                                               # one-hot row
    ids, pr, _, _ = synera.confidence_topk(x, 8)
    n, mass = synera.topp_count(pr, top_p)
    torch.cuda.synchronize()
    prh = pr.cpu().numpy()
    for r in range(x.shape[0]):
        want_n, want_mass = oracle.topp_count(prh[r], top_p)
        assert int(n[r]) == want_n, r
        assert abs(float(mass[r]) - want_mass) <= 1e-6
    assert int(n[7]) == 8 and int(n[8]) == 1
    with pytest.raises(synera.SyneraError):
        synera.topp_count(pr, 0.0)


def _check_nucleus(x_t, top_p, name):
    """Full-vocabulary nucleus against the oracle.  Where the oracle's running sum clears top_p by more than 1e-5
    on both sides of the cut, the size and the cut logit must agree exactly and the mass to 1e-5.  Elsewhere the
    size is an integer decided within rounding of a tie: the reported size must then be A valid nucleus size,
    i.e. the oracle's sorted probabilities reach top_p - 2e-6 with that many tokens and stay below top_p + 2e-6
    with one fewer."""
    synera = _synera()
    n, mass, cut = synera.nucleus(x_t, top_p)
    torch.cuda.synchronize()
    x = x_t.detach().to("cpu", torch.float32).numpy().astype(np.float64)
    n, mass, cut = n.cpu().numpy(), mass.cpu().numpy(), cut.cpu().numpy()
    loose = 0
    for r in range(x.shape[0]):
        wn, wmass, wcut, gap = oracle.nucleus_row(x[r], top_p)
        if gap >= 1e-5:
            assert int(n[r]) == wn, (name, r, int(n[r]), wn)
            assert abs(float(mass[r]) - wmass) <= 1e-5, (name, r)
            assert float(cut[r]) == wcut, (name, r)
            continue
        loose += 1
        order, pr = oracle.topk_row(x[r], x.shape[1])
        cum = np.cumsum(pr)
        g = int(n[r])
        assert 1 <= g <= x.shape[1], (name, r)
        assert cum[g - 1] >= top_p - 2e-6 and (g == 1 or cum[g - 2] < top_p + 2e-6), (name, r, g, wn)
        assert abs(float(mass[r]) - cum[g - 1]) <= 1e-5 and float(cut[r]) == x[r][order[g - 1]], (name, r)
    return loose


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("rows,vocab", [(3, 8), (5, 1000), (4, 32000), (2, 128256), (6, 1037)])
def test_nucleus_matches_oracle(dtype, rows, vocab):
    g = torch.Generator(device=DEV).manual_seed(rows * 7919 + vocab)
    wide = (vocab + 7) // 8 * 8
    x = (torch.randn((rows, wide), generator=g, device=DEV) * 3).to(dtype)[:, :vocab]
    for top_p in (0.05, 0.5, 0.9, 0.99, 0.9999):         # the last ones cut deep in the tail, among tiny probabilities
        _check_nucleus(x, top_p, f"{rows}x{vocab} p={top_p}")
    assert _check_nucleus(x, 0.05, "clear of ties") + _check_nucleus(x, 0.5, "clear of ties") <= 2


def test_nucleus_ties_one_hot_masked_and_uniform_rows():
    synera = _synera()
    V = 4096
    x = torch.zeros((6, V), device=DEV)
    x[1, 5] = 3.0; x[1, 4000] = 3.0; x[1, 17] = 3.0          # three tied leaders
    x[2, :] = (torch.arange(V, device=DEV) % 7).float()      # plateaus
    x[3, V - 1] = 50.0                                        # one-hot
    x[4, :] = float("-inf"); x[4, 10:20] = torch.arange(10, device=DEV).float()   # masked row: ten live tokens
    x[5, ::2] = 1.0
    for top_p in (0.3, 0.5, 0.75, 0.999):
        _check_nucleus(x, top_p, f"special p={top_p}")
    n, mass, cut = synera.nucleus(x, 0.5)
    assert int(n[0]) == V // 2 and int(n[3]) == 1 and float(cut[3]) == 50.0
    n, _, _ = synera.nucleus(x, 1.0)
    assert int(n[4]) <= 10
    # the nucleus is a prefix of the top-k order: its mass equals the sum of the first n list entries
    g = torch.Generator(device=DEV).manual_seed(3)
    y = torch.randn((16, 32000), generator=g, device=DEV) * 4
    n, mass, cut = synera.nucleus(y, 0.9)
    ids, pr, _, _ = synera.confidence_topk(y, 256)
    torch.cuda.synchronize()
    for r in range(16):
        k = int(n[r])
        if k <= 256:
            assert abs(float(pr[r, :k].sum()) - float(mass[r])) < 1e-5
            assert float(y[r, ids[r, k - 1].long()]) == float(cut[r])
    with pytest.raises(synera.SyneraError):
        synera.nucleus(y, 0.0)
    with pytest.raises(synera.SyneraError):
        synera.nucleus(y, 1.5)
