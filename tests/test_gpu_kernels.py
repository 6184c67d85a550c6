"""GPU parity of the stand-alone entry points (confidence, KV append, GEMM) through the C ABI."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _synera():
    import paper_2511_07423_amd as synera
    return synera


def _check_conf(logits_t, name):
    synera = _synera()
    ids, p, H = synera.confidence(logits_t)
    torch.cuda.synchronize()
    x = logits_t.detach().to("cpu", torch.float32).numpy().astype(np.float64)
    wi, wp, wH, mg = oracle.confidence(x)
    ids, p, H = ids.cpu().numpy(), p.cpu().numpy(), H.cpu().numpy()
    assert np.array_equal(ids, wi), f"{name}: argmax differs at rows {np.nonzero(ids != wi)[0][:8]}"
    assert np.all(np.abs(p - wp) <= 1e-4 * wp + 1e-12), f"{name}: prob rel err {np.max(np.abs(p - wp) / wp):.3e}"
    assert np.all(np.abs(H - wH) <= 1e-3 * wH + 1e-6), f"{name}: entropy err {np.max(np.abs(H - wH)):.3e}"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("rows,vocab", [(1, 8), (3, 40), (5, 1000), (7, 4096), (4, 32000), (2, 128256), (9, 1037)])
def test_confidence_matches_oracle(dtype, rows, vocab):
    g = torch.Generator(device=DEV).manual_seed(rows * 100003 + vocab)
    wide = (vocab + 7) // 8 * 8                      # rows must start 16-byte aligned; the tail may be ragged
    x = (torch.randn((rows, wide), generator=g, device=DEV) * 3).to(dtype)[:, :vocab]
    _check_conf(x, f"{rows}x{vocab}")


def test_confidence_workload_recipe_strided_and_ties():
    synera = _synera()
    x = wl.draw_confidence_logits(64, 128256, 3.0, 10.0, 42, DEV, torch.bfloat16)
    _check_conf(x, "c5b recipe")
    # rows taken from a wider buffer (stride > vocab), f32
    wide = torch.randn((6, 2048), device=DEV)
    _check_conf(wide[:, :1000], "strided")
    # exact ties: lowest id wins, also across threads / wavefronts / vector lanes
    t = torch.zeros((4, 5000), device=DEV)
    t[0, [4097, 13, 4999]] = 2.0
    t[1, [4999]] = 1.0
    t[2, :] = -7.5
    t[3, [1027, 1026]] = 0.5
    ids, p, H = synera.confidence(t)
    assert ids.cpu().tolist() == [13, 4999, 0, 1026]
    assert p[2].item() == pytest.approx(1 / 5000, rel=1e-5) and H[2].item() == pytest.approx(math.log(5000), rel=1e-5)
    # peaked rows: p -> 1, H -> 0
    t = torch.full((2, 4096), -50.0, device=DEV)
    t[0, 7] = 50.0
    t[1, 4095] = 0.0
    ids, p, H = synera.confidence(t)
    assert ids.cpu().tolist() == [7, 4095] and p[0].item() == 1.0 and abs(H[0].item()) < 1e-6
    # empty input is a no-op
    ids, _, _ = synera.confidence(torch.empty((0, 128), device=DEV))
    assert ids.numel() == 0


def test_rows_without_finite_entries_report_token_zero():
    """A row of NaN logits must not produce an id outside the vocabulary (it would be followed as a
    token id by a caller that feeds corrections back in)."""
    synera = _synera()
    t = torch.full((3, 4096), float("nan"), device=DEV)
    t[1] = torch.randn(4096, device=DEV)
    ids, _, _ = synera.confidence(t)
    ids = ids.cpu().tolist()
    assert ids[0] == 0 and ids[2] == 0 and 0 <= ids[1] < 4096


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_masked_logits_carry_probability_zero_and_finite_entropy(dtype):
    """Rows filtered by top-k / top-p masking hold -inf almost everywhere: most threads of the block see nothing but
    -inf, others a mix; probability and entropy must be those of the finite entries alone."""
    synera = _synera()
    g = torch.Generator(device=DEV).manual_seed(17)
    x = (torch.randn((6, 32000), generator=g, device=DEV) * 3).to(dtype)
    keep = [torch.tensor([5]), torch.tensor([31999, 0]), torch.arange(100, 140), torch.randint(0, 32000, (50,), generator=g, device=DEV).cpu(),
            torch.arange(0, 32000, 7), torch.arange(31990, 32000)]
    for r, idx in enumerate(keep):
        m = torch.full((32000,), float("-inf"), device=DEV, dtype=dtype)
        m[idx.to(DEV)] = x[r, idx.to(DEV)]
        x[r] = m
    _check_conf(x, "masked rows")
    ids, p, H = synera.confidence(x)
    assert p[0].item() == 1.0 and H[0].item() == 0.0
    tk_id, tk_p, margin, Hk = synera.confidence_topk(x, 4)
    torch.cuda.synchronize()
    assert torch.isfinite(Hk).all() and torch.allclose(Hk, H, rtol=1e-5, atol=1e-6)
    assert tk_id[1].cpu().tolist()[:2] == sorted([0, 31999], key=lambda i: (-float(x[1, i]), i))
    assert tk_p[0].cpu().tolist() == [1.0, 0.0, 0.0, 0.0]


def test_confidence_rejects_bad_arguments():
    synera = _synera()
    x = torch.zeros((4, 1001), device=DEV, dtype=torch.bfloat16)   # row stride not 16-byte aligned
    with pytest.raises(synera.SyneraError) as e:
        synera.confidence(x)
    assert e.value.status == synera.EINVAL


def _mini_shape():
    return wl.ModelShape("mini", 2, 128, 4, 2, 64, 256, 256)


def test_kv_append_is_bit_exact_and_touches_nothing_else():
    synera = _synera()
    shape = _mini_shape()
    head = wl.draw_head_weights(shape, 9, DEV)
    layers = [wl.draw_layer_weights(shape, 9, l, DEV) for l in range(shape.n_layers)]
    rng = np.random.default_rng(3)
    B, n_pages, max_pages = 5, 40, 6
    perm = rng.permutation(n_pages)
    bt = perm[: B * max_pages].reshape(B, max_pages).astype(np.int32)
    start = np.array([0, 3, 16, 31, 40], np.int32)
    n_new = np.array([33, 1, 16, 2, 50], np.int32)
    ver = synera.Verifier(shape, head, layers, max_batch=B, max_tokens=64, max_pages=max_pages)
    kp = torch.full((2, n_pages, 2, 16, 64), float("nan"), dtype=torch.bfloat16, device=DEV)
    vp = torch.full((2, n_pages, 2, 64, 16), float("nan"), dtype=torch.bfloat16, device=DEV)
    okv = oracle.PagedKV(2, n_pages, 2, 64)
    nan_bits = int(torch.tensor(float("nan"), dtype=torch.bfloat16).view(torch.int16).item()) & 0xFFFF
    okv.k[:] = nan_bits
    okv.v[:] = nan_bits
    for layer in range(2):
        k = wl.draw_normal_bf16((int(n_new.sum()), 2, 64), 1.0, 100 + layer, DEV)
        v = wl.draw_normal_bf16((int(n_new.sum()), 2, 64), 1.0, 200 + layer, DEV)
        ver.kv_append(layer, start, n_new, k, v, bt, n_pages, kp, vp)
        at = 0
        for i in range(B):
            rows = slice(at, at + int(n_new[i]))
            okv.append_many(layer, bt[i], int(start[i]), k[rows].float().cpu().numpy(), v[rows].float().cpu().numpy())
            at += int(n_new[i])
    torch.cuda.synchronize()
    assert np.array_equal(kp.view(torch.int16).cpu().numpy().view(np.uint16), okv.k)
    assert np.array_equal(vp.view(torch.int16).cpu().numpy().view(np.uint16), okv.v)
    # error paths: nothing is launched, the pools stay as they were
    before = kp.clone()
    bad = bt.copy()
    bad[1, 0] = bt[0, 0]
    for kwargs, code in ((dict(block_table=bad), synera.ERANGE), (dict(layer=2), synera.EINVAL),
                         (dict(n_new=np.array([33, 1, 16, 2, 57], np.int32)), synera.ENOSPC)):
        args = dict(layer=0, ctx_len=start, n_new=n_new, k=k, v=v, block_table=bt, n_pages_in_pool=n_pages,
                    k_pool=kp, v_pool=vp)
        args.update(kwargs)
        with pytest.raises(synera.SyneraError) as e:
            ver.kv_append(**args)
        assert e.value.status == code
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), kp.view(torch.int16))
    ver.close()


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (16, 256, 256), (130, 384, 512), (128, 4096, 4096),
                                   (544, 1024, 14336), (257, 32000, 256)])
def test_gemm_matches_float64(M, N, K):
    synera = _synera()
    x = wl.draw_normal_bf16((M, K), 1.0, 11 * M + K, DEV).float() * 1.37
    a, al = synera.split_pair(x)
    w = wl.draw_normal_bf16((N, K), 0.02, 13 * N + K, DEV)
    c = synera.gemm_pair(a, al, w)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, M - 1], np.random.default_rng(M).integers(0, M, 6)]))
    want = (a[rows].double() + al[rows].double()).cpu() @ w.double().cpu().T
    got = c[rows].double().cpu()
    scale = 0.02 * math.sqrt(K)
    assert torch.isfinite(c).all()
    assert (got - want).abs().max().item() < 6e-9 * K + 2e-7
    # full comparison against the fp32 library product on the device (looser: its own rounding)
    ref = x @ w.float().T
    assert (c - ref).abs().max().item() < 1e-3 * scale + 1e-5


def test_pair_carries_22_bits_and_weights_of_any_magnitude_below_256_are_exact():
    """The fp16 pair must reproduce an fp32 activation to 2^-22 (elements far below the row's scale included: their
    low parts are subnormal in fp16), and the weight's path bf16 -> fp16 with a raised exponent must be exact
    from 2^-22 up to 255."""
    synera = _synera()
    M, N, K = 48, 256, 512
    g = torch.Generator(device=DEV).manual_seed(5)
    x = torch.randn((M, K), generator=g, device=DEV) * torch.exp2(torch.randint(-12, 6, (M, K), generator=g, device=DEV).float())
    a, al = synera.split_pair(x)
    assert ((a.double() + al.double()) - x.double()).abs().max().item() <= 2.0 ** -22 * x.abs().max().item()
    mag = torch.exp2(torch.randint(-21, 8, (N, K), generator=g, device=DEV).float())
    w = (mag * (1 + torch.rand((N, K), generator=g, device=DEV) * 0.99) * (torch.randint(0, 2, (N, K), generator=g, device=DEV) * 2 - 1)).to(torch.bfloat16)
    w[0, :] = 0
    w[1, 0] = 255.0
    c = synera.gemm_pair(a, al, w)
    torch.cuda.synchronize()
    xd, wd = a.double() + al.double(), w.double()
    want = xd @ wd.T
    bound = 2e-6 * (xd.abs() @ wd.abs().T) + 1e-30       # fp32 accumulation of K terms; nothing of order 2^-8 (a bf16 step)
    assert ((c.double() - want).abs() <= bound).all()
    assert (c[:, 0] == 0).all()


@pytest.mark.parametrize("tile", [-1, 1, 5, 8, 9, 12, 17, 103, 112, 201, 205, 301, 309])
@pytest.mark.parametrize("M,N,K", [(1, 256, 64), (97, 512, 1024), (532, 1024, 4096), (545, 1792, 512), (272, 32000, 256)])
def test_gemm_on_the_high_part_alone(tile, M, N, K):
    """The single-term form (the LM head's): exactly the product of the fp16 high part with the weights."""
    synera = _synera()
    g = torch.Generator(device=DEV).manual_seed(3 * M + N + K)
    a = torch.randn((M, K), generator=g, device=DEV).to(torch.float16)
    w = wl.draw_normal_bf16((N, K), 0.02, 19 * N + K, DEV)
    synera.debug_set_gemm_tile(tile)
    try:
        c = synera.gemm_pair(a, None, w)
        torch.cuda.synchronize()
    finally:
        synera.debug_set_gemm_tile(-1)
    want = a.double() @ w.double().T
    assert (c.double() - want).abs().max().item() < 6e-9 * K + 2e-7


# tiles: rows / 16 (1..17) with 256 columns, 100 + rows / 16 (1..12) with 128 columns, + 200 for two MFMA K steps
# per stage (256 columns: 1..5, 128 columns: 1..9); -1 = the planner's choice
@pytest.mark.parametrize("tile", [-1] + list(range(1, 18)) + list(range(101, 113)) + list(range(201, 206)) + list(range(301, 310)))
@pytest.mark.parametrize("M,N,K", [(1, 256, 64), (97, 512, 1024), (289, 768, 320), (532, 1024, 4096), (600, 4096, 1792),
                                   (532, 1792, 1024), (97, 1792, 320), (545, 1792, 512)])
def test_gemm_every_tile_and_epilogue(tile, M, N, K):
    """(hi, lo) activations through each tile configuration: store, residual add, SwiGLU; compared with the
    float64 product of the same operands."""
    synera = _synera()
    g = torch.Generator(device=DEV).manual_seed(1000 * M + N + K)
    x = torch.randn((M, K), generator=g, device=DEV)
    a, al = synera.split_pair(x)
    w = wl.draw_normal_bf16((N, K), 0.02, 17 * N + K, DEV)
    xd = a.double() + al.double()
    want = xd @ w.double().T
    # fp32 accumulation of 2K products of size ~0.02: measured ~1.7e-9 K; one missing term of the lo half of
    # one K step (an accumulator read before its last MFMA landed) is ~1e-5 and must not pass
    tol = 6e-9 * K + 2e-7
    synera.debug_set_gemm_tile(tile)
    try:
        c = synera.gemm_pair(a, al, w)
        base = torch.randn((M, N), generator=g, device=DEV)
        c_add = base.clone()
        synera.debug_gemm_epilogue(a, al, w, None, c_add, None, 1)
        half = N // 2
        act_hi = torch.empty((M, half), dtype=torch.float16, device=DEV)
        act_lo = torch.empty_like(act_hi)
        synera.debug_gemm_epilogue(a, al, w[:half].contiguous(), w[half:].contiguous(), act_hi, act_lo, 2)
        torch.cuda.synchronize()
    finally:
        synera.debug_set_gemm_tile(-1)
    assert (c.double() - want).abs().max().item() < tol
    assert (c_add.double() - (base.double() + want)).abs().max().item() < tol + 1e-6
    gate, up = want[:, :half], want[:, half:]
    glu = gate / (1 + torch.exp(-gate)) * up
    got = (act_hi.double() + act_lo.double()) / 8.0
    # elementwise: d(silu(g) u) <= 1.1 |u| dg + |g| du, fast-exp error, and the fp16 pair's 2^-22 relative rounding
    # (its low part goes subnormal for tiny products: 2^-25 / 8 absolute)
    bound = tol * (1.1 * up.abs() + gate.abs()) + (2.0 ** -21 + 2e-6) * glu.abs() + 1e-8
    assert ((got - glu).abs() - bound).max().item() < 0


def _pairs(hi, lo):
    """[M][K] high and low parts -> [M][K / 32][hi 32 | lo 32], the form the decoder layers hand activations over in."""
    M, K = hi.shape
    return torch.stack([hi.view(M, K // 32, 32), lo.view(M, K // 32, 32)], dim=2).contiguous()


@pytest.mark.parametrize("tile", [-1] + list(range(1, 18)) + list(range(101, 113)))
@pytest.mark.parametrize("M,N,K", [(1, 256, 64), (97, 512, 1024), (289, 768, 320), (532, 1024, 4096), (600, 4096, 1792),
                                   (545, 1792, 512)])
def test_gemm_paired_activation_layout(tile, M, N, K):
    """The activation pair as one array of whole 128-byte lines (hi and lo of a K block side by side): same MFMAs in
    the same order as the two-array form, so a forced tile must give the same bits; the planner's own choice
    (tile -1, which may differ between the forms) is held to the float64 product."""
    synera = _synera()
    g = torch.Generator(device=DEV).manual_seed(77 * M + N + K)
    x = torch.randn((M, K), generator=g, device=DEV)
    a, al = synera.split_pair(x)
    ap = _pairs(a, al)
    w = wl.draw_normal_bf16((N, K), 0.02, 23 * N + K, DEV)
    half = N // 2
    w0, w1 = w[:half].contiguous(), w[half:].contiguous()
    base = torch.randn((M, N), generator=g, device=DEV)
    synera.debug_set_gemm_tile(tile)
    try:
        c = torch.full((M, N), float("nan"), device=DEV)
        synera.debug_gemm_epilogue(a, al, w, None, c, None, 0)
        c_add = base.clone()
        synera.debug_gemm_epilogue(a, al, w, None, c_add, None, 1)
        act_hi = torch.empty((M, half), dtype=torch.float16, device=DEV)
        act_lo = torch.empty_like(act_hi)
        synera.debug_gemm_epilogue(a, al, w0, w1, act_hi, act_lo, 2)
        cp = torch.full((M, N), float("nan"), device=DEV)
        synera.debug_gemm_paired(ap, w, None, cp, 0)
        cp_add = base.clone()
        synera.debug_gemm_paired(ap, w, None, cp_add, 1)
        actp = torch.full((M, half // 32, 2, 32), float("nan"), dtype=torch.float16, device=DEV)
        synera.debug_gemm_paired(ap, w0, w1, actp, 2)
        torch.cuda.synchronize()
    finally:
        synera.debug_set_gemm_tile(-1)
    want = (a.double() + al.double()) @ w.double().T
    tol = 6e-9 * K + 2e-7
    assert (cp.double() - want).abs().max().item() < tol
    if tile > 0:
        assert torch.equal(cp, c) and torch.equal(cp_add, c_add)
        assert torch.equal(actp[:, :, 0].reshape(M, half), act_hi) and torch.equal(actp[:, :, 1].reshape(M, half), act_lo)
    else:
        assert (cp_add.double() - (base.double() + want)).abs().max().item() < tol + 1e-6
        got = (actp[:, :, 0].double() + actp[:, :, 1].double()).reshape(M, half)
        ref = act_hi.double() + act_lo.double()
        assert (got - ref).abs().max().item() <= 8 * tol * 4 + 2.0 ** -20 * ref.abs().max().item()


@pytest.mark.parametrize("tile", [-1, 4, 8, 9, 13, 17, 104, 108, 112, 204, 205, 304, 308, 309])
@pytest.mark.parametrize("M,N,K", [(97, 512, 1024), (289, 768, 320), (532, 1024, 4096), (545, 4096, 1792), (532, 1792, 2048),
                                   (24, 1792, 4096)])
def test_gemm_stored_k_slices_sum_to_the_product(tile, M, N, K):
    """K split into stored slices (the mode the decoder layers use): the slices, added in order, give the
    product; a planner that does not split returns it whole.  The slices are stored, never accumulated, so two
    runs agree bit for bit."""
    synera = _synera()
    g = torch.Generator(device=DEV).manual_seed(7 * M + N + K)
    x = torch.randn((M, K), generator=g, device=DEV)
    a, al = synera.split_pair(x)
    w = wl.draw_normal_bf16((N, K), 0.02, 13 * N + K, DEV)
    want = (a.double() + al.double()) @ w.double().T
    synera.debug_set_gemm_tile(tile)
    try:
        parts = synera.debug_gemm_slices(a, al, w).clone()
        again = synera.debug_gemm_slices(a, al, w)
        torch.cuda.synchronize()
    finally:
        synera.debug_set_gemm_tile(-1)
    assert 1 <= parts.shape[0] <= 8
    if tile > 0 and K >= 1024 and (M + 16 * (tile % 100) - 1) // (16 * (tile % 100)) * (N // (128 if tile > 100 else 256)) <= 128:
        assert parts.shape[0] > 1          # few tiles, at least 32 K steps: a forced tile splits here
    assert torch.equal(parts, again)
    assert (parts.double().sum(0) - want).abs().max().item() < 6e-9 * K + 2e-7


def test_gemm_rejects_unsupported_shapes():
    synera = _synera()
    a = torch.zeros((4, 96), dtype=torch.float16, device=DEV)
    w = torch.zeros((128, 96), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(synera.SyneraError) as e:
        synera.gemm_pair(a, a, w)
    assert e.value.status == synera.EUNSUP
