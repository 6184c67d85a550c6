"""The projection GEMM's entry point that allocates nothing (synera_gemm_pair_static) against the entry point it
is a variant of (synera_debug_gemm_slices, whose caller brings the slice workspace): same slices, summed in the
same order, so the results must agree bit for bit; two calls in a row, the second smaller, share the static
array.  Collected last: a failure here must not hide the other GPU tests."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _expected(synera, a, al, w):
    parts = synera.debug_gemm_slices(a, al, w)
    want = parts[0].clone()
    for s in range(1, parts.shape[0]):            # in order, as the static variant sums them
        want += parts[s]
    return want, parts.shape[0]


def test_static_workspace_gemm_matches_the_workspace_argument_form_on_two_calls_in_a_row():
    import paper_2511_07423_amd as synera
    g = torch.Generator(device=DEV).manual_seed(99)
    shapes = [(96, 4096, 4096), (24, 1792, 2048)]          # the second call is smaller and reuses the array
    inputs = []
    for M, N, K in shapes:
        x = torch.randn((M, K), generator=g, device=DEV)
        a, al = synera.split_pair(x)
        w = wl.draw_normal_bf16((N, K), 0.02, 31 * N + K, DEV)
        inputs.append((a, al, w, torch.full((M, N), float("nan"), device=DEV)))
    want = [_expected(synera, a, al, w) for a, al, w, _ in inputs]
    assert want[0][1] > 1 and want[1][1] > 1                # both calls really go through K slices
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for a, al, w, out in inputs:                            # back to back on one stream
        synera.gemm_pair_static(a, al, w, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for (a, al, w, out), (exp, _) in zip(inputs, want):
        assert torch.equal(out, exp)
        ref = (a.double() + al.double()) @ w.double().T
        assert (out.double() - ref).abs().max().item() < 6e-9 * a.shape[1] + 2e-7
    # once more in the other order: what the larger call left in the array must not leak into the smaller one
    for a, al, w, out in reversed(inputs):
        out.fill_(float("nan"))
        synera.gemm_pair_static(a, al, w, out)
    torch.cuda.synchronize()
    for (a, al, w, out), (exp, _) in zip(inputs, want):
        assert torch.equal(out, exp)


def test_static_workspace_gemm_rejects_what_does_not_fit():
    import paper_2511_07423_amd as synera
    M, N, K = 129, 4096, 64                                 # 129 x 4096 > 524288 outputs
    a = torch.zeros((M, K), dtype=torch.float16, device=DEV)
    w = torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((M, N), device=DEV)
    with pytest.raises(synera.SyneraError) as e:
        synera.gemm_pair_static(a, a, w, out)
    assert e.value.status == synera.ENOSPC
    with pytest.raises(synera.SyneraError) as e:
        synera.gemm_pair_static(a[:4, :], a[:4, :], w[:100], out[:4, :100].contiguous())
    assert e.value.status == synera.EUNSUP
    assert M * N > synera.STATIC_GEMM_MAX_OUT
