"""Host logic of the projection GEMM's tile planner (no GPU call): the plans of the headline batch, and
properties every plan must have for the launch to be valid."""
import pytest

import paper_2511_07423_amd as synera

STORE, ADD, SWIGLU = 0, 1, 2
# the projections of one decoder layer and the LM head at the 8B shape (Section 6.1's cloud model class)
D, F, QKV, VOCAB = 4096, 14336, 6144, 32000


def test_headline_batch_plans():
    """532 draft rows: every projection on 256-column tall tiles; the few-tile ones split K into stored slices."""
    T = 532
    assert synera.debug_gemm_plan(T, QKV, D, STORE) == (272, 256, 5)
    assert synera.debug_gemm_plan(T, D, D, ADD) == (144, 256, 4)
    assert synera.debug_gemm_plan(T, 2 * F, D, SWIGLU) == (272, 256, 1)
    assert synera.debug_gemm_plan(T, D, F, ADD) == (272, 256, 8)
    assert synera.debug_gemm_plan(T, VOCAB, D, STORE, stored_slices=False) == (272, 256, 1)
    for n, k, e in ((QKV, D, STORE), (D, D, ADD), (2 * F, D, SWIGLU), (D, F, ADD)):
        assert synera.debug_gemm_plan_bk(T, n, k, e) == 32          # the tall tiles fill the LDS with 64-byte rows


def test_small_batches_take_the_narrow_tiles():
    """About 140 rows: 128-column tiles double the blocks that stream the weights, and those tiles are short
    enough for two MFMA K steps per stage (half the barriers, full 128-byte rows per copy)."""
    for n, k, e in ((QKV, D, STORE), (D, D, ADD), (2 * F, D, SWIGLU), (D, F, ADD)):
        assert synera.debug_gemm_plan(144, n, k, e)[1] == 128
        assert synera.debug_gemm_plan_bk(144, n, k, e) == 64
        assert synera.debug_gemm_plan_bk(128, n, k, e) == 64


def test_decode_sized_batches_use_tiles_of_their_own_height_and_never_atomics():
    """Below 128 rows the tile is as tall as the batch (one M tile); K may only be split into stored slices,
    and without a slice buffer (the stand-alone mode) it is not split at all: no path adds with atomics."""
    for M in (1, 8, 16, 17, 64, 96):
        for n, k, e in ((QKV, D, STORE), (D, D, ADD), (2 * F, D, SWIGLU), (D, F, ADD), (VOCAB, D, STORE)):
            bm, bn, split = synera.debug_gemm_plan(M, n, k, e)
            assert bm == (M + 15) // 16 * 16
            assert synera.debug_gemm_plan(M, n, k, e, stored_slices=False)[2] == 1


@pytest.mark.parametrize("stored", [True, False])
@pytest.mark.parametrize("M", [1, 17, 96, 97, 130, 200, 333, 532, 777, 1030, 2048])
@pytest.mark.parametrize("N,K,epi", [(QKV, D, STORE), (D, D, ADD), (2 * F, D, SWIGLU), (D, F, ADD), (VOCAB, D, STORE),
                                     (128, 64, STORE), (1792, 4096, ADD), (8320, 8320, STORE)])
def test_plans_are_launchable(M, N, K, epi, stored):
    bm, bn, split = synera.debug_gemm_plan(M, N, K, epi, stored)
    assert bm % 16 == 0 and bn in (128, 256) and N % bn == 0
    assert 1 <= split <= K // 32
    if epi == SWIGLU:
        assert split == 1
    assert split <= 8                           # SYNERA_MAX_GEMM_SLICES
    bk = synera.debug_gemm_plan_bk(M, N, K, epi, stored)
    assert bk in (32, 64) and K % bk == 0
    if bk == 64:                                # three stages of (2 bm + bn) rows of 128 bytes fit the 160 KB of LDS
        assert 3 * (2 * bm + bn) * 128 <= 163840
    if not stored:
        assert split == 1


def test_plan_rejects_bad_shapes():
    with pytest.raises(synera.SyneraError):
        synera.debug_gemm_plan(0, 128, 64)
    with pytest.raises(synera.SyneraError):
        synera.debug_gemm_plan(16, 192, 64)     # N % 128
    with pytest.raises(synera.SyneraError):
        synera.debug_gemm_plan(16, 384, 64, SWIGLU)   # N % 256 for SwiGLU
    with pytest.raises(synera.SyneraError):
        synera.debug_gemm_plan(16, 128, 96)     # K % 64
