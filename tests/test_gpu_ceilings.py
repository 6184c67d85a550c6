"""The ceiling-measurement kernels: the copy moves every byte, the MFMA loop computes what its operands say
(constant operands: each of the 4 accumulators receives iters x 4 MFMAs of 16 products 1.0 x 2^-7), and the
reported FLOP count is the loop's."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2511_07423_amd as synera
from paper_2511_07423_amd import binding

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_bytes", [16, 16 * 1001, 1 << 20, (1 << 24) + 16 * 77])
def test_copy_moves_every_byte(n_bytes):
    g = torch.Generator(device="cuda:0").manual_seed(n_bytes)
    src = torch.randint(0, 256, (n_bytes,), dtype=torch.uint8, device="cuda:0", generator=g)
    dst = torch.zeros(n_bytes + 64, dtype=torch.uint8, device="cuda:0")
    moved = synera.measure_hbm_copy(dst[:n_bytes], src)
    torch.cuda.synchronize()
    assert moved == 2 * n_bytes
    assert torch.equal(dst[:n_bytes], src)
    assert int(dst[n_bytes:].sum()) == 0          # nothing past the end


@pytest.mark.parametrize("n_bytes", [16, 16 * 1001, (1 << 24) + 16 * 77, (1 << 26) + 16 * 5])
def test_read_stream_touches_every_piece_once(n_bytes):
    """Each lane's output word is the xor of exactly the pieces the header assigns to it."""
    g = torch.Generator(device="cuda:0").manual_seed(n_bytes + 1)
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (n_bytes // 4,), dtype=torch.int32, device="cuda:0", generator=g)
    lanes = synera.MEASURE_READ_BLOCKS * 256
    out = torch.full((lanes,), 0x5A5A5A5A, dtype=torch.int32, device="cuda:0")
    assert synera.measure_hbm_read(out, src) == n_bytes
    torch.cuda.synchronize()
    pieces = np.bitwise_xor.reduce(src.cpu().numpy().reshape(-1, 4), axis=1)          # one word per 16-byte piece
    blocks = synera.MEASURE_READ_BLOCKS
    seg = -(-len(pieces) // blocks)
    seg_pad = -(-seg // 256) * 256
    want = np.zeros((blocks, 256), np.int32)
    for b in range(blocks):
        part = pieces[b * seg:(b + 1) * seg]
        if len(part) == 0:
            break
        padded = np.zeros(seg_pad, np.int32)
        padded[:len(part)] = part
        want[b] = np.bitwise_xor.reduce(padded.reshape(-1, 256), axis=0)
    assert np.array_equal(out.cpu().numpy().reshape(blocks, 256), want)


@pytest.mark.parametrize("blocks,iters", [(1, 1), (3, 7), (256, 1000)])
def test_mfma_loop_constant_operands(blocks, iters):
    out = torch.full((blocks * 256,), -1.0, dtype=torch.float32, device="cuda:0")
    flops = synera.measure_mfma_bf16(out, blocks, iters, random_operands=False)
    torch.cuda.synchronize()
    assert flops == blocks * 4 * iters * 16 * 2 * 32 * 32 * 16
    assert torch.equal(out, torch.full_like(out, 2.0 * iters))


@pytest.mark.parametrize("blocks,iters", [(1, 1), (3, 7), (256, 1000)])
def test_mfma_f16_loop_constant_operands(blocks, iters):
    """The loop on the projection kernel's own MFMA: 1.0 x 2^-7 over K = 32, four MFMAs per accumulator and
    iteration, eight accumulators summed per lane."""
    out = torch.full((blocks * 256,), -1.0, dtype=torch.float32, device="cuda:0")
    flops = synera.measure_mfma_f16(out, blocks, iters, random_operands=False)
    torch.cuda.synchronize()
    assert flops == blocks * 4 * iters * 32 * 2 * 16 * 16 * 32
    assert torch.equal(out, torch.full_like(out, 8.0 * iters))


def test_mfma_f16_loop_random_operands_is_finite_and_deterministic():
    a = torch.empty(8 * 256, dtype=torch.float32, device="cuda:0")
    b = torch.empty_like(a)
    synera.measure_mfma_f16(a, 8, 500, random_operands=True)
    synera.measure_mfma_f16(b, 8, 500, random_operands=True)
    torch.cuda.synchronize()
    assert torch.isfinite(a).all() and torch.equal(a, b)
    assert a.abs().max() > 0


def test_mfma_loop_random_operands_is_finite_and_deterministic():
    a = torch.empty(8 * 256, dtype=torch.float32, device="cuda:0")
    b = torch.empty_like(a)
    synera.measure_mfma_bf16(a, 8, 500, random_operands=True)
    synera.measure_mfma_bf16(b, 8, 500, random_operands=True)
    torch.cuda.synchronize()
    assert torch.isfinite(a).all() and torch.equal(a, b)
    assert a.abs().max() > 0


def test_bad_arguments_are_refused():
    buf = torch.zeros(1024, dtype=torch.float32, device="cuda:0")
    lib, p = binding._lib, buf.data_ptr()
    assert lib.synera_measure_hbm_copy(None, p, 16, None) == synera.EINVAL
    assert lib.synera_measure_hbm_copy(p, p + 2048, 24, None) == synera.EINVAL        # not a multiple of 16
    assert lib.synera_measure_hbm_copy(p + 4, p + 2048, 16, None) == synera.EINVAL    # misaligned
    assert lib.synera_measure_hbm_read(None, p, 16, None) == synera.EINVAL
    assert lib.synera_measure_hbm_read(p, p + 8, 16, None) == synera.EINVAL           # misaligned source
    assert lib.synera_measure_mfma_bf16(None, 1, 1, 0, None, None) == synera.EINVAL
    assert lib.synera_measure_mfma_bf16(p, 0, 1, 0, None, None) == synera.EINVAL
    assert lib.synera_measure_mfma_bf16(p, 4097, 1, 0, None, None) == synera.EINVAL
    assert lib.synera_measure_mfma_bf16(p, 1, 200001, 0, None, None) == synera.EINVAL
    assert lib.synera_measure_mfma_f16(None, 1, 1, 0, None, None) == synera.EINVAL
    assert lib.synera_measure_mfma_f16(p, 4097, 1, 0, None, None) == synera.EINVAL
    with pytest.raises(ValueError):
        synera.measure_mfma_bf16(buf, 8, 1)       # out too small for 8 blocks
