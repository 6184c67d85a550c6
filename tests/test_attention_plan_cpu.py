"""Host logic of the chunk attention's work plan (no GPU): whatever the number of persistent blocks and the mix of
stream lengths, every 32-key tile of every (request, row group, KV head) stream is executed exactly once, by a
program the kernel can walk: shares tile the program, positions come in pairs or singles as the share's class
wants, tiles name the request's own pages, and streams cut across blocks own distinct partial slots."""
import numpy as np
import pytest

import paper_2511_07423_amd as synera
import workloads as wl

KIND, LAST = 7, 8
PAD, KV, Q = 0, 1, 2


def _check_plan(shape, n_blocks, ctx, unc, nd, bt):
    pl = synera.debug_attention_plan(shape, n_blocks, ctx, unc, nd, bt)
    shares, prog, units, cuts = pl["shares"], pl["prog"], pl["units"], pl["cuts"]
    G, Hkv = shape.n_q_heads // shape.n_kv_heads, shape.n_kv_heads
    chunk = unc + nd
    cu = np.concatenate([[0], np.cumsum(chunk)])
    assert 1 <= len(shares) <= n_blocks
    at = 0
    seen = {}                                   # (tok0, kh) -> list of (first tile, end tile, unit)
    for begin, n_pos, rbn, _ in shares:
        assert begin == at and n_pos > 0 and rbn in (2, 4) and n_pos % (4 // rbn) == 0
        at += n_pos
        kp = 4 // rbn
        i, end = begin, begin + n_pos
        while i < end:
            # a stream's share: its query positions ...
            tag, tok0, nrows, c = prog[i]
            assert tag & KIND == Q and c & 255 == 0
            u, kh = tag >> 4, c >> 8
            assert (rbn == 4) == (nrows > 32) and 1 <= nrows <= 64 and nrows % G == 0
            if rbn == 4:
                assert tuple(prog[i + 1]) == (tag, tok0, nrows, 32 | (kh << 8))
            else:
                assert prog[i + 1][0] & KIND == PAD
            i += 2
            req = int(np.searchsorted(cu, tok0, side="right") - 1)
            j0, ntok = tok0 - cu[req], nrows // G
            keys = int(ctx[req] + j0 + ntok)
            assert j0 + ntok <= chunk[req]
            ut = units[u]
            assert (ut[0], ut[1], ut[2], ut[5]) == (tok0, nrows, ctx[req] + j0, kh) and 0 <= kh < Hkv
            # ... then its key tiles, padded to whole iterations, the last iteration flagged
            first = i
            tiles = []
            while i < end and prog[i][0] & KIND == KV:
                t_tag, pa, pb, k0 = prog[i]
                assert t_tag >> 4 == kh and k0 % 32 == 0
                t = k0 // 32
                pages = (keys + 15) // 16
                assert pa == bt[req][2 * t] and pb == (bt[req][2 * t + 1] if 2 * t + 1 < pages else pa)
                tiles.append(t)
                i += 1
            assert tiles and tiles == list(range(tiles[0], tiles[0] + len(tiles)))
            if (i - first) % kp:
                assert prog[i][0] & KIND == PAD
                i += 1
            flagged = [j for j in range(first, i) if prog[j][0] & LAST]
            assert flagged == [i - kp]
            assert ut[3] == min(keys, 32 * (tiles[-1] + 1))
            seen.setdefault((tok0, kh), []).append((tiles[0], tiles[-1] + 1, u, keys, ut[4], nrows))
    assert at == len(prog)
    # every stream: all KV heads, tiles 0 .. n once, partial slots iff cut
    groups = set()
    tg = max(1, 64 // G)
    for r in range(len(ctx)):
        for j0 in range(0, int(chunk[r]), tg):
            groups.add(int(cu[r] + j0))
    assert {k[0] for k in seen} == groups and len(seen) == len(groups) * Hkv
    slots = []
    n_cut = 0
    for (tok0, kh), parts in seen.items():
        parts.sort()
        keys = parts[0][3]
        assert parts[0][0] == 0 and parts[-1][1] == (keys + 31) // 32
        assert all(a[1] == b[0] for a, b in zip(parts, parts[1:]))
        if len(parts) == 1:
            assert parts[0][4] == -1
        else:
            n_cut += 1
            mine = [p[4] for p in parts]
            cut = [c for c in cuts if c[2] == tok0 and c[4] == kh]
            assert len(cut) == 1 and cut[0][1] == len(parts) and cut[0][3] == parts[0][5]
            assert sorted(mine) == list(range(cut[0][0], cut[0][0] + len(parts)))
            slots += mine
    assert n_cut == len(cuts) and len(set(slots)) == len(slots) and (not slots or max(slots) < 2 * n_blocks)
    return pl


def _batch(rng, B, max_ctx, max_chunk=32):
    ctx = rng.integers(0, max_ctx + 1, B).astype(np.int32)
    nd = rng.integers(1, max_chunk + 1, B).astype(np.int32)
    unc = np.array([rng.integers(0, max_chunk - k + 1) for k in nd], np.int32)
    need = (ctx + unc + nd + 15) // 16
    bt = np.full((B, int(need.max()) + 1), -1, np.int32)
    perm = rng.permutation(int(need.sum()) + 3)
    at = 0
    for i in range(B):
        bt[i, :need[i]] = perm[at:at + need[i]]
        at += int(need[i])
    return ctx, unc, nd, bt


@pytest.mark.parametrize("n_blocks", [2, 3, 7, 64, 512])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_batches(seed, n_blocks):
    rng = np.random.default_rng(100 + seed)
    shape = [wl.LLAMA_8B, wl.ModelShape("mini_gqa", 3, 128, 4, 2, 64, 256, 256), wl.ModelShape("mha", 2, 256, 4, 4, 64, 1024, 4096)][seed]
    _check_plan(shape, n_blocks, *_batch(rng, [40, 12, 5][seed], [3000, 700, 130][seed]))


@pytest.mark.parametrize("cfg", [1, 2, 3, 5])
def test_task_workloads(cfg):
    rec = wl.config(cfg)
    b = wl.draw_batch(rec)
    B = len(b["ctx_len"])
    pl = _check_plan(rec.shape, 512, b["ctx_len"], np.zeros(B, np.int32), b["n_draft"], b["block_table"])
    n = pl["shares"][:, 1].astype(np.int64) // (4 // pl["shares"][:, 2])
    if cfg in (3, 5):                           # enough work for every block: balanced within each class
        assert len(pl["shares"]) == 512
        for rbn in (2, 4):
            m = n[pl["shares"][:, 2] == rbn]
            assert len(m) == 0 or m.max() <= 1.25 * m.mean() + 4


def test_edge_batches():
    shape = wl.LLAMA_8B
    one = np.ones(1, np.int32)
    bt = np.arange(4, dtype=np.int32)[None]
    _check_plan(shape, 512, 0 * one, 0 * one, one, bt)                 # empty context, one draft
    _check_plan(shape, 512, 0 * one, 0 * one, 32 * one, bt)            # a full chunk against nothing
    _check_plan(shape, 3, 31 * one, 16 * one, 16 * one, bt)            # context + chunk = the whole block table
    with pytest.raises(synera.SyneraError):
        _check_plan(shape, 3, 40 * one, 16 * one, 16 * one, bt)        # beyond it
    with pytest.raises(synera.SyneraError):
        _check_plan(shape, 1, one, 0 * one, one, bt)                   # one block per class of streams at least
