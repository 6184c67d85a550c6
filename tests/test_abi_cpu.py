"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and the host
validation (the only logic that runs without a GPU) returns the documented codes."""
import ctypes
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(synera_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    import paper_2511_07423_amd as synera
    lib = ctypes.CDLL(synera.lib_path())
    names = _declared_symbols()
    assert {"synera_verify", "synera_confidence", "synera_kv_append", "synera_create", "synera_destroy",
            "synera_validate_batch", "synera_gemm_pair", "synera_version", "synera_strerror",
            "synera_sched_create", "synera_sched_next", "synera_sched_commit"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None, n
    assert synera.version() == 100
    lib.synera_strerror.restype = ctypes.c_char_p
    assert b"range" in lib.synera_strerror(-2)


def test_validate_batch_codes():
    import paper_2511_07423_amd as s
    bt = np.arange(12, dtype=np.int32).reshape(3, 4)
    ok = dict(ctx_len=[10, 20, 0], n_first=[4, 1, 16], n_second=[0, 3, 0], block_table=bt, n_pages_in_pool=12,
              max_batch=4, max_tokens=64)
    assert s.validate_batch(**ok) == s.OK
    assert s.validate_batch(**dict(ok, n_first=[4, 0, 16])) == s.EINVAL            # k < 1
    assert s.validate_batch(**dict(ok, n_second=[0, -1, 0])) == s.EINVAL           # u < 0
    assert s.validate_batch(**dict(ok, ctx_len=[10, -1, 0])) == s.ERANGE           # negative length
    assert s.validate_batch(**dict(ok, n_first=[4, 1, 30], n_second=[0, 3, 3])) == s.EUNSUP   # chunk > 32
    assert s.validate_batch(**dict(ok, max_batch=2)) == s.ENOSPC
    assert s.validate_batch(**dict(ok, max_tokens=23)) == s.ENOSPC                 # 4 + 4 + 16 = 24 tokens
    assert s.validate_batch(**dict(ok, max_tokens=24)) == s.OK
    assert s.validate_batch(**dict(ok, ctx_len=[10, 62, 0])) == s.ENOSPC           # needs 5 pages, table has 4
    assert s.validate_batch(**dict(ok, ctx_len=[10, 60, 0])) == s.OK               # exactly 64 positions
    bad = bt.copy(); bad[1, 1] = 12
    assert s.validate_batch(**dict(ok, block_table=bad)) == s.ERANGE               # page id outside the pool
    bad = bt.copy(); bad[1, 0] = -1
    assert s.validate_batch(**dict(ok, block_table=bad)) == s.ERANGE
    dup = bt.copy(); dup[2, 0] = 4                                                 # page 4 belongs to request 1
    assert s.validate_batch(**dict(ok, block_table=dup)) == s.ERANGE
    unused = bt.copy(); unused[0, 3] = -1; unused[2, 1:] = 999                    # beyond the needed pages: ignored
    assert s.validate_batch(**dict(ok, block_table=unused)) == s.OK
    assert s.validate_batch(**dict(ok, n_second=None)) == s.OK
    big = dict(ok, n_first=[400, 1, 1], n_second=None, ctx_len=[0, 0, 0], max_tokens=1 << 40)
    assert s.validate_batch(**big, chunk_limit=0) == s.ENOSPC                      # 400 rows need 25 pages
    assert s.validate_batch(**dict(big, n_first=[64, 1, 1]), chunk_limit=0) == s.OK


def test_workload_draws_are_valid_batches():
    import paper_2511_07423_amd as s
    import workloads as wl
    for n, rec in wl.CONFIGS.items():
        b = wl.draw_batch(rec)
        assert len(b["ctx_len"]) == rec.batch
        assert b["ctx_len"].min() >= rec.ctx_lo and b["ctx_len"].max() <= rec.ctx_hi
        assert b["n_draft"].min() >= rec.k_lo and b["n_draft"].max() <= rec.k_hi
        st = s.validate_batch(b["ctx_len"], b["n_draft"], b["n_uncached"], b["block_table"], b["n_pages"],
                              rec.batch, int(b["n_draft"].sum()))
        assert st == s.OK, (n, st)
        again = wl.draw_batch(rec)
        assert np.array_equal(b["block_table"], again["block_table"])             # seeded
        if rec.permute_pages:
            assert (np.diff(b["block_table"][0, :4]) != 1).any()
