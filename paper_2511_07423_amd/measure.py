"""Kernel-level measurements of the standalone entry points (not the end-to-end benchmark, which is
bench.py at the repository root):

    python -m paper_2511_07423_amd.measure confidence   # synera_confidence on a 2048 x 128256 logits block
    python -m paper_2511_07423_amd.measure gemm [M ...] # the four projection shapes of the 8B decoder at M = 532, 1152, 2048
    python -m paper_2511_07423_amd.measure sched        # host time of the scheduler per iteration (no GPU needed)
    python -m paper_2511_07423_amd.measure ceilings     # what this GPU gives: device copy (HBM), register-resident MFMA loop
    python -m paper_2511_07423_amd.measure blocks       # the gate/up tile (272 x 256, K = 4096) on 2 .. 448 blocks, random and zero activations

Each line gives the average launch time over HIP events on the launch stream and the achieved rate
against MI355X's peak (HBM 8 TB/s; dense fp16 / bf16 MFMA 2.5 PFLOP/s, algorithmic FLOPs).  Inputs are seeded
and synthetic (workloads/)."""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _time(fn, n=20, warm=3):
    import torch
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def confidence():
    import torch
    import paper_2511_07423_amd as synera
    import workloads as wl
    from workloads import shapes
    for dtype, name in ((torch.float32, "f32"), (torch.bfloat16, "bf16")):
        x = wl.draw_confidence_logits(shapes.C5B_ROWS, shapes.C5B_VOCAB, shapes.C5B_STD, shapes.C5B_BOOST_HI,
                                      wl.config(5).seed, "cuda:0", dtype)
        ms = _time(lambda: synera.confidence(x))
        nbytes = x.numel() * x.element_size()
        print(json.dumps({"kernel": "synera_confidence", "rows": shapes.C5B_ROWS, "vocab": shapes.C5B_VOCAB,
                          "dtype": name, "bytes": nbytes, "avg_launch_ms": ms, "bound": "hbm",
                          "achieved_GBs": nbytes / ms / 1e6, "peak_GBs": 8000.0, "frac": nbytes / ms / 1e6 / 8000.0}))
        for k in (8, 64, 256):
            ms = _time(lambda: synera.confidence_topk(x, k))
            print(json.dumps({"kernel": f"synera_confidence_topk (k = {k})", "rows": shapes.C5B_ROWS, "vocab": shapes.C5B_VOCAB,
                              "dtype": name, "bytes": nbytes, "avg_launch_ms": ms, "bound": "hbm",
                              "achieved_GBs": nbytes / ms / 1e6, "peak_GBs": 8000.0, "frac": nbytes / ms / 1e6 / 8000.0}))
        ms = _time(lambda: synera.nucleus(x, 0.9))            # one read for the maximum and the sum, four for the radix search
        print(json.dumps({"kernel": "synera_nucleus (top_p = 0.9)", "rows": shapes.C5B_ROWS, "vocab": shapes.C5B_VOCAB,
                          "dtype": name, "bytes": nbytes, "avg_launch_ms": ms, "bound": "hbm",
                          "achieved_GBs": nbytes / ms / 1e6, "peak_GBs": 8000.0, "frac": nbytes / ms / 1e6 / 8000.0}))


def gemm():
    import torch
    import paper_2511_07423_amd as synera
    import workloads as wl
    shapes = (("qkv", 6144, 4096), ("o", 4096, 4096), ("gate_up (store epilogue)", 28672, 4096), ("down", 4096, 14336))
    ws = {}
    for M in [int(v) for v in sys.argv[2:]] or [532, 1152, 2048]:
        for name, N, K in shapes:
            x = torch.randn((M, K), generator=torch.Generator(device="cuda:0").manual_seed(7), device="cuda:0")
            a, al = synera.split_pair(x)
            if name not in ws:                                 # three copies, rotated: no cache reuse
                ws[name] = [wl.draw_normal_bf16((N, K), 0.02, 100 + i, "cuda:0") for i in range(3)]
            w3 = ws[name]
            c = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
            it = iter(range(10 ** 9))
            ms = _time(lambda: synera.gemm_pair(a, al, w3[next(it) % 3], out=c), n=18)
            fl = 2.0 * M * N * K
            print(json.dumps({"kernel": "synera_gemm_pair", "shape": name, "M": M, "N": N, "K": K, "avg_launch_ms": ms,
                              "bound": "mfma", "achieved_TFLOPs": fl / ms / 1e9, "executed_TFLOPs": 2 * fl / ms / 1e9,
                              "peak_TFLOPs": 2500.0, "frac": fl / ms / 1e9 / 2500.0}))


def measured_ceilings(copy_bytes=1 << 30, mfma_iters=20000):
    """The chip's measured rates next to the published ones: a 1 GiB device copy (HBM moves 2 GiB) and the
    register-resident bf16 MFMA loop on 256 blocks, with constant and with random operands."""
    import torch
    import paper_2511_07423_amd as synera
    src = torch.zeros(copy_bytes // 4, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    moved = [0]

    def copy():
        moved[0] = synera.measure_hbm_copy(dst, src)
    ms = _time(copy, n=10)
    res = {"hbm_copy_GBs": moved[0] / ms / 1e6}
    del dst
    words = torch.empty(synera.MEASURE_READ_BLOCKS * 256, dtype=torch.int32, device="cuda:0")

    def read():
        moved[0] = synera.measure_hbm_read(words, src)
    ms = _time(read, n=10)
    res["hbm_read_GBs"] = moved[0] / ms / 1e6
    res["hbm_peak_GBs"] = 8000.0
    del src, words
    out = torch.empty(256 * 256, dtype=torch.float32, device="cuda:0")
    for key, rnd in (("mfma_bf16_constant_operands_TFLOPs", False), ("mfma_bf16_random_operands_TFLOPs", True)):
        flops = [0]

        def loop():
            flops[0] = synera.measure_mfma_bf16(out, 256, mfma_iters, rnd)
        ms = _time(loop, n=5, warm=2)
        res[key] = flops[0] / ms / 1e9
    res["mfma_bf16_peak_TFLOPs"] = 2500.0
    # the instruction the projection kernel issues (16x16x32 fp16, 4 passes), 32 per iteration
    for key, rnd in (("mfma_f16_constant_operands_TFLOPs", False), ("mfma_f16_random_operands_TFLOPs", True)):
        flops = [0]

        def loop16():
            flops[0] = synera.measure_mfma_f16(out, 256, mfma_iters // 2, rnd)
        ms = _time(loop16, n=5, warm=2)
        res[key] = flops[0] / ms / 1e9
    return res


def blocks():
    """What limits the gate/up projection: the same work per block (a 272 x 256 tile of the SwiGLU projection over
    K = 4096, weights rotated over three copies) on 2, 56, 112, 224 and 448 blocks, with random operands, with zero
    activations and with all operands zero (same instruction stream and memory traffic, less and less switching power).  A lone pair of blocks shows what the
    kernel's own structure costs on one compute unit; more blocks add the shared memory system and the chip's
    power management."""
    import torch
    import paper_2511_07423_amd as synera
    import workloads as wl
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(1)
    tile = int(sys.argv[2]) if len(sys.argv) > 2 else 17          # 17: four wavefronts; 217: the same tile on eight
    K = int(sys.argv[3]) if len(sys.argv) > 3 else 4096           # row pitch of both operands = 2 K bytes
    synera.debug_set_gemm_tile(tile)
    try:
        for M, N in ((272, 512), (272, 14336), (272, 28672), (272, 57344), (532, 28672), (544, 57344)):
            x = torch.randn((M, K), generator=g, device=dev)
            a, al = synera.split_pair(x, 64.0)
            ws = [(wl.draw_normal_bf16((N // 2, K), 0.02, 5 + i, dev), wl.draw_normal_bf16((N // 2, K), 0.02, 50 + i, dev))
                  for i in range(3)]
            hi = torch.empty((M, N // 2), dtype=torch.float16, device=dev)
            lo = torch.empty_like(hi)
            for operands in ("random", "zero activations", "all zero"):
                if operands != "random":
                    a.zero_()
                    al.zero_()
                if operands == "all zero":
                    for w in ws:
                        w[0].zero_()
                        w[1].zero_()
                it = iter(range(10 ** 9))

                def launch():
                    w = ws[next(it) % 3]
                    synera.debug_gemm_epilogue(a, al, w[0], w[1], hi, lo, 2)
                ms = _time(launch, n=60, warm=5)
                tiles = ((M + 271) // 272) * (N // 256)
                executed = 4.0 * 272 * ((M + 271) // 272) * N * K        # padded rows, both terms
                print(json.dumps({"kernel": "proj_kernel<17, 4, 2, true>" if tile == 17 else f"tile {tile}", "M": M,
                                  "N": N, "K": K, "blocks": tiles, "operands": operands, "avg_launch_us": ms * 1e3,
                                  "executed_TFLOPs": executed / ms / 1e9,
                                  "executed_TFLOPs_per_busy_CU": executed / ms / 1e9 / min(tiles, 256),
                                  "peak_TFLOPs_per_CU": 2500.0 / 256}), flush=True)
    finally:
        synera.debug_set_gemm_tile(-1)


def ceilings():
    print(json.dumps({"what": "measured ceilings (device copy and read-only stream of 1 GiB; 256 blocks x 4 wavefronts x 20000 x 16 MFMA 32x32x16 bf16, x 10000 x 32 MFMA 16x16x32 fp16)",
                      **measured_ceilings()}))


def sched():
    """Host cost of the verification-aware scheduler on the headline batch shape: 64 active requests with the
    context lengths of that workload; every round all 64 submit a verification (1 uncached token + their
    drafts), one iteration forms the batch and its block tables, and the commit books the accept lengths.
    Reported per iteration, wall clock around the Python calls and the module's own counter (C++ only)."""
    import time
    import numpy as np
    import paper_2511_07423_amd as synera
    import workloads as wl
    b = wl.draw_batch(wl.config(3))
    B = len(b["ctx_len"])
    max_pages = int(b["max_pages"]) + 8
    s = synera.Scheduler(B * max_pages, max_pages, B, 64 * B)
    for i in range(B):
        s.submit_prefill(i, int(b["ctx_len"][i]))
    while True:                                   # register the contexts (no engine behind it)
        kind, out = s.next()
        if kind == synera.SCHED_IDLE:
            break
        s.commit()
    rng = np.random.default_rng(0)
    base = s.stats()["host_ns"]
    rounds, t0 = 50, time.perf_counter()
    for _ in range(rounds):
        for i in range(B):
            s.submit_verify(i, 1, int(b["n_draft"][i]))
        kind, out = s.next()
        assert kind == synera.SCHED_VERIFY and len(out["request_id"]) == B
        s.commit(rng.integers(0, 2, B).astype(np.int32))
    wall = (time.perf_counter() - t0) / rounds
    inner = (s.stats()["host_ns"] - base) / rounds
    print(json.dumps({"what": "synera_sched iteration, 64 verification requests", "requests": B,
                      "block_table_columns": max_pages, "python_wall_us_per_iteration": wall * 1e6,
                      "module_us_per_iteration": inner / 1e3}))


if __name__ == "__main__":
    which = sys.argv[1] if len(sys.argv) > 1 else "confidence"
    {"confidence": confidence, "gemm": gemm, "sched": sched, "ceilings": ceilings, "blocks": blocks}[which]()
