#!/usr/bin/env python3
"""Benchmark of the batched-verify hot path on one MI355X.

A step is one synera_verify call over the whole batch of the headline workload (the ragged
selective-offload batch on the 8B shape: 64 requests, contexts log-uniform in [128, 4096], chunk
lengths uniform in 1..16, bf16 weights).  Everything is synthetic and seeded; weights, KV pools,
block tables, tokens and drafts are resident in HBM before the timed region starts (the call's
own small metadata upload is part of the step).  Drafts come from the library's own greedy chain
(draft j is the current greedy token with the config's match probability, else a random token).

Prints ONE JSON line: verified draft tokens/s, plus
  roofline     - the dominant kernel (gate/up projection + SiLU*mul) timed with HIP events inside
                 the timed region, its algorithmic FLOPs against the dense bf16 MFMA peak;
  stages       - the same fields for every projection, the attention kernel and the vocabulary
                 reduction, each timed with HIP events in a few further steps of the same process;
  cpu_baseline - the CPU oracle timed on a bounded sample of the same workload (this leg is the
                 only place the benchmark touches the oracle).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch (read + written) of the stage kernels on the default workload, from the two rocprofv3
# --pmc passes (FETCH_SIZE, WRITE_SIZE) whose summary, commands and copy-kernel calibration are in
# profiles/gemm_attention_c3_8b_b64_hbm_traffic.md.  Counters cannot be read from inside this process, so the
# roofline objects carry the profiled figure -- but only while the build being timed still launches what was
# profiled: PROFILED_PLAN is the tile plan of the five projections and the attention work plan on that
# workload as they were when the counters were read; if the planners of the library being timed answer
# differently, the traffic fields are null.
PROFILED_WORKLOAD = "c3_8b_b64_ragged"
PROFILED_PLAN = "qkv=272x256pair/5;o=144x256pair/4;gate_up=272x256pair/1;down=272x256pair/8;lm_head=272x256/1;attention=512sh/21270pos/258cut"
MEASURED_TRAFFIC_BYTES = {          # read + written, per launch
    "gate_up": 341.0e6 + 30.5e6,        # 305 - 456 MB read from launch to launch
    "down": 361.9e6 + 69.7e6,
    "qkv": 122.0e6 + 65.4e6,
    "o": 103.6e6 + 34.9e6,
    "attention": 333.0e6 + 15.7e6,
    "lm_head": 302.0e6 + 68.1e6,
}


def plan_fingerprint(synera, shape, b, T):
    """What the library's planners launch for this workload: tile rows x columns / K slices of the five
    projections, and shares / positions / cut streams of the attention work plan."""
    import numpy as np
    d, f, V, qkv = shape.d_model, shape.d_ffn, shape.vocab, shape.q_dim + 2 * shape.kv_dim
    parts = []
    for name, n, k, epi, stored in (("qkv", qkv, d, 0, True), ("o", d, shape.q_dim, 1, True), ("gate_up", 2 * f, d, 2, True),
                                    ("down", d, f, 1, True), ("lm_head", V, d, 0, False)):
        bm, bn, split = synera.debug_gemm_plan(T, n, k, epi, stored)
        # two MFMA K steps per stage, or one with the layers' activation pairs as one array of whole lines
        form = "k64" if synera.debug_gemm_plan_bk(T, n, k, epi, stored) == 64 else ("pair" if stored else "")
        parts.append(f"{name}={bm}x{bn}{form}/{split}")
    plan = synera.debug_attention_plan(shape, 512, b["ctx_len"], np.zeros(len(b["ctx_len"]), np.int32), b["n_draft"],
                                       b["block_table"])
    parts.append(f"attention={len(plan['shares'])}sh/{len(plan['prog'])}pos/{len(plan['cuts'])}cut")
    return ";".join(parts)


def build_workload(cfg_no, device):
    import numpy as np
    import torch
    import paper_2511_07423_amd as synera
    import workloads as wl

    rec = wl.config(cfg_no)
    shape = rec.shape
    b = wl.draw_batch(rec)
    B = len(b["ctx_len"])
    rnd = wl.draw_draft_randoms(rec, B)
    head = wl.draw_head_weights(shape, rec.seed, device)
    layers = [wl.draw_layer_weights(shape, rec.seed, l, device) for l in range(shape.n_layers)]
    pool_dims = (shape.n_layers, b["n_pages"], shape.n_kv_heads)
    k_pool = torch.zeros(pool_dims + (wl.PAGE_SIZE, shape.head_dim), dtype=torch.bfloat16, device=device)
    v_pool = torch.zeros(pool_dims + (shape.head_dim, wl.PAGE_SIZE), dtype=torch.bfloat16, device=device)
    ver = synera.Verifier(shape, head, layers, max_batch=B, max_tokens=int(b["n_draft"].sum()) + B,
                          max_pages=b["max_pages"])
    # cached context: N(0,1) K/V at positions 0..L-2, then a real decode of a random token at L-1
    L = b["ctx_len"]
    n_fill = (L - 1).astype(np.int32)
    zeros = np.zeros(B, np.int32)
    for l in range(shape.n_layers):
        kr, vr = wl.draw_context_kv(shape, rec.seed, l, int(n_fill.sum()), device)
        ver.kv_append(l, zeros, n_fill, kr, vr, b["block_table"], b["n_pages"], k_pool, v_pool)
        torch.cuda.synchronize()
    last = torch.from_numpy(rnd["last_ctx_tok"]).to(device)
    out = ver.verify(n_fill, zeros, np.ones(B, np.int32), last, torch.zeros(B, dtype=torch.int32, device=device),
                     b["block_table"], b["n_pages"], k_pool, v_pool, want_logits=False)
    anchor = out["argmax"].clone()
    # drafts from the library's own greedy chain
    anchors = anchor.cpu().numpy()
    drafts = [[] for _ in range(B)]
    greedy = [int(a) for a in anchors]
    for j in range(int(b["n_draft"].max())):
        live = [i for i in range(B) if b["n_draft"][i] > j]
        for i in live:
            drafts[i].append(greedy[i] if rnd["u"][i][j] < rec.p_match else int(rnd["tok"][i][j]))
        toks = torch.tensor([t for i in live for t in drafts[i]], dtype=torch.int32, device=device)
        o = ver.verify(L[live], np.zeros(len(live), np.int32), np.full(len(live), j + 1, np.int32), toks,
                       anchor[live], b["block_table"][live], b["n_pages"], k_pool, v_pool, want_logits=False)
        am = o["argmax"].cpu().numpy()
        for n, i in enumerate(live):
            greedy[i] = int(am[(n + 1) * (j + 1) - 1])
    tokens = torch.tensor([t for d in drafts for t in d], dtype=torch.int32, device=device)
    return dict(rec=rec, shape=shape, batch=b, head=head, layers=layers, ver=ver, k_pool=k_pool, v_pool=v_pool,
                tokens=tokens, anchor=anchor, drafts=drafts, rnd=rnd)


def cpu_baseline(w, device):
    """Times oracle.verify_chunks (numpy float64 on the host cores) on the first half of the batch's requests
    through the full decoder, LM head and verification.  Each request carries its last context
    token as one uncached token, so the oracle's call is self-contained (it computes q(x|prefix) itself)."""
    import numpy as np
    import oracle
    import workloads as wl

    rec, shape, b = w["rec"], w["shape"], w["batch"]
    B = len(b["ctx_len"])
    n_req = max(1, B // 2) if shape.n_layers * shape.layer_params <= 8e9 else max(1, B // 16)
    to_np = lambda t: t.detach().to("cpu").float().numpy()                     # noqa: E731
    head = {k: to_np(v) for k, v in w["head"].items()}
    lay = [{k: to_np(v) for k, v in w["layers"][l].items()} for l in range(shape.n_layers)]
    L = b["ctx_len"]
    n_fill = (L - 1).astype(np.int64)
    starts = np.concatenate([[0], np.cumsum(n_fill)])
    pages = [p for i in range(n_req) for p in b["block_table"][i] if p >= 0]
    model = oracle.OracleModel(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                               shape.d_ffn, shape.vocab, head["embed"], lay, head["final_norm"], head["lm_head"],
                               rope_base=shape.rope_base, rms_eps=shape.rms_eps)      # the oracle's default: float64
    kv = oracle.PagedKV(shape.n_layers, b["n_pages"], shape.n_kv_heads, shape.head_dim, pages=pages)
    for l in range(shape.n_layers):
        kr, vr = wl.draw_context_kv(shape, rec.seed, l, int(n_fill.sum()), device)
        kr, vr = to_np(kr[: int(starts[n_req])]), to_np(vr[: int(starts[n_req])])
        for i in range(n_req):
            sl = slice(int(starts[i]), int(starts[i + 1]))
            kv.append_many(l, b["block_table"][i], 0, kr[sl], vr[sl])
    reqs = [{"block_table": b["block_table"][i], "ctx_len": int(L[i]) - 1,
             "uncached": [int(w["rnd"]["last_ctx_tok"][i])], "drafts": w["drafts"][i], "anchor": -1}
            for i in range(n_req)]
    n_tok = int(b["n_draft"][:n_req].sum())
    t0 = time.perf_counter()
    oracle.verify_chunks(model, kv, reqs)
    dt = time.perf_counter() - t0
    # the threads the oracle's matrix products really ran on: numpy's BLAS pool
    blas, cores = "unknown BLAS", int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    try:
        from threadpoolctl import threadpool_info
        pools = [p for p in threadpool_info() if p.get("user_api") == "blas"]
        if pools:
            blas = f"{pools[0].get('internal_api')} {pools[0].get('version')}"
            cores = int(pools[0].get("num_threads", cores))
    except Exception:                                                           # noqa: BLE001 (reporting only)
        pass
    return {"value": n_tok / dt, "unit": "verified draft tokens/s", "cores": cores, "kind": "oracle",
            "sample": (f"oracle.verify_chunks (numpy float64, {blas}, {cores} threads) on {n_req} of {B} requests "
                       f"({n_tok} draft tokens, their real contexts), all {shape.n_layers} layers + LM head + "
                       f"verification: {dt:.1f}s")}


def roof_fields(o):
    keep = ("kernel", "bound", "achieved", "peak", "unit", "frac", "algorithmic", "algorithmic_unit", "traffic",
            "avg_launch_ms", "launches")
    return {k: o[k] for k in keep}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload number (3 = the headline ragged batch-64 8B config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="also print per-stage times to stderr")
    ap.add_argument("--stage", default="gate_up", help="kernel stage the roofline object reports")
    ap.add_argument("--stage-steps", type=int, default=5,
                    help="further steps per stage for the `stages` array (each stage bracketed in its own steps)")
    ap.add_argument("--print-plan", action="store_true", help="print the planners' fingerprint for this workload and exit")
    ap.add_argument("--gemm-tile", type=int, default=-1,
                    help="tuning: force one projection tile for the timed steps (rows/16, +100 for 128 columns)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one plain 1 GiB device copy (a known-size dispatch to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (requests are independent, so N GPUs would each verify a "
              "disjoint share of the batch with no exchange step); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2511_07423_amd as synera
    assert torch.cuda.is_available(), "bench.py needs the GPU; there is no CPU path"
    device = "cuda:0"
    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=device)     # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    w = build_workload(args.config, device)
    b, ver, shape = w["batch"], w["ver"], w["shape"]
    B = len(b["ctx_len"])
    T = int(b["n_draft"].sum())
    zeros = np.zeros(B, np.int32)
    ctx, nd, bt = (np.ascontiguousarray(b[k], dtype=np.int32) for k in ("ctx_len", "n_draft", "block_table"))
    out = {"logits": None, "argmax": torch.empty(T, dtype=torch.int32, device=device),
           "top1_prob": torch.empty(T, dtype=torch.float32, device=device),
           "entropy": torch.empty(T, dtype=torch.float32, device=device),
           "accept_len": torch.empty(B, dtype=torch.int32, device=device),
           "correction": torch.empty(B, dtype=torch.int32, device=device)}

    def step():
        ver.verify_into(ctx, zeros, nd, w["tokens"], w["anchor"], bt, b["n_pages"], w["k_pool"], w["v_pool"], out)

    if args.print_plan:
        print(plan_fingerprint(synera, shape, b, T))
        return
    synera.debug_set_gemm_tile(args.gemm_tile)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stage = synera.STAGES[args.stage]
    ver.profile_begin(stage)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_launch, stage_ms = ver.profile_end()
    ms_per_step = dt * 1000.0 / args.steps
    accepted = int(out["accept_len"].sum().item())

    d, f, V = shape.d_model, shape.d_ffn, shape.vocab
    qd, kd = shape.q_dim, shape.kv_dim
    stage_flops = {"qkv": 2.0 * T * d * (qd + 2 * kd), "o": 2.0 * T * qd * d, "gate_up": 2.0 * T * d * 2 * f,
                   "down": 2.0 * T * f * d, "lm_head": 2.0 * T * d * V}
    stage_bytes = {"attention": float((b["ctx_len"] + b["n_draft"]).sum()) * 2 * shape.kv_dim * 2,
                   "confidence": float(T) * V * 4}
    fingerprint = plan_fingerprint(synera, shape, b, T)
    traffic_valid = w["rec"].name == PROFILED_WORKLOAD and fingerprint == PROFILED_PLAN and args.gemm_tile < 0

    def stage_object(name, n_launch, total_ms):
        """The roofline fields of one stage from its HIP-event time: algorithmic FLOPs (2 T params) against the dense
        bf16 MFMA peak for the projections, algorithmic bytes (K/V read once per KV head; the logits once)
        against the HBM peak for attention and the vocabulary reduction."""
        avg_ms = total_ms / max(n_launch, 1)
        if name in stage_flops:
            ach = stage_flops[name] / (avg_ms * 1e-3) / 1e12
            o = {"kernel": name, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                 "frac": ach / MFMA_BF16_PEAK_TFLOPS, "algorithmic": stage_flops[name], "algorithmic_unit": "FLOP per launch"}
        else:
            ach = stage_bytes[name] / (avg_ms * 1e-3) / 1e9
            o = {"kernel": name, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": ach / HBM_PEAK_GBS, "algorithmic": stage_bytes[name], "algorithmic_unit": "bytes per launch"}
        o["traffic"] = MEASURED_TRAFFIC_BYTES.get(name) if traffic_valid else None
        o["avg_launch_ms"] = avg_ms
        o["launches"] = n_launch
        return o

    roof = stage_object(args.stage, n_launch, stage_ms)
    if roof["bound"] == "mfma":
        roof["note"] = ("algorithmic FLOPs 2*T*params; the kernel issues twice that (fp16 hi + lo activation pairs "
                        "against bf16 weights widened to fp16)")
    # the same ceiling measured on this machine, in this process (published peak stays the denominator of frac)
    from paper_2511_07423_amd.measure import measured_ceilings
    meas = measured_ceilings()
    if roof["bound"] == "mfma":
        roof["peak_measured"] = meas["mfma_f16_random_operands_TFLOPs"]
        roof["peak_measured_note"] = ("register-resident loop of the kernel's own MFMA (16x16x32 fp16), random operands "
                                      "(constant operands: %.0f; the 32x32x16 bf16 form: %.0f random, %.0f constant)"
                                      % (meas["mfma_f16_constant_operands_TFLOPs"], meas["mfma_bf16_random_operands_TFLOPs"],
                                         meas["mfma_bf16_constant_operands_TFLOPs"]))
    else:
        roof["peak_measured"] = meas["hbm_read_GBs"]
        roof["peak_measured_note"] = ("read-only stream over 1 GiB (plain device copy, read + written bytes: %.0f)"
                                      % meas["hbm_copy_GBs"])
    roof["traffic_unit"] = "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-kernel calibrated)"
    roof["traffic_plan"] = {"profiled": PROFILED_PLAN, "this_build": fingerprint,
                            "note": "traffic is null unless the planners still launch what the counters were read on"}
    # the other kernels of the step, each bracketed by HIP events in a few further steps of the same process
    stages = []
    for name in ("qkv", "attention", "o", "gate_up", "down", "lm_head", "confidence") if args.stage_steps > 0 else ():
        if name == args.stage:
            stages.append(dict(roof_fields(roof)))
            continue
        ver.profile_begin(synera.STAGES[name])
        for _ in range(args.stage_steps):
            step()
        torch.cuda.synchronize()
        n, ms = ver.profile_end()
        stages.append(stage_object(name, n, ms))
    res = {"metric": "verified draft tokens/sec (8B-shape bf16, batch 64) + % of HBM/MFMA roofline",
           "value": T / (ms_per_step * 1e-3), "unit": "verified draft tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16",
           "dtype_note": ("bf16 weights and KV cache (the metric's model type); matrix-core operands: fp16 (hi, lo) activation "
                          "pairs against the bf16 weights widened exactly to fp16, bf16 pairs against the bf16 cache in "
                          "attention; fp32 accumulation and residual stream"),
           "data": "synthetic",
           "config": {"workload": w["rec"].name, "requests": B, "draft_tokens": T,
                      "context_tokens": int(b["ctx_len"].sum()), "accepted_plus_correction_tokens": accepted + B,
                      "shape": shape.name},
           "roofline": roof, "stages": stages}
    if args.breakdown:                      # extra passes, one stage bracketed at a time (stderr, not the JSON line)
        total = 0.0
        for name, sid in synera.STAGES.items():
            if sid == 0:
                continue
            ver.profile_begin(sid)
            for _ in range(args.steps):
                step()
            torch.cuda.synchronize()
            n, ms = ver.profile_end()
            total += ms / args.steps
            print(f"[breakdown] {name:12s} {ms / args.steps:8.3f} ms/step  {n // args.steps:4d} launches/step  "
                  f"{ms / max(n, 1) * 1e3:9.1f} us/launch", file=sys.stderr, flush=True)
        print(f"[breakdown] stages sum {total:.3f} ms/step vs {ms_per_step:.3f} ms/step wall", file=sys.stderr)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, device)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
