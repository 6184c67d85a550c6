"""Which (hi, lo) activation pairs need their low part?  A measurement, run by name on the GPU machine:

    python tests/ablate_low_parts.py [config number, default 3] [oracle-followed requests, default 10]

Builds the full-size workload once (the oracle follows a sample of the requests through its own draft chain, as
in test_gpu_fullsize.py), then runs the same verify with the low part of one site at a time written as zeros
(synera_debug_set_lo_off: numerically the second matrix-core term of that product dropped) and prints
max |dlogit| against the float64 oracle for each.  A site whose line stays at the baseline could run on a single
term; the 2e-2 tolerance with a 1.5x margin is the gate.  Not collected by pytest (a measurement, not a test).
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import numpy as np  # noqa: E402

import gpu_harness as gh  # noqa: E402
import paper_2511_07423_amd as synera  # noqa: E402
import workloads as wl  # noqa: E402


def main():
    n = int(sys.argv[1]) if len(sys.argv) > 1 else 3
    n_oracle = int(sys.argv[2]) if len(sys.argv) > 2 else 10
    rec = wl.config(n)
    weights = gh.draw_weights(rec.shape, wl.config(2).seed if rec.shape.name == wl.LLAMA_8B.name else rec.seed, "cuda:0")
    case = gh.build_case(rec, "cuda:0", n_oracle=n_oracle, weights=weights, verbose=True)
    sites = ["qkv_in", "gate_up_in", "down_in", "o_in", "lm_head_in", "q", "p"]
    runs = [("default (pairs; LM head: high part)", [])] + [(f"no lo at {s}", [s]) for s in sites] + \
           [("no lo at any projection input", ["qkv_in", "gate_up_in", "down_in", "o_in", "lm_head_in"]),
            ("no lo at q and p", ["q", "p"]), ("lo kept at the LM head too", ["keep_lm_head"]), ("default again", [])]
    print(f"config {n} ({rec.name}): {len(case.sampled)} requests followed by the oracle, "
          f"{int(sum(case.batch['n_draft'][i] for i in case.sampled))} rows", flush=True)
    print(f"{'variant':34s} {'max|dlogit|':>12s} {'rms dlogit':>12s} {'argmax rows differing':>22s}", flush=True)
    for name, off in runs:
        case.verifier.debug_set_lo_off(off)
        out = gh.run_verify(case)
        cu = np.concatenate([[0], np.cumsum(case.batch["n_draft"])])
        worst, sq, cnt, flips = 0.0, 0.0, 0, 0
        for i in case.sampled:
            want = case.want_rows[i]
            d = out["logits"][int(cu[i]):int(cu[i + 1])].astype(np.float64) - want
            worst = max(worst, float(np.abs(d).max()))
            sq += float((d * d).sum())
            cnt += d.size
            flips += int((out["argmax"][int(cu[i]):int(cu[i + 1])] != want.argmax(axis=1)).sum())
        print(f"{name:34s} {worst:12.3e} {np.sqrt(sq / cnt):12.3e} {flips:22d}", flush=True)
    case.verifier.debug_set_lo_off(0)
    case.verifier.close()


if __name__ == "__main__":
    main()
