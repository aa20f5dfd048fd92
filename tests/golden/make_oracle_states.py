#!/usr/bin/env python3
"""Writes tests/golden/oracle_states_cfg<N>.json: what the CPU oracle computes along its OWN
decoding trajectory on the full-size benchmark configurations (full depth, full width, full
vocabulary), so that the GPU parity tests can compare against the oracle without spending
minutes of oracle forwards on the GPU machine.

Imports only `oracle/` and the seeded input generators (`psd_inputs`); nothing of the HIP
library.  Run on the CPU (about 40 GB of host memory for an 8B-parameter shape):

    python tests/golden/make_oracle_states.py --config 3 --iterations 2
    python tests/golden/make_oracle_states.py --config 4 --iterations 1
    python tests/golden/make_oracle_states.py --config 5 --iterations 1

Per configuration the file holds, for sequence 0 of the workload and the first block, every
state the oracle's model is called on during the first iterations of Alg. 1 -- the stage-1
state and the K drafts of the batched verification (Sec. 3.2; Eq. 1; Eq. 2) -- with, per state:

  tokens      the state itself, int [N]
  top1, conf  the oracle's (x_hat, c) tables on the block, sentinels included (Sec. 3.1);
              conf as the fp32 value both sides decide on
  runner_up   id of the second-largest logit per block row ([M] excluded)
  margin      top-1 minus runner-up logit per row (exact arithmetic, fp64)
  cols, z     a seeded sample of vocabulary columns and the exact logits there, [L, len(cols)];
              z_top1 / z_runner_up: the logits of the two leading tokens of every row
  bf16        (first and last state of the first iteration only) the same network evaluated
              by the oracle in fp64 with only the contraction operands rounded to bf16:
              its logits at the sampled entries, and max-abs / rms of its difference from
              exact arithmetic over ALL L x V logits.  That is the noise floor of any bf16
              evaluation of this network; the GPU test calibrates its tolerance with it.

and per iteration the oracle's decisions on its own tables (T, sigma, m, accepted, k*, the
post-verification commit and the next state).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import psd_inputs as inp                      # noqa: E402
from oracle import psd_oracle as orc          # noqa: E402

N_SAMPLE_COLS = 24


def state_record(host, tokens, bs, L, cols, kind, with_bf16):
    shape = host.shape
    top1, conf, z = orc.forward_confidence(host, tokens, bs, L, return_logits=True)
    zz = z.copy()
    zz[:, shape.mask_id] = -np.inf
    order = np.argsort(-zz, axis=-1, kind="stable")[:, :2]
    lead, second = order[:, 0], order[:, 1]
    rows = np.arange(L)
    rec = {
        "kind": kind,
        "tokens": [int(t) for t in tokens],
        "top1": [int(t) for t in top1],
        "conf": [float(c) for c in conf],                       # fp32 values, exactly representable in JSON
        "runner_up": [int(t) for t in second],
        "margin": [float(m) for m in (zz[rows, lead] - zz[rows, second])],
        "z_top1": [float(v) for v in z[rows, lead]],
        "z_runner_up": [float(v) for v in z[rows, second]],
        "z": [[float(v) for v in z[r, cols]] for r in range(L)],
        "logit_std": float(z.std()),
    }
    if with_bf16:
        zb = orc.block_logits(host, tokens, bs, L, operands="bf16")
        diff = zb - z
        rec["bf16"] = {
            "z": [[float(v) for v in zb[r, cols]] for r in range(L)],
            "max_abs_all": float(np.abs(diff).max()),
            "rms_all": float(np.sqrt(np.mean(diff * diff))),
        }
    return rec, top1, conf


def run(config, iterations, seq, out_path):
    w = inp.WORKLOADS[config]
    shape, N, bs, L, K = w.shape, w.seq_len, w.prompt_len, w.block_len, w.n_drafts
    t0 = time.perf_counter()
    host = inp.draw_model(shape, N, threads=8)
    print(f"[golden] config {config}: weights drawn after {time.perf_counter() - t0:.0f} s", flush=True)
    policy, graph = orc.Policy(w.tau, w.k_min, w.k_max), orc.chain_graph(K)
    cols = sorted(int(c) for c in np.random.default_rng(1000 + config).choice(shape.vocab - 1, N_SAMPLE_COLS, replace=False))
    x = inp.initial_state(w)[seq]
    out = {
        "config": config, "sequence": seq, "block_start": bs, "L": L, "K": K, "N": N, "vocab": shape.vocab,
        "tau": w.tau, "k_min": w.k_min, "k_max": w.k_max, "cols": cols, "states": [], "iterations": [],
        "written_by": "tests/golden/make_oracle_states.py (oracle only, fp64)",
    }
    for it in range(iterations):
        rec, top1, conf = state_record(host, x, bs, L, cols, "stage1", with_bf16=(it == 0))
        rec["iteration"] = it
        out["states"].append(rec)
        print(f"[golden] config {config} iteration {it}: stage-1 state done after {time.perf_counter() - t0:.0f} s", flush=True)
        x1, transfer = orc.select_unmask(x, bs, L, top1, conf, policy, shape.mask_id)
        sigma, m, drafts = orc.build_drafts(x1, bs, L, top1, conf, graph, shape.mask_id)
        dec = {"iteration": it, "stage1_state": len(out["states"]) - 1, "transfer_mask": [int(t) for t in transfer],
               "sigma": [int(s) for s in sigma], "m": int(m)}
        if m == 0:
            dec["next_tokens"] = [int(t) for t in x1]
            out["iterations"].append(dec)
            x = x1
            break
        v_top1, v_conf, first = [], [], len(out["states"])
        for k in range(K):
            rec, t1, c1 = state_record(host, drafts[k], bs, L, cols, "draft", with_bf16=(it == 0 and k == K - 1))
            rec["iteration"], rec["node"] = it, k
            out["states"].append(rec)
            v_top1.append(t1)
            v_conf.append(c1)
            print(f"[golden] config {config} iteration {it}: draft {k} done after {time.perf_counter() - t0:.0f} s", flush=True)
        v_top1, v_conf = np.stack(v_top1), np.stack(v_conf)
        accepted, k_star = orc.hierarchical_accept(drafts, bs, L, sigma, m, graph, policy, v_top1, v_conf, shape.mask_id)
        x2, n_post = orc.advance(drafts, k_star, bs, L, v_top1, v_conf, policy, shape.mask_id)
        dec.update({"draft_states": list(range(first, first + K)), "accepted": [int(a) for a in accepted],
                    "k_star": int(k_star), "n_postverify": int(n_post), "next_tokens": [int(t) for t in x2]})
        out["iterations"].append(dec)
        x = x2
    out["seconds"] = round(time.perf_counter() - t0)
    with open(out_path, "w") as f:
        json.dump(out, f, separators=(",", ":"))
        f.write("\n")
    print(f"[golden] wrote {out_path} ({os.path.getsize(out_path)} bytes) after {time.perf_counter() - t0:.0f} s", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, required=True, choices=[2, 3, 4, 5])
    ap.add_argument("--iterations", type=int, default=1)
    ap.add_argument("--sequence", type=int, default=0)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    out = args.out or os.path.join(os.path.dirname(os.path.abspath(__file__)), f"oracle_states_cfg{args.config}.json")
    run(args.config, args.iterations, args.sequence, out)


if __name__ == "__main__":
    main()
