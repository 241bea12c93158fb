"""Batch / beam sweeps and the graph on / off ablation of the decoder on one MI355X.

Shaped like the paper's Tab. 2 (decoder-only RTFx against batch size, greedy vs beam) and Tab. 3
(RTFx against beam size), and its Tab. 1 rows with and without graph replay, on the synthetic
RNN-T (or TDT) workload of `synth_inputs` (no trained model or dataset is available, so only the
speed columns exist).  Prints markdown tables.

    python -m paper_2506_00185_amd.sweep [--model rnnt|tdt] [--algo alsd|aes] [--repeats 3]
"""
from __future__ import annotations

import argparse
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="rnnt", choices=["rnnt", "tdt"])
    ap.add_argument("--algo", default="alsd", choices=["alsd", "aes"])
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--batches", default="1,4,8,16,32")
    ap.add_argument("--beams", default="1,2,4,6,8,12")
    args = ap.parse_args()

    import torch
    import synth_inputs as S
    import paper_2506_00185_amd as A

    base = S.config(3 if args.model == "tdt" else 2)
    base = dict(base, algo=args.algo, T=125, T_min=125, gamma=float("inf"))
    batches = [int(x) for x in args.batches.split(",")]
    beams = [int(x) for x in args.beams.split(",")]
    w = S.make_weights(base)
    Bmax, Kmax = max(batches), max(beams)
    L = S.make_lengths(dict(base, B=Bmax))
    enc = S.make_enc(dict(base, B=Bmax), L)
    d_enc = torch.as_tensor(enc).cuda().contiguous()
    d_len = torch.as_tensor(L).cuda().contiguous()

    def run(dec, B, K):
        dec.decode(d_enc[:B].contiguous(), d_len[:B].contiguous(), beam=K)
        r = dec.results()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.repeats):
            dec.decode(d_enc[:B].contiguous(), d_len[:B].contiguous(), beam=K)
            r = dec.results()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.repeats
        return S.audio_seconds(L[:B]) / dt, dt * 1e3, int(r["n_steps"].max())

    decs = {g: A.BeamDecoder(base, w, max_B=Bmax, max_T=base["T"], max_beam=Kmax, use_graph=g) for g in (True, False)}
    print(f"# {args.model.upper()} {args.algo.upper()}++, T = {base['T']} frames per utterance, synthetic weights, one MI355X\n")
    print("## RTFx against batch size (graph replay)\n")
    print("| batch | " + " | ".join(f"beam {k}" for k in beams) + " | beam 4 / beam 1 time |")
    print("|---|" + "---|" * (len(beams) + 1))
    for B in batches:
        row, ms = [], {}
        for K in beams:
            rtfx, m, steps = run(decs[True], B, K)
            ms[K] = m
            row.append(f"{rtfx:.0f}")
        ratio = f"{ms[4] / ms[1]:.2f}" if 4 in ms and 1 in ms else "-"
        print(f"| {B} | " + " | ".join(row) + f" | {ratio} |")
    print("\n## Graph replay against plain launches (batch %d)\n" % Bmax)
    print("| beam | steps | graph ms | plain ms | plain / graph |")
    print("|---|---|---|---|---|")
    for K in beams:
        _, mg, steps = run(decs[True], Bmax, K)
        _, mp, _ = run(decs[False], Bmax, K)
        print(f"| {K} | {steps} | {mg:.2f} | {mp:.2f} | {mp / mg:.2f} |")


if __name__ == "__main__":
    main()
