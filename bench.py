#!/usr/bin/env python3
"""Benchmark of the batched beam-search path on one MI355X.

A "step" is one pass of the whole hot path over one batch: encoder projection,
then the data-dependent number of beam-search steps (joint, selection / tree /
recombination, prediction network, optional LM), then the back-trace, plus the
copy of the n-best lists to the host.  The workload is the RNN-T ALSD++ case of
batch 32, T = 125 frames (10 s of audio each), beam 4, float32, with synthetic
inputs of the model's shapes resident in HBM before the clock starts.

Prints ONE JSON line: metric = RTFx (audio seconds decoded per wall second).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X, dense fp32 matrix
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def gate_tiles_in_projection_launch(c: dict, M: int) -> int:
    """How many of the 4P / 32 gate tiles of W_hh h ride in the projection launch (the rest are in the main
    launch): the library's rule, restated here to count each launch's FLOPs."""
    from paper_2506_00185_amd.binding import block_map
    m_tiles = (M + 31) // 32
    if c["P"] % 128 == 0 and M >= 8 and (c["H"] // 32) * m_tiles * 2 <= 256:
        return 0  # projection split in two along k, all gate tiles in the main launch
    for b_end in range(4 * c["P"] // 32, 0, -1):
        if block_map(c["H"] // 32, m_tiles, 0, b_end, m_tiles)[0] <= 256:
            return b_end
    return 0


def kernel_flops(name: str, c: dict, M: int, B: int, T: int) -> float:
    """Algorithmic floating-point operations of one launch (multiply-add = 2)."""
    nd = len(c["durations"])
    joint = 2.0 * M * c["H"] * (c["V"] + 1 + nd)
    # recurrent half of the LSTM gates; the embedding half is a table made at create
    recurrent = 2.0 * M * c["P"] * 4 * c["P"] if c["pred"] == "lstm" else 0.0
    in_proj = gate_tiles_in_projection_launch(c, M) / (4 * c["P"] / 32) if c["pred"] == "lstm" else 0.0
    if name == "k_step_main":  # joint blocks and recurrent-product blocks share the launch
        return joint + recurrent * (1.0 - in_proj)
    if name == "joint":
        return joint
    if name in ("k_pred_proj", "k_pred_proj_half"):
        return (2.0 * M * c["P"] * c["H"] + recurrent * in_proj) if c["pred"] == "lstm" else 0.0
    if name == "k_joint_big":  # token columns only; blank and duration rows are done by the row kernel
        return 2.0 * M * c["H"] * c["V"]
    if name.startswith("k_gemm_nt"):
        return 2.0 * B * T * c["D"] * c["H"]
    return 0.0


def kernel_bytes(name: str, c: dict, M: int) -> float:
    """Algorithmic HBM bytes of one launch of the kernels that are bound by memory traffic."""
    if name == "k_row_select":  # one read of the float32 logits of every hypothesis
        return 4.0 * M * c["V"] + (4.0 * M * c["V"] if c["lm"] else 0.0)
    return 0.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="workload id (2 = the headline case)")
    ap.add_argument("--variant", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--no-graph", action="store_true", help="launch the step kernels one by one")
    ap.add_argument("--lm-rule", type=int, default=4, choices=[3, 4], help="LM fusion rule (workloads with an LM)")
    ap.add_argument("--lm-prune", default="late", choices=["late", "early"])
    ap.add_argument("--tdt-pairs", action="store_true", help="TDT workloads: every (symbol, duration) pair a candidate")
    ap.add_argument("--algo", default=None, choices=["alsd", "aes"], help="override the workload's search algorithm")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-utts", type=int, default=16, help="utterances the oracle decodes for the CPU baseline")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this size five times (scale for the FETCH_SIZE / "
                         "WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (utterances would be sharded "
              "across GPUs with no collective in the loop); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as S
    import paper_2506_00185_amd as A

    assert torch.cuda.is_available(), "needs an MI355X"
    if args.copy_calibration:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.arange(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_MiB": args.copy_calibration, "bytes_read": n * 4, "bytes_written": n * 4}))
        return
    c = S.config(args.config, prec=args.variant if args.config == 2 else S.CONFIGS[args.config]["prec"])
    if args.tdt_pairs:
        assert c["model"] == "tdt", "--tdt-pairs needs a TDT workload (config 3)"
        c["tdt_pairs"] = True
    if args.algo:
        c["algo"] = args.algo
        if args.algo == "alsd":
            c["gamma"] = float("inf")  # the prune margin belongs to AES++
    w = S.make_weights(c)
    L = S.make_lengths(c)
    enc = S.make_enc(c, L)
    lm = None
    if c["lm"]:
        lm = A.NGramLM(S.make_lm(c["V"], c["lm"]["order"], c["lm"]["n_target"], c["lm"]["zipf_s"], 1000 * c["id"] + 3))
    dec = A.BeamDecoder(c, w, use_graph=not args.no_graph, lm_rule=args.lm_rule, lm_prune=args.lm_prune)
    d_enc = torch.as_tensor(enc).cuda().contiguous()
    d_len = torch.as_tensor(L).cuda().contiguous()
    audio_s = S.audio_seconds(L)
    B, T, K = c["B"], c["T"], c["beam"]

    def one_pass(beam=None):
        dec.decode(d_enc, d_len, beam=beam, lm=lm, lm_weight=c["lm_weight"])
        return dec.results()

    for _ in range(args.warmup):
        r = one_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        r = one_pass()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / args.steps * 1e3
    value = audio_s * args.steps / dt
    n_steps = int(r["n_steps"].max())
    gpu_ms = dec.last_decode_ms()

    # same kernels at beam 1 (greedy)
    for _ in range(2):
        one_pass(beam=1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(max(3, args.steps // 2)):
        r1 = one_pass(beam=1)
    torch.cuda.synchronize()
    ms_beam1 = (time.perf_counter() - t0) / max(3, args.steps // 2) * 1e3

    # per-kernel durations, HIP events on the decode's stream (one kernel at a time, no graph)
    dec.set_profiling(True)
    one_pass()
    kt = dec.kernel_times()
    dec.set_profiling(False)
    kernels = {n: dict(total_ms=round(t, 4), launches=k, avg_us=round(t / k * 1e3, 3) if k else None,
                       tflops=round(kernel_flops(n, c, B * K, B, T) / (t / k * 1e-3) / 1e12, 3) if k and t > 0 else None,
                       gbs=round(kernel_bytes(n, c, B * K) / (t / k * 1e-3) / 1e9, 1) if k and t > 0 else None)
               for n, (t, k) in kt.items() if k}
    loop = {n: v for n, v in kernels.items()
            if n in ("k_step_main", "k_select", "k_lstm_pointwise", "k_pred_proj", "k_pred_proj_half", "k_lm_rows",
                     "k_joint_big", "k_row_select")}
    dom = max(loop, key=lambda n: loop[n]["total_ms"])
    flops = kernel_flops(dom, c, B * K, B, T)
    nbytes = kernel_bytes(dom, c, B * K)
    if nbytes:
        achieved = nbytes / (loop[dom]["avg_us"] * 1e-6) / 1e9
        roofline = dict(kernel=dom, bound="hbm", achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBS, 5), traffic=None, avg_us=loop[dom]["avg_us"],
                        bytes_per_launch=nbytes)
    else:
        # the fused kernels contract on the fp32 matrix instructions, k_joint_big on the bf16 ones
        peak = PEAK_BF16_MFMA_TFLOPS if dom == "k_joint_big" else PEAK_FP32_MFMA_TFLOPS
        achieved = flops / (loop[dom]["avg_us"] * 1e-6) / 1e12 if flops else 0.0
        roofline = dict(kernel=dom, bound="mfma", achieved=round(achieved, 3), peak=peak, unit="TFLOP/s",
                        frac=round(achieved / peak, 5), traffic=None, avg_us=loop[dom]["avg_us"],
                        flops_per_launch=flops)
    # HBM bytes per launch of that kernel, from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries
    tpath = os.path.join(ROOT, "profiles", "%s_%s_traffic.json" % (c["name"], dom))
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        roofline["traffic"] = round(tj["fetch_bytes"] + tj["write_bytes"])
        roofline["traffic_source"] = os.path.relpath(tpath, ROOT)
    # utilisation of the matrix cores by the launch that holds the joint
    if "k_joint_big" in loop:
        joint_util = (kernel_flops("k_joint_big", c, B * K, B, T) / (loop["k_joint_big"]["avg_us"] * 1e-6) / 1e12
                      / PEAK_BF16_MFMA_TFLOPS)
    else:  # the joint shares its launch with the recurrent product
        joint_util = (kernel_flops("k_step_main", c, B * K, B, T) / (loop["k_step_main"]["avg_us"] * 1e-6) / 1e12
                      / PEAK_FP32_MFMA_TFLOPS)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_utt = min(args.cpu_utts, B)
        olm = oracle.LM(S.make_lm(c["V"], c["lm"]["order"], c["lm"]["n_target"], c["lm"]["zipf_s"],
                                  1000 * c["id"] + 3)) if c["lm"] else None
        t0 = time.perf_counter()
        o = oracle.decode(dict(c, B=n_utt), w, enc[:n_utt], L[:n_utt], lm=olm, lm_weight=c["lm_weight"],
                          lm_rule=args.lm_rule, lm_prune=args.lm_prune)
        cdt = time.perf_counter() - t0
        cpu = dict(value=round(S.audio_seconds(L[:n_utt]) / cdt, 2), unit="audio-s/s", cores=int(o["threads"]),
                   kind="oracle", sample=f"first {n_utt} of {B} utterances of the same workload, {cdt:.1f} s wall")
        # the sampled utterances double as a check of this run
        same = sum(int(np.array_equal(o["tokens"][b, 0, :o["lens"][b, 0]], r["tokens"][b, 0, :r["lens"][b, 0]]))
                   for b in range(n_utt))
        cpu["best_hypothesis_identical"] = f"{same}/{n_utt}"

    out = {
        "metric": "batched beam decode throughput (audio-s/s, RTFx) at beam %d" % K,
        "value": round(value, 1), "unit": "audio-s/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if c["prec"] == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": c["name"] + ("" if c["prec"] == "f32" or args.config != 2 else "_bf16joint"),
                   "B": B, "T": T, "beam": K, "algo": c["algo"], "V": c["V"], "max_symbols": c["s"],
                   "graph": not args.no_graph, "audio_s_per_pass": audio_s,
                   **({"lm_rule": args.lm_rule, "lm_prune": args.lm_prune} if c["lm"] else {}),
                   **({"tdt_pairs": True} if c.get("tdt_pairs") else {})},
        "beam_search_steps": n_steps, "us_per_beam_step": round(gpu_ms * 1e3 / max(n_steps, 1), 3),
        "gpu_ms_per_pass": round(gpu_ms, 4), "beam1_ms_per_pass": round(ms_beam1, 4),
        "beam_over_greedy": round(ms / ms_beam1, 4), "joint_launch_mfma_util": round(joint_util, 5),
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
