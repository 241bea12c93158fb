#!/usr/bin/env python3
"""Benchmark of the batched beam-search path on one MI355X.

A "step" is one pass of the whole hot path over one batch: encoder projection,
then the data-dependent number of beam-search steps (joint, selection / tree /
recombination, prediction network, optional LM), then the back-trace, plus the
copy of the n-best lists to the host.  The headline workload is the RNN-T ALSD++
case of batch 32, T = 125 frames (10 s of audio each), beam 4, float32, with
synthetic inputs of the model's shapes resident in HBM before the clock starts.
The other workloads (tiny, bf16-joint variant, TDT AES++, LM fusion, large
stateless) are measured the same way with fewer passes and reported under
"workloads" in the same line.

Prints ONE JSON line: metric = RTFx (audio seconds decoded per wall second).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X, dense fp32 matrix
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

LOOP_KERNELS = ("k_step_main", "k_select", "k_lstm_pointwise", "k_pred_proj", "k_lm_rows", "k_joint_big", "k_row_select",
                "k_utt_select", "k_stateless_pre")


def gate_tiles_in_projection_launch(c: dict, M: int) -> int:
    """How many of the 4P / 32 gate tiles of W_hh h ride in the projection launch (the rest are in the main
    launch): the library's rule, restated here to count each launch's FLOPs."""
    from paper_2506_00185_amd.binding import block_map
    m_tiles = (M + 31) // 32
    if c["P"] % 128 == 0 and M >= 8 and (c["H"] // 32) * m_tiles * 2 <= 200:
        return 0  # projection split in two along k, all gate tiles in the main launch
    for b_end in range(4 * c["P"] // 32, 0, -1):
        if block_map(c["H"] // 32, m_tiles, 0, b_end, m_tiles)[0] <= 256:
            return b_end
    return 0


def uses_materialized_path(c: dict, M: int) -> bool:
    return c["prec"] == "bf16" and c["pred"] == "stateless" and c["V"] >= 2048 and M >= 128


def kernel_flops(name: str, c: dict, M: int, B: int, T: int) -> float:
    """Algorithmic floating-point operations of one launch (multiply-add = 2)."""
    nd = len(c["durations"])
    joint = 2.0 * M * c["H"] * (c["V"] + 1 + nd)
    # recurrent half of the LSTM gates; the embedding half is a table made at create
    recurrent = 2.0 * M * c["P"] * 4 * c["P"] if c["pred"] == "lstm" else 0.0
    in_proj = gate_tiles_in_projection_launch(c, M) / (4 * c["P"] / 32) if c["pred"] == "lstm" else 0.0
    if name == "k_step_main":  # joint blocks and recurrent-product blocks share the launch
        return joint + recurrent * (1.0 - in_proj)
    if name == "k_pred_proj":
        return (2.0 * M * c["P"] * c["H"] + recurrent * in_proj) if c["pred"] == "lstm" else 0.0
    if name == "k_joint_big":  # token columns only; blank and duration rows are done by the row kernel
        return 2.0 * M * c["H"] * c["V"]
    if name.startswith("k_gemm_tiled"):
        return 2.0 * B * T * c["D"] * c["H"]
    return 0.0


def kernel_bytes(name: str, c: dict, M: int, B: int, T: int, K: int, steps: int) -> float:
    """Algorithmic HBM bytes of one launch: every operand and result once (weights included: the caches that hold
    them do not survive a kernel boundary)."""
    H, P, V, D = c["H"], c["P"], c["V"], c["D"]
    nd = len(c["durations"])
    n_chunks = (V + 1 + nd + 31) // 32
    lm = 4.0 * M * V if c["lm"] else 0.0
    lstm = c["pred"] == "lstm"
    in_proj = gate_tiles_in_projection_launch(c, M) / (4 * P / 32) if lstm else 0.0
    state = 64.0 * M                      # hypothesis state read and written by the selection
    tree = 12.0 * M                       # parent, token, merged-into
    if name == "k_step_main":
        lists = M * n_chunks * (8.0 * K + 8.0)
        rec = (4.0 * 4 * P * P + 4.0 * M * P + 4.0 * M * 4 * P) * (1.0 - in_proj) if lstm else 0.0
        return 4.0 * n_chunks * 32 * H + 4.0 * M * H + 2 * lists + rec + lm + state + tree
    # LM rows (unigram row read, row written) ride in the projection launch while a row is at most 16 KiB, else in the
    # cell-update launch
    lm_in_proj = 4.0 * V <= 16 * 1024
    if name == "k_lstm_pointwise":        # R, G rows, c in / out, h out
        return M * P * (16.0 + 16.0 + 4.0 + 4.0 + 4.0) + (0.0 if lm_in_proj else 2 * lm)
    if name == "k_pred_proj":
        rec = (4.0 * 4 * P * P + 4.0 * M * P + 4.0 * M * 4 * P) * in_proj if lstm else 0.0
        return 4.0 * H * P + 4.0 * M * P + 4.0 * M * H + 4.0 * M * H + rec + (2 * lm if lm_in_proj else 0.0)
    if name == "k_lm_rows":
        return 2 * lm
    if name == "k_select":                # stand-alone selection from one list per hypothesis
        return M * (8.0 * K + 8.0 + 4.0 * (1 + nd)) + state + tree
    if name in ("k_row_select", "k_utt_select"):
        # without an LM: the chunk statistics (8 bytes per 32 columns) and about 2 K chunks of 128 bytes per row;
        # with one: one read of the float32 logits and of the LM rows.  Then the tail: selection and activations
        Npad = (V + 255) // 256 * 256
        scan = 4.0 * M * Npad + lm if c["lm"] else M * (8.0 * Npad / 32 + 2 * K * 128.0)
        return scan + M * (8.0 * K + 8.0 + 4.0 * (1 + nd)) + state + tree + M * H * (4.0 * (1 + c["ctx"]) + 2.0)
    if name == "k_stateless_pre":
        return M * H * (4.0 * (1 + c["ctx"]) + (2.0 if uses_materialized_path(c, M) else 4.0))
    if name == "k_joint_big":
        Npad, Hb = (V + 255) // 256 * 256, (H + 63) // 64 * 64
        return 2.0 * Npad * Hb + 2.0 * M * Hb + 4.0 * M * Npad + 8.0 * M * Npad / 32  # logits and chunk statistics out
    if name.startswith("k_gemm_tiled"):
        return 4.0 * (B * T * D + H * D + B * T * H)
    if name == "k_backtrace":
        return 8.0 * M * steps + 12.0 * M + 4.0 * M * (T * c["s"] + 1) * 0.25
    return 0.0


def kernel_bound(name: str, c: dict) -> tuple:
    """(bound, peak, unit) of a kernel: the contractions against the matrix-core peak of the type they multiply in,
    everything else against HBM."""
    if name == "k_joint_big":
        return "mfma", PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"
    if name in ("k_step_main", "k_pred_proj"):  # the recurrent product (most of the launch's FLOPs) is float32 always
        return "mfma", PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"
    if name.startswith("k_gemm_tiled"):
        return "mfma", PEAK_BF16_MFMA_TFLOPS if c["prec"] == "bf16" else PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"
    return "hbm", PEAK_HBM_GBS, "GB/s"


def measure(S, A, torch, cid: int, variant: str, steps: int, warmup: int, args, want_cpu: bool) -> dict:
    """One workload: timed passes, the same kernels at beam 1, per-kernel durations, roofline of the dominant kernel."""
    import numpy as np
    c = S.config(cid, prec=variant if cid == 2 else S.CONFIGS[cid]["prec"])
    if args.tdt_pairs and c["model"] == "tdt":
        c["tdt_pairs"] = True
    if args.algo:
        c["algo"] = args.algo
        if args.algo == "alsd":
            c["gamma"] = float("inf")  # the prune margin belongs to AES++
    if args.beam:
        c["beam"] = args.beam
    w = S.make_weights(c)
    L = S.make_lengths(c)
    enc = S.make_enc(c, L)
    lm = lm_arrays = None
    if c["lm"]:
        lm_arrays = S.make_lm(c["V"], c["lm"]["order"], c["lm"]["n_target"], c["lm"]["zipf_s"], 1000 * c["id"] + 3)
        lm = A.NGramLM(lm_arrays)
    dec = A.BeamDecoder(c, w, use_graph=not args.no_graph, lm_rule=args.lm_rule, lm_prune=args.lm_prune,
                        async_enqueue=args.async_enqueue, persistent=args.single_launch)
    d_enc = torch.as_tensor(enc).cuda().contiguous()
    d_len = torch.as_tensor(L).cuda().contiguous()
    audio_s = S.audio_seconds(L)
    B, T, K = c["B"], c["T"], c["beam"]

    def one_pass(beam=None):
        dec.decode(d_enc, d_len, beam=beam, lm=lm, lm_weight=c["lm_weight"])
        return dec.results()

    for _ in range(warmup):
        r = one_pass()
    torch.cuda.synchronize()
    per_pass = []
    t0 = time.perf_counter()
    for _ in range(steps):
        t1 = time.perf_counter()
        r = one_pass()  # (results() waits for the decode and copies the n-best lists)
        per_pass.append((time.perf_counter() - t1) * 1e3)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / steps * 1e3
    value = audio_s * steps / dt
    n_steps = int(r["n_steps"].max())
    gpu_ms = dec.last_decode_ms()

    # same kernels at beam 1 (greedy)
    n1 = max(3, steps // 2)
    for _ in range(2):
        one_pass(beam=1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n1):
        one_pass(beam=1)
    torch.cuda.synchronize()
    ms_beam1 = (time.perf_counter() - t0) / n1 * 1e3

    # per-kernel durations, HIP events on the decode's stream (one kernel at a time, no graph)
    dec.set_profiling(True)
    one_pass()
    kt = dec.kernel_times()
    dec.set_profiling(False)
    M = B * K
    kernels = {}
    for n, (t, k) in kt.items():
        if not k:
            continue
        us = t / k * 1e3
        fl, by = kernel_flops(n, c, M, B, T), kernel_bytes(n, c, M, B, T, K, n_steps)
        bound, peak, unit = kernel_bound(n, c)
        ent = dict(total_ms=round(t, 4), launches=k, avg_us=round(us, 3), bound=bound)
        if fl:
            ent["tflops"] = round(fl / (us * 1e-6) / 1e12, 3)
        if by:
            ent["gbs"] = round(by / (us * 1e-6) / 1e9, 1)
            ent["bytes_per_launch"] = round(by)
        ent["frac_of_bound"] = round((ent.get("tflops", 0.0) if bound == "mfma" else ent.get("gbs", 0.0)) / peak, 5)
        kernels[n] = ent
    loop = {n: v for n, v in kernels.items() if n in LOOP_KERNELS}
    dom = max(loop, key=lambda n: loop[n]["total_ms"])
    bound, peak, unit = kernel_bound(dom, c)
    work = kernel_flops(dom, c, M, B, T) if bound == "mfma" else kernel_bytes(dom, c, M, B, T, K, n_steps)
    achieved = work / (loop[dom]["avg_us"] * 1e-6) / (1e12 if bound == "mfma" else 1e9)
    roofline = dict(kernel=dom, bound=bound, achieved=round(achieved, 3), peak=peak, unit=unit,
                    frac=round(achieved / peak, 5), traffic=None, avg_us=loop[dom]["avg_us"],
                    timing="HIP events around each plain launch (holds the dispatch latency after the previous command)")
    roofline["flops_per_launch" if bound == "mfma" else "bytes_per_launch"] = work
    # from the committed rocprofv3 summaries: HBM bytes per launch (FETCH_SIZE / WRITE_SIZE) and the kernel's duration
    # inside the replayed graph
    name = c["name"] + ("_bf16joint" if cid == 2 and variant == "bf16" else "")
    tpath = os.path.join(ROOT, "profiles", "%s_%s_traffic.json" % (name, dom))
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        roofline["traffic"] = round(tj["fetch_bytes"] + tj["write_bytes"])
        roofline["traffic_source"] = os.path.relpath(tpath, ROOT)
    gpath = os.path.join(ROOT, "profiles", "%s_in_graph.json" % name)
    if os.path.exists(gpath):
        with open(gpath) as f:
            gj = json.load(f)
        if dom in gj.get("kernels", {}):
            us = gj["kernels"][dom]["avg_us"]
            ach = work / (us * 1e-6) / (1e12 if bound == "mfma" else 1e9)
            roofline["in_graph"] = dict(avg_us=us, achieved=round(ach, 3), frac=round(ach / peak, 5),
                                        source=os.path.relpath(gpath, ROOT))
    out = dict(
        value=round(value, 1), unit="audio-s/s", steps=steps, warmup=warmup, ms_per_step=round(ms, 4),
        ms_per_step_median=round(statistics.median(per_pass), 4), ms_per_step_min=round(min(per_pass), 4),
        dtype="f32" if c["prec"] == "f32" else "bf16",
        config={"workload": name, "B": B, "T": T, "beam": K, "algo": c["algo"], "V": c["V"], "max_symbols": c["s"],
                "graph": not args.no_graph, "audio_s_per_pass": audio_s,
                **({"lm_rule": args.lm_rule, "lm_prune": args.lm_prune} if c["lm"] else {}),
                **({"tdt_pairs": True} if c.get("tdt_pairs") else {}),
                **({"async_enqueue": True} if args.async_enqueue else {}),
                **({"step_loop": "single launch"} if args.single_launch else {})},
        beam_search_steps=n_steps, us_per_beam_step=round(gpu_ms * 1e3 / max(n_steps, 1), 3),
        gpu_ms_per_pass=round(gpu_ms, 4), beam1_ms_per_pass=round(ms_beam1, 4), beam_over_greedy=round(ms / ms_beam1, 4),
        roofline=roofline, kernels=kernels)
    joint = "k_joint_big" if "k_joint_big" in loop else "k_step_main"
    out["joint_launch_mfma_util"] = loop[joint]["frac_of_bound"]
    if want_cpu:
        import oracle
        n_utt = min(args.cpu_utts, B)
        olm = oracle.LM(lm_arrays) if lm_arrays is not None else None
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
        out["cpu_baseline"] = cpu
    dec.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="workload id (2 = the headline case)")
    ap.add_argument("--variant", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--no-graph", action="store_true", help="launch the step kernels one by one")
    ap.add_argument("--async-enqueue", action="store_true", help="enqueue the upper bound of steps without following the device")
    ap.add_argument("--single-launch", action="store_true",
                    help="the whole step loop as one launch (persistent_kernel) where it applies, instead of the "
                         "replayed graph of per-step kernels")
    ap.add_argument("--lm-rule", type=int, default=4, choices=[3, 4], help="LM fusion rule (workloads with an LM)")
    ap.add_argument("--lm-prune", default="late", choices=["late", "early"])
    ap.add_argument("--tdt-pairs", action="store_true", help="TDT workloads: every (symbol, duration) pair a candidate")
    ap.add_argument("--algo", default=None, choices=["alsd", "aes"], help="override the workload's search algorithm")
    ap.add_argument("--beam", type=int, default=0, help="override the workload's beam (the paper's Tab. 2 uses 6)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-workloads", action="store_true", help="only the workload named by --config")
    ap.add_argument("--cpu-utts", type=int, default=16, help="utterances the oracle decodes for the CPU baseline")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this size five times (scale for the FETCH_SIZE / "
                         "WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (utterances would be sharded "
              "across GPUs with no collective in the loop); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

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

    head = measure(S, A, torch, args.config, args.variant, args.steps, args.warmup, args, not args.no_cpu_baseline)
    out = {
        "metric": "batched beam decode throughput (audio-s/s, RTFx) at beam %d" % head["config"]["beam"],
        "value": head["value"], "unit": "audio-s/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
    }
    for k in ("config", "ms_per_step_median", "ms_per_step_min", "beam_search_steps", "us_per_beam_step", "gpu_ms_per_pass",
              "beam1_ms_per_pass", "beam_over_greedy", "joint_launch_mfma_util", "roofline"):
        out[k] = head[k]
    out["cpu_baseline"] = head.get("cpu_baseline")
    out["kernels"] = head["kernels"]
    # the other workloads, fewer passes each; no oracle leg (the parity tests compare them with the oracle)
    if not args.no_workloads and args.config == 2 and args.variant == "f32":
        others = {}
        for cid, variant in ((1, "f32"), (2, "bf16"), (3, "f32"), (4, "f32"), (5, "bf16")):
            m = measure(S, A, torch, cid, variant, 3, 1, args, False)
            others[m["config"]["workload"]] = m
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
