"""Parity on randomly drawn small workloads: every selection form (beams 1 to 16), both models, both algorithms, both
prediction networks, both precisions, the fused and the materialised-logits path, prune margins, the prefix search and
n-gram fusion meet shapes that no hand-written case has (odd vocabularies, one to six 32-wide tiles per dimension,
batches that leave tiles ragged).  Each case is the same check as the hand-written ones: trees identical up to a near
tie of the oracle, then the step-by-step walk of the GPU's own tree.

bf16 bars: the noise of a logit from operands rounded on one side only grows as the joint gets narrower (its weights
are ~ N(0, 9 / H)), so the near-tie bar and the score tolerance of the full-width workloads (5e-3, 2e-2 at H = 640) are
scaled by sqrt(640 / H) here, the near-tie bar by another 1.5."""
from __future__ import annotations

import numpy as np
import pytest

import synth_inputs as S
from gpu_common import compare, gpu_decode, make_walk

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def amd():
    import paper_2506_00185_amd as A
    A.load_library()
    return A


def draw_case(rng):
    model = str(rng.choice(["rnnt", "tdt"]))
    algo = str(rng.choice(["alsd", "aes"]))
    pred = str(rng.choice(["lstm", "stateless"]))
    prec = str(rng.choice(["f32", "bf16"]))
    beam = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 16]))
    H, P, D = 32 * int(rng.integers(1, 7)), 32 * int(rng.integers(1, 7)), 32 * int(rng.integers(1, 4))
    T = int(rng.integers(5, 18))
    kw = dict(model=model, algo=algo, pred=pred, prec=prec, beam=beam, V=int(rng.integers(12, 400)), H=H, P=P, E=P, D=D,
              B=int(rng.integers(1, 10)), T=T, T_min=max(1, T // 3), s=int(rng.integers(1, 5)),
              gamma=float(rng.choice([np.inf, 1.5, 3.0])) if algo == "aes" else float("inf"),
              blank_bias=float(rng.choice([2.0, 3.0])))
    if model == "tdt":
        kw["durations"] = (0, 1, 2, 3, 4)
    if pred == "stateless":
        kw["ctx"] = 2
    lm_w = float(rng.choice([0.0, 0.0, 0.3])) if np.isinf(kw["gamma"]) else 0.0  # (an LM with a finite margin is refused)
    prefix = bool(algo == "aes" and lm_w == 0.0 and rng.random() < 0.3)
    if prefix:
        kw["aes_prefix"] = True
    path = "materialized" if (pred == "stateless" and prec == "bf16" and rng.random() < 0.6) else "fused"
    return S.custom_config(**kw), path, lm_w, prefix, int(rng.integers(1, 1 << 30))


@pytest.mark.parametrize("seed", [101, 102, 103])
def test_random_small_workloads(amd, oracle, seed):
    rng = np.random.default_rng(seed)
    for case in range(100):
        c, path, lm_w, prefix, wseed = draw_case(rng)
        print(f"seed {seed} case {case}: {c['model']} {c['algo']} {c['pred']} {c['prec']} beam {c['beam']} V {c['V']} "
              f"H {c['H']} P {c['P']} D {c['D']} B {c['B']} T {c['T']} s {c['s']} gamma {c['gamma']} lm {lm_w} "
              f"prefix {prefix} {path} weights {wseed}", flush=True)
        w = S.perturb_biases(S.make_weights(c, wseed), wseed + 1)  # (so that a dropped bias term shows)
        L = S.make_lengths(c, wseed + 2)
        enc = S.make_enc(c, L, wseed + 3)
        glm = olm = None
        if lm_w:
            lm = S.make_lm(V=c["V"], order=3, n_target=min(3000, c["V"] ** 2 // 3), zipf_s=1.1, seed=wseed + 4)
            glm, olm = amd.NGramLM(lm), oracle.LM(lm)
        wf = max(1.0, (640.0 / c["H"]) ** 0.5)
        tol, tie = (2e-2 * wf, 7.5e-3 * wf) if c["prec"] == "bf16" else (1e-3, 1e-4)
        dec = amd.BeamDecoder(c, w, joint_path=path)
        g = gpu_decode(dec, enc, L, lm=glm, lm_weight=lm_w)
        assert g["rc"] == 0
        o = oracle.decode(c, w, enc, L, lm=olm, lm_weight=lm_w, log=True)
        walk = None if prefix else make_walk(oracle, c, w, enc, L, g, tol, lm=olm, lm_weight=lm_w)
        full, exempt = compare(g, o, tol, tie, walk=walk)
        assert full + exempt == c["B"]
