"""The step-by-step tree walk that the GPU parity tests apply to trees that left the oracle's (tree_check.py),
tried on the CPU: the oracle's own logged tree must pass it, and a tree with one planted defect must not."""
import numpy as np
import pytest

import synth_inputs as S
from tree_check import check_tree

CASES = {
    "rnnt_alsd": dict(V=9, T=10, s=2, beam=4, algo="alsd"),
    "rnnt_aes_margin": dict(V=9, T=10, s=2, beam=4, algo="aes", gamma=1.5),
    "tdt_aes_margin": dict(V=7, T=14, s=2, beam=4, algo="aes", gamma=2.3, model="tdt", durations=(0, 1, 2, 3, 4)),
    "stateless_bf16": dict(V=12, T=9, s=2, beam=6, algo="aes", pred="stateless", ctx=2, prec="bf16"),
    "lm_late": dict(V=12, T=9, s=3, beam=5, algo="alsd"),
    "lm_early_eq3": dict(V=12, T=9, s=3, beam=5, algo="alsd"),
}


def _run(oracle, name):
    kw = CASES[name]
    c = S.custom_config(B=2, T_min=kw["T"] - 3, H=32, P=32, E=32, D=32, **kw)
    w = S.perturb_biases(S.make_weights(c, 40), 41)
    L = S.make_lengths(c, 42)
    enc = S.make_enc(c, L, 43)
    lm, extra = None, {}
    if name.startswith("lm"):
        lm = oracle.LM(S.make_lm(V=c["V"], order=3, n_target=300, zipf_s=1.1, seed=44))
        extra = dict(lm_weight=0.4)
        if name == "lm_early_eq3":
            extra.update(lm_rule=3, lm_prune="early")
    o = oracle.decode(c, w, enc, L, lm=lm, log=True, **extra)
    return c, w, L, enc, lm, extra, o


def _walk(oracle, c, w, L, enc, lm, extra, o, b, parent=None, token=None, merged=None, scores=None, slack=1e-9):
    n = int(o["n_steps"][b])
    sc = o["scores"][b] if scores is None else scores
    nbest = [(tuple(int(x) for x in o["tokens"][b, j, :o["lens"][b, j]]), float(sc[j]))
             for j in range(c["beam"]) if o["lens"][b, j] >= 0]
    return check_tree(oracle, c, w, enc[b], int(L[b]),
                      o["log_parent"][b, :n] if parent is None else parent,
                      o["log_token"][b, :n] if token is None else token,
                      o["log_merged"][b, :n] if merged is None else merged, n, nbest, slack=slack, tol=1e-9,
                      lm=lm, lm_weight=extra.get("lm_weight", 0.0), lm_rule=extra.get("lm_rule", 4),
                      lm_prune=extra.get("lm_prune", "late"))


@pytest.mark.parametrize("name", list(CASES))
def test_the_oracles_own_tree_passes_the_walk(oracle, name):
    c, w, L, enc, lm, extra, o = _run(oracle, name)
    for b in range(2):
        r = _walk(oracle, c, w, L, enc, lm, extra, o, b)
        assert r["steps_checked"] == o["n_steps"][b] and not r["stopped_at_duration_tie"]
        assert r["max_score_diff"] < 1e-9


@pytest.mark.parametrize("name", ["rnnt_alsd", "tdt_aes_margin", "lm_late"])
def test_a_planted_defect_in_the_tree_fails_the_walk(oracle, name):
    c, w, L, enc, lm, extra, o = _run(oracle, name)
    b, n, K, V = 0, int(o["n_steps"][0]), c["beam"], c["V"]
    P, Tk, M = (o[k][b, :n].copy() for k in ("log_parent", "log_token", "log_merged"))
    # a kept token replaced by one that was not kept at that step
    st = next(i for i in range(2, n) if (Tk[i] >= 0).any())
    j = int(np.nonzero(Tk[st] >= 0)[0][-1])
    used = {int(x) for x in Tk[st][P[st] == P[st][j]]}
    bad = Tk.copy()
    bad[st, j] = next(v for v in range(V) if v not in used)
    with pytest.raises(AssertionError):
        _walk(oracle, c, w, L, enc, lm, extra, o, b, token=bad)
    # a slot left empty although candidates exist
    bad_p, bad_t, bad_m = P.copy(), Tk.copy(), M.copy()
    full = next(i for i in range(n) if (P[i] >= 0).all())
    bad_p[full, K - 1], bad_t[full, K - 1], bad_m[full, K - 1] = -1, -3, -1
    with pytest.raises(AssertionError):
        _walk(oracle, c, w, L, enc, lm, extra, o, b, parent=bad_p, token=bad_t, merged=bad_m)
    # a recombination that did not happen / happened
    bad_m = M.copy()
    live = np.argwhere(M >= 0)
    i, j = (int(x) for x in live[len(live) // 2])
    bad_m[i, j] = j - 1 if M[i, j] == j and j > 0 else (j if M[i, j] != j else -1)
    with pytest.raises(AssertionError):
        _walk(oracle, c, w, L, enc, lm, extra, o, b, merged=bad_m)
    # a reported score off by more than the tolerance
    with pytest.raises(AssertionError):
        _walk(oracle, c, w, L, enc, lm, extra, o, b, scores=o["scores"][b] + 1e-6)
    # a blank recorded for a waiting / finished hypothesis (or the reverse)
    stay = np.argwhere(Tk == -2)
    if len(stay):
        bad = Tk.copy()
        bad[tuple(stay[0])] = -1
        with pytest.raises(AssertionError):
            _walk(oracle, c, w, L, enc, lm, extra, o, b, token=bad)
