"""Pins for the CPU oracle: each checks it against something other than itself
(exhaustive enumeration, a textbook forward recursion, a standalone greedy
decoder, library layers, closed forms, the paper's merge example)."""
import math
import os

import numpy as np
import pytest
import torch

import synth_inputs as S
from refmodel import (RefModel, aes_bucketed, aes_frame_synchronous, replay_step_margins, alsd_two_stage, TableModel, dict_lm, dict_lm_score, enumerate_alignments, forward_dp, greedy,
                      logaddexp, py_hash)

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _small(seed, **kw):
    c = S.custom_config(**kw)
    w = S.perturb_biases(S.make_weights(c, seed), seed + 1)
    L = S.make_lengths(c, seed + 2)
    enc = S.make_enc(c, L, seed + 3)
    return c, w, L, enc


def _ref_logp_fn(c, w, enc_b):
    m = RefModel(c, w)
    f = [m.f_proj(enc_b[t]) for t in range(enc_b.shape[0])]
    return lambda t, toks: m.logp(f[t], toks)


def _nbest(r, b=0):
    out = {}
    for j in range(r["lens"].shape[1]):
        n = r["lens"][b, j]
        if n >= 0:
            key = tuple(int(x) for x in r["tokens"][b, j, :n])
            assert key not in out, "the same transcript twice in the n-best: a merge was missed"
            out[key] = r["scores"][b, j]
    return out


# ---------------------------------------------------------------- whole loop

@pytest.mark.parametrize("V,T,s,beam", [(2, 4, 2, 1024), (3, 3, 2, 2048), (16, 3, 1, 8192)])
@pytest.mark.parametrize("algo", ["alsd", "aes"])
def test_unpruned_beam_equals_exhaustive_enumeration(oracle, V, T, s, beam, algo):
    c, w, L, enc = _small(100 + V, V=V, T=T, s=s, beam=beam, algo=algo)
    fn = _ref_logp_fn(c, w, enc[0])
    want = enumerate_alignments(fn, T, V, s)
    r = oracle.decode(c, w, enc, L)
    assert r["n_cut"][0] == 0, "beam too small for the exhaustive comparison"
    assert r["collisions"][0] == 0
    got = _nbest(r)
    assert set(got) == set(want)
    for y, sc in want.items():
        assert abs(got[y] - sc) < 1e-9, (y, got[y], sc)
    total = sum(math.exp(v) for v in got.values())
    assert total <= 1.0 + 1e-12
    assert r["max_logp"][0] <= 1e-12
    # ranked by score
    live = r["scores"][0][r["lens"][0] >= 0]
    assert np.all(np.diff(live) <= 0)


def test_alsd_and_aes_agree_when_nothing_is_pruned(oracle):
    c, w, L, enc = _small(7, V=3, T=4, s=2, beam=16384)
    a = _nbest(oracle.decode(c, w, enc, L, algo=oracle.ALSD))
    b = _nbest(oracle.decode(c, w, enc, L, algo=oracle.AES))
    assert set(a) == set(b)
    for y in a:
        assert abs(a[y] - b[y]) < 1e-9


def test_nbest_scores_equal_forward_recursion(oracle):
    c, w, L, enc = _small(21, V=3, T=4, s=2, beam=6, H=16, P=16, E=16, D=16)
    fn = _ref_logp_fn(c, w, enc[0])
    big = dict(c, beam=16384)
    # with pruning the scores are lower bounds; without it they equal the forward sum
    r = oracle.decode(big, w, enc, L)
    assert r["n_cut"][0] == 0
    got = _nbest(r)
    ranked = sorted(got, key=lambda y: -got[y])[:40] + [()]
    for y in ranked:
        assert abs(got[y] - forward_dp(fn, 4, 3, 2, y)) < 1e-9
    rp = _nbest(oracle.decode(c, w, enc, L))
    for y, sc in rp.items():
        assert sc <= forward_dp(fn, 4, 3, 2, y) + 1e-9


@pytest.mark.parametrize("algo", ["alsd", "aes"])
@pytest.mark.parametrize("cfg", [1, "tdt", "stateless"])
def test_beam_one_is_greedy(oracle, cfg, algo):
    if cfg == 1:
        c = S.config(1, beam=1, algo=algo)
        w, L = S.make_weights(c), S.make_lengths(c)
        enc = S.make_enc(c, L)
    elif cfg == "tdt":
        c, w, L, enc = _small(31, model="tdt", durations=(0, 1, 2, 3, 4), V=6, T=30, s=2, beam=1, algo=algo,
                              H=16, P=16, E=16, D=16)
    else:
        c, w, L, enc = _small(32, pred="stateless", ctx=2, V=6, T=25, s=3, beam=1, algo=algo, H=16, P=16, E=16,
                              D=16)
    fn = _ref_logp_fn(c, w, enc[0])
    toks, score = greedy(fn, int(L[0]), c["V"], c["s"], c["durations"])
    r = oracle.decode(c, w, enc, L)
    n = r["lens"][0, 0]
    assert tuple(r["tokens"][0, 0, :n]) == toks
    assert abs(r["scores"][0, 0] - score) < 1e-9


@pytest.mark.parametrize("K", [2, 3, 5])
def test_aes_with_pruning_equals_two_set_frame_loop(oracle, K):
    """AES++ with a real (pruning) beam against the frame/round loop with open and
    waiting sets; this is what tells the waiting rule from the length-synchronous one."""
    differs = 0
    for seed in range(6):
        c, w, L, enc = _small(200 + seed, V=4, T=7, s=2, beam=K, algo="aes", H=12, P=12, E=12, D=12)
        fn = _ref_logp_fn(c, w, enc[0])
        want = aes_frame_synchronous(fn, 7, 4, 2, K)
        r = oracle.decode(c, w, enc, L)
        got = _nbest(r)
        assert set(got) == set(want), seed
        for y in want:
            assert abs(got[y] - want[y]) < 1e-9
        alsd = _nbest(oracle.decode(c, w, enc, L, algo=oracle.ALSD))
        differs += set(alsd) != set(got) or any(abs(alsd[y] - got[y]) > 1e-6 for y in got)
    assert differs > 0, "the cases do not separate AES from ALSD"



@pytest.mark.parametrize("gamma", [math.inf, 2.3, 0.7])
@pytest.mark.parametrize("K", [2, 3, 5])
def test_tdt_aes_with_a_pruning_beam_and_margin_equals_the_bucketed_two_set_loop(oracle, K, gamma):
    """The regime of the TDT workload: AES++ on a TDT model (per-hypothesis frame index, one duration per symbol)
    with a beam that really prunes and a finite prune margin, against the frame-by-frame loop with one waiting
    set per landing frame."""
    durations = (0, 1, 2, 3, 4)
    differs_alsd = differs_margin = cut = 0
    for seed in range(5):
        c, w, L, enc = _small(230 + seed, model="tdt", durations=durations, V=4, T=9, s=2, beam=K, algo="aes",
                              gamma=gamma, H=12, P=12, E=12, D=12)
        w["b_out"][5:] = 0.0   # durations of every size, token and blank often disagree: hypotheses spread over frames
        w["W_out"][5:] *= 4.0
        fn = _ref_logp_fn(c, w, enc[0])
        want = aes_bucketed(fn, 9, 4, 2, K, durations, gamma)
        r = oracle.decode(c, w, enc, L)
        got = _nbest(r)
        assert set(got) == set(want), (seed, got, want)
        for y in want:
            assert abs(got[y] - want[y]) < 1e-9
        cut += int(r["n_cut"][0])
        alsd = _nbest(oracle.decode(dict(c, gamma=math.inf), w, enc, L, algo=oracle.ALSD))
        differs_alsd += set(alsd) != set(got) or any(abs(alsd[y] - got[y]) > 1e-6 for y in got)
        free = _nbest(oracle.decode(dict(c, gamma=math.inf), w, enc, L))
        differs_margin += set(free) != set(got) or any(abs(free[y] - got[y]) > 1e-6 for y in got)
    assert cut > 0 or (gamma < 1.0 and K >= 5), "the beam never pruned"  # (a tight margin leaves fewer than 5 candidates)
    assert differs_alsd > 0, "the cases do not separate AES from ALSD"
    assert gamma > 1.0 or differs_margin > 0, "the margin never mattered"  # (2.3 rarely reaches into a narrow beam)


@pytest.mark.parametrize("K,gamma", [(3, 1.0), (4, 2.3)])
def test_rnnt_aes_with_margin_equals_the_bucketed_two_set_loop(oracle, K, gamma):
    differs = 0
    for seed in range(5):
        c, w, L, enc = _small(260 + seed, V=5, T=7, s=2, beam=K, algo="aes", gamma=gamma, H=12, P=12, E=12, D=12)
        fn = _ref_logp_fn(c, w, enc[0])
        want = aes_bucketed(fn, 7, 5, 2, K, (), gamma)
        got = _nbest(oracle.decode(c, w, enc, L))
        assert set(got) == set(want), seed
        for y in want:
            assert abs(got[y] - want[y]) < 1e-9
        # without a margin the bucketed loop is the classical one
        a, b = aes_bucketed(fn, 7, 5, 2, K), aes_frame_synchronous(fn, 7, 5, 2, K)
        assert set(a) == set(b) and all(abs(a[y] - b[y]) < 1e-12 for y in a)
        differs += set(a) != set(want)
    assert differs > 0, "the margin never mattered"


@pytest.mark.parametrize("model", ["rnnt", "tdt"])
def test_prune_margin_belongs_to_aes_only(oracle, model):
    """ALSD++ with a prune margin in its configuration is ALSD++: nothing pruned -> the exhaustive sums."""
    durations = (0, 1, 2) if model == "tdt" else ()
    c, w, L, enc = _small(270, model=model, durations=durations, V=2, T=4, s=2, beam=4096, algo="alsd", gamma=0.5)
    fn = _ref_logp_fn(c, w, enc[0])
    want = enumerate_alignments(fn, 4, 2, 2, durations)
    r = oracle.decode(c, w, enc, L)
    assert r["n_cut"][0] == 0
    got = _nbest(r)
    assert set(got) == set(want)
    for y in want:
        assert abs(got[y] - want[y]) < 1e-9
    # while under AES++ the same margin does cut
    assert set(_nbest(oracle.decode(c, w, enc, L, algo=oracle.AES))) != set(want)


# ------------------------------------------- AES++ maximum-length prefix search

@pytest.mark.parametrize("V,T,s,beam", [(2, 4, 2, 1024), (3, 3, 2, 2048)])
def test_prefix_search_leaves_the_unpruned_result_exact(oracle, V, T, s, beam):
    """With nothing pruned the prefix search may not change anything: every score is still the sum over the
    alignments of its transcript (a reading that moved an expansion's score into the longer hypothesis as well
    would count those alignments twice and fail here)."""
    c, w, L, enc = _small(100 + V, V=V, T=T, s=s, beam=beam, algo="aes", aes_prefix=True)
    fn = _ref_logp_fn(c, w, enc[0])
    want = enumerate_alignments(fn, T, V, s)
    r = oracle.decode(c, w, enc, L)
    assert r["n_cut"][0] == 0 and r["collisions"][0] == 0
    got = _nbest(r)
    assert set(got) == set(want)
    for y, sc in want.items():
        assert abs(got[y] - sc) < 1e-9, (y, got[y], sc)
    assert sum(math.exp(v) for v in got.values()) <= 1.0 + 1e-12


@pytest.mark.parametrize("model,K,gamma,V", [("rnnt", 2, math.inf, 3), ("rnnt", 3, math.inf, 3), ("rnnt", 5, 2.0, 3),
                                             ("tdt", 3, math.inf, 3), ("tdt", 3, 4.0, 3), ("rnnt", 2, math.inf, 7),
                                             ("rnnt", 3, math.inf, 9)])
def test_prefix_search_with_a_pruning_beam_equals_the_two_set_loop(oracle, model, K, gamma, V):
    """With a real beam the prefix search changes which candidates are kept; against the frame / round loop with
    dictionaries of transcripts."""
    durations = (0, 1, 2) if model == "tdt" else ()
    changed = 0
    for seed in range(24 if (V > 3 or model == "tdt") else 8):
        c, w, L, enc = _small(500 + seed, model=model, durations=durations, V=V, T=8, s=3, beam=K, algo="aes",
                              gamma=gamma, aes_prefix=True, H=12, P=12, E=12, D=12, blank_bias=0.5)
        if durations:
            # even seeds: mostly duration 0 (expansions stay in the frame); odd seeds: all durations occur
            w["b_out"][V + 1:] = [1.5, 0.0, 0.0] if seed % 2 == 0 else [0.2, 0.4, 0.0]
            if seed % 2:
                w["W_out"][V + 1:] *= 4.0
        fn = _ref_logp_fn(c, w, enc[0])
        want = aes_bucketed(fn, 8, V, 3, K, durations, gamma, prefix=True)
        got = _nbest(oracle.decode(c, w, enc, L))
        assert set(got) == set(want), (seed, got, want)
        for y in want:
            assert abs(got[y] - want[y]) < 1e-9
        plain = _nbest(oracle.decode(dict(c, aes_prefix=False), w, enc, L))
        changed += set(plain) != set(got) or any(abs(plain[y] - got[y]) > 1e-6 for y in got)
    assert changed > 0 or model == "tdt", "the prefix search never changed a decision on these cases"


def test_prefix_credit_needs_one_of_the_beam_best_expansions(oracle):
    """A hand-made table (two context classes by hash parity, beam 2) where "" and "a" stand in frame 1 together
    and "a" is only the THIRD best token after "": no credit, the two best expansions of "" fill the beam.  A
    credit for that expansion would lift "ab" into the beam instead (key -1.8 + 0.51 against -1.5 and -1.6)."""
    V, NEG = 3, -8.0
    tok = np.full((1, 2, 2, V + 1), NEG, np.float32)
    tok[0, 0, 0] = [-0.3, NEG, NEG, -1.0]      # frame 0 after "":  a, then blank
    tok[0, 0, 1] = [NEG, NEG, NEG, -1.0]       # frame 0 after "a": blank
    tok[0, 1, 0] = [-0.7, -0.5, -0.6, -3.0]    # frame 1 after "":  b, c, a
    tok[0, 1, 1] = [-0.9, -0.5, -0.7, -3.0]    # frame 1 after "a"
    tok += np.random.default_rng(3).uniform(0, 2e-3, tok.shape).astype(np.float32)  # no exact ties anywhere
    assert py_hash(()) % 2 == 0 and py_hash((0,)) % 2 == 1
    c = S.custom_config(B=1, T=2, V=V, beam=2, s=2, algo="aes", aes_prefix=True)
    L = np.array([2], np.int32)
    r = oracle.decode(c, None, None, L, injected=(tok, None), log=True)
    # step 2 is the step in question: "" in slot 0 (-1.0), "a" in slot 1 (-1.3), both open in frame 1
    np.testing.assert_array_equal(r["log_parent"][0, 2], [0, 0])
    np.testing.assert_array_equal(r["log_token"][0, 2], [1, 2])
    tm = TableModel(tok[0], None, V, py_hash)
    want = aes_bucketed(tm.logp_at, 2, V, 2, 2, prefix=True)
    got = _nbest(r)
    assert set(got) == set(want)
    for y in want:
        assert abs(got[y] - want[y]) < 1e-12
    # with "a" as the second best token after "" the credit exists (0.575) and lifts "ab" (-1.225) and "ac" (-1.425)
    # over the expansions of "" (-1.5, -1.55, -1.6)
    tok[0, 1, 0] = [-0.55, -0.5, -0.6, -3.0]
    tok[0, 1, 0] += np.float32(1e-3) * np.arange(4, dtype=np.float32)
    r2 = oracle.decode(c, None, None, L, injected=(tok, None), log=True)
    np.testing.assert_array_equal(r2["log_parent"][0, 2], [1, 1])
    np.testing.assert_array_equal(r2["log_token"][0, 2], [1, 2])


def test_prefix_search_is_an_aes_option(oracle):
    c, w, L, enc = _small(520, V=3, T=8, s=3, beam=3, algo="alsd", aes_prefix=True, H=12, P=12, E=12, D=12)
    a, b = oracle.decode(c, w, enc, L), oracle.decode(dict(c, aes_prefix=False), w, enc, L)
    np.testing.assert_array_equal(a["scores"], b["scores"])
    np.testing.assert_array_equal(a["tokens"], b["tokens"])


# ------------------------------------------------------- near-tie report

def test_step_margin_report_on_a_hand_made_table(oracle):
    """log_gap of a two-frame, one-token table worked out by hand (beam 2, s = 1, ALSD++):
    step 0: candidates a = -0.25, blank = -1.75, both kept                        -> 1.5
    step 1: slot 0 = "a" (forced blank, frame 0): -2.0; slot 1 = "" at frame 1: a -2.25, blank -2.75; kept -2.0,
            -2.25, first discarded -2.75                                          -> min(0.25, 0.5) = 0.25
    step 2: slot 0 = "a" at frame 1: a -2.5, blank -3.0; slot 1 = "a" with one symbol in frame 1 (forced blank)
            -3.25; kept -2.5, -3.0, discarded -3.25                               -> 0.25
    step 3: slot 0 = "aa" forced blank -3.5; slot 1 = "a" finished, stays -3.0    -> 0.5"""
    c = S.custom_config(B=1, T=2, V=1, beam=2, s=1, algo="alsd")
    tok = np.array([[[[-0.25, -1.75]], [[-0.5, -1.0]]]], np.float32)
    r = oracle.decode(c, None, None, np.array([2], np.int32), injected=(tok, None), log=True)
    assert r["n_steps"][0] == 4
    np.testing.assert_allclose(r["log_gap"][0, :4], [1.5, 0.25, 0.25, 0.5], rtol=0, atol=1e-12)
    assert r["min_gap"][0] == 0.25
    assert _nbest(r) == {(0,): -3.0, (0, 0): -3.5}


@pytest.mark.parametrize("name,kw", [
    ("rnnt_alsd", dict(V=5, T=8, s=2, beam=3, algo="alsd")),
    ("rnnt_aes_margin", dict(V=5, T=8, s=2, beam=3, algo="aes", gamma=1.5)),
    ("tdt_aes_margin", dict(V=4, T=10, s=2, beam=4, algo="aes", gamma=2.3, model="tdt", durations=(0, 1, 2, 3, 4))),
    ("tdt_alsd", dict(V=4, T=10, s=2, beam=5, algo="alsd", model="tdt", durations=(0, 1, 2, 3, 4))),
    ("stateless_aes", dict(V=6, T=8, s=3, beam=4, algo="aes", pred="stateless", ctx=2)),
])
def test_step_margin_report_equals_an_independent_replay(oracle, name, kw):
    """The per-step margin the oracle reports (the parity tests forgive a divergence only at a step whose margin
    was small) against margins recomputed from library layers along the oracle's own logged tree: ranking gaps
    down to the first discarded candidate, duration arg-max margins, distance from the prune margin."""
    seen_cut = 0
    for seed in range(4):
        c, w, L, enc = _small(300 + 7 * seed, B=2, T_min=kw["T"] - 3, H=12, P=12, E=12, D=12, **kw)
        r = oracle.decode(c, w, enc, L, log=True)
        for b in range(2):
            fn = _ref_logp_fn(c, w, enc[b])
            n = int(r["n_steps"][b])
            want = replay_step_margins(fn, int(L[b]), c["V"], c["s"], c["beam"], c["algo"], c["durations"], c["gamma"],
                                       r["log_parent"][b], r["log_token"][b], r["log_merged"][b], n)
            np.testing.assert_allclose(r["log_gap"][b, :n], want, rtol=0, atol=1e-9)
            assert abs(r["min_gap"][b] - min(want)) < 1e-9
            seen_cut += int(r["n_cut"][b] > 0)
    assert seen_cut > 0


# ------------------------------------------------------------------- TDT

def test_tdt_duration_always_one_is_brute_force_over_symbols(oracle):
    # duration head pinned to "1": every symbol, blank or not, consumes one frame,
    # so an alignment is any string of T symbols and transcripts never share one.
    V, T = 3, 4
    c, w, L, enc = _small(41, model="tdt", durations=(0, 1, 2), V=V, T=T, s=2, beam=1024, algo="aes")
    w = dict(w)
    b = w["b_out"].copy()
    b[V + 1:] = [-60.0, 60.0, -60.0]
    w["b_out"] = b
    m = RefModel(c, w)
    f = [m.f_proj(enc[0, t]) for t in range(T)]
    want = {}
    import itertools
    for seq in itertools.product(range(V + 1), repeat=T):
        toks, lp = (), 0.0
        for t, v in enumerate(seq):
            logp, dl = m.logp(f[t], toks)
            lp += logp[v] + dl[1]
            if v != V:
                toks = toks + (v,)
        want[toks] = logaddexp(want.get(toks, -math.inf), lp)
    r = oracle.decode(c, w, enc, L)
    assert r["n_cut"][0] == 0
    got = _nbest(r)
    assert set(got) == set(want)
    for y in want:
        assert abs(got[y] - want[y]) < 1e-9


def test_tdt_unpruned_equals_enumeration_with_duration_rule(oracle):
    V, T, s = 2, 5, 2
    c, w, L, enc = _small(43, model="tdt", durations=(0, 1, 2, 3, 4), V=V, T=T, s=s, beam=4096, algo="aes")
    fn = _ref_logp_fn(c, w, enc[0])
    want = enumerate_alignments(fn, T, V, s, c["durations"])
    r = oracle.decode(c, w, enc, L)
    assert r["n_cut"][0] == 0
    got = _nbest(r)
    assert set(got) == set(want)
    for y in want:
        assert abs(got[y] - want[y]) < 1e-9


# ------------------------------------------------------------ network numerics

def test_lstm_joint_and_projections_match_library_layers(oracle):
    c, w, L, enc = _small(51, V=11, T=3, H=24, P=20, E=12, D=28)
    m = RefModel(c, w)
    f = oracle.enc_proj(c, w, enc[0, 1])
    np.testing.assert_allclose(f, m.f_proj(enc[0, 1]).numpy(), rtol=0, atol=1e-12)
    h, cc = np.zeros(c["P"]), np.zeros(c["P"])
    toks = ()
    for tok in [c["V"], 3, 7, 0]:
        h, cc = oracle.lstm_step(c, w, h, cc, tok)
        if tok != c["V"]:
            toks = toks + (tok,)
        g_ref, state = m.pred(toks)
        np.testing.assert_allclose(h, state[0][0].numpy(), atol=1e-12)
        np.testing.assert_allclose(cc, state[1][0].numpy(), atol=1e-12)
        g = oracle.pred_proj(c, w, h)
        np.testing.assert_allclose(g, g_ref.numpy(), atol=1e-12)
        z = oracle.joint(c, w, f, g)
        lp_ref, _ = m.logp(torch.tensor(f), toks)
        tot, lp, a_t, a_b = oracle.score_row(c, z=z)
        np.testing.assert_allclose(lp, lp_ref, atol=1e-12)
        np.testing.assert_allclose(tot, lp_ref, atol=1e-12)
        assert (a_t, a_b) == (0, 1)
        assert abs(np.exp(lp).sum() - 1) < 1e-12


def test_stateless_prediction_network(oracle):
    c, w, L, enc = _small(52, pred="stateless", ctx=2, V=9, H=12, P=10, E=10, D=8)
    m = RefModel(c, w)
    for toks in [(), (4,), (4, 2), (4, 2, 8)]:
        np.testing.assert_allclose(oracle.stateless_pred(c, w, toks), m.pred(toks)[0].numpy(), atol=1e-12)


def test_bf16_operand_rounding_matches_library_cast(oracle):
    c, w, L, enc = _small(53, prec="bf16", V=5, H=16, P=12, E=12, D=20)
    rb = lambda a: torch.tensor(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float64)
    f = oracle.enc_proj(c, w, enc[0, 0])
    f_ref = (rb(w["W_enc"]) @ rb(enc[0, 0]) + torch.tensor(w["b_enc"], dtype=torch.float64)).numpy()
    np.testing.assert_allclose(f, f_ref, atol=1e-12)
    h = np.random.default_rng(0).standard_normal(c["P"])
    g = oracle.pred_proj(c, w, h)
    g_ref = (rb(w["W_pred"]) @ rb(h) + torch.tensor(w["b_pred"], dtype=torch.float64)).numpy()
    np.testing.assert_allclose(g, g_ref, atol=1e-12)
    z = oracle.joint(c, w, f, g)
    a = torch.relu(torch.tensor(f + g))
    z_ref = (rb(w["W_out"]) @ rb(a.numpy()) + torch.tensor(w["b_out"], dtype=torch.float64)).numpy()
    np.testing.assert_allclose(z, z_ref, atol=1e-12)
    # the decode path with pre-rounded matrices gives what the per-call rounding gives
    cb = dict(c, beam=1, T=6, B=1)
    Lb = np.array([6], np.int32)
    encb = S.make_enc(cb, Lb, 5)
    r = oracle.decode(cb, w, encb, Lb)
    fn_tok, score = None, 0.0
    toks, t, sym, hh, cc = (), 0, 0, *oracle.lstm_step(cb, w, np.zeros(c["P"]), np.zeros(c["P"]), c["V"])
    while t < 6:
        z = oracle.joint(cb, w, oracle.enc_proj(cb, w, encb[0, t]), oracle.pred_proj(cb, w, hh))
        lp = z[: c["V"] + 1] - np.log(np.exp(z[: c["V"] + 1]).sum())
        v = int(np.argmax(lp)) if sym < cb["s"] else c["V"]
        score += lp[v]
        if v == c["V"]:
            t, sym = t + 1, 0
        else:
            toks, sym = toks + (v,), sym + 1
            hh, cc = oracle.lstm_step(cb, w, hh, cc, v)
    assert tuple(r["tokens"][0, 0, : r["lens"][0, 0]]) == toks
    assert abs(r["scores"][0, 0] - score) < 1e-9


# ------------------------------------------------------------ selection, hash

def test_topk_is_the_head_of_a_stable_sort(oracle):
    rng = np.random.default_rng(3)
    for n, K in [(10, 3), (68, 4), (4100, 8), (50, 50)]:
        v = np.round(rng.standard_normal(n), 1)  # many ties
        v[rng.integers(0, n, n // 5)] = -np.inf
        want = np.lexsort((np.arange(n), -v))[:K]
        np.testing.assert_array_equal(oracle.topk(v, K), want)


def test_hash_is_eq1_with_big_integers(oracle):
    rng = np.random.default_rng(4)
    for n in [0, 1, 2, 7, 300]:
        toks = rng.integers(0, 8192, n)
        assert oracle.hash_tokens(toks) == py_hash([int(x) for x in toks])
    # order matters, token 0 is not absorbed by the empty hash
    assert oracle.hash_tokens([0]) != oracle.hash_tokens([])
    assert oracle.hash_tokens([1, 2]) != oracle.hash_tokens([2, 1])
    assert oracle.hash_tokens([5]) == 6


def _parse_golden():
    rows = []
    for line in open(os.path.join(GOLD, "merge_example.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            a, y = [x.strip() for x in line.split("->")]
            rows.append((a, y))
    return rows


def test_paper_merge_example_collapses_and_merges(oracle):
    """The paper's three alignments of "ab" (blank in different places) must end
    up in one slot whose score is the log-sum of all alignments of "ab"."""
    rows = _parse_golden()
    assert len(rows) == 3
    for a, y in rows:
        assert a.replace("0", "") == y == "ab"
    V, T, s, C = 2, 4, 2, 4  # a = 0, b = 1; four frames so that every listed alignment can be completed
    tok, _ = S.make_injected(1, T, C, V, 0, seed=9, levels=200)
    c = S.custom_config(V=V, T=T, s=s, beam=2048)
    L = np.array([T], np.int32)
    r = oracle.decode(c, None, None, L, injected=(tok, None), log=True)
    assert r["n_cut"][0] == 0
    table = TableModel(tok[0], None, V, py_hash)
    want = enumerate_alignments(table.logp_at, T, V, s)
    got = _nbest(r)
    assert abs(got[(0, 1)] - want[(0, 1)]) < 1e-9
    # each listed alignment, completed with blanks, is one of the summed paths
    sym = {"a": 0, "b": 1, "0": V}
    for a, _ in rows:
        seq = [sym[ch] for ch in a]
        while seq.count(V) < T:
            seq.append(V)
        t, toks, lp, n_in_frame = 0, (), 0.0, 0
        for v in seq:
            lp += table.logp_at(t, toks)[0][v]
            if v == V:
                t, n_in_frame = t + 1, 0
            else:
                toks, n_in_frame = toks + (v,), n_in_frame + 1
                assert n_in_frame <= s
        assert t == T and toks == (0, 1)
        assert lp <= got[(0, 1)] + 1e-12
    # merges did happen and were logged
    n = r["n_steps"][0]
    merged = r["log_merged"][0, :n]
    slots = np.arange(merged.shape[1])[None, :]
    assert np.any((merged >= 0) & (merged != slots))


def test_injected_unpruned_equals_enumeration_and_key_is_exact(oracle):
    V, T, s, C = 3, 4, 2, 5
    tok, _ = S.make_injected(1, T, C, V, 0, seed=11, levels=300)
    c = S.custom_config(V=V, T=T, s=s, beam=16384)
    L = np.array([T], np.int32)
    r = oracle.decode(c, None, None, L, injected=(tok, None))
    assert r["n_cut"][0] == 0 and r["collisions"][0] == 0
    want = enumerate_alignments(TableModel(tok[0], None, V, py_hash).logp_at, T, V, s)
    got = _nbest(r)
    assert set(got) == set(want)
    for y in want:
        assert abs(got[y] - want[y]) < 1e-9


def test_log_replays_to_the_explicit_transcripts(oracle):
    """Walking (parent, token) back through the step log reproduces the explicit
    token vectors of every slot at every snapshot: the tree rule of Sec. 2.1."""
    c = S.config(1)
    w, L = S.make_weights(c), S.make_lengths(c)
    enc = S.make_enc(c, L)
    for algo in (oracle.ALSD, oracle.AES):
        r = oracle.decode(c, w, enc, L, algo=algo, log=True, snap_every=5)
        K = c["beam"]
        n = r["n_steps"][0]
        for i in range(n // 5):
            step = (i + 1) * 5
            for k in range(K):
                want_len = r["snap_lens"][0, i, k]
                if want_len < 0:
                    continue
                toks, slot = [], k
                for st in range(step - 1, -1, -1):
                    tk = r["log_token"][0, st, slot]
                    if tk >= 0:
                        toks.append(tk)
                    slot = r["log_parent"][0, st, slot]
                    assert slot >= 0
                toks.reverse()
                assert toks == list(r["snap_tokens"][0, i, k, :want_len])


def test_slot_bookkeeping_invariants(oracle):
    c = S.config(1)
    w, L = S.make_weights(c), S.make_lengths(c)
    enc = S.make_enc(c, L)
    for algo in (oracle.ALSD, oracle.AES):
        r = oracle.decode(c, w, enc, L, algo=algo, log=True)
        n = r["n_steps"][0]
        assert n <= c["T"] * (c["s"] + 1)
        assert r["max_logp"][0] <= 0
        assert r["collisions"][0] == 0
        p, t, m = r["log_parent"][0, :n], r["log_token"][0, :n], r["log_merged"][0, :n]
        assert p.shape[1] == c["beam"]  # exactly Beam slots at every step
        assert np.all((p >= -1) & (p < c["beam"]))
        assert np.all((t >= -3) & (t < c["V"]))
        assert np.all((p == -1) == (t == -3))
        assert np.all(m <= np.arange(c["beam"])[None, :])
        # at most s tokens without leaving a frame
        toks = r["tokens"][0, 0, : r["lens"][0, 0]]
        assert len(toks) <= c["T"] * c["s"]


def test_prune_margin_and_frame_limit(oracle):
    c = S.custom_config(V=6, s=2, gamma=1.0, algo="aes")
    z = np.array([2.0, 1.5, 0.5, -1.0, 0.9, 1.01, 0.0])  # blank last
    lp = z - np.log(np.exp(z).sum())
    tot, logp, _, _ = oracle.score_row(c, z=z, apply_gamma=True)
    np.testing.assert_allclose(logp, lp, atol=1e-12)
    keep = lp >= lp.max() - 1.0
    assert np.all(np.isneginf(tot[~keep])) and np.allclose(tot[keep], lp[keep])
    assert keep.sum() == 3
    tot, _, _, _ = oracle.score_row(c, z=z, apply_gamma=True, forced_blank=True)
    assert np.all(np.isneginf(tot[:6])) and abs(tot[6] - lp[6]) < 1e-12  # blank restored although pruned
    tot, _, _, _ = oracle.score_row(c, z=z, apply_gamma=False)
    np.testing.assert_allclose(tot, lp, atol=1e-12)


def test_tdt_duration_rule(oracle):
    c = S.custom_config(model="tdt", durations=(0, 1, 2, 3, 4), V=3)
    z = np.array([0.3, -0.2, 0.1, 0.5, 2.0, 0.1, 1.9, -1.0, 0.2])  # 3 tokens, blank, 5 durations
    lp = z[:4] - np.log(np.exp(z[:4]).sum())
    dl = z[4:] - np.log(np.exp(z[4:]).sum())
    tot, logp, a_t, a_b = oracle.score_row(c, z=z)
    assert (a_t, a_b) == (0, 2)  # best duration is 0 for tokens; blank takes the best one that advances
    np.testing.assert_allclose(tot[:3], lp[:3] + dl[0], atol=1e-12)
    assert abs(tot[3] - (lp[3] + dl[2])) < 1e-12
    np.testing.assert_allclose(logp, lp, atol=1e-12)


# ------------------------------------------------------------------------ LM

@pytest.fixture(scope="module")
def small_lm():
    return S.make_lm(V=12, order=4, n_target=1000, zipf_s=1.1, seed=77)


def test_lm_query_equals_dictionary_backoff(oracle, small_lm):
    d = dict_lm(small_lm)
    assert 900 <= len(d) <= 2500
    lm = oracle.LM(small_lm)
    rng = np.random.default_rng(5)
    stored3 = [k for k in d if len(k) == 3]
    cases = [(), (3,), (3, 4), (0, 0, 0), (11, 10, 9, 8, 7)] + [tuple(rng.integers(0, 12, n)) for n in (1, 2, 3, 5)
                                                                for _ in range(6)]
    cases += [stored3[i] for i in range(0, len(stored3), max(1, len(stored3) // 10))]
    for toks in cases:
        toks = tuple(int(x) for x in toks)
        got = lm.query(toks, 12)
        ctx = toks[-3:] if len(toks) >= 3 else toks
        want = np.array([math.log(10.0) * dict_lm_score(d, ctx, v) for v in range(12)])
        np.testing.assert_allclose(got, want, atol=1e-12)
        assert np.all(got < 0)


def test_fusion_rules(oracle):
    V = 5
    c = S.custom_config(V=V)
    rng = np.random.default_rng(6)
    z = rng.standard_normal(V + 1) * 2
    lp = z - np.log(np.exp(z).sum())
    q = rng.random(V)
    lm_row = np.log(q / q.sum())  # a normalised LM distribution
    lam = 0.7
    tot, logp, _, _ = oracle.score_row(c, z=z, lm_row=lm_row, lm_weight=lam)
    nb = math.log(1 - math.exp(lp[V]))
    np.testing.assert_allclose(tot[:V], lp[:V] + lam * (nb + lm_row), atol=1e-12)  # Eq. (4), tokens
    assert abs(tot[V] - (1 + lam) * lp[V]) < 1e-12  # Eq. (4), blank
    assert np.all(tot <= 0)
    # "preserves total probability": the rescaled LM mass over tokens is 1 - p_blank
    assert abs(np.exp(nb + lm_row).sum() - (1 - math.exp(lp[V]))) < 1e-12
    tot3, _, _, _ = oracle.score_row(c, z=z, lm_row=lm_row, lm_weight=lam, lm_rule=3)
    np.testing.assert_allclose(tot3[:V], lp[:V] + lam * lm_row, atol=1e-12)  # Eq. (3)
    assert abs(tot3[V] - lp[V]) < 1e-12
    tot0, _, _, _ = oracle.score_row(c, z=z, lm_row=lm_row, lm_weight=0.0)
    np.testing.assert_allclose(tot0, lp, atol=1e-12)
    # blank probability close to one: ln(1 - p_blank) stays finite and accurate
    z2 = np.array([-40.0] * V + [0.0])
    tot2, lp2, _, _ = oracle.score_row(c, z=z2, lm_row=lm_row, lm_weight=1.0)
    assert np.all(np.isfinite(tot2))
    assert abs((tot2[0] - lp2[0] - lm_row[0]) - (math.log(V) - 40.0)) < 1e-9


def test_lm_weight_zero_is_the_run_without_lm(oracle, small_lm):
    c, w, L, enc = _small(61, V=12, T=12, s=2, beam=4, H=16, P=16, E=16, D=16)
    lm = oracle.LM(small_lm)
    a = oracle.decode(c, w, enc, L)
    b = oracle.decode(c, w, enc, L, lm=lm, lm_weight=0.0)
    np.testing.assert_array_equal(a["tokens"], b["tokens"])
    np.testing.assert_array_equal(a["scores"], b["scores"])
    d = oracle.decode(c, w, enc, L, lm=lm, lm_weight=0.5)
    assert d["max_logp"][0] <= 0
    assert not np.array_equal(a["scores"], d["scores"])


def test_fused_beam_one_is_greedy_on_fused_scores(oracle, small_lm):
    c, w, L, enc = _small(62, V=12, T=10, s=2, beam=1, H=16, P=16, E=16, D=16)
    d = dict_lm(small_lm)
    lam = 0.4
    base = _ref_logp_fn(c, w, enc[0])

    def fused(t, toks):
        lp, _ = base(t, toks)
        ctx = toks[-3:]
        lmrow = np.array([math.log(10.0) * dict_lm_score(d, ctx, v) for v in range(12)])
        nb = math.log(1 - math.exp(lp[12]))
        out = lp.copy()
        out[:12] = lp[:12] + lam * (nb + lmrow)
        out[12] = (1 + lam) * lp[12]
        return out, None

    toks, score = greedy(fused, 10, 12, 2)
    r = oracle.decode(c, w, enc, L, lm=oracle.LM(small_lm), lm_weight=lam)
    assert tuple(r["tokens"][0, 0, : r["lens"][0, 0]]) == toks
    assert abs(r["scores"][0, 0] - score) < 1e-9


def _fused_fn(base, d, V, lam, rule):
    """Fused increments of Eq. (3) / Eq. (4) from a dictionary LM (order 4)."""
    def fused(t, toks):
        lp, _ = base(t, toks)
        lmrow = np.array([math.log(10.0) * dict_lm_score(d, toks[-3:], v) for v in range(V)])
        out = lp.copy()
        if rule == 4:
            out[:V] = lp[:V] + lam * (math.log(1 - math.exp(lp[V])) + lmrow)
            out[V] = (1 + lam) * lp[V]
        else:
            out[:V] = lp[:V] + lam * lmrow
        return out
    return fused


@pytest.mark.parametrize("rule", [3, 4])
def test_early_pruning_changes_nothing_when_nothing_is_pruned(oracle, rule):
    lm_small = S.make_lm(V=3, order=3, n_target=30, zipf_s=1.1, seed=78)
    c, w, L, enc = _small(63, V=3, T=3, s=2, beam=2048, H=16, P=16, E=16, D=16)
    lm = oracle.LM(lm_small)
    late = oracle.decode(c, w, enc, L, lm=lm, lm_weight=0.6, lm_rule=rule)
    early = oracle.decode(c, w, enc, L, lm=lm, lm_weight=0.6, lm_rule=rule, lm_prune="early")
    assert late["n_cut"][0] == 0 and early["n_cut"][0] == 0
    a, b = _nbest(late), _nbest(early)
    assert a.keys() == b.keys() and len(a) > 20
    for k in a:
        assert abs(a[k] - b[k]) < 1e-9


@pytest.mark.parametrize("rule", [3, 4])
def test_early_pruning_beam_one_follows_the_transducer_and_pays_the_fused_score(oracle, small_lm, rule):
    c, w, L, enc = _small(64, V=12, T=10, s=2, beam=1, H=16, P=16, E=16, D=16)
    d = dict_lm(small_lm)
    lam = 0.8
    base = _ref_logp_fn(c, w, enc[0])
    fused = _fused_fn(base, d, 12, lam, rule)
    toks, _ = greedy(base, 10, 12, 2)
    # the same walk again, adding up what the fused rule charges for each of its choices
    t, cur, sym, score = 0, (), 0, 0.0
    while t < 10:
        lp, _ = base(t, cur)
        v = int(np.argmax(lp)) if sym < 2 else 12
        score += fused(t, cur)[v]
        if v == 12:
            t, sym = t + 1, 0
        else:
            cur, sym = cur + (v,), sym + 1
    assert cur == toks
    r = oracle.decode(c, w, enc, L, lm=oracle.LM(small_lm), lm_weight=lam, lm_rule=rule, lm_prune="early")
    assert tuple(r["tokens"][0, 0, : r["lens"][0, 0]]) == toks
    assert abs(r["scores"][0, 0] - score) < 1e-9
    # late pruning at this weight takes another path, or the two modes could not be told apart here
    late = oracle.decode(c, w, enc, L, lm=oracle.LM(small_lm), lm_weight=lam, lm_rule=rule)
    assert tuple(late["tokens"][0, 0, : late["lens"][0, 0]]) != toks


@pytest.mark.parametrize("rule,K", [(4, 3), (3, 5)])
def test_early_pruning_with_a_real_beam_equals_the_two_stage_loop(oracle, small_lm, rule, K):
    c, w, L, enc = _small(65, V=12, T=7, s=2, beam=K, H=16, P=16, E=16, D=16)
    d = dict_lm(small_lm)
    lam = 0.7
    base = _ref_logp_fn(c, w, enc[0])
    want = alsd_two_stage(base, _fused_fn(base, d, 12, lam, rule), 7, 12, 2, K)
    r = oracle.decode(c, w, enc, L, lm=oracle.LM(small_lm), lm_weight=lam, lm_rule=rule, lm_prune="early")
    assert r["n_cut"][0] > 0
    got = _nbest(r)
    assert got.keys() == want.keys()
    for k in got:
        assert abs(got[k] - want[k]) < 1e-9


# ------------------------------------------- TDT with every (symbol, duration) pair as a candidate

@pytest.mark.parametrize("algo", ["alsd", "aes"])
def test_tdt_pairs_unpruned_equals_enumeration_over_pairs(oracle, algo):
    c, w, L, enc = _small(66, model="tdt", durations=(0, 1, 2), V=2, T=3, s=2, beam=8192, algo=algo, tdt_pairs=True)
    fn = _ref_logp_fn(c, w, enc[0])
    want = enumerate_alignments(fn, 3, 2, 2, durations=(0, 1, 2), pairs=True)
    r = oracle.decode(c, w, enc, L)
    assert r["n_cut"][0] == 0 and r["collisions"][0] == 0
    got = _nbest(r)
    assert set(got) == set(want) and len(want) > 10
    for y, sc in want.items():
        assert abs(got[y] - sc) < 1e-9, (y, got[y], sc)
    # more probability mass than with one duration per symbol, which drops every other pair
    one = _nbest(oracle.decode(dict(c, tdt_pairs=False), w, enc, L))
    assert all(got[y] > one[y] - 1e-12 for y in one) and any(got[y] > one[y] + 1e-6 for y in one)
    assert sum(math.exp(v) for v in got.values()) <= 1.0 + 1e-12


def test_tdt_pairs_beam_one_equals_the_one_duration_rule(oracle):
    """The best pair of a hypothesis is (best symbol, its best duration): at beam 1 the two rules coincide."""
    c, w, L, enc = _small(67, model="tdt", durations=(0, 1, 2, 3), V=9, T=12, s=2, beam=1)
    a = oracle.decode(c, w, enc, L)
    b = oracle.decode(dict(c, tdt_pairs=True), w, enc, L)
    np.testing.assert_array_equal(a["tokens"], b["tokens"])
    np.testing.assert_allclose(a["scores"], b["scores"], atol=1e-12)
    toks, score = greedy(_ref_logp_fn(c, w, enc[0]), 12, 9, 2, durations=(0, 1, 2, 3))
    assert tuple(b["tokens"][0, 0, : b["lens"][0, 0]]) == toks and abs(b["scores"][0, 0] - score) < 1e-9
