"""Validity of a hypothesis tree that has left the oracle's own tree.

Beam search is a heuristic: once the GPU and the oracle have taken a different decision at a step where two
candidates were within rounding of each other, their trees legitimately differ from there on and cannot be compared
slot by slot any more.  What can still be checked is that every later step of the GPU's tree is a correct step of the
method given the hypotheses the GPU itself held: the walk below follows the GPU's logged tree (parent slot, token,
merged-into slot per step), rebuilds every hypothesis with the oracle's unit entry points (encoder projection, LSTM
step / stateless network, prediction projection, joint, per-row score rule, LM query) in float64, and asserts at
every step that
  * the candidates the GPU kept are a top-Beam set of all candidates of that step up to ``slack`` (no discarded
    candidate is better than a kept one by more than ``slack``; nothing is left out while a slot stays empty),
    in descending order up to ``slack``.  The library's accumulated scores may differ from the walk's by the score
    tolerance, so candidates of two different hypotheses can legitimately swap within twice that: the callers
    pass ``slack`` = 2 x their score tolerance;
  * waiting / finished hypotheses are carried over with the "stay" code and forced blanks are blanks;
  * recombination is exact: merged-into equals the lowest earlier slot with the same (transcript, frame, symbols in
    frame), decided on explicit transcripts;
and at the end that the n-best transcripts and scores the library reports are those of the walk, within ``tol``.
TDT: a walk ends early, and says so, when the GPU's choice depended on a duration arg-max that was itself a near
tie (the tree does not record durations).  Nothing here calls the HIP library.
"""
from __future__ import annotations

import math

import numpy as np


def logaddexp(a, b):
    if a == -math.inf:
        return b
    if b == -math.inf:
        return a
    m = max(a, b)
    return m + math.log(math.exp(a - m) + math.exp(b - m))


class UnitModel:
    """The Transducer of one utterance through the oracle's unit entry points, cached by transcript."""

    def __init__(self, oracle, c, w, enc_b, lm=None, lm_weight=0.0, lm_rule=4):
        self.o, self.c, self.enc = oracle, dict(c), enc_b
        self.V, self.nd = c["V"], len(c["durations"])
        self.lm, self.lam, self.lm_rule = lm, lm_weight, lm_rule
        self.rounded = c["prec"] == "bf16"
        self.w = dict(w)
        if self.rounded:  # round the joint's matrices once (library cast; the oracle's own rounding is pinned to it)
            import torch
            for k in ("W_enc", "W_pred", "W_out"):
                self.w[k] = torch.tensor(np.asarray(w[k], np.float32)).bfloat16().float().numpy()
        self._f, self._pred, self._lm, self._z = {}, {}, {}, {}

    def f(self, t):
        if t not in self._f:
            self._f[t] = self.o.enc_proj(self.c, self.w, self.enc[t], rounded=self.rounded)
        return self._f[t]

    def pred(self, toks):
        """(g, (h, c)) for a transcript (LSTM fed with the start symbol first)."""
        if toks in self._pred:
            return self._pred[toks]
        c = self.c
        if c["pred"] == "lstm":
            if len(toks) == 0:
                z = np.zeros(c["P"])
                st = self.o.lstm_step(c, self.w, z, z, self.V)
            else:
                st = self.o.lstm_step(c, self.w, *self.pred(toks[:-1])[1], toks[-1])
            g = self.o.pred_proj(c, self.w, st[0], rounded=self.rounded)
        else:
            st = None
            g = self.o.stateless_pred(c, self.w, list(toks), rounded=self.rounded)
        self._pred[toks] = (g, st)
        return self._pred[toks]

    def lm_row(self, toks):
        if self.lm is None:
            return None
        if toks not in self._lm:
            self._lm[toks] = self.lm.query(list(toks), self.V)
        return self._lm[toks]

    def row(self, t, toks, apply_gamma, forced, with_lm=True):
        """tot [V + 1] (masks and TDT duration term included), logp, frames advanced by a token / by blank, and the
        smallest margin of the two duration arg-maxes."""
        if (t, toks) not in self._z:
            self._z = {k: v for k, v in self._z.items() if k[0] >= t - 8}  # frames long left behind are not needed
            self._z[(t, toks)] = self.o.joint(self.c, self.w, self.f(t), self.pred(toks)[0], rounded=self.rounded)
        z = self._z[(t, toks)]
        tot, logp, adv_tok, adv_blank = self.o.score_row(
            self.c, z=z, lm_row=self.lm_row(toks) if with_lm else None, lm_weight=self.lam if with_lm else 0.0,
            lm_rule=self.lm_rule, apply_gamma=apply_gamma, forced_blank=forced)
        dmargin = math.inf
        if self.nd:
            d = z[self.V + 1:]
            dur = self.c["durations"]
            best = int(np.argmax(d))
            ok = [i for i in range(self.nd) if dur[i] >= 1]
            best_b = ok[int(np.argmax(d[ok]))]
            for i in range(self.nd):
                if i != best:
                    dmargin = min(dmargin, d[best] - d[i])
                if i != best_b and dur[i] >= 1:
                    dmargin = min(dmargin, d[best_b] - d[i])
        return tot, logp, adv_tok, adv_blank, dmargin


def check_tree(oracle, c, w, enc_b, T_b, parent, token, merged, n_steps, nbest, slack, tol, lm=None, lm_weight=0.0,
               lm_rule=4, lm_prune="late"):
    """Walk one utterance.  parent / token / merged: [S, K] arrays of the library's tree dump for this utterance;
    nbest: list of (transcript tuple, score) the library reported, best first.  Returns a dict with the number of
    steps verified and whether the walk stopped early at a duration near tie."""
    assert not c.get("tdt_pairs"), "the walk knows the one-duration rule only"
    assert not c.get("aes_prefix"), "the walk ranks by the new scores: it does not know the prefix credit"
    K, V, s = parent.shape[1], c["V"], c["s"]
    algo, gamma = c["algo"], c["gamma"]
    m = UnitModel(oracle, c, w, enc_b, lm, lm_weight, lm_rule)
    early = lm is not None and lm_prune == "early"
    dead = dict(live=False, toks=(), t=0, sym=0, score=-math.inf)
    slots = [dict(live=True, toks=(), t=0, sym=0, score=0.0)] + [dict(dead) for _ in range(K - 1)]
    use_gamma = algo == "aes" and math.isfinite(gamma)
    for st in range(n_steps):
        open_t = [h["t"] for h in slots if h["live"] and h["t"] < T_b]
        assert open_t, f"step {st}: the tree goes on although every hypothesis has finished"
        t_cur = min(open_t)
        # per slot: ranking key and new score of every symbol (-inf = no such candidate), and which symbols sit within
        # rounding of the prune margin (kept or dropped, both are right)
        val, key, unsure, adv, kind, dmargin = {}, {}, {}, {}, {}, {}
        for k, h in enumerate(slots):
            if not h["live"]:
                kind[k] = 0
                continue
            val[k] = np.full(V + 1, -np.inf)
            key[k] = np.full(V + 1, -np.inf)
            unsure[k] = np.zeros(V + 1, bool)
            if not (h["t"] < T_b and (algo == "alsd" or h["t"] == t_cur)):
                kind[k] = 1
                val[k][V] = key[k][V] = h["score"]
                continue
            kind[k] = 2
            forced = h["sym"] >= s
            tot, logp, a_t, a_b, dm = m.row(h["t"], h["toks"], algo == "aes", forced)
            rank = m.row(h["t"], h["toks"], algo == "aes", forced, with_lm=False)[0] if early else tot
            adv[k], dmargin[k] = (a_t, a_b), dm
            val[k], key[k] = h["score"] + tot, h["score"] + rank
            if use_gamma and not forced:
                near = np.abs(logp - (logp.max() - gamma)) < slack
                if near.any():
                    t2 = m.row(h["t"], h["toks"], False, forced)[0]
                    r2 = m.row(h["t"], h["toks"], False, forced, with_lm=False)[0] if early else t2
                    val[k] = np.where(near, h["score"] + t2, val[k])
                    key[k] = np.where(near, h["score"] + r2, key[k])
                    unsure[k] = near
        kept = []
        for j in range(K):
            p, code = int(parent[st][j]), int(token[st][j])
            if p < 0:
                assert code == -3 and int(merged[st][j]) == -1, (st, j, p, code)
                continue
            assert kind.get(p, 0) != 0, f"step {st} slot {j}: parent {p} is an empty slot"
            assert (code == -2) == (kind[p] == 1), f"step {st} slot {j}: code {code} for a parent of kind {kind[p]}"
            cand = (p, V if code < 0 else code)
            assert key[p][cand[1]] > -np.inf, f"step {st} slot {j}: candidate {cand} is masked (frame limit / prune margin)"
            assert cand not in [x for x, _ in kept], f"step {st}: candidate {cand} kept twice"
            kept.append((cand, j))
        # what was discarded although it certainly is a candidate
        rest_best, rest_at = -np.inf, None
        for k in key:
            r = np.where(unsure[k], -np.inf, key[k])
            for (p, v), _ in kept:
                if p == k:
                    r[v] = -np.inf
            i = int(np.argmax(r))
            if r[i] > rest_best:
                rest_best, rest_at = float(r[i]), (k, i)
        if len(kept) < K:
            assert rest_best == -np.inf, f"step {st}: slots left empty although candidate {rest_at} exists"
        else:
            worst = min(key[p][v] for (p, v), _ in kept)
            assert rest_best <= worst + slack, (
                f"step {st}: discarded candidate {rest_at} ({rest_best:.6f}) beats kept {worst:.6f} by more than {slack}")
        ks = [key[p][v] for (p, v), _ in kept]
        assert all(ks[i] >= ks[i + 1] - slack for i in range(len(ks) - 1)), f"step {st}: kept candidates out of order"
        # TDT: the frames a kept candidate advances by come from a duration arg-max the tree does not record
        if m.nd and any(kind[p] == 2 and dmargin[p] < slack for (p, _), _ in kept):
            return dict(steps_checked=st, stopped_at_duration_tie=True)
        new = [dict(dead) for _ in range(K)]
        for (p, v), j in kept:
            h = slots[p]
            n = dict(h, score=float(val[p][v]))
            if kind[p] == 1:
                pass
            elif v == V:
                n.update(t=min(h["t"] + adv[p][1], T_b), sym=0)
            else:
                n.update(toks=h["toks"] + (v,), t=min(h["t"] + adv[p][0], T_b), sym=h["sym"] + 1 if adv[p][0] == 0 else 0)
            new[j] = n
        for j in range(K):
            if not new[j]["live"]:
                continue
            same = [i for i in range(j) if new[i]["live"] and (new[i]["toks"], new[i]["t"], new[i]["sym"]) ==
                    (new[j]["toks"], new[j]["t"], new[j]["sym"])]
            want = same[0] if same else j
            assert int(merged[st][j]) == want, f"step {st} slot {j}: merged into {int(merged[st][j])}, expected {want}"
            if same:
                new[want]["score"] = logaddexp(new[want]["score"], new[j]["score"])
                new[j] = dict(dead)
        slots = new
    assert not any(h["live"] and h["t"] < T_b for h in slots) or n_steps >= T_b * (s + 1), "the tree ends too early"
    mine = {}
    for h in slots:
        if h["live"]:
            assert h["toks"] not in mine
            mine[h["toks"]] = h["score"]
    got = dict(nbest)
    assert len(got) == len(nbest), "the same transcript twice in the n-best list"
    assert set(got) == set(mine), (sorted(got), sorted(mine))
    for y, sc in got.items():
        assert abs(sc - mine[y]) <= tol, (y, sc, mine[y])
    sc = [x for _, x in nbest]
    assert all(sc[i] >= sc[i + 1] for i in range(len(sc) - 1)), "n-best not sorted"
    return dict(steps_checked=n_steps, stopped_at_duration_tie=False,
                max_score_diff=max(abs(x - mine[y]) for y, x in got.items()))
