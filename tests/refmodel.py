"""Independent checkers for the CPU oracle.

Nothing here calls the oracle or the HIP library.  The Transducer is evaluated
with PyTorch CPU library routines in float64 (``LSTMCell``, ``linear``,
``log_softmax``), and the search space is walked exhaustively: every alignment
of the lattice is enumerated and summed per transcript, which is what a beam
search that prunes nothing must reproduce (hypotheses with identical
transcripts are merged: Methods, first paragraph, and Sec. 2.1 of the paper).
"""
from __future__ import annotations

import math

import numpy as np
import torch


def logaddexp(a, b):
    if a == -math.inf:
        return b
    if b == -math.inf:
        return a
    m = max(a, b)
    return m + math.log(math.exp(a - m) + math.exp(b - m))


class RefModel:
    """float64 Transducer built from library layers."""

    def __init__(self, c, w):
        self.c = c
        self.V = c["V"]
        self.nd = len(c["durations"])
        t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
        self.W_enc, self.b_enc = t(w["W_enc"]), t(w["b_enc"])
        self.W_pred, self.b_pred = t(w["W_pred"]), t(w["b_pred"])
        self.W_out, self.b_out = t(w["W_out"]), t(w["b_out"])
        self.emb = t(w["emb"])
        if c["pred"] == "lstm":
            cell = torch.nn.LSTMCell(c["E"], c["P"]).double()
            with torch.no_grad():
                cell.weight_ih.copy_(t(w["W_ih"]))
                cell.weight_hh.copy_(t(w["W_hh"]))
                cell.bias_ih.copy_(t(w["b_ih"]))
                cell.bias_hh.copy_(t(w["b_hh"]))
            self.cell = cell
        self._pred_cache = {}

    def f_proj(self, enc_t):
        return torch.nn.functional.linear(torch.tensor(np.asarray(enc_t), dtype=torch.float64),
                                          self.W_enc, self.b_enc)

    def pred(self, tokens: tuple):
        """Prediction-network output (after W_pred) and state for a transcript."""
        if tokens in self._pred_cache:
            return self._pred_cache[tokens]
        c = self.c
        with torch.no_grad():
            if c["pred"] == "lstm":
                if len(tokens) == 0:
                    h0 = torch.zeros(1, c["P"], dtype=torch.float64)
                    state = self.cell(self.emb[self.V][None], (h0, h0.clone()))
                else:
                    _, prev = self.pred(tokens[:-1])
                    state = self.cell(self.emb[tokens[-1]][None], prev)
                h = state[0][0]
            else:
                h = torch.zeros(c["P"], dtype=torch.float64)
                for i in range(c["ctx"]):
                    tok = tokens[len(tokens) - 1 - i] if len(tokens) - 1 - i >= 0 else self.V
                    h = h + self.emb[i, tok]
                state = None
            g = torch.nn.functional.linear(h, self.W_pred, self.b_pred)
        self._pred_cache[tokens] = (g, state)
        return g, state

    def logp(self, f_t, tokens: tuple):
        """(token log-probs [V+1], duration log-probs [nd] or None)"""
        g, _ = self.pred(tokens)
        with torch.no_grad():
            z = torch.nn.functional.linear(torch.relu(f_t + g), self.W_out, self.b_out)
            lp = torch.log_softmax(z[: self.V + 1], dim=0).numpy()
            dl = torch.log_softmax(z[self.V + 1:], dim=0).numpy() if self.nd else None
        return lp, dl


class TableModel:
    """Log-probabilities read from a table [T, C, V+1] by class = hash mod C
    (mirrors the injected mode of the decoders)."""

    def __init__(self, tok, dur, V, hash_fn):
        self.tok, self.dur, self.V, self.hash_fn = tok, dur, V, hash_fn
        self.C = tok.shape[1]

    def logp_at(self, t, tokens):
        cls = self.hash_fn(tokens) % self.C
        return (self.tok[t, cls].astype(np.float64),
                None if self.dur is None else self.dur[t, cls].astype(np.float64))


def py_hash(tokens, base=1000003, mod=2 ** 31 - 1):
    """Eq. (1) with arbitrary-precision integers; token fed as v + 1."""
    h = 0
    for v in tokens:
        h = (h * base + (v + 1)) % mod
    return h


def duration_rule(dlogp, durations):
    """The decoders' reading for TDT: tokens take the most likely duration, blank
    the most likely one that advances at least a frame (ties -> first)."""
    best = int(np.argmax(dlogp))
    ok = [i for i, d in enumerate(durations) if d >= 1]
    best_b = ok[int(np.argmax([dlogp[i] for i in ok]))]
    return durations[best], dlogp[best], durations[best_b], dlogp[best_b]


def enumerate_alignments(logp_fn, T, V, s, durations=(), pairs=False):
    """Sum of alignment probabilities per transcript, by depth-first enumeration.

    ``pairs`` (TDT): every (symbol, duration) pair is a step of its own, blank only with
    durations >= 1, instead of one duration per symbol chosen by ``duration_rule``.

    ``logp_fn(t, tokens) -> (logp [V+1], dlogp or None)``.  An alignment ends
    when it has consumed T frames; at most ``s`` tokens are emitted without
    leaving a frame, after which only blank is possible (with its own
    log-probability).  Returns {transcript tuple: log-sum}.
    """
    totals = {}

    def rec(t, toks, sym, lp):
        if t >= T:
            totals[toks] = logaddexp(totals.get(toks, -math.inf), lp)
            return
        logp, dlogp = logp_fn(t, toks)
        if durations and pairs:
            for i, d in enumerate(durations):
                if d >= 1:
                    rec(min(t + d, T), toks, 0, lp + logp[V] + dlogp[i])
                if sym < s:
                    for v in range(V):
                        rec(min(t + d, T), toks + (v,), sym + 1 if d == 0 else 0, lp + logp[v] + dlogp[i])
            return
        if durations:
            adv_tok, x_tok, adv_blank, x_blank = duration_rule(dlogp, durations)
        else:
            adv_tok, x_tok, adv_blank, x_blank = 0, 0.0, 1, 0.0
        rec(min(t + adv_blank, T), toks, 0, lp + logp[V] + x_blank)
        if sym < s:
            for v in range(V):
                rec(min(t + adv_tok, T), toks + (v,), sym + 1 if adv_tok == 0 else 0, lp + logp[v] + x_tok)

    rec(0, (), 0, 0.0)
    return totals


def forward_dp(logp_fn, T, V, s, y):
    """Transducer forward variable for one transcript y with at most s tokens per
    frame: alpha[t][u][c] = log-probability of having emitted y[:u], standing at
    frame t, with c tokens emitted in it.  Blank: (t,u,c)->(t+1,u,0); token:
    (t,u,c)->(t,u+1,c+1) if c < s.  Returns log P(y) = alpha[T][U][0]."""
    U = len(y)
    NEG = -math.inf
    alpha = [[[NEG] * (s + 1) for _ in range(U + 1)] for _ in range(T + 1)]
    alpha[0][0][0] = 0.0
    for t in range(T):
        for u in range(U + 1):
            logp, _ = logp_fn(t, tuple(y[:u]))
            for c in range(s + 1):
                a = alpha[t][u][c]
                if a == NEG:
                    continue
                alpha[t + 1][u][0] = logaddexp(alpha[t + 1][u][0], a + logp[V])
                if u < U and c < s:
                    alpha[t][u + 1][c + 1] = logaddexp(alpha[t][u + 1][c + 1], a + logp[y[u]])
    return alpha[T][U][0]


def greedy(logp_fn, T, V, s, durations=()):
    """Standalone greedy decoder: per frame take the argmax, at most s tokens
    before blank is forced (with its own log-probability)."""
    t, toks, sym, score = 0, (), 0, 0.0
    while t < T:
        logp, dlogp = logp_fn(t, toks)
        if durations:
            adv_tok, x_tok, adv_blank, x_blank = duration_rule(dlogp, durations)
        else:
            adv_tok, x_tok, adv_blank, x_blank = 0, 0.0, 1, 0.0
        cand = logp.copy()
        cand[:V] += x_tok
        cand[V] += x_blank
        v = int(np.argmax(cand)) if sym < s else V
        score += cand[v]
        if v == V:
            t, sym = t + adv_blank, 0
        else:
            toks = toks + (v,)
            sym = sym + 1 if adv_tok == 0 else 0
            t += adv_tok
    return toks, score


def dict_lm(lm):
    """{(tokens...): (log10 p, log10 backoff)}"""
    d = {}
    for row, n, p, b in zip(lm["tokens"], lm["order"], lm["log10_prob"], lm["log10_backoff"]):
        d[tuple(int(x) for x in row[:n])] = (float(p), float(b))
    return d


def dict_lm_score(d, ctx: tuple, v: int) -> float:
    """ARPA back-off in log10 with a dictionary of tuples."""
    if ctx + (v,) in d:
        return d[ctx + (v,)][0]
    if not ctx:
        return -99.0
    bo = d[ctx][1] if ctx in d else 0.0
    return bo + dict_lm_score(d, ctx[1:], v)


def aes_frame_synchronous(logp_fn, T, V, s, K):
    """Frame-synchronous expansion search written as the classical two-set loop
    (Sec. 2.2, "AES"): per frame, hypotheses still emitting in the frame (open)
    are expanded round by round, those that emitted blank (closed) wait for the
    frame to end; every round keeps the K best of all expansions and waiting
    hypotheses, then merges equal transcripts among the waiting ones.  At most
    s tokens per frame; no prune margin.  Returns {transcript: score}."""
    closed = {(): 0.0}
    for t in range(T):
        open_, closed = closed, {}
        for rnd in range(s + 1):
            if not open_:
                break
            cands = []
            for toks, sc in open_.items():
                logp, _ = logp_fn(t, toks)
                cands.append((sc + logp[V], "closed", toks))
                if rnd < s:
                    for v in range(V):
                        cands.append((sc + logp[v], "open", toks + (v,)))
            for toks, sc in closed.items():
                cands.append((sc, "closed", toks))
            cands.sort(key=lambda x: -x[0])
            open_, closed = {}, {}
            for sc, kind, toks in cands[:K]:
                if kind == "open":
                    assert toks not in open_
                    open_[toks] = sc
                else:
                    closed[toks] = logaddexp(closed.get(toks, -math.inf), sc)
    return closed


def aes_bucketed(logp_fn, T, V, s, K, durations=(), gamma=math.inf, prefix=False):
    """The two-set loop of ``aes_frame_synchronous`` for models whose symbols carry durations (TDT), and with a
    prune margin.  A hypothesis that leaves frame t by a blank or by a token of duration d >= 1 is put into the
    waiting set of the frame it lands on (``bucket[t + d]``, clamped at T = finished); tokens of duration 0 keep it
    open in the frame for the next round, at most ``s`` of them.  Frames are visited in order; the hypotheses
    waiting at a frame become its open set; every round expands all open hypotheses by one symbol (one duration
    per symbol: ``duration_rule``), lets every waiting hypothesis of every later frame compete with its score as
    it is, keeps the K best, and merges equal transcripts that wait at the same frame.  ``gamma``: a symbol
    (blank included) whose log-probability is more than gamma below the best one of its hypothesis is not
    expanded; a blank forced by the frame limit is kept.
    ``prefix``: maximum-length prefix search.  If the open set of a round holds both y and y + (v,), and the
    expansion of y by v stays in the frame and is one of the K best token expansions of y, the expansions of
    y + (v,) are RANKED as if its score also held that expansion's score; the scores themselves are unchanged (the
    expansion competes on its own and is merged with y + (v,) when both have left the frame).
    Returns {transcript: score} of the finished set."""
    bucket = {t: {} for t in range(T + 1)}
    bucket[0][()] = 0.0
    for t in range(T):
        open_, bucket[t] = bucket[t], {}
        rnd = 0
        while open_:
            cands = []  # (ranking key, score, landing frame or None = stays open, transcript)
            tok_vals, stays = {}, {}
            rows = {}
            for toks, sc in open_.items():
                logp, dlogp = logp_fn(t, toks)
                if durations:
                    adv_tok, x_tok, adv_blank, x_blank = duration_rule(dlogp, durations)
                else:
                    adv_tok, x_tok, adv_blank, x_blank = 0, 0.0, 1, 0.0
                floor = max(logp) - gamma
                forced = rnd >= s
                row = []
                if forced or logp[V] >= floor:
                    row.append((sc + logp[V] + x_blank, min(t + adv_blank, T), toks))
                vals = {}
                if not forced:
                    for v in range(V):
                        if logp[v] >= floor:
                            vals[v] = sc + logp[v] + x_tok
                            row.append((vals[v], None if adv_tok == 0 else min(t + adv_tok, T), toks + (v,)))
                rows[toks], tok_vals[toks], stays[toks] = row, vals, adv_tok == 0
            for toks, sc in open_.items():
                delta = 0.0
                if prefix and toks and toks[:-1] in open_ and stays[toks[:-1]]:
                    vals, v = tok_vals[toks[:-1]], toks[-1]
                    if v in vals and sum(1 for u, x in vals.items() if x > vals[v] or (x == vals[v] and u < v)) < K:
                        delta = logaddexp(sc, vals[v]) - sc
                cands += [(val + delta, val, land, y) for val, land, y in rows[toks]]
            for tw in range(t + 1, T + 1):
                for toks, sc in bucket[tw].items():
                    cands.append((sc, sc, tw, toks))
            cands.sort(key=lambda x: -x[0])
            if len(cands) > K:
                assert cands[K - 1][0] != cands[K][0], "exact tie at the cut: the case cannot pin the order"
            open_ = {}
            for tw in range(t + 1, T + 1):
                bucket[tw] = {}
            for _, sc, land, toks in cands[:K]:
                if land is None:
                    assert toks not in open_
                    open_[toks] = sc
                else:
                    bucket[land][toks] = logaddexp(bucket[land].get(toks, -math.inf), sc)
            rnd += 1
    return bucket[T]


def alsd_two_stage(logp_fn, fused_fn, T, V, s, K):
    """Alignment-length synchronous search with early pruning, written with dictionaries
    (Sec. 2.3, "Early/late pruning"): at every step all expansions of the unfinished hypotheses
    are ranked by the Transducer's score alone, the K best are kept and only those are charged
    the fused (Transducer + LM) increment.  Hypotheses that have consumed all frames compete with
    their score as it is.  Equal (transcript, frame, symbols in frame) are merged by log-sum.
    At most s tokens per frame.  ``fused_fn(t, toks)`` returns the fused increments [V + 1].
    Returns {transcript: score} of the hypotheses alive at the end."""
    hyps = {((), 0, 0): 0.0}
    for _ in range(T * (s + 1)):
        if all(t >= T for (_, t, _) in hyps):
            break
        cands = []
        for (toks, t, sym), sc in hyps.items():
            if t >= T:
                cands.append((sc, sc, (toks, t, sym)))
                continue
            logp, _ = logp_fn(t, toks)
            fused = fused_fn(t, toks)
            cands.append((sc + logp[V], sc + fused[V], (toks, t + 1, 0)))
            if sym < s:
                for v in range(V):
                    cands.append((sc + logp[v], sc + fused[v], (toks + (v,), t, sym + 1)))
        cands.sort(key=lambda x: -x[0])
        hyps = {}
        for _, val, node in cands[:K]:
            hyps[node] = logaddexp(hyps.get(node, -math.inf), val)
    out = {}
    for (toks, t, sym), sc in hyps.items():
        assert toks not in out
        out[toks] = sc
    return out


def replay_step_margins(logp_fn, T, V, s, K, algo, durations, gamma, log_parent, log_token, log_merged, n_steps):
    """Walks one utterance along a decoder's logged tree (parent slot, token code, merged-into slot per step) and
    recomputes, from the model alone, the smallest margin by which any decision of each step was taken:
      * the gaps between consecutive candidates in the ranking, down to the gap between the last kept and the
        first discarded one (kept candidates' order decides the slot numbers, the last gap decides the cut);
      * TDT, one duration per symbol: the margins of the two duration arg-maxes of every expanded hypothesis;
      * AES with a finite prune margin: for every symbol of a hypothesis that is expanded freely (not forced to
        blank) whose unmasked candidate would rank within 1e-3 of the cut or better, the distance of its
        log-probability from the margin's threshold.
    Slots follow the unified step: dead slots have no candidate; a live hypothesis that is finished or (AES) not at
    the earliest frame has the single candidate "stay"; candidates are ordered by (value desc, k (V + 1) + v asc).
    Also checks that the logged selection IS the head of that ranking whenever the step's margin is clear.
    Returns the list of margins, one per step."""
    slots = [dict(live=(k == 0), toks=(), t=0, sym=0, score=0.0 if k == 0 else -math.inf) for k in range(K)]
    out = []
    for st in range(n_steps):
        open_t = [h["t"] for h in slots if h["live"] and h["t"] < T]
        assert open_t, "the log goes on after the utterance has finished"
        t_cur = min(open_t)
        margin = math.inf
        cands = []       # (value, flat index)
        unmasked = {}    # flat index -> (value without the prune margin, distance from the margin's threshold)
        adv = {}
        for k, h in enumerate(slots):
            if not h["live"]:
                continue
            if not (h["t"] < T and (algo == "alsd" or h["t"] == t_cur)):
                cands.append((h["score"], k * (V + 1) + V))
                continue
            logp, dlogp = logp_fn(h["t"], h["toks"])
            x_tok = x_blank = 0.0
            adv[k] = (0, 1)
            if durations:
                best = max(range(len(durations)), key=lambda d: (dlogp[d], -d))
                adv_ok = [d for d in range(len(durations)) if durations[d] >= 1]
                best_b = max(adv_ok, key=lambda d: (dlogp[d], -d))
                for d in range(len(durations)):
                    if d != best:
                        margin = min(margin, dlogp[best] - dlogp[d])
                    if d != best_b and durations[d] >= 1:
                        margin = min(margin, dlogp[best_b] - dlogp[d])
                x_tok, x_blank = dlogp[best], dlogp[best_b]
                adv[k] = (durations[best], durations[best_b])
            forced = h["sym"] >= s
            floor = max(logp) - gamma if algo == "aes" else -math.inf
            for v in range(V + 1):
                val = h["score"] + logp[v] + (x_blank if v == V else x_tok)
                masked = (forced and v < V) or (not (forced and v == V) and logp[v] < floor)
                cands.append((-math.inf if masked else val, k * (V + 1) + v))
                if algo == "aes" and math.isfinite(gamma) and not forced:
                    unmasked[k * (V + 1) + v] = (val, abs(logp[v] - floor))
        cands.sort(key=lambda c: (-c[0], c[1]))
        finite = [c for c in cands if c[0] > -math.inf]
        for i in range(min(K, len(finite) - 1)):
            margin = min(margin, finite[i][0] - finite[i + 1][0])
        cut = finite[K - 1][0] if len(finite) >= K else -math.inf
        for val, dist in unmasked.values():
            if val >= cut - 1e-3:
                margin = min(margin, dist)
        out.append(margin)
        # the logged step
        new = []
        for j in range(K):
            p, code = int(log_parent[st][j]), int(log_token[st][j])
            if p < 0:
                new.append(dict(live=False, toks=(), t=0, sym=0, score=-math.inf))
                continue
            h = slots[p]
            v = V if code < 0 else code
            if margin > 1e-9:
                assert j < len(finite) and finite[j][1] == p * (V + 1) + v, (st, j, finite[:K], p, code)
            val = dict((i, x) for x, i in finite)[p * (V + 1) + v]
            n = dict(h, score=val)
            if code == -2:
                pass
            elif code == -1:
                n.update(t=min(h["t"] + adv[p][1], T), sym=0)
            else:
                n.update(toks=h["toks"] + (code,), t=min(h["t"] + adv[p][0], T),
                         sym=h["sym"] + 1 if adv[p][0] == 0 else 0)
            new.append(n)
        if margin > 1e-9:
            assert sum(1 for n in new if n["live"]) == min(K, len(finite))
        for j in range(K):
            m = int(log_merged[st][j])
            if new[j]["live"] and m != j:
                assert 0 <= m < j and (new[m]["toks"], new[m]["t"], new[m]["sym"]) == (
                    new[j]["toks"], new[j]["t"], new[j]["sym"])
                new[m]["score"] = logaddexp(new[m]["score"], new[j]["score"])
                new[j] = dict(live=False, toks=(), t=0, sym=0, score=-math.inf)
        slots = new
    return out
