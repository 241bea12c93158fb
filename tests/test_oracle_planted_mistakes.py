"""Each plausible mistake, planted in a private copy of the oracle's source and
compiled on the CPU, must make at least one pin fail.  This is the evidence that
the pins constrain every part of the oracle and not only its happy path."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rnnt_oracle.c")

MISTAKES = [
    ("merge key without the symbols-in-frame count",
     "nxt[i].t == nxt[j].t && nxt[i].sym == nxt[j].sym", "nxt[i].t == nxt[j].t"),
    ("merge keeps the maximum instead of the log-sum",
     "nxt[i].score = logaddexp(nxt[i].score, nxt[j].score);",
     "nxt[i].score = nxt[i].score > nxt[j].score ? nxt[i].score : nxt[j].score;"),
    ("frame limit off by one", "const int forced = hy->sym >= s;", "const int forced = hy->sym > s;"),
    ("symbol counter not reset when a TDT token advances",
     "nh->sym = adv_tok[k] == 0 ? nh->sym + 1 : 0;", "nh->sym = nh->sym + 1;"),
    ("blank takes the tokens' duration", "tot[V] += dl[best_b];", "tot[V] += dl[best];"),
    ("frame index not clamped", "if (nh->t > T_b) nh->t = T_b;", ""),
    ("AES waiting rule dropped", "int active = hy->t < T_b && (J->algo == 0 || hy->t == t_cur);",
     "int active = hy->t < T_b;"),
    ("recurrent bias dropped", "gate[q] = gi[r] + (double)w->b_ih[r] + gh[r] + (double)w->b_hh[r];",
     "gate[q] = gi[r] + (double)w->b_ih[r] + gh[r];"),
    ("forget and input gates swapped", "double cn = fg * c_in[p] + ig * gg;", "double cn = ig * c_in[p] + fg * gg;"),
    ("ReLU dropped", "a[j] = opnd(c, s > 0.0 ? s : 0.0);", "a[j] = opnd(c, s);"),
    ("blank not rescored under fusion", "tot[V] = (lm && c->lm_rule != 3) ? (1.0 + lambda) * logp[V] : logp[V];",
     "tot[V] = logp[V];"),
    ("non-blank mass term dropped", "else tot[v] = logp[v] + lambda * (nb + lm[v]);",
     "else tot[v] = logp[v] + lambda * lm[v];"),
    ("back-off weight ignored", "double bo = c >= 0 ? (double)lm->backoff[c] : 0.0;", "double bo = 0.0;"),
    ("back-off drops the newest token instead of the oldest", "return bo + lm_q10(lm, ctx + 1, n - 1, v);",
     "return bo + lm_q10(lm, ctx, n - 1, v);"),
    ("hash feeds the raw token", "(uint64_t)nh->hash * ORC_HASH_BASE + (uint64_t)(v + 1)",
     "(uint64_t)nh->hash * ORC_HASH_BASE + (uint64_t)(v)"),
    ("ties broken by the higher index", "return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);",
     "return x->idx > y->idx ? -1 : (x->idx < y->idx ? 1 : 0);"),
    ("prune margin applied to the fused score's maximum only for tokens", "for (int v = 0; v <= V; ++v)\n      if (logp[v] < mx - c->gamma) tot[v] = -INFINITY;",
     "for (int v = 0; v < V; ++v)\n      if (logp[v] < mx - c->gamma) tot[v] = -INFINITY;"),
    ("bf16 rounding truncates", "u += 0x7fffu + lsb;", "u += 0;"),
    ("early pruning ranks by the fused score",
     "cand[((int64_t)k * (V + 1) + v) * nd + d].key = hy->score + tot_asr[v] + x;", ""),
    ("blank may stand still when every pair is a candidate",
     "double x = pairs ? ((v == V && c->durations[d] < 1) ? -INFINITY : dl[d]) : 0.0;", "double x = pairs ? dl[d] : 0.0;"),
    ("a pair advances by the best duration instead of its own",
     "if (pairs) adv_tok[k] = adv_blank[k] = c->durations[dsel]; /* the pair's own duration */", ""),
    ("early pruning keeps the Transducer's score as the new score", "nh->score = cand[j].val;", "nh->score = cand[j].key;"),
    ("near-tie report looks at the kept candidates only", "for (int i = 0; i < K && i + 1 < n_cand; ++i)",
     "for (int i = 0; i + 1 < K && i + 1 < n_cand; ++i)"),
    ("duration margin left out of the near-tie report", "    if (gap_out) {\n      for (int d = 0; d < c->n_dur; ++d) {",
     "    if (0) {\n      for (int d = 0; d < c->n_dur; ++d) {"),
    ("distance from the prune margin left out of the near-tie report",
     "if (J->algo == 1 && isfinite(c->gamma) && !pairs) {\n      /* a token close", "if (0) {\n      /* a token close"),
    ("prune margin applied under ALSD++ too", "const int use_gamma = J->algo == 1;", "const int use_gamma = 1;"),
    ("prefix search adds the expansion's score to the longer hypothesis as well (alignments counted twice)",
     "for (int u = 0; u <= V; ++u) cand[((int64_t)i * (V + 1) + u) * nd].key += delta;",
     "for (int u = 0; u <= V; ++u) { cand[((int64_t)i * (V + 1) + u) * nd].key += delta; "
     "cand[((int64_t)i * (V + 1) + u) * nd].val += delta; }"),
    ("prefix credit also for an expansion that is not among the Beam best of its hypothesis",
     "if (better < K) add = logaddexp(add, credit);", "add = logaddexp(add, credit);"),
    ("prefix credit also for an expansion that leaves the frame", "          if (adv_tok[j] != 0) continue;\n", ""),
    ("AES++ opens the frame of the first unfinished slot instead of the earliest frame",
     "        if (cur[k].t < t_cur) t_cur = cur[k].t;", "        if (t_cur == T_b) t_cur = cur[k].t;"),
]


@pytest.mark.parametrize("name,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(SRC).read()
    assert src.count(old) >= 1, "the oracle's source changed: update this mistake"
    mutated = tmp_path / "mutated.c"
    mutated.write_text(src.replace(old, new, 1))
    lib = tmp_path / "libmutated.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(lib), str(mutated),
                           "-lm"])
    env = dict(os.environ, RNNT_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True)
    assert r.returncode != 0, f"no pin noticed: {name}"
    assert "failed" in r.stdout
