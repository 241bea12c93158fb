"""Shared helpers of the GPU parity tests: run the HIP library and the CPU
oracle on the same seeded inputs and compare them."""
from __future__ import annotations

import numpy as np


def to_gpu(a, dtype=None):
    import torch
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda().contiguous()


def gpu_decode(dec, enc, lengths, want_tree=True, check=True, **kw):
    import torch
    dec.decode(to_gpu(enc, torch.float32), to_gpu(lengths, torch.int32), **kw)
    r = dec.results(check=check)
    if want_tree:
        r.update(dec.dump_tree(int(r["n_steps"].max()) + 1))
    return r


def gpu_decode_injected(dec, tok, dur, lengths, **kw):
    import torch
    dec.decode_injected(to_gpu(tok, torch.float32), to_gpu(dur, torch.float32) if dur is not None else None,
                        to_gpu(lengths, torch.int32), **kw)
    r = dec.results()
    r.update(dec.dump_tree(int(r["n_steps"].max()) + 1))
    return r


def make_walk(oracle, c, w, enc, L, g, tol, lm=None, lm_weight=0.0, lm_rule=4, lm_prune="late"):
    """walk(gb): step-by-step validity check of the GPU's own tree of batch row ``gb`` (see tree_check.py)."""
    from tree_check import check_tree

    def walk(gb):
        n = int(g["n_steps"][gb])
        nbest = [(tuple(int(x) for x in g["tokens"][gb, j, :g["lens"][gb, j]]), float(g["scores"][gb, j]))
                 for j in range(g["lens"].shape[1]) if g["lens"][gb, j] >= 0]
        return check_tree(oracle, c, w, enc[gb], int(L[gb]), g["parent"][:n, gb], g["token"][:n, gb],
                          g["merged"][:n, gb], n, nbest, slack=2 * tol, tol=tol, lm=lm, lm_weight=lm_weight,
                          lm_rule=lm_rule, lm_prune=lm_prune)
    return walk


def compare(g, o, tol, tie, exact_tree=False, rows=None, walk=None):
    """GPU result ``g`` against oracle result ``o`` (decoded with log=True).

    Per utterance: the trees (parent, token, merged_into of every live slot) must
    be identical up to a step at which the oracle took its decision by a margin
    below ``tie``: the first step where the two trees differ must itself be such
    a step.  If they are identical throughout, step counts and token sequences
    must be identical and scores within ``tol``.  An utterance whose tree leaves
    the oracle's at a near tie cannot be compared with the oracle's from there on;
    ``walk`` (see ``make_walk``) then checks the GPU's own tree step by step,
    from the first step to the last, and its n-best list.
    ``exact_tree``: no exemption at all.  ``rows``: GPU batch rows that the
    oracle rows correspond to.  Returns (n_full_match, n_left_the_oracles_tree).
    """
    B = o["lens"].shape[0]
    rows = list(range(B)) if rows is None else rows
    full, exempt = 0, 0
    left = []
    for ob, gb in enumerate(rows):
        n = int(o["n_steps"][ob])
        gaps = o["log_gap"][ob, :n]
        near = np.nonzero(gaps < tie)[0]
        first_tie = n if (exact_tree or near.size == 0) else int(near[0])
        ng = int(g["n_steps"][gb])
        diverged_at = None
        for st in range(min(n, ng)):
            op, ot, om = o["log_parent"][ob, st], o["log_token"][ob, st], o["log_merged"][ob, st]
            gp, gt, gm = g["parent"][st, gb], g["token"][st, gb], g["merged"][st, gb]
            live = op >= 0
            same = (np.array_equal(live, gp >= 0) and np.array_equal(op[live], gp[live])
                    and np.array_equal(ot[live], gt[live]) and np.array_equal(om[live], gm[live]))
            if not same:
                diverged_at = st
                break
        if diverged_at is None and ng != n:
            diverged_at = min(n, ng)
        if diverged_at is not None:
            at = min(diverged_at, n - 1)
            assert diverged_at >= first_tie and gaps[at] < tie, (
                f"utterance {gb}: tree differs at step {diverged_at}, where the oracle's margin was {gaps[at]:.3g} "
                f"(allowed below {tie}; first near tie at {first_tie}); "
                f"oracle {o['log_parent'][ob, diverged_at]} {o['log_token'][ob, diverged_at]} "
                f"gpu {g['parent'][diverged_at, gb]} {g['token'][diverged_at, gb]}")
            exempt += 1
            left.append(gb)
            continue
        np.testing.assert_array_equal(g["lens"][gb], o["lens"][ob])
        for j in range(o["lens"].shape[1]):
            L = o["lens"][ob, j]
            if L < 0:
                assert np.isneginf(g["scores"][gb, j])
                continue
            np.testing.assert_array_equal(g["tokens"][gb, j, :L], o["tokens"][ob, j, :L])
            assert abs(g["scores"][gb, j] - o["scores"][ob, j]) <= tol, (
                gb, j, g["scores"][gb, j], o["scores"][ob, j])
        full += 1
    if walk is not None and left:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, len(left))) as pool:  # the oracle's C routines release the GIL
            reports = list(pool.map(walk, left))
        print(f"walked {len(left)} trees that left the oracle's: steps checked {[r['steps_checked'] for r in reports]}, "
              f"stopped at a duration near tie {sum(r['stopped_at_duration_tie'] for r in reports)}, largest score "
              f"difference {max([r.get('max_score_diff', 0.0) for r in reports]):.3g}")
    return full, exempt
