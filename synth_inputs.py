"""Seeded synthetic inputs for the batched Transducer beam-search hot path.

This module only draws random numbers and lays them out in arrays.  It holds
none of the method's arithmetic (no joint, no softmax, no search, no LM
back-off): the CPU oracle and the HIP library both receive what it returns and
share nothing else.

The paper evaluates on trained Fast Conformer Transducer models (BPE vocabulary
of 1024 tokens, 80 ms encoder frames) with n-gram LMs built from ARPA files
(Experimental Setup section).  None of that data is available, so the arrays
made here take the *shapes* of those models and stand in for them.

Seeds: ``1000 * config + part`` with part 0 = encoder output, 1 = weights,
2 = lengths, 3 = language model, 4 = injected log-probability tables.
"""
from __future__ import annotations

import numpy as np

FRAME_SECONDS = 0.08  # one encoder frame covers 80 ms of audio

# name -> workload description.  Keys follow the notation of the method:
# B utterances, T frames, D encoder dim, H joint hidden, P prediction hidden,
# E embedding dim, V tokens (blank id = V), s = max symbols per frame.
CONFIGS = {
    1: dict(name="c1_tiny_rnnt_alsd", model="rnnt", pred="lstm", prec="f32",
            B=1, T=20, T_min=20, D=64, H=64, P=64, E=64, V=16, durations=(),
            beam=4, s=3, algo="alsd", gamma=float("inf"), blank_bias=2.0,
            lm=None, lm_weight=0.0, ctx=0),
    2: dict(name="c2_rnnt_alsd_b32", model="rnnt", pred="lstm", prec="f32",
            B=32, T=125, T_min=125, D=1024, H=640, P=640, E=640, V=1024,
            durations=(), beam=4, s=5, algo="alsd", gamma=float("inf"),
            blank_bias=3.0, lm=None, lm_weight=0.0, ctx=0),
    3: dict(name="c3_tdt_aes_b64", model="tdt", pred="lstm", prec="f32",
            B=64, T=250, T_min=50, D=1024, H=640, P=640, E=640, V=1024,
            durations=(0, 1, 2, 3, 4), beam=4, s=2, algo="aes", gamma=2.3,
            blank_bias=3.0, lm=None, lm_weight=0.0, ctx=0),
    4: dict(name="c4_rnnt_alsd_lm_b32", model="rnnt", pred="lstm", prec="f32",
            B=32, T=125, T_min=125, D=1024, H=640, P=640, E=640, V=1024,
            durations=(), beam=8, s=5, algo="alsd", gamma=float("inf"),
            blank_bias=3.0, lm=dict(order=4, n_target=2_000_000, zipf_s=1.1),
            lm_weight=0.3, ctx=0),
    5: dict(name="c5_stateless_aes_b128", model="rnnt", pred="stateless",
            prec="bf16", B=128, T=250, T_min=250, D=1024, H=640, P=640, E=640,
            V=8192, durations=(), beam=10, s=2, algo="aes",
            gamma=float("inf"), blank_bias=3.0, lm=None, lm_weight=0.0, ctx=2),
}


def config(idx: int, **overrides) -> dict:
    """A copy of workload ``idx`` with fields replaced by ``overrides``."""
    c = dict(CONFIGS[idx])
    c["id"] = idx
    c.update(overrides)
    return c


def custom_config(**fields) -> dict:
    """A small workload of arbitrary shape (used by the shrunken test cases)."""
    c = dict(name="custom", model="rnnt", pred="lstm", prec="f32", B=1, T=4,
             T_min=None, D=8, H=8, P=8, E=8, V=2, durations=(), beam=4, s=2,
             algo="alsd", gamma=float("inf"), blank_bias=2.0, lm=None,
             lm_weight=0.0, ctx=0, id=0)
    c.update(fields)
    if c["T_min"] is None:
        c["T_min"] = c["T"]
    return c


def _normal(rng, shape, fan_in):
    return (rng.standard_normal(shape) / np.sqrt(fan_in)).astype(np.float32)


def make_weights(c: dict, seed: int | None = None) -> dict:
    """Random-initialised Transducer weights, row-major float32.

    All matrices ~ N(0, 1/fan_in).  The token rows of the output layer are
    scaled by 3 and the blank bias is raised so that the synthetic model emits
    a mix of blanks and tokens; TDT duration rows stay unscaled and their bias
    favours duration 1.  The embedding row of the start-of-sequence symbol
    (row V) is zero.
    """
    if seed is None:
        seed = 1000 * c["id"] + 1
    rng = np.random.default_rng(seed)
    D, H, P, E, V = c["D"], c["H"], c["P"], c["E"], c["V"]
    nd = len(c["durations"])
    w = {}
    w["W_enc"] = _normal(rng, (H, D), D)
    w["b_enc"] = np.zeros(H, np.float32)
    w["W_pred"] = _normal(rng, (H, P), P)
    w["b_pred"] = np.zeros(H, np.float32)
    W_out = _normal(rng, (V + 1 + nd, H), H)
    W_out[: V + 1] *= 3.0
    w["W_out"] = W_out
    b_out = np.zeros(V + 1 + nd, np.float32)
    b_out[V] = c["blank_bias"]
    if nd:
        for i, d in enumerate(c["durations"]):
            if d == 1:
                b_out[V + 1 + i] = 2.0
    w["b_out"] = b_out
    if c["pred"] == "lstm":
        emb = rng.standard_normal((V + 1, E)).astype(np.float32)
        emb[V] = 0.0
        w["emb"] = emb
        w["W_ih"] = _normal(rng, (4 * P, E), E)
        w["W_hh"] = _normal(rng, (4 * P, P), P)
        w["b_ih"] = np.zeros(4 * P, np.float32)
        w["b_hh"] = np.zeros(4 * P, np.float32)
    else:
        emb = rng.standard_normal((c["ctx"], V + 1, P)).astype(np.float32)
        emb /= np.sqrt(c["ctx"])
        emb[:, V] = 0.0
        w["emb"] = emb
    return w


def perturb_biases(w: dict, seed: int, scale: float = 0.1) -> dict:
    """Replace the all-zero biases by small random ones (keeps the blank and
    duration offsets).  The workload recipes have zero biases, which would hide
    a dropped bias term; the small test cases use this variant."""
    rng = np.random.default_rng(seed)
    out = dict(w)
    for k in ("b_enc", "b_pred", "b_out", "b_ih", "b_hh"):
        if k in w:
            out[k] = (w[k] + scale * rng.standard_normal(w[k].shape)).astype(np.float32)
    return out


def make_lengths(c: dict, seed: int | None = None) -> np.ndarray:
    """Frames per utterance: all T, or uniform in [T_min, T]."""
    if seed is None:
        seed = 1000 * c["id"] + 2
    rng = np.random.default_rng(seed)
    if c["T_min"] == c["T"]:
        return np.full(c["B"], c["T"], np.int32)
    return rng.integers(c["T_min"], c["T"] + 1, size=c["B"]).astype(np.int32)


def make_enc(c: dict, lengths: np.ndarray | None = None,
             seed: int | None = None) -> np.ndarray:
    """Encoder output [B, T, D] ~ N(0, 1), zero beyond each utterance's length."""
    if seed is None:
        seed = 1000 * c["id"] + 0
    rng = np.random.default_rng(seed)
    enc = rng.standard_normal((c["B"], c["T"], c["D"])).astype(np.float32)
    if lengths is not None:
        for b, n in enumerate(lengths):
            enc[b, int(n):] = 0.0
    return enc


def audio_seconds(lengths: np.ndarray) -> float:
    return float(np.sum(lengths)) * FRAME_SECONDS


def make_injected(B: int, T: int, C: int, V: int, nd: int, seed: int,
                  levels: int = 640, blank_boost: int = 0):
    """Log-probability tables that replace the joint network in index-parity
    tests: ``tok[b, t, c, v]`` and ``dur[b, t, c, d]`` are negative multiples
    of 2**-6, so that float32 and float64 sums of a few hundred of them are
    exact.  ``blank_boost`` moves the blank column towards 0 by that many
    levels (more blanks, shorter outputs)."""
    rng = np.random.default_rng(seed)
    tok = -(rng.integers(1, levels, size=(B, T, C, V + 1)).astype(np.float32)) / 64.0
    if blank_boost:
        tok[..., V] = np.minimum(tok[..., V] + blank_boost / 64.0, -1.0 / 64.0)
    dur = None
    if nd:
        dur = -(rng.integers(1, 256, size=(B, T, C, nd)).astype(np.float32)) / 64.0
    return tok, dur


def make_lm(V: int, order: int, n_target: int, zipf_s: float, seed: int) -> dict:
    """A synthetic back-off n-gram model in ARPA terms (log10 values).

    All V unigrams are present.  Highest-order n-grams are drawn with tokens
    i.i.d. Zipf(s) over ranks 1..V (token = rank - 1); each is inserted together
    with its prefixes of 2..order-1 tokens, until about ``n_target`` distinct
    n-grams exist.  log10 p ~ U(-6, -0.5); back-off weights ~ U(-1, 0) for every
    order below the highest (0 for the highest).

    Returns ``tokens`` [n, order] int32 (-1 padded on the right), ``order``
    [n] int8, ``log10_prob`` and ``log10_backoff`` [n] float32.
    """
    if order > 1 and n_target > sum(V ** n for n in range(1, order + 1)):
        raise ValueError(f"a vocabulary of {V} tokens has fewer than {n_target} n-grams of orders up to {order}")
    rng = np.random.default_rng(seed)
    ranks = np.arange(1, V + 1, dtype=np.float64)
    pz = ranks ** (-zipf_s)
    pz /= pz.sum()
    bits = int(np.ceil(np.log2(V + 1)))
    assert bits * order <= 60, "packed n-gram key would overflow"

    def pack(tok, n):  # tok [m, order] with first n columns valid
        key = np.full(tok.shape[0], n, np.int64)
        for j in range(order):
            col = tok[:, j].astype(np.int64) + 1 if j < n else np.zeros(tok.shape[0], np.int64)
            key = (key << bits) | col
        return key

    uni = np.full((V, order), -1, np.int32)
    uni[:, 0] = np.arange(V)
    keys = [pack(uni, 1)]
    rows = [uni]
    ords = [np.full(V, 1, np.int8)]
    total = V
    batch = max(1024, n_target // 16)
    known = np.empty(0, np.int64)
    idle = 0
    while total < n_target and order > 1:
        draw = rng.choice(V, size=(batch, order), p=pz).astype(np.int32)
        new_rows, new_keys, new_ords = [], [], []
        for n in range(2, order + 1):
            r = draw.copy()
            r[:, n:] = -1
            new_rows.append(r)
            new_keys.append(pack(r, n))
            new_ords.append(np.full(batch, n, np.int8))
        r = np.concatenate(new_rows)
        k = np.concatenate(new_keys)
        o = np.concatenate(new_ords)
        k_u, first = np.unique(k, return_index=True)
        fresh = ~np.isin(k_u, known)
        sel = first[fresh]
        # keep whole draws together: a kept n-gram's prefixes are kept as well
        known = np.union1d(known, k_u[fresh])
        rows.append(r[sel])
        keys.append(k[sel])
        ords.append(o[sel])
        total += sel.size
        idle = idle + 1 if sel.size == 0 else 0
        if idle >= 200:  # (frequent tokens only: the rare n-grams that are left would take for ever to draw)
            raise ValueError(f"{n_target} distinct n-grams not reached with {V} tokens (stuck at {total})")
    tokens = np.concatenate(rows)
    order_arr = np.concatenate(ords)
    key = np.concatenate(keys)
    perm = np.argsort(key, kind="stable")
    tokens, order_arr = tokens[perm], order_arr[perm]
    n = tokens.shape[0]
    prob = rng.uniform(-6.0, -0.5, size=n).astype(np.float32)
    bo = rng.uniform(-1.0, 0.0, size=n).astype(np.float32)
    bo[order_arr == order] = 0.0
    return dict(tokens=np.ascontiguousarray(tokens), order=order_arr,
                log10_prob=prob, log10_backoff=bo, max_order=order, V=V)
