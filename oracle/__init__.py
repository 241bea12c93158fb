"""ctypes front end of the CPU oracle (``rnnt_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
CPU-baseline leg of the benchmark, never by the HIP library or its binding.
Argument marshalling only; every number comes out of the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rnnt_oracle.c")
_LIB = os.path.join(_HERE, "librnnt_oracle.so")

ALSD, AES = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over utterances)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Config(C.Structure):
    _fields_ = [("model", C.c_int32), ("pred", C.c_int32), ("prec", C.c_int32),
                ("D", C.c_int32), ("H", C.c_int32), ("P", C.c_int32), ("E", C.c_int32), ("V", C.c_int32),
                ("n_dur", C.c_int32), ("durations", C.c_int32 * 8), ("ctx", C.c_int32),
                ("max_symbols", C.c_int32), ("lm_rule", C.c_int32), ("lm_prune", C.c_int32), ("tdt_pairs", C.c_int32), ("aes_prefix", C.c_int32),
                ("gamma", C.c_double)]


_WNAMES = ["W_enc", "b_enc", "W_pred", "b_pred", "W_out", "b_out", "emb", "W_ih", "W_hh", "b_ih", "b_hh"]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WNAMES]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # RNNT_ORACLE_LIB: a separately compiled copy (the planted-mistake tests use it)
        _lib = C.CDLL(os.environ.get("RNNT_ORACLE_LIB") or build())
        _lib.orc_lm_create.restype = C.c_void_p
        _lib.orc_hash_tokens.restype = C.c_uint32
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def make_config(c: dict, lm_rule: int = 4, lm_prune: str = "late") -> _Config:
    cfg = _Config()
    cfg.model = 1 if c["model"] == "tdt" else 0
    cfg.pred = 1 if c["pred"] == "stateless" else 0
    cfg.prec = 1 if c["prec"] == "bf16" else 0
    cfg.D, cfg.H, cfg.P, cfg.E, cfg.V = c["D"], c["H"], c["P"], c["E"], c["V"]
    cfg.n_dur = len(c["durations"])
    for i, d in enumerate(c["durations"]):
        cfg.durations[i] = d
    cfg.ctx = c["ctx"]
    cfg.max_symbols = c["s"]
    cfg.lm_rule = lm_rule
    cfg.lm_prune = {"late": 0, "early": 1}[lm_prune]
    cfg.tdt_pairs = 1 if c.get("tdt_pairs") else 0
    cfg.aes_prefix = 1 if c.get("aes_prefix") else 0
    cfg.gamma = c["gamma"]
    return cfg


class Weights:
    """Keeps the float32 arrays alive next to the pointer struct."""

    def __init__(self, w: dict):
        self.arrays = {k: _f32(v) for k, v in w.items()}
        self.struct = _Weights()
        for n in _WNAMES:
            setattr(self.struct, n, _ptr(self.arrays.get(n)))


class LM:
    def __init__(self, lm: dict):
        self.order = int(lm["max_order"])
        toks = _i32(lm["tokens"])
        self.handle = C.c_void_p(lib().orc_lm_create(
            C.c_int(self.order), C.c_int64(toks.shape[0]), _ptr(toks),
            _ptr(np.ascontiguousarray(lm["order"], dtype=np.int8)),
            _ptr(_f32(lm["log10_prob"])), _ptr(_f32(lm["log10_backoff"]))))

    def query(self, tokens, V: int) -> np.ndarray:
        """Natural-log LM score of every token after the transcript ``tokens``."""
        t = _i32(np.asarray(tokens, dtype=np.int32).reshape(-1))
        out = np.empty(V, np.float64)
        lib().orc_lm_query(self.handle, _ptr(t), C.c_int(t.size), C.c_int(V), _ptr(out))
        return out

    def __del__(self):
        try:
            lib().orc_lm_destroy(self.handle)
        except Exception:
            pass


def decode(c: dict, w: dict | None, enc, lengths, beam=None, algo=None, lm: LM | None = None,
           lm_weight: float = 0.0, lm_rule: int = 4, injected=None, log=False, snap_every=0, lm_prune: str = "late",
           n_threads=0) -> dict:
    """Run the oracle on a batch.  ``injected`` = (tok_logp [B,T,C,V+1], dur_logp or None)."""
    L = lib()
    cfg = make_config(c, lm_rule, lm_prune)
    beam = c["beam"] if beam is None else beam
    algo = (AES if c["algo"] == "aes" else ALSD) if algo is None else algo
    lengths = _i32(lengths)
    B = lengths.shape[0]
    V, s = c["V"], c["s"]
    W = Weights(w) if w is not None else Weights({})
    if injected is not None:
        tok, dur = injected
        tok = _f32(tok)
        dur = _f32(dur) if dur is not None else None
        T, Cc = tok.shape[1], tok.shape[2]
        enc_a = None
    else:
        enc_a = _f32(enc)
        T = enc_a.shape[1]
        tok = dur = None
        Cc = 1
    Tmax = int(lengths.max()) if B else 0
    assert Tmax <= T
    cap = Tmax * max(s, 1) + 1
    S_cap = Tmax * (s + 1) + 1
    tokens = np.full((B, beam, cap), -1, np.int32)
    lens = np.zeros((B, beam), np.int32)
    scores = np.zeros((B, beam), np.float64)
    n_steps = np.zeros(B, np.int32)
    lp = lt = lm_ = lg = None
    if log:
        lp = np.full((B, S_cap, beam), -9, np.int32)
        lt = np.full((B, S_cap, beam), -9, np.int32)
        lm_ = np.full((B, S_cap, beam), -9, np.int32)
        lg = np.full((B, S_cap), np.inf, np.float64)
    st = sl = None
    n_snap = 0
    if snap_every:
        n_snap = S_cap // snap_every + 1
        st = np.full((B, n_snap, beam, cap), -1, np.int32)
        sl = np.full((B, n_snap, beam), -9, np.int32)
    min_gap = np.zeros(B, np.float64)
    coll = np.zeros(B, np.int64)
    n_cut = np.zeros(B, np.int64)
    max_logp = np.zeros(B, np.float64)
    used = L.orc_decode(C.byref(cfg), C.byref(W.struct), _ptr(enc_a), _ptr(lengths), C.c_int(B), C.c_int(T),
                        C.c_int(beam), C.c_int(algo), lm.handle if lm is not None else None,
                        C.c_double(lm_weight), _ptr(tok), _ptr(dur), C.c_int(Cc), _ptr(tokens), C.c_int(cap),
                        _ptr(lens), _ptr(scores), _ptr(n_steps), _ptr(lp), _ptr(lt), _ptr(lm_), _ptr(lg), C.c_int(S_cap),
                        _ptr(st), _ptr(sl), C.c_int(snap_every), C.c_int(n_snap), _ptr(min_gap), _ptr(coll),
                        _ptr(n_cut), _ptr(max_logp), C.c_int(n_threads))
    return dict(tokens=tokens, lens=lens, scores=scores, n_steps=n_steps, log_parent=lp, log_token=lt,
                log_merged=lm_, log_gap=lg, snap_tokens=st, snap_lens=sl, min_gap=min_gap, collisions=coll, n_cut=n_cut,
                max_logp=max_logp, threads=used, cap=cap)


# ---- unit-level entry points (for the pins) ---------------------------------

def enc_proj(c, w, enc_t, rounded=False):
    """``rounded``: the joint's weight matrices in ``w`` have been rounded to bf16 already (same result, faster)."""
    cfg, W = make_config(c), Weights(w)
    out = np.empty(c["H"], np.float64)
    fn = lib().orc_enc_proj_rounded if rounded else lib().orc_enc_proj
    fn(C.byref(cfg), C.byref(W.struct), _ptr(_f32(enc_t)), _ptr(out))
    return out


def lstm_step(c, w, h, cc, token):
    cfg, W = make_config(c), Weights(w)
    h2, c2 = np.empty(c["P"], np.float64), np.empty(c["P"], np.float64)
    lib().orc_lstm_step(C.byref(cfg), C.byref(W.struct), _ptr(_f64(h)), _ptr(_f64(cc)), C.c_int(int(token)),
                        _ptr(h2), _ptr(c2))
    return h2, c2


def pred_proj(c, w, h, rounded=False):
    cfg, W = make_config(c), Weights(w)
    out = np.empty(c["H"], np.float64)
    fn = lib().orc_pred_proj_rounded if rounded else lib().orc_pred_proj
    fn(C.byref(cfg), C.byref(W.struct), _ptr(_f64(h)), _ptr(out))
    return out


def stateless_pred(c, w, tokens, rounded=False):
    cfg, W = make_config(c), Weights(w)
    t = _i32(np.asarray(tokens, dtype=np.int32).reshape(-1))
    out = np.empty(c["H"], np.float64)
    fn = lib().orc_stateless_pred_rounded if rounded else lib().orc_stateless_pred
    fn(C.byref(cfg), C.byref(W.struct), _ptr(t), C.c_int(t.size), _ptr(out))
    return out


def joint(c, w, f, g, rounded=False):
    cfg, W = make_config(c), Weights(w)
    out = np.empty(c["V"] + 1 + len(c["durations"]), np.float64)
    fn = lib().orc_joint_rounded if rounded else lib().orc_joint
    fn(C.byref(cfg), C.byref(W.struct), _ptr(_f64(f)), _ptr(_f64(g)), _ptr(out))
    return out


def score_row(c, z=None, logp=None, dlogp=None, lm_row=None, lm_weight=0.0, lm_rule=4, apply_gamma=False,
              forced_blank=False):
    """Per-hypothesis candidate scores; returns (tot [V+1], logp [V+1], adv_tok, adv_blank)."""
    cfg = make_config(c, lm_rule)
    V = c["V"]
    tot, lp = np.empty(V + 1, np.float64), np.empty(V + 1, np.float64)
    a1, a2 = C.c_int(0), C.c_int(0)
    z_a = _f64(z) if z is not None else None
    lp_in = _f64(logp) if logp is not None else None
    dl_in = _f64(dlogp) if dlogp is not None else None
    lm_a = _f64(lm_row) if lm_row is not None else None
    lib().orc_score_row(C.byref(cfg), _ptr(z_a), _ptr(lp_in), _ptr(dl_in), _ptr(lm_a), C.c_double(lm_weight),
                        C.c_int(int(apply_gamma)), C.c_int(int(forced_blank)), _ptr(tot), _ptr(lp),
                        C.byref(a1), C.byref(a2), None, None)
    return tot, lp, a1.value, a2.value


def topk(values, K):
    v = _f64(values).reshape(-1)
    out = np.empty(K, np.int64)
    lib().orc_topk(_ptr(v), C.c_int64(v.size), C.c_int(K), _ptr(out))
    return out


def hash_tokens(tokens) -> int:
    t = _i32(np.asarray(tokens, dtype=np.int32).reshape(-1))
    return int(lib().orc_hash_tokens(_ptr(t), C.c_int(t.size)))
