"""ctypes binding of the rnnt_beam C ABI.  Same names as the C entry points;
argument marshalling only."""
from __future__ import annotations

import ctypes as C
import math
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librnnt_beam.so")

ALSD, AES = 0, 1

EXPORTS = ["rnnt_beam_create", "rnnt_lm_create", "rnnt_beam_decode", "rnnt_beam_results",
           "rnnt_beam_decode_injected", "rnnt_beam_dump_tree", "rnnt_beam_debug_encproj", "rnnt_lm_debug_query",
           "rnnt_beam_last_decode_ms", "rnnt_beam_set_profiling", "rnnt_beam_kernel_times", "rnnt_beam_last_error",
           "rnnt_beam_destroy", "rnnt_lm_destroy", "rnnt_beam_debug_block_map", "rnnt_beam_decode_static", "rnnt_beam_debug_set_spin_limit"]


class RnntBeamError(RuntimeError):
    pass


def block_map(a_tiles, a_m, b_begin, b_end, b_m):
    """Host logic, no GPU: (grid, role[], ntile[], mtile[]) of the per-step launches' block -> item mapping."""
    lib = load_library()
    n = lib.rnnt_beam_debug_block_map(a_tiles, a_m, b_begin, b_end, b_m, None, None, None, 0)
    if n < 0:
        raise RnntBeamError(f"rnnt_beam_debug_block_map: {n}")
    role, nt, mt = (np.full(n, -7, np.int32) for _ in range(3))
    lib.rnnt_beam_debug_block_map(a_tiles, a_m, b_begin, b_end, b_m, role.ctypes.data_as(C.c_void_p),
                                  nt.ctypes.data_as(C.c_void_p), mt.ctypes.data_as(C.c_void_p), n)
    return n, role, nt, mt


class _Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("model", C.c_int32), ("pred", C.c_int32), ("prec", C.c_int32),
                ("D", C.c_int32), ("H", C.c_int32), ("P", C.c_int32), ("E", C.c_int32), ("V", C.c_int32),
                ("n_durations", C.c_int32), ("durations", C.c_int32 * 8), ("stateless_context", C.c_int32),
                ("max_B", C.c_int32), ("max_T", C.c_int32), ("max_beam", C.c_int32), ("max_symbols", C.c_int32),
                ("prune_margin", C.c_float), ("use_graph", C.c_int32), ("joint_path", C.c_int32),
                ("lm_rule", C.c_int32), ("lm_early_pruning", C.c_int32), ("tdt_all_pairs", C.c_int32),
                ("async_enqueue", C.c_int32), ("aes_prefix_search", C.c_int32),
                ("persistent_kernel", C.c_int32)]


_WNAMES = ["W_enc", "b_enc", "W_pred", "b_pred", "W_out", "b_out", "emb", "W_ih", "W_hh", "b_ih", "b_hh"]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WNAMES]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RnntBeamError(f"{_LIB_PATH} is missing: build it with `python -m paper_2506_00185_amd.build` "
                                "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime (same soname as the system one).  It must be in the
        # process first, so that this library binds to it instead of starting a second runtime,
        # which would not see the GPU.
        import torch  # noqa: F401
        lib = C.CDLL(_LIB_PATH)
        lib.rnnt_beam_last_error.restype = C.c_char_p
        lib.rnnt_beam_last_error.argtypes = [C.c_void_p]
        lib.rnnt_beam_last_decode_ms.restype = C.c_float
        lib.rnnt_beam_last_decode_ms.argtypes = [C.c_void_p]
        lib.rnnt_beam_destroy.argtypes = [C.c_void_p]
        lib.rnnt_lm_destroy.argtypes = [C.c_void_p]
        _lib = lib
    return _lib


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RnntBeamError("no GPU visible: the rnnt_beam library runs on an MI355X only")
    return torch


def _check(rc, handle=None):
    if rc < 0:
        msg = load_library().rnnt_beam_last_error(handle)
        raise RnntBeamError(f"rnnt_beam error {rc}: {msg.decode() if msg else ''}")
    return rc


class NGramLM:
    """rnnt_lm_create / rnnt_lm_destroy."""

    def __init__(self, lm: dict):
        lib = load_library()
        _torch()
        toks = np.ascontiguousarray(lm["tokens"], dtype=np.int32)
        order = np.ascontiguousarray(lm["order"], dtype=np.int8)
        prob = np.ascontiguousarray(lm["log10_prob"], dtype=np.float32)
        bo = np.ascontiguousarray(lm["log10_backoff"], dtype=np.float32)
        self.V = int(lm["V"])
        self.order = int(lm["max_order"])
        self.handle = C.c_void_p()
        rc = lib.rnnt_lm_create(C.c_int32(self.order), C.c_int64(toks.shape[0]), toks.ctypes.data_as(C.c_void_p),
                                order.ctypes.data_as(C.c_void_p), prob.ctypes.data_as(C.c_void_p),
                                bo.ctypes.data_as(C.c_void_p), C.c_int32(self.V), C.byref(self.handle))
        if rc < 0:
            raise RnntBeamError(f"rnnt_lm_create failed with {rc}")

    def debug_query(self, ctx_tokens) -> np.ndarray:
        """rnnt_lm_debug_query: ctx_tokens [n, order-1], most recent first, -1 = none."""
        ctx = np.ascontiguousarray(ctx_tokens, dtype=np.int32).reshape(-1, max(self.order - 1, 1))
        out = np.empty((ctx.shape[0], self.V), np.float32)
        rc = load_library().rnnt_lm_debug_query(self.handle, ctx.ctypes.data_as(C.c_void_p), C.c_int32(ctx.shape[0]),
                                                out.ctypes.data_as(C.c_void_p))
        if rc < 0:
            raise RnntBeamError(f"rnnt_lm_debug_query failed with {rc}")
        return out

    def __del__(self):
        try:
            if self.handle:
                load_library().rnnt_lm_destroy(self.handle)
        except Exception:
            pass


class BeamDecoder:
    """rnnt_beam_create / decode / results / destroy for one model."""

    def __init__(self, c: dict, w: dict, max_B=None, max_T=None, max_beam=None, use_graph=True, device="cuda:0",
                 joint_path="auto", lm_rule=4, lm_prune="late", async_enqueue=False, persistent=False):
        lib = load_library()
        torch = _torch()
        self.device = torch.device(device)
        self.c = dict(c)
        cfg = _Config()
        cfg.struct_size = C.sizeof(_Config)
        cfg.model = 1 if c["model"] == "tdt" else 0
        cfg.pred = 1 if c["pred"] == "stateless" else 0
        cfg.prec = 1 if c["prec"] == "bf16" else 0
        cfg.D, cfg.H, cfg.P, cfg.E, cfg.V = c["D"], c["H"], c["P"], c["E"], c["V"]
        cfg.n_durations = len(c["durations"])
        for i, d in enumerate(c["durations"]):
            cfg.durations[i] = d
        cfg.stateless_context = c["ctx"]
        cfg.max_B = max_B or c["B"]
        cfg.max_T = max_T or c["T"]
        cfg.max_beam = max_beam or c["beam"]
        cfg.max_symbols = c["s"]
        cfg.prune_margin = c["gamma"] if math.isfinite(c["gamma"]) else float("inf")
        cfg.use_graph = 1 if use_graph else 0
        cfg.joint_path = {"auto": 0, "fused": 1, "materialized": 2}[joint_path]
        cfg.lm_rule = lm_rule
        cfg.lm_early_pruning = {"late": 0, "early": 1}[lm_prune]
        cfg.tdt_all_pairs = 1 if c.get("tdt_pairs") else 0
        cfg.async_enqueue = 1 if async_enqueue else 0
        cfg.aes_prefix_search = 1 if c.get("aes_prefix") else 0
        cfg.persistent_kernel = 1 if persistent else 0
        self.cfg = cfg
        self._w = {k: torch.as_tensor(np.ascontiguousarray(v, dtype=np.float32)).to(self.device)
                   for k, v in w.items()}
        ws = _Weights()
        for n in _WNAMES:
            setattr(ws, n, self._w[n].data_ptr() if n in self._w else None)
        self.handle = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = lib.rnnt_beam_create(C.byref(cfg), C.byref(ws), C.byref(self.handle))
        if rc < 0:
            msg = lib.rnnt_beam_last_error(None)
            raise RnntBeamError(f"rnnt_beam_create failed with {rc}: {msg.decode() if msg else ''}")
        self._w = None  # the library re-packed them
        self._keep = None
        self._shape = None

    # -- rnnt_beam_decode ----------------------------------------------------
    def decode(self, enc, lengths, beam=None, algo=None, lm: NGramLM | None = None, lm_weight=0.0, stream=None):
        """enc: CUDA float32 tensor [B, T, D]; lengths: CUDA int32 tensor [B]."""
        torch = _torch()
        assert enc.is_cuda and enc.dtype == torch.float32 and enc.is_contiguous()
        assert lengths.is_cuda and lengths.dtype == torch.int32 and lengths.is_contiguous()
        B, T, D = enc.shape
        assert D == self.c["D"] and lengths.shape[0] == B
        beam = self.c["beam"] if beam is None else beam
        algo = (AES if self.c["algo"] == "aes" else ALSD) if algo is None else algo
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._keep = (enc, lengths, lm)
        self._shape = (B, beam)
        rc = load_library().rnnt_beam_decode(self.handle, C.c_void_p(enc.data_ptr()), C.c_void_p(lengths.data_ptr()),
                                             C.c_int32(B), C.c_int32(T), C.c_int32(beam), C.c_int32(algo),
                                             lm.handle if lm is not None else None, C.c_float(lm_weight),
                                             C.c_void_p(s.cuda_stream))
        _check(rc, self.handle)

    # -- rnnt_beam_decode_static ---------------------------------------------
    def decode_static(self, enc, lengths, tokens, lens, scores, n_steps, flags=None, beam=None, algo=None,
                      lm: NGramLM | None = None, lm_weight=0.0, stream=None):
        """All arrays are CUDA tensors owned by the caller: tokens int32 [B, beam, cap], lens int32 [B, beam],
        scores float64 [B, beam], n_steps int32 [B], flags int32 [2] or None.  Returns without waiting."""
        torch = _torch()
        assert enc.is_cuda and enc.dtype == torch.float32 and enc.is_contiguous()
        assert lengths.is_cuda and lengths.dtype == torch.int32 and lengths.is_contiguous()
        B, T, D = enc.shape
        beam = self.c["beam"] if beam is None else beam
        algo = (AES if self.c["algo"] == "aes" else ALSD) if algo is None else algo
        assert tokens.is_cuda and tokens.dtype == torch.int32 and tokens.is_contiguous() and tokens.shape[:2] == (B, beam)
        assert lens.is_cuda and lens.dtype == torch.int32 and lens.is_contiguous() and lens.shape == (B, beam)
        assert scores.is_cuda and scores.dtype == torch.float64 and scores.is_contiguous() and scores.shape == (B, beam)
        assert n_steps.is_cuda and n_steps.dtype == torch.int32 and n_steps.shape == (B,)
        assert flags is None or (flags.is_cuda and flags.dtype == torch.int32 and flags.numel() >= 2)
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._keep = (enc, lengths, lm, tokens, lens, scores, n_steps, flags)
        rc = load_library().rnnt_beam_decode_static(
            self.handle, C.c_void_p(enc.data_ptr()), C.c_void_p(lengths.data_ptr()), C.c_int32(B), C.c_int32(T),
            C.c_int32(beam), C.c_int32(algo), lm.handle if lm is not None else None, C.c_float(lm_weight),
            C.c_void_p(tokens.data_ptr()), C.c_int32(tokens.shape[2]), C.c_void_p(lens.data_ptr()),
            C.c_void_p(scores.data_ptr()), C.c_void_p(n_steps.data_ptr()),
            C.c_void_p(flags.data_ptr()) if flags is not None else None, C.c_void_p(s.cuda_stream))
        _check(rc, self.handle)

    def decode_injected(self, tok_logp, dur_logp, lengths, beam=None, algo=None, stream=None):
        torch = _torch()
        assert tok_logp.is_cuda and tok_logp.dtype == torch.float32 and tok_logp.is_contiguous()
        B, T, Cc, V1 = tok_logp.shape
        assert V1 == self.c["V"] + 1
        beam = self.c["beam"] if beam is None else beam
        algo = (AES if self.c["algo"] == "aes" else ALSD) if algo is None else algo
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        self._keep = (tok_logp, dur_logp, lengths)
        self._shape = (B, beam)
        rc = load_library().rnnt_beam_decode_injected(
            self.handle, C.c_void_p(tok_logp.data_ptr()),
            C.c_void_p(dur_logp.data_ptr()) if dur_logp is not None else None, C.c_int32(Cc),
            C.c_void_p(lengths.data_ptr()), C.c_int32(B), C.c_int32(T), C.c_int32(beam), C.c_int32(algo),
            C.c_void_p(s.cuda_stream))
        _check(rc, self.handle)

    # -- rnnt_beam_results ---------------------------------------------------
    def results(self, cap=None, check=True) -> dict:
        B, K = self._shape
        cap = cap or (self.cfg.max_T * self.cfg.max_symbols + 1)
        tokens = np.full((B, K, cap), -1, np.int32)
        lens = np.zeros((B, K), np.int32)
        scores = np.zeros((B, K), np.float64)
        steps = np.zeros(B, np.int32)
        rc = load_library().rnnt_beam_results(self.handle, tokens.ctypes.data_as(C.c_void_p), C.c_int32(cap),
                                              lens.ctypes.data_as(C.c_void_p), scores.ctypes.data_as(C.c_void_p),
                                              steps.ctypes.data_as(C.c_void_p))
        if check:
            _check(rc, self.handle)
        return dict(tokens=tokens, lens=lens, scores=scores, n_steps=steps, rc=rc)

    def dump_tree(self, s_cap) -> dict:
        B, K = self._shape
        arrs = [np.empty((s_cap, B, K), np.int32) for _ in range(3)]
        rc = load_library().rnnt_beam_dump_tree(self.handle, *[a.ctypes.data_as(C.c_void_p) for a in arrs],
                                                C.c_int32(s_cap))
        _check(rc, self.handle)
        return dict(parent=arrs[0], token=arrs[1], merged=arrs[2])

    def debug_encproj(self, B, T) -> np.ndarray:
        out = np.empty((B * T, self.c["H"]), np.float32)
        rc = load_library().rnnt_beam_debug_encproj(self.handle, out.ctypes.data_as(C.c_void_p), C.c_int64(out.size))
        _check(rc, self.handle)
        return out

    def debug_set_spin_limit(self, polls: int):
        _check(load_library().rnnt_beam_debug_set_spin_limit(self.handle, C.c_int32(polls)), self.handle)

    def last_decode_ms(self) -> float:
        return float(load_library().rnnt_beam_last_decode_ms(self.handle))

    def set_profiling(self, on: bool):
        _check(load_library().rnnt_beam_set_profiling(self.handle, C.c_int32(1 if on else 0)), self.handle)

    def kernel_times(self) -> dict:
        n_cap = 16
        names = (C.c_char_p * n_cap)()
        ms = (C.c_float * n_cap)()
        calls = (C.c_int32 * n_cap)()
        n = load_library().rnnt_beam_kernel_times(self.handle, names, ms, calls, C.c_int32(n_cap))
        _check(n, self.handle)
        return {names[i].decode(): (float(ms[i]), int(calls[i])) for i in range(n)}

    def close(self):
        if getattr(self, "handle", None):
            load_library().rnnt_beam_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
