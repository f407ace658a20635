"""ctypes front-end of the CPU oracle (oracle/wind_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg; never by the product package, with which it shares no code.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Iterable, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wind_oracle.c")
_LIB = os.path.join(_HERE, "libwind_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math: sums stay in index order, in fp64."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


class _Model(C.Structure):
    _fields_ = [
        ("D", C.c_int32), ("E", C.c_int32), ("Hp", C.c_int32), ("L", C.c_int32),
        ("Hj", C.c_int32), ("V", C.c_int32),
        ("emb", C.c_void_p),
        ("w_ih", C.c_void_p * 4), ("w_hh", C.c_void_p * 4),
        ("b_ih", C.c_void_p * 4), ("b_hh", C.c_void_p * 4),
        ("w_enc", C.c_void_p), ("b_enc", C.c_void_p),
        ("w_pred", C.c_void_p), ("b_pred", C.c_void_p),
        ("w_out", C.c_void_p), ("b_out", C.c_void_p),
    ]


class _Eval(C.Structure):
    _fields_ = [
        ("t", C.c_int32), ("u", C.c_int32), ("label", C.c_int32), ("top1", C.c_int32),
        ("top2", C.c_int32), ("v1", C.c_double), ("v2", C.c_double), ("vlabel", C.c_double),
    ]


EVAL_DTYPE = np.dtype(
    {"names": ["t", "u", "label", "top1", "top2", "v1", "v2", "vlabel"],
     "formats": ["<i4", "<i4", "<i4", "<i4", "<i4", "<f8", "<f8", "<f8"],
     "offsets": [_Eval.t.offset, _Eval.u.offset, _Eval.label.offset, _Eval.top1.offset,
                 _Eval.top2.offset, _Eval.v1.offset, _Eval.v2.offset, _Eval.vlabel.offset],
     "itemsize": C.sizeof(_Eval)})

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


class Oracle:
    """Holds one model (fp32 numpy arrays, see wind_inputs.make_weights) for the C oracle."""

    def __init__(self, D: int, E: int, Hp: int, L: int, Hj: int, V: int, weights: Dict[str, np.ndarray]):
        self.D, self.E, self.Hp, self.L, self.Hj, self.V = D, E, Hp, L, Hj, V
        self.w = {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in weights.items()}
        m = _Model()
        m.D, m.E, m.Hp, m.L, m.Hj, m.V = D, E, Hp, L, Hj, V
        w = self.w
        assert w["emb"].shape == (V + 1, E) and w["w_out"].shape == (V + 1, Hj)
        assert w["w_enc"].shape == (Hj, D) and w["w_pred"].shape == (Hj, Hp)
        m.emb = _p(w["emb"])
        for l in range(L):
            assert w[f"w_ih{l}"].shape == (4 * Hp, E if l == 0 else Hp)
            assert w[f"w_hh{l}"].shape == (4 * Hp, Hp)
            m.w_ih[l] = w[f"w_ih{l}"].ctypes.data
            m.w_hh[l] = w[f"w_hh{l}"].ctypes.data
            m.b_ih[l] = w[f"b_ih{l}"].ctypes.data
            m.b_hh[l] = w[f"b_hh{l}"].ctypes.data
        m.w_enc, m.b_enc = _p(w["w_enc"]), _p(w["b_enc"])
        m.w_pred, m.b_pred = _p(w["w_pred"]), _p(w["b_pred"])
        m.w_out, m.b_out = _p(w["w_out"]), _p(w["b_out"])
        self._m = m

    @classmethod
    def from_config(cls, cfg, weights):
        return cls(cfg.D, cfg.E, cfg.Hp, cfg.L, cfg.Hj, cfg.V, weights)

    # ---- model pieces -------------------------------------------------------------------
    def decoder_step(self, token: int, h: np.ndarray, c: np.ndarray) -> None:
        assert h.dtype == np.float64 and c.dtype == np.float64 and h.size == self.L * self.Hp
        lib().oracle_decoder_step(C.byref(self._m), C.c_int(token), _p(h), _p(c))

    def decoder_from_scratch(self, hyp: Iterable[int]) -> np.ndarray:
        hyp = np.ascontiguousarray(list(hyp), dtype=np.int32)
        g = np.zeros(self.Hp, dtype=np.float64)
        lib().oracle_decoder_from_scratch(C.byref(self._m), _p(hyp), C.c_int(hyp.size), _p(g))
        return g

    def joiner(self, frame: np.ndarray, g: np.ndarray) -> np.ndarray:
        frame = np.ascontiguousarray(frame, dtype=np.float32)
        g = np.ascontiguousarray(g, dtype=np.float64)
        assert frame.shape == (self.D,) and g.shape == (self.Hp,)
        out = np.zeros(self.V + 1, dtype=np.float64)
        lib().oracle_joiner(C.byref(self._m), _p(frame), _p(g), _p(out))
        return out

    def encoder_projection(self, frame: np.ndarray) -> np.ndarray:
        """W_enc f + b_enc, the encoder half of the joiner's hidden vector ([Hj], fp64)."""
        frame = np.ascontiguousarray(frame, dtype=np.float32)
        assert frame.shape == (self.D,)
        out = np.zeros(self.Hj, dtype=np.float64)
        lib().oracle_encoder_projection(C.byref(self._m), _p(frame), _p(out))
        return out

    # ---- Algorithm 1 ---------------------------------------------------------------------
    def greedy(self, enc: np.ndarray, S: int, forced: Optional[List[Tuple[int, int, int]]] = None,
               want_log: bool = True):
        """enc [len, D].  Returns (tokens, frames, log) with log a structured array of evaluations."""
        enc = np.ascontiguousarray(enc, dtype=np.float32)
        n = enc.shape[0]
        cap = max(1, n * S)
        tokens = np.zeros(cap, np.int32)
        frames = np.zeros(cap, np.int32)
        count = C.c_int32(0)
        f = np.ascontiguousarray(forced if forced else np.zeros((0, 3)), dtype=np.int32).reshape(-1, 3)
        log_cap = n * (S + 1) + 1
        log = np.zeros(log_cap if want_log else 1, dtype=EVAL_DTYPE)
        n_log = C.c_int32(0)
        rc = lib().oracle_greedy(C.byref(self._m), _p(enc), C.c_int(n), C.c_int(S), _p(f), C.c_int(f.shape[0]),
                                 _p(tokens), _p(frames), C.c_int(cap), C.byref(count),
                                 _p(log) if want_log else None, C.c_int(log_cap), C.byref(n_log))
        assert rc == 0
        k = count.value
        return tokens[:k].copy(), frames[:k].copy(), log[: n_log.value].copy()

    def greedy_batch(self, enc: np.ndarray, lengths: np.ndarray, S: int,
                     forced: Optional[List[Tuple[int, int, int, int]]] = None,
                     want_log: bool = False, threads: int = 0):
        """enc [B,T,D].  Returns (list of tokens, list of frames, list of logs or None)."""
        enc = np.ascontiguousarray(enc, dtype=np.float32)
        lengths = np.ascontiguousarray(lengths, dtype=np.int32)
        B, T, D = enc.shape
        assert D == self.D and lengths.shape == (B,) and (B == 0 or int(lengths.max()) <= T)
        cap = max(1, T * S)
        tokens = np.zeros((B, cap), np.int32)
        frames = np.zeros((B, cap), np.int32)
        counts = np.zeros(B, np.int32)
        f = np.ascontiguousarray(forced if forced else np.zeros((0, 4)), dtype=np.int32).reshape(-1, 4)
        log_cap = T * (S + 1) + 1
        log = np.zeros((B, log_cap) if want_log else (1, 1), dtype=EVAL_DTYPE)
        n_log = np.zeros(B, np.int32)
        bad = lib().oracle_greedy_batch(C.byref(self._m), _p(enc), _p(lengths), C.c_int(B), C.c_int(T), C.c_int(S),
                                        _p(f), C.c_int(f.shape[0]), _p(tokens), _p(frames), C.c_int(cap),
                                        _p(counts), _p(log) if want_log else None, C.c_int(log_cap),
                                        _p(n_log), C.c_int(threads))
        assert bad == 0
        toks = [tokens[b, : counts[b]].copy() for b in range(B)]
        frs = [frames[b, : counts[b]].copy() for b in range(B)]
        logs = [log[b, : n_log[b]].copy() for b in range(B)] if want_log else None
        return toks, frs, logs

    # ---- Algorithm 2 ---------------------------------------------------------------------
    def wind(self, enc: np.ndarray, W: int, S: int):
        """enc [len, D].  Returns (tokens, frames, calls [n,2] = (t, n), jump histogram [W+1])."""
        enc = np.ascontiguousarray(enc, dtype=np.float32)
        n = enc.shape[0]
        cap = max(1, n * S)
        tokens = np.zeros(cap, np.int32)
        frames = np.zeros(cap, np.int32)
        count = C.c_int32(0)
        calls_cap = n * (S + 1) + 1
        calls = np.zeros((calls_cap, 2), np.int32)
        n_calls = C.c_int32(0)
        hist = np.zeros(W + 1, np.int64)
        rc = lib().oracle_wind(C.byref(self._m), _p(enc), C.c_int(n), C.c_int(W), C.c_int(S),
                               _p(tokens), _p(frames), C.c_int(cap), C.byref(count),
                               _p(calls), C.c_int(calls_cap), C.byref(n_calls), _p(hist))
        assert rc == 0
        k = count.value
        return tokens[:k].copy(), frames[:k].copy(), calls[: n_calls.value].copy(), hist


def num_threads() -> int:
    return int(lib().oracle_num_threads())
