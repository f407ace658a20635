"""ctypes binding of include/wind.h.  Argument marshalling only: every step of decoding runs in
the HIP kernels of libwind.so.  torch supplies device memory and the stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
WIND_MAX_LAYERS = 4
WIND_MAX_WINDOW = 64
WIND_F32, WIND_BF16 = 0, 1
WIND_OK, WIND_ERR_ARG, WIND_ERR_HIP, WIND_ERR_OVERFLOW, WIND_ERR_UNSUPPORTED, WIND_ERR_UNFINISHED = 0, -1, -2, -3, -4, -5

EXPORTS = ("wind_load_weights", "wind_free", "wind_greedy_decode", "wind_sequential_decode",
           "wind_greedy_decode_async", "wind_get_stats", "wind_debug_joint_logits", "wind_set_option", "wind_last_error",
           "wind_get_kernel_times", "wind_get_joint_launches", "wind_get_call_times", "wind_beam_window_scores", "wind_beam_decode",
           "wind_workspace_bytes", "wind_debug_enc_proj", "wind_debug_joint_keys", "wind_beam_window_scores_static",
           "wind_get_loop_info")
PREFIX_MODES = {"off": 0, "keep": 1, "remove": 2}
KERNEL_NAMES = ("enc_proj", "build_z", "joint", "decide", "lstm", "pred_proj")


class WindError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"wind error {code}: {msg}")
        self.code = code


class _Weights(C.Structure):
    _fields_ = [
        ("D", C.c_int32), ("E", C.c_int32), ("Hp", C.c_int32), ("L", C.c_int32), ("Hj", C.c_int32),
        ("V", C.c_int32), ("dtype", C.c_int32),
        ("emb", C.c_void_p),
        ("w_ih", C.c_void_p * WIND_MAX_LAYERS), ("w_hh", C.c_void_p * WIND_MAX_LAYERS),
        ("b_ih", C.c_void_p * WIND_MAX_LAYERS), ("b_hh", C.c_void_p * WIND_MAX_LAYERS),
        ("w_enc", C.c_void_p), ("b_enc", C.c_void_p), ("w_pred", C.c_void_p), ("b_pred", C.c_void_p),
        ("w_out", C.c_void_p), ("b_out", C.c_void_p),
    ]


class WindStats(C.Structure):
    _fields_ = [
        ("iterations", C.c_int64), ("windows", C.c_int64), ("rows", C.c_int64), ("useful_rows", C.c_int64),
        ("labels", C.c_int64), ("forced_advances", C.c_int64), ("rechecks", C.c_int64),
        ("jump_hist", C.c_int64 * (WIND_MAX_WINDOW + 1)),
    ]


class WindBeamStats(C.Structure):
    _fields_ = [
        ("rounds", C.c_int64), ("hyps_scored", C.c_int64), ("decoder_steps", C.c_int64), ("completions", C.c_int64),
        ("completion_rows", C.c_int64), ("max_pending", C.c_int64), ("nodes", C.c_int64),
    ]


_I32P = C.POINTER(C.c_int32)
BEAM_ROUND_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_int, C.c_int, C.c_int, _I32P, _I32P, _I32P, C.POINTER(C.c_double), _I32P,
                            C.c_int, _I32P, _I32P, C.POINTER(C.c_float))


def lib_path() -> str:
    return os.path.join(_HERE, "libwind.so")


_lib = None


def load_library():
    """Loads libwind.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} is missing: run `python -m paper_2505_13765_amd.build` first")
        lib = C.CDLL(path)
        lib.wind_last_error.restype = C.c_char_p
        lib.wind_load_weights.argtypes = [C.POINTER(_Weights), C.c_void_p, C.POINTER(C.c_void_p)]
        lib.wind_free.argtypes = [C.c_void_p]
        lib.wind_greedy_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        lib.wind_sequential_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        lib.wind_greedy_decode_async.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t,
                                                 C.c_int64, C.c_void_p]
        lib.wind_get_stats.argtypes = [C.c_void_p, C.POINTER(WindStats)]
        lib.wind_debug_joint_logits.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        lib.wind_set_option.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
        lib.wind_get_kernel_times.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        lib.wind_debug_enc_proj.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        lib.wind_debug_joint_keys.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                              C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_void_p]
        lib.wind_get_call_times.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        lib.wind_get_loop_info.argtypes = [C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        lib.wind_get_joint_launches.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_int,
                                                C.POINTER(C.c_int)]
        lib.wind_beam_window_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.wind_beam_window_scores_static.argtypes = lib.wind_beam_window_scores.argtypes
        lib.wind_workspace_bytes.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
        lib.wind_beam_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                         C.c_void_p, C.c_void_p, C.c_int, _I32P, C.POINTER(C.c_double),
                                         C.POINTER(WindBeamStats), C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = lib
    return _lib


def _check(rc: int, allow_overflow: bool = False) -> int:
    if rc == WIND_OK or (allow_overflow and rc == WIND_ERR_OVERFLOW):
        return rc
    raise WindError(rc, load_library().wind_last_error().decode())


def _stream_ptr() -> int:
    import torch

    return int(torch.cuda.current_stream().cuda_stream)


class WindModel:
    """Owns a wind_model handle.  `weights` are fp32 numpy arrays named as in wind_inputs.make_weights."""

    def __init__(self, D: int, E: int, Hp: int, L: int, Hj: int, V: int, dtype: str,
                 weights: Dict[str, np.ndarray]):
        self._lib = load_library()
        self.D, self.E, self.Hp, self.L, self.Hj, self.V = D, E, Hp, L, Hj, V
        w = {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in weights.items()}
        ws = _Weights()
        ws.D, ws.E, ws.Hp, ws.L, ws.Hj, ws.V = D, E, Hp, L, Hj, V
        ws.dtype = {"f32": WIND_F32, "bf16": WIND_BF16}[dtype]
        ws.emb = w["emb"].ctypes.data
        for l in range(min(L, WIND_MAX_LAYERS)):
            ws.w_ih[l] = w[f"w_ih{l}"].ctypes.data
            ws.w_hh[l] = w[f"w_hh{l}"].ctypes.data
            ws.b_ih[l] = w[f"b_ih{l}"].ctypes.data
            ws.b_hh[l] = w[f"b_hh{l}"].ctypes.data
        ws.w_enc, ws.b_enc = w["w_enc"].ctypes.data, w["b_enc"].ctypes.data
        ws.w_pred, ws.b_pred = w["w_pred"].ctypes.data, w["b_pred"].ctypes.data
        ws.w_out, ws.b_out = w["w_out"].ctypes.data, w["b_out"].ctypes.data
        h = C.c_void_p()
        _check(self._lib.wind_load_weights(C.byref(ws), _stream_ptr(), C.byref(h)))
        self._h = h

    @classmethod
    def from_config(cls, cfg, weights):
        return cls(cfg.D, cfg.E, cfg.Hp, cfg.L, cfg.Hj, cfg.V, cfg.dtype, weights)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.wind_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, key: str, value: int) -> None:
        _check(self._lib.wind_set_option(self._h, key.encode(), int(value)))

    def greedy_decode(self, enc_out, lengths, W: Optional[int], S: int, out_tokens, out_frames, out_counts,
                      allow_overflow: bool = False) -> int:
        """enc_out [B,T,D] float32 cuda, lengths [B] int32 cuda, outputs [B,cap] / [B] int32 cuda.
        W=None calls wind_sequential_decode."""
        B, T, D = enc_out.shape
        assert D == self.D and enc_out.is_contiguous() and lengths.is_contiguous()
        cap = out_tokens.shape[1]
        args = (self._h, enc_out.data_ptr(), lengths.data_ptr(), B, T)
        tail = (S, out_tokens.data_ptr(), out_frames.data_ptr(), out_counts.data_ptr(), cap, _stream_ptr())
        if W is None:
            rc = self._lib.wind_sequential_decode(*args, *tail)
        else:
            rc = self._lib.wind_greedy_decode(*args, W, *tail)
        return _check(rc, allow_overflow)

    def greedy_decode_async(self, enc_out, lengths, W: int, S: int, out_tokens, out_frames, out_counts, workspace,
                            max_iterations: int) -> None:
        """wind_greedy_decode_async: enqueues on the current stream and returns; `workspace` is a device tensor
        of at least workspace_bytes(B, T, W) bytes.  stats() completes the call and raises on its errors."""
        B, T, _ = enc_out.shape
        _check(self._lib.wind_greedy_decode_async(self._h, enc_out.data_ptr(), lengths.data_ptr(), int(B), int(T), int(W),
                                                  int(S), out_tokens.data_ptr(), out_frames.data_ptr(),
                                                  out_counts.data_ptr(), int(out_tokens.shape[1]), workspace.data_ptr(),
                                                  int(workspace.numel() * workspace.element_size()), int(max_iterations),
                                                  _stream_ptr()))

    def decode(self, enc_out, lengths, W: Optional[int], S: int, cap: Optional[int] = None):
        """Convenience wrapper: allocates outputs with torch and returns per-utterance numpy lists."""
        import torch

        B, T, _ = enc_out.shape
        cap = cap or max(1, T * S)
        tok = torch.zeros((B, cap), dtype=torch.int32, device=enc_out.device)
        frm = torch.zeros((B, cap), dtype=torch.int32, device=enc_out.device)
        cnt = torch.zeros((B,), dtype=torch.int32, device=enc_out.device)
        self.greedy_decode(enc_out, lengths, W, S, tok, frm, cnt)
        tok, frm, cnt = tok.cpu().numpy(), frm.cpu().numpy(), cnt.cpu().numpy()
        return [tok[b, : cnt[b]] for b in range(B)], [frm[b, : cnt[b]] for b in range(B)]

    def workspace_bytes(self, B: int, T: int, W: int) -> int:
        n = C.c_size_t(0)
        _check(self._lib.wind_workspace_bytes(self._h, int(B), int(T), int(W), C.byref(n)))
        return int(n.value)

    def stats(self) -> WindStats:
        s = WindStats()
        _check(self._lib.wind_get_stats(self._h, C.byref(s)))
        return s

    def kernel_times(self):
        """{kernel: (total ms, launches)} accumulated since option "profile" was last set."""
        ms = (C.c_double * len(KERNEL_NAMES))()
        n = (C.c_int64 * len(KERNEL_NAMES))()
        _check(self._lib.wind_get_kernel_times(self._h, ms, n))
        return {k: (ms[i], n[i]) for i, k in enumerate(KERNEL_NAMES)}

    def call_times(self):
        """(total ms, loop-only ms) of the last decode call, device time from events on its stream."""
        a, b = C.c_double(0), C.c_double(0)
        _check(self._lib.wind_get_call_times(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def loop_info(self):
        """(workgroups of the resident loop kernel in the last decode call, or 0; whether they shared one L2)."""
        g, one = C.c_int(0), C.c_int(0)
        _check(self._lib.wind_get_loop_info(self._h, C.byref(g), C.byref(one)))
        return int(g.value), bool(one.value)

    def joint_launches(self):
        """(rows, us) of every joint launch of the last decode made with option "profile" = 1."""
        n = C.c_int(0)
        _check(self._lib.wind_get_joint_launches(self._h, (C.c_int32 * 1)(), (C.c_float * 1)(), 0, C.byref(n)))
        rows = (C.c_int32 * max(n.value, 1))()
        us = (C.c_float * max(n.value, 1))()
        _check(self._lib.wind_get_joint_launches(self._h, rows, us, n.value, C.byref(n)))
        return list(rows[:n.value]), list(us[:n.value])

    def beam_window_scores_static(self, enc_window, dec_out, K: int, out):
        """wind_beam_window_scores_static: enqueues on the current stream and returns; `out` = three device
        tensors (labels, jumps int32 [Bh, K]; scores fp32 [Bh, K]) that the caller reads after a synchronise."""
        n, Bh = int(enc_window.shape[0]), int(dec_out.shape[0])
        lab, jmp, sc = out
        _check(self._lib.wind_beam_window_scores_static(self._h, enc_window.data_ptr(), n, dec_out.data_ptr(), Bh, int(K),
                                                        lab.data_ptr(), jmp.data_ptr(), sc.data_ptr(), _stream_ptr()))

    def beam_window_scores(self, enc_window, dec_out, K: int, out=None):
        """wind_beam_window_scores on device tensors enc_window [n, D] and dec_out [Bh, Hp] (fp32).
        Returns (labels, jumps, scores) as numpy arrays [Bh, K]; with `out` = three device tensors the
        results are left there and nothing is copied back."""
        import torch

        n, Bh = int(enc_window.shape[0]), int(dec_out.shape[0])
        if out is None:
            lab = torch.zeros((Bh, K), dtype=torch.int32, device=enc_window.device)
            jmp = torch.zeros((Bh, K), dtype=torch.int32, device=enc_window.device)
            sc = torch.zeros((Bh, K), dtype=torch.float32, device=enc_window.device)
        else:
            lab, jmp, sc = out
        _check(self._lib.wind_beam_window_scores(self._h, enc_window.data_ptr(), n, dec_out.data_ptr(), Bh, int(K),
                                                 lab.data_ptr(), jmp.data_ptr(), sc.data_ptr(), _stream_ptr()))
        if out is not None:
            return None
        return lab.cpu().numpy(), jmp.cpu().numpy(), sc.cpu().numpy()

    def beam_decode(self, enc_out, N: int, K: int, S: int, prefix_step: str = "keep", cap: Optional[int] = None,
                    trace: Optional[list] = None):
        """wind_beam_decode on a device tensor enc_out [T, D] (fp32).  Returns (tokens, frames, score,
        stats).  With `trace` = a list, every pass appends a dict: t, n, hyps = [(tokens, frames, score,
        sym)], expansions = per hypothesis [(label, jump, score)]."""
        T = int(enc_out.shape[0])
        assert enc_out.is_contiguous() and (T == 0 or int(enc_out.shape[1]) == self.D)
        cap = cap if cap is not None else max(1, T * S)
        tok = np.zeros(max(cap, 1), np.int32)
        frm = np.zeros(max(cap, 1), np.int32)
        cnt, score, st = C.c_int32(0), C.c_double(0.0), WindBeamStats()

        def on_round(_user, t, n, n_hyps, hyp_len, hyp_tokens, hyp_frames, hyp_score, hyp_sym, Kc, labels, jumps, scores):
            hyps, exps, o = [], [], 0
            for b in range(n_hyps):
                ln = hyp_len[b]
                hyps.append((tuple(hyp_tokens[o:o + ln]), tuple(hyp_frames[o:o + ln]), hyp_score[b], hyp_sym[b]))
                o += ln
                exps.append([(labels[b * Kc + k], jumps[b * Kc + k], scores[b * Kc + k]) for k in range(Kc)
                             if labels[b * Kc + k] >= 0])
            trace.append({"t": t, "n": n, "hyps": hyps, "expansions": exps})

        cb = BEAM_ROUND_FN(on_round) if trace is not None else None
        rc = self._lib.wind_beam_decode(self._h, enc_out.data_ptr() if T else None, T, int(N), int(K), int(S),
                                        PREFIX_MODES[prefix_step], tok.ctypes.data, frm.ctypes.data, int(cap),
                                        C.byref(cnt), C.byref(score), C.byref(st),
                                        C.cast(cb, C.c_void_p) if cb is not None else None, None, _stream_ptr())
        _check(rc)
        return tok[: cnt.value].copy(), frm[: cnt.value].copy(), score.value, st

    def debug_enc_proj(self, enc_out, lengths):
        """e [B, T, Hj] fp32 (numpy) as a decode call computes it; rows past an utterance's end are unspecified."""
        import torch

        B, T, _ = enc_out.shape
        out = torch.zeros((B, T, self.Hj), dtype=torch.float32, device=enc_out.device)
        _check(self._lib.wind_debug_enc_proj(self._h, enc_out.data_ptr(), lengths.data_ptr(), B, T, out.data_ptr(),
                                             _stream_ptr()))
        return out.cpu().numpy()

    def debug_joint_keys(self, enc_out, lengths, W: int):
        """(keys [B*W, nparts, 4] fp32 numpy, part_width): the joint kernel's output for the first iteration
        (largest, second, third key of the part, one unused word)."""
        import torch

        B, T, _ = enc_out.shape
        nparts, width = C.c_int32(0), C.c_int32(0)
        _check(self._lib.wind_debug_joint_keys(self._h, None, None, B, T, int(W), None, C.byref(nparts), C.byref(width),
                                               _stream_ptr()))
        out = torch.zeros((B * W, nparts.value, 4), dtype=torch.float32, device=enc_out.device)
        _check(self._lib.wind_debug_joint_keys(self._h, enc_out.data_ptr(), lengths.data_ptr(), B, T, int(W),
                                               out.data_ptr(), C.byref(nparts), C.byref(width), _stream_ptr()))
        return out.cpu().numpy(), int(width.value)

    def debug_joint_logits(self, enc_out, b: int, t0: int, n: int, prefix: Sequence[int], exact: bool):
        import torch

        B, T, _ = enc_out.shape
        pre = np.ascontiguousarray(list(prefix), dtype=np.int32)
        out = torch.zeros((n, self.V + 1), dtype=torch.float32, device=enc_out.device)
        _check(self._lib.wind_debug_joint_logits(self._h, enc_out.data_ptr(), B, T, b, t0, n,
                                                 pre.ctypes.data if pre.size else None, int(pre.size),
                                                 1 if exact else 0, out.data_ptr(), _stream_ptr()))
        return out.cpu().numpy()
