"""ctypes access to the plain-C oracle (oracle/tts_oracle.c).

TEST INFRASTRUCTURE: only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this.  Argument marshalling only; all arithmetic is
in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build as _build

_DIM_FIELDS = ("n_mel", "prenet_dim", "enc_dim", "att_rnn_dim", "dec_rnn_dim", "att_dim",
               "loc_filters", "loc_kernel", "loc_in_channels")
_W_FIELDS = ("prenet1", "prenet2", "att_w_ih", "att_w_hh", "att_b", "q_w", "mem_w", "loc_conv",
             "loc_w", "v", "dec_w_ih", "dec_w_hh", "dec_b", "mel_w", "mel_b", "stop_w", "stop_b")

_fp = C.POINTER(C.c_float)
_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int)


class OrcDims(C.Structure):
    _fields_ = [(n, C.c_int) for n in _DIM_FIELDS]


class OrcWeights(C.Structure):
    _fields_ = [(n, _fp) for n in _W_FIELDS]


_lib = None


def load(path: str) -> C.CDLL:
    """Load one build of the oracle and declare its entry points."""
    L = C.CDLL(path)
    _declare(L)
    return L


def use_library(L: Optional[C.CDLL]) -> Optional[C.CDLL]:
    """Swap the library every function below calls (tests of the pins themselves
    point them at deliberately broken builds); returns the previous one."""
    global _lib
    prev, _lib = _lib, L
    return prev


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.OUT
        if (not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC)
                or os.path.getmtime(path) < os.path.getmtime(_build.SRC_POSTNET)):
            _build.build(force=True)
        _lib = load(path)
    return _lib


def _declare(L: C.CDLL) -> None:
    L.orc_prenet.argtypes = [C.POINTER(OrcDims), _fp, _fp, _dp, _dp]
    L.orc_lstm_cell.argtypes = [C.c_int, C.c_int, _fp, _fp, _fp, _dp, _dp, _dp]
    L.orc_memory_projection.argtypes = [C.POINTER(OrcDims), _fp, _fp, C.c_int, C.c_int, _dp]
    L.orc_location_features.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, _fp, _dp, _dp]
    L.orc_lsa.argtypes = [C.POINTER(OrcDims), C.POINTER(OrcWeights), C.c_int, _fp, _dp, _dp, _dp, _dp,
                          _dp, _dp, _dp]
    L.orc_projection.argtypes = [C.POINTER(OrcDims), C.POINTER(OrcWeights), _dp, _dp, _dp, _dp]
    L.orc_request_new.restype = C.c_void_p
    L.orc_request_new.argtypes = [C.POINTER(OrcDims), C.POINTER(OrcWeights), _fp, C.c_int, C.c_int,
                                  C.c_int, C.c_double]
    L.orc_request_free.argtypes = [C.c_void_p]
    L.orc_request_step.argtypes = [C.c_void_p, _dp, _dp]
    L.orc_request_get.argtypes = [C.c_void_p, C.c_int, _dp]
    L.orc_request_set.argtypes = [C.c_void_p, C.c_int, _dp]
    L.orc_request_frames.argtypes = [C.c_void_p]
    L.orc_request_finished.argtypes = [C.c_void_p]
    L.orc_pool_decode.argtypes = [C.POINTER(OrcDims), C.POINTER(OrcWeights), C.c_int,
                                  C.POINTER(_fp), _ip, _ip, C.c_int, C.c_int, C.c_double, C.c_int,
                                  _dp, _dp, _ip]
    L.orc_conv5.argtypes = [C.c_int, C.c_int, C.c_int, _fp, _fp, _dp, C.c_int, _dp]
    L.orc_postnet.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(_fp), C.POINTER(_fp), C.c_int, _dp, _dp]
    L.orc_postnet_chunk.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(_fp), C.POINTER(_fp), C.c_int, C.c_int,
                                    _dp, _dp]


def _f(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_fp)


def _d(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def make_dims(dims: Dict[str, int]) -> OrcDims:
    return OrcDims(*[int(dims[n]) for n in _DIM_FIELDS])


class Weights:
    """Keeps the fp32 arrays alive and exposes the C struct."""

    def __init__(self, w: Dict[str, np.ndarray]):
        self.arrays = {n: np.ascontiguousarray(w[n], dtype=np.float32) for n in _W_FIELDS}
        self.c = OrcWeights(*[_f(self.arrays[n]) for n in _W_FIELDS])


STATE = dict(m=0, a=1, w_last=2, w_acc=3, h_att=4, c_att=5, h_dec=6, c_dec=7, PM=8)


def prenet(dims, W1, W2, m):
    d = make_dims(dims)
    m = np.ascontiguousarray(m, np.float64)
    p = np.zeros(dims["prenet_dim"], np.float64)
    lib().orc_prenet(C.byref(d), _f(np.ascontiguousarray(W1, np.float32)),
                     _f(np.ascontiguousarray(W2, np.float32)), _d(m), _d(p))
    return p


def lstm_cell(W_ih, W_hh, b, x, h, c):
    W_ih = np.ascontiguousarray(W_ih, np.float32)
    W_hh = np.ascontiguousarray(W_hh, np.float32)
    b = np.ascontiguousarray(b, np.float32)
    hid = W_hh.shape[1]
    in_dim = W_ih.shape[1]
    assert W_ih.shape[0] == 4 * hid and W_hh.shape[0] == 4 * hid and b.shape[0] == 4 * hid
    x = np.ascontiguousarray(x, np.float64)
    h = np.array(h, np.float64)
    c = np.array(c, np.float64)
    assert x.shape == (in_dim,) and h.shape == (hid,) and c.shape == (hid,)
    lib().orc_lstm_cell(in_dim, hid, _f(W_ih), _f(W_hh), _f(b), _d(x), _d(h), _d(c))
    return h, c


def memory_projection(dims, mem_w, F, round_bf16=False):
    d = make_dims(dims)
    F = np.ascontiguousarray(F, np.float32)
    mem_w = np.ascontiguousarray(mem_w, np.float32)
    L = F.shape[0]
    PM = np.zeros((L, dims["att_dim"]), np.float64)
    lib().orc_memory_projection(C.byref(d), _f(mem_w), _f(F), L, int(round_bf16), _d(PM))
    return PM


def location_features(K, u):
    K = np.ascontiguousarray(K, np.float32)
    u = np.ascontiguousarray(u, np.float64)
    n_filt, n_ch, ksz = K.shape
    assert u.shape[0] == n_ch
    L = u.shape[1]
    loc = np.zeros((L, n_filt), np.float64)
    lib().orc_location_features(L, n_filt, n_ch, ksz, _f(K), _d(u), _d(loc))
    return loc


def lsa(dims, weights: Weights, F, PM, h_att, w_last, w_acc):
    d = make_dims(dims)
    F = np.ascontiguousarray(F, np.float32)
    L = F.shape[0]
    PM = np.ascontiguousarray(PM, np.float64)
    h_att = np.ascontiguousarray(h_att, np.float64)
    w_last = np.ascontiguousarray(w_last, np.float64)
    w_acc = np.ascontiguousarray(w_acc, np.float64)
    assert PM.shape == (L, dims["att_dim"]) and w_last.shape == (L,) and w_acc.shape == (L,)
    e = np.zeros(L, np.float64)
    w = np.zeros(L, np.float64)
    ctx = np.zeros(dims["enc_dim"], np.float64)
    lib().orc_lsa(C.byref(d), C.byref(weights.c), L, _f(F), _d(PM), _d(h_att), _d(w_last), _d(w_acc),
                  _d(e), _d(w), _d(ctx))
    return e, w, ctx


def projection(dims, weights: Weights, h_dec, ctx):
    d = make_dims(dims)
    h_dec = np.ascontiguousarray(h_dec, np.float64)
    ctx = np.ascontiguousarray(ctx, np.float64)
    mel = np.zeros(dims["n_mel"], np.float64)
    stop = C.c_double(0.0)
    lib().orc_projection(C.byref(d), C.byref(weights.c), _d(h_dec), _d(ctx), _d(mel), C.byref(stop))
    return mel, stop.value


class Request:
    """One request decoded alone: the reference for any pooled run."""

    def __init__(self, dims, weights: Weights, F, n_steps, pm_round_bf16=False, stop_threshold=-1.0):
        self.dims = dims
        self._w = weights
        self._F = np.ascontiguousarray(F, np.float32)
        self.L = self._F.shape[0]
        d = make_dims(dims)
        self._h = lib().orc_request_new(C.byref(d), C.byref(weights.c), _f(self._F), self.L, int(n_steps),
                                        int(pm_round_bf16), float(stop_threshold))
        if not self._h:
            raise ValueError("orc_request_new rejected its arguments")

    def step(self):
        mel = np.zeros(self.dims["n_mel"], np.float64)
        stop = C.c_double(0.0)
        ok = lib().orc_request_step(self._h, _d(mel), C.byref(stop))
        return (mel, stop.value) if ok else None

    def get(self, name: str) -> np.ndarray:
        n = lib().orc_request_get(self._h, STATE[name], None)
        out = np.zeros(n, np.float64)
        lib().orc_request_get(self._h, STATE[name], _d(out))
        return out

    def set(self, name: str, value) -> None:
        v = np.ascontiguousarray(value, np.float64).ravel()
        n = lib().orc_request_get(self._h, STATE[name], None)
        assert v.shape[0] == n
        lib().orc_request_set(self._h, STATE[name], _d(v))

    @property
    def frames(self) -> int:
        return lib().orc_request_frames(self._h)

    @property
    def finished(self) -> bool:
        return bool(lib().orc_request_finished(self._h))

    def close(self):
        if self._h:
            lib().orc_request_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pool_decode(dims, weights: Weights, F_list: Sequence[np.ndarray], n_steps: Sequence[int], window: int,
                pm_round_bf16: bool = False, stop_threshold: float = -1.0, n_threads: int = 1):
    """Each request decoded alone for min(n_steps[i], window) frames.

    Returns (mel [n, window, n_mel] float64 with NaN past the last frame,
    stop [n, window], frames [n], threads actually used).
    """
    n = len(F_list)
    d = make_dims(dims)
    Fs = [np.ascontiguousarray(f, np.float32) for f in F_list]
    Fp = (_fp * n)(*[_f(f) for f in Fs])
    L = np.array([f.shape[0] for f in Fs], np.int32)
    ns = np.ascontiguousarray(n_steps, np.int32)
    mel = np.full((n, window, dims["n_mel"]), np.nan, np.float64)
    stop = np.full((n, window), np.nan, np.float64)
    frames = np.zeros(n, np.int32)
    used = lib().orc_pool_decode(C.byref(d), C.byref(weights.c), n, Fp,
                                 L.ctypes.data_as(_ip), ns.ctypes.data_as(_ip), int(window),
                                 int(pm_round_bf16), float(stop_threshold), int(n_threads),
                                 _d(mel), _d(stop), frames.ctypes.data_as(_ip))
    return mel, stop, frames, used


# ---- PostNet (oracle/postnet_oracle.c)
class PostnetWeights:
    """conv_w[l]: [c_out, c_in, 5], conv_b[l]: [c_out], fp32."""

    def __init__(self, conv_w: Sequence[np.ndarray], conv_b: Sequence[np.ndarray]):
        self.w = [np.ascontiguousarray(a, np.float32) for a in conv_w]
        self.b = [np.ascontiguousarray(a, np.float32) for a in conv_b]
        self.n_layers = len(self.w)
        self.n_mel = self.w[0].shape[1]
        self.channels = self.w[0].shape[0]
        assert self.w[-1].shape[0] == self.n_mel and all(a.shape[2] == 5 for a in self.w)
        self.wp = (_fp * self.n_layers)(*[_f(a) for a in self.w])
        self.bp = (_fp * self.n_layers)(*[_f(a) for a in self.b])


def conv5(w, b, x, apply_tanh=False):
    w = np.ascontiguousarray(w, np.float32)
    b = np.ascontiguousarray(b, np.float32)
    x = np.ascontiguousarray(x, np.float64)
    T, c_in = x.shape
    c_out = w.shape[0]
    assert w.shape == (c_out, c_in, 5) and b.shape == (c_out,)
    y = np.zeros((T, c_out), np.float64)
    lib().orc_conv5(T, c_in, c_out, _f(w), _f(b), _d(x), int(apply_tanh), _d(y))
    return y


def postnet(W: PostnetWeights, mel):
    mel = np.ascontiguousarray(mel, np.float64)
    T = mel.shape[0]
    out = np.zeros((T, W.n_mel), np.float64)
    lib().orc_postnet(W.n_layers, W.n_mel, W.channels, W.wp, W.bp, T, _d(mel), _d(out))
    return out


def postnet_chunk(W: PostnetWeights, mel_so_far, s: int):
    """Chunk [s, e) with e = len(mel_so_far)."""
    mel = np.ascontiguousarray(mel_so_far, np.float64)
    e = mel.shape[0]
    out = np.zeros((e - s, W.n_mel), np.float64)
    lib().orc_postnet_chunk(W.n_layers, W.n_mel, W.channels, W.wp, W.bp, int(s), int(e), _d(mel), _d(out))
    return out
