"""ctypes access to the plain-C oracle (oracle/*.c).

TEST INFRASTRUCTURE: only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this.  The arithmetic of the decoder step, the
PostNet, the generator and the encoder is in the C files and this module only
marshals their arguments; the one piece of the method written here is
VocoderStream, the response rule of Eq. 3 / Eq. 4 (which samples a chunk's
response carries, the equal-power fade against the previous tail, the
write-back), plain numpy in double precision with its own pins in
tests/test_vocoder_oracle.py.
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


class OrcGenerator(C.Structure):
    _fields_ = [("n_mel", C.c_int), ("c0", C.c_int), ("n_stages", C.c_int), ("n_blocks", C.c_int),
                ("n_pairs", C.c_int), ("k_pre", C.c_int), ("k_post", C.c_int),
                ("rates", _ip), ("block_k", _ip), ("dils", _ip), ("slope", C.c_double),
                ("pre_w", _fp), ("pre_b", _fp), ("post_w", _fp), ("post_b", _fp),
                ("up_w", C.POINTER(_fp)), ("up_b", C.POINTER(_fp)),
                ("res_w", C.POINTER(_fp)), ("res_b", C.POINTER(_fp))]


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
    L.orc_conv1d.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _fp, _fp, _dp, _dp]
    L.orc_conv_transpose1d.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _fp, _fp, _dp, _dp]
    L.orc_generator.argtypes = [C.POINTER(OrcGenerator), C.c_int, _dp, _dp]
    L.orc_fade.argtypes = [C.c_int, _dp, _dp]
    _ipp, _fpp = C.POINTER(_ip), C.POINTER(_fp)
    L.orc_encoder_embed.argtypes = [C.c_int, C.c_int, C.c_int, _fpp, _ipp, _dp]
    L.orc_encoder_conv_relu.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, _fp, _fp, _dp, _dp]
    L.orc_bilstm.argtypes = [C.c_int, C.c_int, C.c_int, _fp, _fp, _fp, _fp, _fp, _fp, _dp, _dp]
    L.orc_encoder.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, _fpp, _ipp, C.c_int, C.c_int, _fpp, _fpp,
                              _fp, _fp, _fp, _fp, _fp, _fp, _dp]
    L.orc_crossfade.argtypes = [C.c_int, _dp, _dp, _dp]


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


# ---- vocoder (oracle/vocoder_oracle.c)
class VocoderWeights:
    """w: dict with pre_w [c0, n_mel, 7], pre_b, post_w [1, c_last, 7], post_b, up_w[s] [c_in, c_in / 2, 2 u_s],
    up_b[s], res_w[s][block][2 pair + {0: dilated, 1: plain}] [c, c, k_block], res_b likewise.  fp32."""

    def __init__(self, w: dict, rates=(8, 8, 2, 2), block_k=(3, 7, 11), dils=(1, 3, 5), slope=0.1):
        c32 = lambda a: np.ascontiguousarray(a, np.float32)
        self.rates, self.block_k, self.dils, self.slope = tuple(rates), tuple(block_k), tuple(dils), float(slope)
        self.pre_w, self.pre_b, self.post_w, self.post_b = c32(w["pre_w"]), c32(w["pre_b"]), c32(w["post_w"]), c32(w["post_b"])
        self.up_w = [c32(a) for a in w["up_w"]]
        self.up_b = [c32(a) for a in w["up_b"]]
        self.res_w = [[[c32(a) for a in blk] for blk in st] for st in w["res_w"]]
        self.res_b = [[[c32(a) for a in blk] for blk in st] for st in w["res_b"]]
        ns, nb, npair = len(self.rates), len(self.block_k), len(self.dils)
        self.n_mel, self.c0 = self.pre_w.shape[1], self.pre_w.shape[0]
        self.hop = int(np.prod(self.rates))
        c = self.c0
        for s_ in range(ns):
            assert self.up_w[s_].shape == (c, c // 2, 2 * self.rates[s_])
            c //= 2
            for b_ in range(nb):
                assert len(self.res_w[s_][b_]) == 2 * npair
                assert all(a.shape == (c, c, self.block_k[b_]) for a in self.res_w[s_][b_])
        assert self.post_w.shape == (1, c, 7) and self.pre_w.shape[2] == 7
        self._rates = (C.c_int * ns)(*self.rates)
        self._bk = (C.c_int * nb)(*self.block_k)
        self._dils = (C.c_int * npair)(*self.dils)
        self._up_w = (_fp * ns)(*[_f(a) for a in self.up_w])
        self._up_b = (_fp * ns)(*[_f(a) for a in self.up_b])
        flat_w = [a for st in self.res_w for blk in st for a in blk]
        flat_b = [a for st in self.res_b for blk in st for a in blk]
        self._res_w = (_fp * len(flat_w))(*[_f(a) for a in flat_w])
        self._res_b = (_fp * len(flat_b))(*[_f(a) for a in flat_b])
        self.c = OrcGenerator(self.n_mel, self.c0, ns, nb, npair, 7, 7,
                              C.cast(self._rates, _ip), C.cast(self._bk, _ip), C.cast(self._dils, _ip), self.slope,
                              _f(self.pre_w), _f(self.pre_b), _f(self.post_w), _f(self.post_b),
                              C.cast(self._up_w, C.POINTER(_fp)), C.cast(self._up_b, C.POINTER(_fp)),
                              C.cast(self._res_w, C.POINTER(_fp)), C.cast(self._res_b, C.POINTER(_fp)))


def conv1d(w, b, x, dil=1):
    """x [T, c_in] -> [T, c_out]; w [c_out, c_in, k], zero 'same' padding."""
    w, b = np.ascontiguousarray(w, np.float32), np.ascontiguousarray(b, np.float32)
    x = np.ascontiguousarray(x, np.float64)
    T, c_in = x.shape
    c_out, _, k = w.shape
    assert w.shape[1] == c_in and k % 2 == 1
    y = np.zeros((T, c_out), np.float64)
    lib().orc_conv1d(T, c_in, c_out, k, int(dil), _f(w), _f(b), _d(x), _d(y))
    return y


def conv_transpose1d(w, b, x, stride, pad):
    """x [T, c_in] -> [T * stride, c_out]; w [c_in, c_out, k] with k - 2 pad = stride."""
    w, b = np.ascontiguousarray(w, np.float32), np.ascontiguousarray(b, np.float32)
    x = np.ascontiguousarray(x, np.float64)
    T, c_in = x.shape
    _, c_out, k = w.shape
    assert w.shape[0] == c_in and k - 2 * pad == stride
    y = np.zeros((T * stride, c_out), np.float64)
    lib().orc_conv_transpose1d(T, c_in, c_out, k, int(stride), int(pad), _f(w), _f(b), _d(x), _d(y))
    return y


def generator(W: VocoderWeights, mel):
    """audio [T * hop] = G(mel [T, n_mel])"""
    mel = np.ascontiguousarray(mel, np.float64)
    T = mel.shape[0]
    assert mel.shape[1] == W.n_mel
    audio = np.zeros(T * W.hop, np.float64)
    lib().orc_generator(C.byref(W.c), T, _d(mel), _d(audio))
    return audio


def fade(n: int):
    al, be = np.zeros(n, np.float64), np.zeros(n, np.float64)
    lib().orc_fade(n, _d(al), _d(be))
    return al, be


def crossfade(head_cur, tail_pre):
    a = np.ascontiguousarray(head_cur, np.float64)
    b = np.ascontiguousarray(tail_pre, np.float64)
    out = np.zeros_like(a)
    lib().orc_crossfade(a.shape[0], _d(a), _d(b), _d(out))
    return out


class VocoderStream:
    """One request's vocoder state across chunks (Sec. 2.2.2 lists it: M_pre, M_cur, S_pre, S_cur).

    chunk(M_cur, last): S_cur = G([tail(M_pre), M_cur]) (Eq. 3, first line; the tail is `overlap` frames, absent for
    the first chunk), the head of S_cur that overlaps the tail of S_pre is fused with it (Eq. 3, second line), then
    M_pre = M_cur, S_pre = S_cur (Eq. 4).  Reading of what a response carries: the overlap region is sent once, fused,
    with the chunk that completes it; so every chunk but the last holds back its final overlap * hop samples, and the
    responses tile the utterance: sum of their lengths = hop * frames."""

    def __init__(self, W: VocoderWeights, overlap: int):
        self.W, self.ov = W, int(overlap)
        self.m_pre = None
        self.s_pre = None

    def chunk(self, m_cur, last: bool):
        m_cur = np.ascontiguousarray(m_cur, np.float64)
        hop, ov = self.W.hop, self.ov
        if self.m_pre is None:
            s_cur = generator(self.W, m_cur)
            body = s_cur
        else:
            tail = self.m_pre[-ov:] if ov else self.m_pre[:0]
            n_ov = tail.shape[0] * hop
            s_cur = generator(self.W, np.concatenate([tail, m_cur], axis=0))
            if n_ov:
                s_cur[:n_ov] = crossfade(s_cur[:n_ov], self.s_pre[-n_ov:])
            body = s_cur
        self.m_pre, self.s_pre = m_cur, s_cur
        if last:
            return body
        hold = min(ov, m_cur.shape[0]) * hop
        return body[: body.shape[0] - hold]


# ---- acoustic encoder (oracle/encoder_oracle.c)
class EncoderWeights:
    """w: dict with tables (list of [vocab_t, dim]), conv_w (list of [dim, dim, 5]), conv_b, and per direction
    d in ('f', 'b'): w_ih_d [4 hid, dim], w_hh_d [4 hid, hid], b_d [4 hid].  fp32."""

    def __init__(self, w: dict):
        c32 = lambda a: np.ascontiguousarray(a, np.float32)
        self.tables = [c32(a) for a in w["tables"]]
        self.conv_w = [c32(a) for a in w["conv_w"]]
        self.conv_b = [c32(a) for a in w["conv_b"]]
        self.lstm = {k: c32(w[k]) for k in ("w_ih_f", "w_hh_f", "b_f", "w_ih_b", "w_hh_b", "b_b")}
        self.dim = self.tables[0].shape[1]
        self.hid = self.lstm["w_hh_f"].shape[1]
        self.ksz = self.conv_w[0].shape[2]
        assert all(t.shape[1] == self.dim for t in self.tables)
        assert all(a.shape == (self.dim, self.dim, self.ksz) for a in self.conv_w)
        assert self.lstm["w_ih_f"].shape == (4 * self.hid, self.dim) and self.lstm["w_hh_b"].shape == (4 * self.hid, self.hid)
        self._tables = (_fp * len(self.tables))(*[_f(a) for a in self.tables])
        self._cw = (_fp * len(self.conv_w))(*[_f(a) for a in self.conv_w])
        self._cb = (_fp * len(self.conv_b))(*[_f(a) for a in self.conv_b])


def _ids(ids, n_tables):
    ids = np.ascontiguousarray(ids, np.int32)
    assert ids.ndim == 2 and ids.shape[0] == n_tables
    rows = [np.ascontiguousarray(ids[t]) for t in range(n_tables)]
    return rows, (_ip * n_tables)(*[r.ctypes.data_as(_ip) for r in rows])


def encoder_embed(W: EncoderWeights, ids):
    rows, ptrs = _ids(ids, len(W.tables))
    L = rows[0].shape[0]
    for r, t in zip(rows, W.tables):
        assert r.min(initial=0) >= 0 and r.max(initial=0) < t.shape[0]
    E = np.zeros((L, W.dim), np.float64)
    lib().orc_encoder_embed(L, W.dim, len(W.tables), C.cast(W._tables, C.POINTER(_fp)), C.cast(ptrs, C.POINTER(_ip)), _d(E))
    return E


def encoder_conv_relu(w, b, x):
    w, b = np.ascontiguousarray(w, np.float32), np.ascontiguousarray(b, np.float32)
    x = np.ascontiguousarray(x, np.float64)
    L, c_in = x.shape
    c_out, _, k = w.shape
    y = np.zeros((L, c_out), np.float64)
    lib().orc_encoder_conv_relu(L, c_in, c_out, k, _f(w), _f(b), _d(x), _d(y))
    return y


def bilstm(lstm: dict, x):
    x = np.ascontiguousarray(x, np.float64)
    L, in_dim = x.shape
    c32 = lambda a: np.ascontiguousarray(a, np.float32)
    w = {k: c32(v) for k, v in lstm.items()}
    hid = w["w_hh_f"].shape[1]
    out = np.zeros((L, 2 * hid), np.float64)
    lib().orc_bilstm(L, in_dim, hid, _f(w["w_ih_f"]), _f(w["w_hh_f"]), _f(w["b_f"]), _f(w["w_ih_b"]), _f(w["w_hh_b"]),
                     _f(w["b_b"]), _d(x), _d(out))
    return out


def encoder(W: EncoderWeights, ids):
    """F_enc [L, 2 hid] of one request from its id sequences ids [n_tables, L] (Eq. 1)."""
    rows, ptrs = _ids(ids, len(W.tables))
    L = rows[0].shape[0]
    for r, t in zip(rows, W.tables):
        assert r.min(initial=0) >= 0 and r.max(initial=0) < t.shape[0]
    out = np.zeros((L, 2 * W.hid), np.float64)
    l = W.lstm
    lib().orc_encoder(L, W.dim, W.hid, len(W.tables), C.cast(W._tables, C.POINTER(_fp)), C.cast(ptrs, C.POINTER(_ip)),
                      len(W.conv_w), W.ksz, C.cast(W._cw, C.POINTER(_fp)), C.cast(W._cb, C.POINTER(_fp)),
                      _f(l["w_ih_f"]), _f(l["w_hh_f"]), _f(l["b_f"]), _f(l["w_ih_b"]), _f(l["w_hh_b"]), _f(l["b_b"]), _d(out))
    return out
