"""Thin ctypes binding of the C-ABI library declared in include/tts_pool.h.

Argument marshalling only: every step of the decoder path runs in the HIP
kernels of libtts_pool.so.  PyTorch is used for the device arena and the
stream, nothing else.  If the library has not been built this module raises;
there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtts_pool.so")

TTS_OK = 0
TTS_E_INVAL, TTS_E_FULL, TTS_E_NOTFOUND, TTS_E_HIP, TTS_E_ARENA, TTS_E_UNSUPPORTED, TTS_E_LOST = -1, -2, -3, -4, -5, -6, -7
DTYPE_F32, DTYPE_BF16 = 0, 1
STATE = dict(m=0, a=1, w_last=2, w_acc=3, h_att=4, c_att=5, h_dec=6, c_dec=7)

_CFG_INT_FIELDS = ("n_mel", "prenet_dim", "enc_dim", "att_rnn_dim", "dec_rnn_dim", "att_dim",
                   "loc_filters", "loc_kernel", "loc_in_channels",
                   "max_pool", "max_enc_len", "max_steps", "chunk_frames",
                   "weight_dtype", "memory_dtype", "use_graph")
WEIGHT_FIELDS = ("prenet1", "prenet2", "att_w_ih", "att_w_hh", "att_b", "q_w", "mem_w", "loc_conv",
                 "loc_w", "v", "dec_w_ih", "dec_w_hh", "dec_b", "mel_w", "mel_b", "stop_w", "stop_b")

# every symbol include/tts_pool.h declares
EXPORTS = (
    "tts_pool_workspace_bytes", "tts_pool_create", "tts_pool_add_request", "tts_pool_add_requests", "tts_pool_step",
    "tts_pool_step_n", "tts_pool_drain_chunk", "tts_pool_get_stop_logits", "tts_pool_retire",
    "tts_pool_get_state", "tts_pool_set_state", "tts_pool_frames", "tts_pool_size", "tts_pool_n_active",
    "tts_pool_span", "tts_pool_moves",
    "tts_pool_sync", "tts_pool_lost", "tts_pool_set_wait_polls", "tts_pool_timing", "tts_pool_elapsed_ms", "tts_pool_kernel_times", "tts_pool_destroy",
    "tts_last_error",
    "tts_book_create", "tts_book_add", "tts_book_step", "tts_book_drain", "tts_book_retire",
    "tts_book_slot", "tts_book_compact", "tts_book_destroy",
    "tts_pool_chunk_window",
    "tts_postnet_workspace_bytes", "tts_postnet_create", "tts_postnet_run", "tts_postnet_run_static", "tts_postnet_elapsed_ms",
    "tts_postnet_destroy",
    "tts_vocoder_workspace_bytes", "tts_vocoder_create", "tts_vocoder_run", "tts_vocoder_elapsed_ms",
    "tts_vocoder_destroy",
    "tts_encoder_workspace_bytes", "tts_encoder_create", "tts_encoder_run", "tts_encoder_elapsed_ms",
    "tts_encoder_destroy",
)

_fp = C.POINTER(C.c_float)
_ip = C.POINTER(C.c_int)
_i64p = C.POINTER(C.c_int64)


class TtsConfig(C.Structure):
    _fields_ = [(n, C.c_int) for n in _CFG_INT_FIELDS] + [("stop_threshold", C.c_float)]


class TtsWeights(C.Structure):
    _fields_ = [(n, _fp) for n in WEIGHT_FIELDS]


class TtsPostnetConfig(C.Structure):
    _fields_ = [("n_mel", C.c_int), ("channels", C.c_int), ("max_columns", C.c_int), ("weight_dtype", C.c_int)]


class TtsPostnetWeights(C.Structure):
    _fields_ = [("conv_w", C.POINTER(C.c_float) * 5), ("conv_b", C.POINTER(C.c_float) * 5)]


class TtsVocoderConfig(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_mel", "c0", "overlap", "max_chunk", "max_requests", "max_batch", "weight_dtype")]


class TtsVocoderWeights(C.Structure):
    _fields_ = [("pre_w", _fp), ("pre_b", _fp), ("up_w", _fp * 4), ("up_b", _fp * 4),
                ("res_w", _fp * 6 * 3 * 4), ("res_b", _fp * 6 * 3 * 4), ("post_w", _fp), ("post_b", _fp)]


class TtsEncoderConfig(C.Structure):
    _fields_ = [("dim", C.c_int), ("hid", C.c_int), ("vocab", C.c_int * 4), ("max_tokens", C.c_int), ("max_len", C.c_int),
                ("weight_dtype", C.c_int)]


class TtsEncoderWeights(C.Structure):
    _fields_ = [("tables", _fp * 4), ("conv_w", _fp * 3), ("conv_b", _fp * 3), ("w_ih", _fp * 2), ("w_hh", _fp * 2), ("b", _fp * 2)]


VOCODER_HOP = 256
VOCODER_FIRST, VOCODER_LAST = 1, 2
POSTNET_CONTEXT = 10      # frames in front of a chunk that can influence it (2 per layer)
TTS_POSTNET_STATIC_MAX_COLUMNS = 4096   # most frames one tts_postnet_run_static call may carry


class TtsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"tts_pool error {code}: {text}")
        self.code = code
        self.text = text


_lib = None


def lib() -> C.CDLL:
    """Load libtts_pool.so (built beforehand by paper_2211_13939_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2211_13939_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    L.tts_pool_workspace_bytes.restype = C.c_size_t
    L.tts_pool_workspace_bytes.argtypes = [C.POINTER(TtsConfig)]
    L.tts_pool_create.argtypes = [C.POINTER(TtsConfig), C.POINTER(TtsWeights), vp, C.c_size_t, vp, C.POINTER(vp)]
    L.tts_pool_add_request.argtypes = [vp, vp, C.c_int, C.c_int, _i64p]
    L.tts_pool_add_requests.argtypes = [vp, C.c_int, C.POINTER(vp), _ip, _ip, _i64p]
    L.tts_pool_step.argtypes = [vp, _ip]
    L.tts_pool_step_n.argtypes = [vp, C.c_int, _i64p]
    L.tts_pool_drain_chunk.argtypes = [vp, C.c_int64, _fp, _ip, _ip]
    L.tts_pool_get_stop_logits.argtypes = [vp, C.c_int64, C.c_int, C.c_int, _fp]
    L.tts_pool_retire.argtypes = [vp, C.c_int64]
    L.tts_pool_get_state.argtypes = [vp, C.c_int64, C.c_int, _fp, C.c_int, _ip]
    L.tts_pool_set_state.argtypes = [vp, C.c_int64, C.c_int, _fp, C.c_int]
    L.tts_pool_frames.argtypes = [vp, C.c_int64, _ip, _ip]
    L.tts_pool_size.argtypes = [vp]
    L.tts_pool_n_active.argtypes = [vp]
    L.tts_pool_span.argtypes = [vp]
    L.tts_pool_moves.restype = C.c_longlong
    L.tts_pool_moves.argtypes = [vp]
    L.tts_pool_sync.argtypes = [vp]
    L.tts_pool_lost.argtypes = [vp, C.c_int64, _ip]
    L.tts_pool_set_wait_polls.argtypes = [vp, C.c_int]
    L.tts_pool_timing.argtypes = [vp, C.c_int]
    L.tts_pool_elapsed_ms.argtypes = [vp, _fp]
    L.tts_pool_kernel_times.argtypes = [vp, C.c_int, _fp, C.c_int, _ip]
    L.tts_pool_destroy.restype = None
    L.tts_pool_destroy.argtypes = [vp]
    L.tts_last_error.restype = C.c_char_p
    L.tts_last_error.argtypes = []
    L.tts_book_create.restype = vp
    L.tts_book_create.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int]
    L.tts_book_add.argtypes = [vp, C.c_int, C.c_int, _i64p]
    L.tts_book_step.argtypes = [vp, _i64p, _ip]
    L.tts_book_drain.argtypes = [vp, C.c_int64, _ip, _ip, _ip]
    L.tts_book_retire.argtypes = [vp, C.c_int64]
    L.tts_book_slot.argtypes = [vp, C.c_int64]
    L.tts_book_compact.argtypes = [vp, C.c_int, _ip, _ip, C.c_int]
    L.tts_book_destroy.restype = None
    L.tts_book_destroy.argtypes = [vp]
    L.tts_pool_chunk_window.argtypes = [vp, C.c_int64, C.c_int, vp, _ip, _ip, _ip]
    L.tts_postnet_workspace_bytes.restype = C.c_size_t
    L.tts_postnet_workspace_bytes.argtypes = [C.POINTER(TtsPostnetConfig)]
    L.tts_postnet_create.argtypes = [C.POINTER(TtsPostnetConfig), C.POINTER(TtsPostnetWeights), vp, C.c_size_t, vp,
                                     C.POINTER(vp)]
    L.tts_postnet_run.argtypes = [vp, vp, _ip, _ip, C.c_int, vp]
    L.tts_postnet_run_static.argtypes = [vp, vp, _ip, _ip, C.c_int, vp]
    L.tts_postnet_elapsed_ms.argtypes = [vp, _fp]
    L.tts_postnet_destroy.restype = None
    L.tts_postnet_destroy.argtypes = [vp]
    L.tts_vocoder_workspace_bytes.restype = C.c_size_t
    L.tts_vocoder_workspace_bytes.argtypes = [C.POINTER(TtsVocoderConfig)]
    L.tts_vocoder_create.argtypes = [C.POINTER(TtsVocoderConfig), C.POINTER(TtsVocoderWeights), vp, C.c_size_t, vp,
                                     C.POINTER(vp)]
    L.tts_vocoder_run.argtypes = [vp, vp, _ip, _ip, _ip, C.c_int, vp, _ip]
    L.tts_vocoder_elapsed_ms.argtypes = [vp, _fp]
    L.tts_vocoder_destroy.restype = None
    L.tts_vocoder_destroy.argtypes = [vp]
    L.tts_encoder_workspace_bytes.restype = C.c_size_t
    L.tts_encoder_workspace_bytes.argtypes = [C.POINTER(TtsEncoderConfig)]
    L.tts_encoder_create.argtypes = [C.POINTER(TtsEncoderConfig), C.POINTER(TtsEncoderWeights), vp, C.c_size_t, vp,
                                     C.POINTER(vp)]
    L.tts_encoder_run.argtypes = [vp, _ip, _ip, C.c_int, vp]
    L.tts_encoder_elapsed_ms.argtypes = [vp, _fp]
    L.tts_encoder_destroy.restype = None
    L.tts_encoder_destroy.argtypes = [vp]
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != TTS_OK:
        raise TtsError(rc, lib().tts_last_error().decode("utf-8", "replace"))


def make_config(dims: Dict[str, int], max_pool: int, max_enc_len: int, max_steps: int, chunk_frames: int = 40,
                bf16: bool = False, memory_bf16: Optional[bool] = None, use_graph: bool = True,
                stop_threshold: float = -1.0) -> TtsConfig:
    if memory_bf16 is None:
        memory_bf16 = bf16
    c = TtsConfig()
    for k, v in dims.items():
        setattr(c, k, int(v))
    c.max_pool, c.max_enc_len, c.max_steps, c.chunk_frames = int(max_pool), int(max_enc_len), int(max_steps), int(chunk_frames)
    c.weight_dtype = DTYPE_BF16 if bf16 else DTYPE_F32
    c.memory_dtype = DTYPE_BF16 if memory_bf16 else DTYPE_F32
    c.use_graph = int(bool(use_graph))
    c.stop_threshold = float(stop_threshold)
    return c


def workspace_bytes(cfg: TtsConfig) -> int:
    return int(lib().tts_pool_workspace_bytes(C.byref(cfg)))


class Pool:
    """tts_pool_* calls on one pool; owns the torch arena and stream."""

    def __init__(self, cfg: TtsConfig, weights: Dict[str, np.ndarray], device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the decoder step has no CPU path")
        self._torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = workspace_bytes(cfg)
        if nbytes == 0:
            _check(TTS_E_INVAL)
        with torch.cuda.device(self.device):
            self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.stream = torch.cuda.Stream(device=self.device)
        self._warr = {n: np.ascontiguousarray(weights[n], dtype=np.float32) for n in WEIGHT_FIELDS}
        w = TtsWeights(*[self._warr[n].ctypes.data_as(_fp) for n in WEIGHT_FIELDS])
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().tts_pool_create(C.byref(cfg), C.byref(w), C.c_void_p(self.arena.data_ptr()), nbytes,
                                         C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self._h = h
        self.n_mel = cfg.n_mel
        self.chunk = cfg.chunk_frames

    # -- the five pool calls
    def add_request(self, enc_out, n_steps: int) -> int:
        """enc_out: numpy fp32 [L, enc_dim] (host) or a torch CUDA fp32 tensor (device)."""
        rid = C.c_int64()
        if isinstance(enc_out, np.ndarray):
            a = np.ascontiguousarray(enc_out, dtype=np.float32)
            ptr, L = a.ctypes.data, a.shape[0]
        else:
            # read by work queued on the pool's stream after this call returns: a temporary copy could be gone by then
            a = enc_out
            assert a.is_cuda and a.dtype == self._torch.float32 and a.is_contiguous()
            ptr, L = a.data_ptr(), a.shape[0]
        _check(lib().tts_pool_add_request(self._h, C.c_void_p(ptr), int(L), int(n_steps), C.byref(rid)))
        return rid.value

    def add_requests(self, enc_outs, n_steps) -> list:
        """Several requests in one call; each enc_out as in add_request."""
        n = len(enc_outs)
        keep, ptrs, Ls = [], (C.c_void_p * max(n, 1))(), (C.c_int * max(n, 1))()
        for i, e in enumerate(enc_outs):
            if isinstance(e, np.ndarray):
                a = np.ascontiguousarray(e, dtype=np.float32)
                ptrs[i] = a.ctypes.data
            else:
                a = e
                assert a.is_cuda and a.dtype == self._torch.float32 and a.is_contiguous()
                ptrs[i] = a.data_ptr()
            Ls[i] = a.shape[0]
            keep.append(a)
        ns = (C.c_int * max(n, 1))(*[int(x) for x in n_steps])
        ids = (C.c_int64 * max(n, 1))()
        _check(lib().tts_pool_add_requests(self._h, n, ptrs, Ls, ns, ids))
        return [ids[i] for i in range(n)]

    def add_request_raw(self, ptr: int, L: int, n_steps: int) -> int:
        rid = C.c_int64()
        _check(lib().tts_pool_add_request(self._h, C.c_void_p(ptr), int(L), int(n_steps), C.byref(rid)))
        return rid.value

    def step(self) -> int:
        n = C.c_int()
        _check(lib().tts_pool_step(self._h, C.byref(n)))
        return n.value

    def step_n(self, n: int) -> int:
        frames = C.c_int64()
        _check(lib().tts_pool_step_n(self._h, int(n), C.byref(frames)))
        return frames.value

    def drain_chunk(self, rid: int) -> Tuple[np.ndarray, bool]:
        buf = np.empty((self.chunk, self.n_mel), np.float32)
        n, fin = C.c_int(), C.c_int()
        _check(lib().tts_pool_drain_chunk(self._h, rid, buf.ctypes.data_as(_fp), C.byref(n), C.byref(fin)))
        return buf[: n.value], bool(fin.value)

    def retire(self, rid: int) -> None:
        _check(lib().tts_pool_retire(self._h, rid))

    # -- helpers
    def stop_logits(self, rid: int, first: int, count: int) -> np.ndarray:
        buf = np.empty(count, np.float32)
        _check(lib().tts_pool_get_stop_logits(self._h, rid, first, count, buf.ctypes.data_as(_fp)))
        return buf

    def get_state(self, rid: int, name: str) -> np.ndarray:
        buf = np.empty(max(self.cfg.max_enc_len, 1024), np.float32)
        n = C.c_int()
        _check(lib().tts_pool_get_state(self._h, rid, STATE[name], buf.ctypes.data_as(_fp), buf.shape[0], C.byref(n)))
        return buf[: n.value].copy()

    def set_state(self, rid: int, name: str, value) -> None:
        v = np.ascontiguousarray(value, np.float32).ravel()
        _check(lib().tts_pool_set_state(self._h, rid, STATE[name], v.ctypes.data_as(_fp), v.shape[0]))

    def set_wait_polls(self, polls: int) -> None:
        _check(lib().tts_pool_set_wait_polls(self._h, int(polls)))

    def frames(self, rid: int) -> Tuple[int, bool]:
        n, fin = C.c_int(), C.c_int()
        _check(lib().tts_pool_frames(self._h, rid, C.byref(n), C.byref(fin)))
        return n.value, bool(fin.value)

    def size(self) -> int:
        return lib().tts_pool_size(self._h)

    def n_active(self) -> int:
        return lib().tts_pool_n_active(self._h)

    def span(self) -> int:
        return lib().tts_pool_span(self._h)

    def moves(self) -> int:
        return lib().tts_pool_moves(self._h)

    def lost(self, rid: int) -> bool:
        """True if the device ended the request early because a step could not be completed for it."""
        v = C.c_int()
        _check(lib().tts_pool_lost(self._h, rid, C.byref(v)))
        return bool(v.value)

    def sync(self) -> None:
        _check(lib().tts_pool_sync(self._h))

    def timing(self, on: bool) -> None:
        _check(lib().tts_pool_timing(self._h, int(on)))

    def elapsed_ms(self) -> float:
        ms = C.c_float()
        _check(lib().tts_pool_elapsed_ms(self._h, C.byref(ms)))
        return ms.value

    KERNEL_NAMES = ("k_lstm_att", "k_lsa", "k_lstm_dec", "k_proj")

    def kernel_times_us(self, n_steps: int) -> Dict[str, float]:
        """Average device time of each kernel over n un-graphed, event-bracketed steps."""
        buf = (C.c_float * 8)()
        nk = C.c_int()
        _check(lib().tts_pool_kernel_times(self._h, int(n_steps), buf, 8, C.byref(nk)))
        out = {self.KERNEL_NAMES[i]: float(buf[i]) for i in range(nk.value)}
        out["event_cost"] = float(buf[nk.value])
        if buf[nk.value + 1] > 0:
            out["k_proj_last_step"] = float(buf[nk.value + 1])
        return out

    def drain_all(self, rid: int) -> np.ndarray:
        """Every remaining frame of a finished request (host convenience loop over drain_chunk)."""
        out = []
        while True:
            chunk, fin = self.drain_chunk(rid)
            if chunk.shape[0]:
                out.append(chunk.copy())
            if fin or chunk.shape[0] == 0:
                break
        return np.concatenate(out, axis=0) if out else np.zeros((0, self.n_mel), np.float32)

    def chunk_window(self, rid: int, context: int, d_dst) -> Tuple[int, int, bool]:
        """Next chunk of `rid` preceded by up to `context` earlier frames, into the CUDA fp32 tensor d_dst
        ([>= context + chunk, n_mel]); returns (context frames copied, chunk frames, finished)."""
        assert d_dst.is_cuda and d_dst.dtype == self._torch.float32 and d_dst.is_contiguous()
        assert d_dst.numel() >= (context + self.chunk) * self.n_mel
        c, n, fin = C.c_int(), C.c_int(), C.c_int()
        _check(lib().tts_pool_chunk_window(self._h, rid, int(context), C.c_void_p(d_dst.data_ptr()), C.byref(c),
                                           C.byref(n), C.byref(fin)))
        return c.value, n.value, bool(fin.value)

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().tts_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Book:
    """Host-only bookkeeping model (tts_book_*): pooling semantics without a device."""

    def __init__(self, max_pool: int, max_enc_len: int, max_steps: int, chunk_frames: int):
        self._h = lib().tts_book_create(max_pool, max_enc_len, max_steps, chunk_frames)
        if not self._h:
            raise ValueError("tts_book_create rejected its arguments")
        self.max_pool = max_pool

    def add(self, L: int, n_steps: int) -> int:
        rid = C.c_int64()
        _check(lib().tts_book_add(self._h, L, n_steps, C.byref(rid)))
        return rid.value

    def step(self):
        ids = (C.c_int64 * self.max_pool)()
        n = C.c_int()
        _check(lib().tts_book_step(self._h, ids, C.byref(n)))
        return [ids[i] for i in range(n.value)]

    def drain(self, rid: int):
        first, n, fin = C.c_int(), C.c_int(), C.c_int()
        _check(lib().tts_book_drain(self._h, rid, C.byref(first), C.byref(n), C.byref(fin)))
        return first.value, n.value, bool(fin.value)

    def retire(self, rid: int) -> None:
        _check(lib().tts_book_retire(self._h, rid))

    def slot(self, rid: int) -> int:
        return lib().tts_book_slot(self._h, rid)

    def compact(self, min_span: int = 16):
        src, dst = (C.c_int * self.max_pool)(), (C.c_int * self.max_pool)()
        n = lib().tts_book_compact(self._h, min_span, src, dst, self.max_pool)
        _check(min(n, 0))
        return [(src[i], dst[i]) for i in range(n)]

    def close(self):
        if self._h:
            lib().tts_book_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_postnet_config(max_columns: int, bf16: bool = False, n_mel: int = 80, channels: int = 512) -> TtsPostnetConfig:
    return TtsPostnetConfig(n_mel, channels, int(max_columns), DTYPE_BF16 if bf16 else DTYPE_F32)


def postnet_workspace_bytes(cfg: TtsPostnetConfig) -> int:
    return int(lib().tts_postnet_workspace_bytes(C.byref(cfg)))


class Postnet:
    """tts_postnet_* calls; owns its torch arena.  `stream` is a torch.cuda.Stream (e.g. a Pool's)."""

    def __init__(self, cfg: TtsPostnetConfig, conv_w, conv_b, stream=None, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the PostNet has no CPU path")
        self._torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = postnet_workspace_bytes(cfg)
        if nbytes == 0:
            _check(TTS_E_INVAL)
        with torch.cuda.device(self.device):
            self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        self._w = [np.ascontiguousarray(a, np.float32) for a in conv_w]
        self._b = [np.ascontiguousarray(a, np.float32) for a in conv_b]
        w = TtsPostnetWeights((_fp * 5)(*[a.ctypes.data_as(_fp) for a in self._w]),
                              (_fp * 5)(*[a.ctypes.data_as(_fp) for a in self._b]))
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().tts_postnet_create(C.byref(cfg), C.byref(w), C.c_void_p(self.arena.data_ptr()), nbytes,
                                            C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self._h = h

    def run_device(self, d_mel, win_len, keep_from, d_out, static: bool = False) -> None:
        """d_mel / d_out: CUDA fp32 tensors (packed windows in, packed chunks out); queued on the stream.
        static: tts_postnet_run_static, the call that allocates nothing (its scratch is the library's static array)."""
        wl = np.ascontiguousarray(win_len, np.int32)
        kf = np.ascontiguousarray(keep_from, np.int32)
        assert d_mel.is_cuda and d_out.is_cuda and d_mel.is_contiguous() and d_out.is_contiguous()
        assert d_mel.numel() >= int(wl.sum()) * self.cfg.n_mel and d_out.numel() >= int((wl - kf).sum()) * self.cfg.n_mel
        fn = lib().tts_postnet_run_static if static else lib().tts_postnet_run
        with self._torch.cuda.device(self.device):
            _check(fn(self._h, C.c_void_p(d_mel.data_ptr()), wl.ctypes.data_as(_ip),
                      kf.ctypes.data_as(_ip), int(wl.shape[0]), C.c_void_p(d_out.data_ptr())))

    def run(self, windows, keep_from) -> list:
        """windows: list of numpy [T_i, n_mel]; returns the post-processed chunks as numpy arrays."""
        torch = self._torch
        wl = [int(w.shape[0]) for w in windows]
        packed = np.ascontiguousarray(np.concatenate(windows, axis=0), np.float32)
        n_out = sum(t - k for t, k in zip(wl, keep_from))
        with torch.cuda.stream(self.stream):
            d_in = torch.from_numpy(packed).to(self.device, non_blocking=False)
            d_out = torch.empty((n_out, self.cfg.n_mel), dtype=torch.float32, device=self.device)
        self.stream.synchronize()
        self.run_device(d_in, wl, keep_from, d_out)
        self.stream.synchronize()
        out = d_out.cpu().numpy()
        res, r = [], 0
        for t, k in zip(wl, keep_from):
            res.append(out[r:r + t - k])
            r += t - k
        return res

    def elapsed_ms(self) -> float:
        ms = C.c_float()
        _check(lib().tts_postnet_elapsed_ms(self._h, C.byref(ms)))
        return ms.value

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().tts_postnet_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_vocoder_config(overlap: int, max_chunk: int, max_requests: int, max_batch: int, bf16: bool = False,
                        n_mel: int = 80, c0: int = 128) -> TtsVocoderConfig:
    return TtsVocoderConfig(n_mel, c0, int(overlap), int(max_chunk), int(max_requests), int(max_batch),
                            DTYPE_BF16 if bf16 else DTYPE_F32)


def vocoder_workspace_bytes(cfg: TtsVocoderConfig) -> int:
    return int(lib().tts_vocoder_workspace_bytes(C.byref(cfg)))


class Vocoder:
    """tts_vocoder_* calls; owns its torch arena.  `weights` is the dict of synth.make_vocoder_weights."""

    def __init__(self, cfg: TtsVocoderConfig, weights: dict, stream=None, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the vocoder has no CPU path")
        self._torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = vocoder_workspace_bytes(cfg)
        if nbytes == 0:
            _check(TTS_E_INVAL)
        with torch.cuda.device(self.device):
            self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        keep = []

        def ptr(a):
            a = np.ascontiguousarray(a, np.float32)
            keep.append(a)
            return a.ctypes.data_as(_fp)

        w = TtsVocoderWeights()
        w.pre_w, w.pre_b, w.post_w, w.post_b = ptr(weights["pre_w"]), ptr(weights["pre_b"]), ptr(weights["post_w"]), ptr(weights["post_b"])
        for s_ in range(4):
            w.up_w[s_], w.up_b[s_] = ptr(weights["up_w"][s_]), ptr(weights["up_b"][s_])
            for b_ in range(3):
                for i in range(6):
                    w.res_w[s_][b_][i] = ptr(weights["res_w"][s_][b_][i])
                    w.res_b[s_][b_][i] = ptr(weights["res_b"][s_][b_][i])
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().tts_vocoder_create(C.byref(cfg), C.byref(w), C.c_void_p(self.arena.data_ptr()), nbytes,
                                            C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self._h = h

    def run_device(self, d_mel, n_frames, state_slot, flags, d_audio) -> list:
        """d_mel: CUDA fp32 [sum n_frames, n_mel] (the chunks back to back); d_audio: CUDA fp32 with room for
        256 * (overlap + n_frames[i]) samples per chunk.  Queued on the stream; returns the responses' lengths."""
        nf = np.ascontiguousarray(n_frames, np.int32)
        sl = np.ascontiguousarray(state_slot, np.int32)
        fl = np.ascontiguousarray(flags, np.int32)
        n = int(nf.shape[0])
        assert sl.shape[0] == n and fl.shape[0] == n
        assert d_mel.is_cuda and d_audio.is_cuda and d_mel.is_contiguous() and d_audio.is_contiguous()
        assert d_mel.dtype == self._torch.float32 and d_audio.dtype == self._torch.float32
        assert d_mel.numel() >= int(nf.sum()) * self.cfg.n_mel
        assert d_audio.numel() >= int((nf + self.cfg.overlap).sum()) * VOCODER_HOP
        out = np.zeros(n, np.int32)
        _check(lib().tts_vocoder_run(self._h, C.c_void_p(d_mel.data_ptr()), nf.ctypes.data_as(_ip), sl.ctypes.data_as(_ip),
                                     fl.ctypes.data_as(_ip), n, C.c_void_p(d_audio.data_ptr()), out.ctypes.data_as(_ip)))
        return [int(x) for x in out]

    def run(self, chunks, state_slot, flags) -> list:
        """chunks: list of numpy [n_i, n_mel]; returns the responses as numpy arrays."""
        torch = self._torch
        nf = [int(c.shape[0]) for c in chunks]
        packed = np.ascontiguousarray(np.concatenate(chunks, axis=0), np.float32)
        with torch.cuda.stream(self.stream):
            d_in = torch.from_numpy(packed).to(self.device, non_blocking=False)
            d_out = torch.empty(sum(n + self.cfg.overlap for n in nf) * VOCODER_HOP, dtype=torch.float32, device=self.device)
        self.stream.synchronize()
        lens = self.run_device(d_in, nf, state_slot, flags, d_out)
        self.stream.synchronize()
        out = d_out.cpu().numpy()
        res, r = [], 0
        for n in lens:
            res.append(out[r:r + n])
            r += n
        return res

    def elapsed_ms(self) -> float:
        ms = C.c_float()
        _check(lib().tts_vocoder_elapsed_ms(self._h, C.byref(ms)))
        return ms.value

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().tts_vocoder_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_encoder_config(max_tokens: int, max_len: int, bf16: bool = False, vocab=(128, 4, 4, 4), dim: int = 512,
                        hid: int = 256) -> TtsEncoderConfig:
    return TtsEncoderConfig(dim, hid, (C.c_int * 4)(*vocab), int(max_tokens), int(max_len), DTYPE_BF16 if bf16 else DTYPE_F32)


def encoder_workspace_bytes(cfg: TtsEncoderConfig) -> int:
    return int(lib().tts_encoder_workspace_bytes(C.byref(cfg)))


class Encoder:
    """tts_encoder_* calls; owns its torch arena.  `weights` is the dict of synth.make_encoder_weights."""

    def __init__(self, cfg: TtsEncoderConfig, weights: dict, stream=None, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the encoder has no CPU path")
        self._torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = encoder_workspace_bytes(cfg)
        if nbytes == 0:
            _check(TTS_E_INVAL)
        with torch.cuda.device(self.device):
            self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        keep = []

        def ptr(a):
            a = np.ascontiguousarray(a, np.float32)
            keep.append(a)
            return a.ctypes.data_as(_fp)

        w = TtsEncoderWeights()
        for t in range(4):
            w.tables[t] = ptr(weights["tables"][t])
        for i in range(3):
            w.conv_w[i], w.conv_b[i] = ptr(weights["conv_w"][i]), ptr(weights["conv_b"][i])
        for d, k in enumerate(("f", "b")):
            w.w_ih[d], w.w_hh[d], w.b[d] = ptr(weights["w_ih_" + k]), ptr(weights["w_hh_" + k]), ptr(weights["b_" + k])
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().tts_encoder_create(C.byref(cfg), C.byref(w), C.c_void_p(self.arena.data_ptr()), nbytes,
                                            C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self._h = h

    def run_device(self, ids_list, d_out) -> list:
        """ids_list: one int array [4, L_i] per request; d_out: CUDA fp32 [>= sum L_i, 2 hid].  Queued on the stream;
        returns the first row of every request in d_out."""
        lens = np.ascontiguousarray([a.shape[1] for a in ids_list], np.int32)
        ids = np.ascontiguousarray(np.concatenate([np.asarray(a, np.int32) for a in ids_list], axis=1))   # [4, total]
        total = int(lens.sum())
        assert ids.shape == (4, total)
        assert d_out.is_cuda and d_out.is_contiguous() and d_out.dtype == self._torch.float32
        assert d_out.numel() >= total * 2 * self.cfg.hid
        _check(lib().tts_encoder_run(self._h, ids.ctypes.data_as(_ip), lens.ctypes.data_as(_ip), int(lens.shape[0]),
                                     C.c_void_p(d_out.data_ptr())))
        return [int(x) for x in np.concatenate([[0], np.cumsum(lens)[:-1]])]

    def run(self, ids_list) -> list:
        """Returns F_enc of every request as numpy [L_i, 2 hid]."""
        torch = self._torch
        total = sum(a.shape[1] for a in ids_list)
        with torch.cuda.stream(self.stream):
            d_out = torch.empty((max(total, 1), 2 * self.cfg.hid), dtype=torch.float32, device=self.device)
        self.stream.synchronize()
        starts = self.run_device(ids_list, d_out)
        self.stream.synchronize()
        out = d_out.cpu().numpy()
        return [out[s:s + a.shape[1]] for s, a in zip(starts, ids_list)]

    def elapsed_ms(self) -> float:
        ms = C.c_float()
        _check(lib().tts_encoder_elapsed_ms(self._h, C.byref(ms)))
        return ms.value

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().tts_encoder_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
