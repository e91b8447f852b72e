"""Seeded synthetic inputs for the pooled decoder step.

This module only *draws numbers*: decoder dimensions, random weights, random
encoder outputs, request lengths, step counts and arrival times.  It contains
none of the decoder's arithmetic and imports neither the HIP binding nor the
CPU oracle, so both can be fed from it.

The paper's own workload (a model trained on a Mandarin corpus, texts of three
length classes with mean durations 2.64 / 4.08 / 7.00 / 4.54 s, Sec. 3.1) is
not available; the workloads below stand in for it with the same shapes:
encoder outputs of a few tens to a few hundred tokens and a few hundred mel
frames per request.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

# Tacotron-2 decoder dimensions ("same model parameters as the original",
# Sec. 3.1); the concrete numbers are this build's workload definition.
DIMS: Dict[str, int] = dict(
    n_mel=80,
    prenet_dim=256,
    enc_dim=512,
    att_rnn_dim=1024,
    dec_rnn_dim=1024,
    att_dim=128,
    loc_filters=32,
    loc_kernel=31,
    loc_in_channels=2,
)

WEIGHT_SEED = 1234
WEIGHT_STD = 0.05

# Field order of the weight struct at the C boundary; tensors are drawn in
# this order from one generator.
WEIGHT_FIELDS = (
    "prenet1", "prenet2",
    "att_w_ih", "att_w_hh", "att_b",
    "q_w", "mem_w", "loc_conv", "loc_w", "v",
    "dec_w_ih", "dec_w_hh", "dec_b",
    "mel_w", "mel_b", "stop_w", "stop_b",
)


def weight_shapes(dims: Dict[str, int] = DIMS) -> Dict[str, tuple]:
    d = dims
    att_in = d["prenet_dim"] + d["enc_dim"]
    dec_in = d["att_rnn_dim"] + d["enc_dim"]
    proj_in = d["dec_rnn_dim"] + d["enc_dim"]
    return {
        "prenet1": (d["prenet_dim"], d["n_mel"]),
        "prenet2": (d["prenet_dim"], d["prenet_dim"]),
        "att_w_ih": (4 * d["att_rnn_dim"], att_in),
        "att_w_hh": (4 * d["att_rnn_dim"], d["att_rnn_dim"]),
        "att_b": (4 * d["att_rnn_dim"],),
        "q_w": (d["att_dim"], d["att_rnn_dim"]),
        "mem_w": (d["att_dim"], d["enc_dim"]),
        "loc_conv": (d["loc_filters"], d["loc_in_channels"], d["loc_kernel"]),
        "loc_w": (d["att_dim"], d["loc_filters"]),
        "v": (d["att_dim"],),
        "dec_w_ih": (4 * d["dec_rnn_dim"], dec_in),
        "dec_w_hh": (4 * d["dec_rnn_dim"], d["dec_rnn_dim"]),
        "dec_b": (4 * d["dec_rnn_dim"],),
        "mel_w": (d["n_mel"], proj_in),
        "mel_b": (d["n_mel"],),
        "stop_w": (1, proj_in),
        "stop_b": (1,),
    }


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result is fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    out = rounded.astype(np.uint32).view(np.float32)
    # NaN/Inf are never drawn here; keep them unchanged if they appear.
    bad = ~np.isfinite(x)
    if bad.any():
        out = out.copy()
        out[bad] = x[bad]
    return out.reshape(x.shape)


def make_weights(seed: int = WEIGHT_SEED, dims: Dict[str, int] = DIMS,
                 bf16: bool = False, std: float = WEIGHT_STD) -> Dict[str, np.ndarray]:
    """Every tensor ~ N(0, std^2) in fp32, drawn in WEIGHT_FIELDS order.

    With ``bf16`` the matrices are then rounded to bfloat16 values (still held
    in fp32 arrays); the bias vectors stay fp32.
    """
    rng = np.random.default_rng(seed)
    shapes = weight_shapes(dims)
    w = {}
    for name in WEIGHT_FIELDS:
        t = (rng.standard_normal(shapes[name]) * std).astype(np.float32)
        if bf16 and not name.endswith("_b"):
            t = round_to_bf16(t)
        w[name] = np.ascontiguousarray(t)
    return w


POSTNET = dict(n_layers=5, kernel=5, channels=512)


def make_postnet_weights(seed: int = 1235, bf16: bool = False, n_mel: int = 80, channels: int = 512,
                         n_layers: int = 5, std: float = 0.05):
    """PostNet stand-in: conv weights [c_out, c_in, 5] and biases [c_out] ~ N(0, std^2) (weights rounded
    to bf16 values when bf16).  Returns (list of weights, list of biases)."""
    rng = np.random.default_rng(seed)
    ws, bs = [], []
    for l in range(n_layers):
        c_in = n_mel if l == 0 else channels
        c_out = n_mel if l == n_layers - 1 else channels
        w = (rng.standard_normal((c_out, c_in, POSTNET["kernel"])) * std).astype(np.float32)
        b = (rng.standard_normal(c_out) * std).astype(np.float32)
        ws.append(np.ascontiguousarray(round_to_bf16(w) if bf16 else w))
        bs.append(np.ascontiguousarray(b))
    return ws, bs


VOCODER = dict(c0=128, rates=(8, 8, 2, 2), block_k=(3, 7, 11), dils=(1, 3, 5), k_pre=7, k_post=7, hop=256)


def make_vocoder_weights(seed: int = 1236, bf16: bool = False, n_mel: int = 80, c0: int = 128,
                         rates=(8, 8, 2, 2), block_k=(3, 7, 11), dils=(1, 3, 5)):
    """Generator stand-in (Sec. 3.1: 128 initial channels, upsampling 8, 8, 2, 2).  Every tensor ~ N(0, (g / sqrt(fan_in))^2)
    with g = 1 for conv_pre, the transposed convolutions and conv_post and g = 0.5 inside the residual blocks,
    biases ~ N(0, 0.02^2), so that activations stay of order one; weights rounded to bf16 values when bf16.
    Returns a dict: pre_w [c0, n_mel, 7], pre_b, up_w[s] [c, c/2, 2 u_s], up_b[s],
    res_w[s][block][2 pair + {0: dilated, 1: plain}] [c, c, k], res_b likewise, post_w [1, c_last, 7], post_b."""
    rng = np.random.default_rng(seed)

    def tensor(shape, fan_in, gain):
        w = (rng.standard_normal(shape) * (gain / np.sqrt(fan_in))).astype(np.float32)
        return np.ascontiguousarray(round_to_bf16(w) if bf16 else w)

    def bias(n):
        return np.ascontiguousarray((rng.standard_normal(n) * 0.02).astype(np.float32))

    w = dict(pre_w=tensor((c0, n_mel, 7), n_mel * 7, 1.0), pre_b=bias(c0), up_w=[], up_b=[], res_w=[], res_b=[])
    c = c0
    for u in rates:
        # every output sample of the transposed convolution sees two taps of every input channel
        w["up_w"].append(tensor((c, c // 2, 2 * u), 2 * c, 1.0))
        w["up_b"].append(bias(c // 2))
        c //= 2
        w["res_w"].append([[tensor((c, c, k), c * k, 0.5) for _ in range(2 * len(dils))] for k in block_k])
        w["res_b"].append([[bias(c) for _ in range(2 * len(dils))] for _ in block_k])
    w["post_w"] = tensor((1, c, 7), c * 7, 1.0)
    w["post_b"] = bias(1)
    return w


ENCODER = dict(dim=512, hid=256, n_conv=3, kernel=5, vocab=(128, 4, 4, 4))


def make_encoder_weights(seed: int = 1237, bf16: bool = False, dim: int = 512, hid: int = 256, n_conv: int = 3,
                         vocab=(128, 4, 4, 4)):
    """Encoder stand-in (Eq. 1): four embedding tables (tokens, pw, pph, iph) ~ N(0, 0.5^2), convolutions
    [dim, dim, 5] ~ N(0, 2 / fan_in) (ReLU keeps the scale), biases ~ N(0, 0.02^2), LSTM matrices ~ N(0, 1 / fan_in)
    per direction with one merged bias ~ N(0, 0.05^2); matrices and tables rounded to bf16 values when bf16."""
    rng = np.random.default_rng(seed)

    def mat(shape, std):
        w = (rng.standard_normal(shape) * std).astype(np.float32)
        return np.ascontiguousarray(round_to_bf16(w) if bf16 else w)

    w = dict(tables=[mat((v, dim), 0.5) for v in vocab],
             conv_w=[mat((dim, dim, ENCODER["kernel"]), np.sqrt(2.0 / (dim * ENCODER["kernel"]))) for _ in range(n_conv)],
             conv_b=[np.ascontiguousarray((rng.standard_normal(dim) * 0.02).astype(np.float32)) for _ in range(n_conv)])
    for d in ("f", "b"):
        w["w_ih_" + d] = mat((4 * hid, dim), 1.0 / np.sqrt(dim))
        w["w_hh_" + d] = mat((4 * hid, hid), 1.0 / np.sqrt(hid))
        w["b_" + d] = np.ascontiguousarray((rng.standard_normal(4 * hid) * 0.05).astype(np.float32))
    return w


def encoder_ids(L: int, seed: int, vocab=(128, 4, 4, 4)) -> np.ndarray:
    """Id sequences of one request, int32 [4, L]: phoneme tokens and the three prosodic-structure tokens."""
    rng = np.random.default_rng([seed, 104729, int(L)])
    return np.stack([rng.integers(0, v, size=L) for v in vocab]).astype(np.int32)


@dataclass
class Workload:
    """One synthetic job: per-request encoder lengths, step counts and outputs."""
    name: str
    bf16: bool
    enc_len: np.ndarray            # [n] int32
    n_steps: np.ndarray            # [n] int32
    seed: int
    arrival_s: Optional[np.ndarray] = None   # [n] float64, streaming load only
    chunk_frames: int = 40
    dims: Dict[str, int] = field(default_factory=lambda: dict(DIMS))
    _enc_cache: Dict[int, np.ndarray] = field(default_factory=dict, repr=False)

    @property
    def n_requests(self) -> int:
        return int(self.enc_len.shape[0])

    def encoder_outputs(self, i: int) -> np.ndarray:
        """F_enc of request i, [L_i, enc_dim] ~ N(0,1) fp32 (bf16 values if bf16)."""
        if i not in self._enc_cache:
            rng = np.random.default_rng([self.seed, 7919, int(i)])
            f = rng.standard_normal((int(self.enc_len[i]), self.dims["enc_dim"])).astype(np.float32)
            if self.bf16:
                f = round_to_bf16(f)
            self._enc_cache[i] = np.ascontiguousarray(f)
        return self._enc_cache[i]

    def drop_cache(self) -> None:
        self._enc_cache.clear()


def workload(name: str) -> Workload:
    """The five workloads of this build.

    c1  1 request, fp32, L = 20, 10 steps
    c2  16 requests, fp32, L ~ U{20..100}, 200 steps each, all join at step 0
    c3  64 requests, bf16, L ~ U{30..300}, steps ~ U{100..600}, pool shrinks
    c4  256 requests, bf16, L ~ U{50..400}, 400 steps each
    c5  Poisson arrivals at 100/s over 10 s, bf16, L ~ U{30..300}, steps = 4 L,
        mel drained in 40-frame chunks
    """
    if name == "c1":
        return Workload("c1", False, np.array([20], np.int32), np.array([10], np.int32), 101)
    if name == "c2":
        rng = np.random.default_rng(102)
        L = rng.integers(20, 101, size=16).astype(np.int32)
        return Workload("c2", False, L, np.full(16, 200, np.int32), 102)
    if name == "c3":
        rng = np.random.default_rng(103)
        L = rng.integers(30, 301, size=64).astype(np.int32)
        n = rng.integers(100, 601, size=64).astype(np.int32)
        return Workload("c3", True, L, n, 103)
    if name == "c4":
        rng = np.random.default_rng(104)
        L = rng.integers(50, 401, size=256).astype(np.int32)
        return Workload("c4", True, L, np.full(256, 400, np.int32), 104)
    if name == "c5":
        rng = np.random.default_rng(105)
        rate, horizon = 100.0, 10.0
        gaps = rng.exponential(1.0 / rate, size=int(rate * horizon * 2))
        t = np.cumsum(gaps)
        t = t[t < horizon]
        n = t.shape[0]
        L = rng.integers(30, 301, size=n).astype(np.int32)
        return Workload("c5", True, L, (4 * L).astype(np.int32), 105, arrival_s=t, chunk_frames=40)
    raise KeyError(name)


def small_workload(n_requests: int, lo: int, hi: int, steps_lo: int, steps_hi: int,
                   seed: int, bf16: bool = False) -> Workload:
    """A free-form job for tests: L ~ U{lo..hi}, steps ~ U{steps_lo..steps_hi}."""
    rng = np.random.default_rng(seed)
    L = rng.integers(lo, hi + 1, size=n_requests).astype(np.int32)
    n = rng.integers(steps_lo, steps_hi + 1, size=n_requests).astype(np.int32)
    return Workload(f"small{seed}", bf16, L, n, seed)
