"""Pins for the vocoder oracle (oracle/vocoder_oracle.c): library routines (torch's conv1d and
conv_transpose1d), impulse responses worked by hand, the generator recomposed from the library routines,
length / locality properties, and the closed forms of the equal-power fade (Sec. 2.1.4, Eq. 3, Eq. 4)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as orc
from paper_2211_13939_amd import synth


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float64))


@pytest.mark.parametrize("c_in,c_out,k,dil,T", [(3, 5, 3, 1, 11), (8, 8, 7, 3, 40), (4, 2, 11, 5, 23), (80, 6, 7, 1, 9)])
def test_conv1d_equals_library_routine(c_in, c_out, k, dil, T):
    rng = np.random.default_rng(k * 100 + dil)
    w = rng.standard_normal((c_out, c_in, k)).astype(np.float32)
    b = rng.standard_normal(c_out).astype(np.float32)
    x = rng.standard_normal((T, c_in))
    want = F.conv1d(_t(x).T[None], _t(w), _t(b), dilation=dil, padding=dil * (k - 1) // 2)[0].T.numpy()
    np.testing.assert_allclose(orc.conv1d(w, b, x, dil), want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("c_in,c_out,stride,T", [(4, 2, 8, 7), (6, 3, 2, 13), (16, 8, 8, 5)])
def test_conv_transpose1d_equals_library_routine(c_in, c_out, stride, T):
    rng = np.random.default_rng(stride * 7 + T)
    k, pad = 2 * stride, stride // 2
    w = rng.standard_normal((c_in, c_out, k)).astype(np.float32)
    b = rng.standard_normal(c_out).astype(np.float32)
    x = rng.standard_normal((T, c_in))
    want = F.conv_transpose1d(_t(x).T[None], _t(w), _t(b), stride=stride, padding=pad)[0].T.numpy()
    got = orc.conv_transpose1d(w, b, x, stride, pad)
    assert got.shape == (T * stride, c_out)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_conv1d_impulse_by_hand():
    """One channel, kernel (1, 2, 3), dilation 2: y[t] = 1 x[t-2] + 2 x[t] + 3 x[t+2]; an impulse at t = 4 gives
    3 at t = 2, 2 at t = 4, 1 at t = 6; at the border the missing neighbour is zero."""
    w = np.array([[[1.0, 2.0, 3.0]]], np.float32)
    b = np.array([0.5], np.float32)
    x = np.zeros((8, 1)); x[4, 0] = 1.0
    y = orc.conv1d(w, b, x, dil=2)[:, 0]
    np.testing.assert_allclose(y, np.array([0, 0, 3, 0, 2, 0, 1, 0]) + 0.5)
    x = np.zeros((8, 1)); x[0, 0] = 1.0; x[7, 0] = 10.0
    y = orc.conv1d(w, b, x, dil=2)[:, 0]
    np.testing.assert_allclose(y, np.array([2, 0, 1, 0, 0, 30, 0, 20]) + 0.5)


def test_conv_transpose1d_impulse_by_hand():
    """Stride 2, kernel 4, padding 1, kernel (1, 2, 3, 4): input t spreads w[j] to output 2 t + j - 1, so an impulse
    at t = 1 of 3 inputs lands as (1, 2, 3, 4) on outputs 1..4; the first input's tap 0 falls off the front."""
    w = np.array([[[1.0, 2.0, 3.0, 4.0]]], np.float32)
    b = np.zeros(1, np.float32)
    x = np.zeros((3, 1)); x[1, 0] = 1.0
    np.testing.assert_allclose(orc.conv_transpose1d(w, b, x, 2, 1)[:, 0], [0, 1, 2, 3, 4, 0])
    x = np.zeros((3, 1)); x[0, 0] = 1.0
    np.testing.assert_allclose(orc.conv_transpose1d(w, b, x, 2, 1)[:, 0], [2, 3, 4, 0, 0, 0])


def _library_generator(w, mel, slope=0.1, rates=(8, 8, 2, 2), block_k=(3, 7, 11), dils=(1, 3, 5)):
    """The generator written with torch's routines (fp64), for the comparison below."""
    x = F.conv1d(_t(mel).T[None], _t(w["pre_w"]), _t(w["pre_b"]), padding=3)
    for s, u in enumerate(rates):
        x = F.conv_transpose1d(F.leaky_relu(x, slope), _t(w["up_w"][s]), _t(w["up_b"][s]), stride=u, padding=u // 2)
        acc = None
        for bk, k in enumerate(block_k):
            r = x
            for i, d in enumerate(dils):
                t = F.conv1d(F.leaky_relu(r, slope), _t(w["res_w"][s][bk][2 * i]), _t(w["res_b"][s][bk][2 * i]),
                             dilation=d, padding=d * (k - 1) // 2)
                t = F.conv1d(F.leaky_relu(t, slope), _t(w["res_w"][s][bk][2 * i + 1]), _t(w["res_b"][s][bk][2 * i + 1]),
                             padding=(k - 1) // 2)
                r = r + t
            acc = r if acc is None else acc + r
        x = acc / len(block_k)
    x = F.conv1d(F.leaky_relu(x, slope), _t(w["post_w"]), _t(w["post_b"]), padding=3)
    return torch.tanh(x)[0, 0].numpy()


def test_generator_equals_composition_of_library_routines():
    w = synth.make_vocoder_weights(seed=5)
    W = orc.VocoderWeights(w)
    rng = np.random.default_rng(3)
    for T in (1, 2, 9):
        mel = rng.standard_normal((T, 80))
        got = orc.generator(W, mel)
        assert got.shape == (T * 256,)
        np.testing.assert_allclose(got, _library_generator(w, mel), rtol=0, atol=1e-11)


def test_generator_small_architecture_and_locality():
    """A narrower generator (16 initial channels, rates 2, 2): output length = 4 T, and a change of one mel frame far
    from a sample does not reach it (the receptive field is finite), while it does change samples next to it."""
    w = synth.make_vocoder_weights(seed=8, c0=16, rates=(2, 2))
    W = orc.VocoderWeights(w, rates=(2, 2))
    rng = np.random.default_rng(4)
    mel = rng.standard_normal((200, 80))
    a = orc.generator(W, mel)
    assert a.shape == (800,) and np.all(np.abs(a) < 1.0)
    mel2 = mel.copy(); mel2[100] += 1.0
    b = orc.generator(W, mel2)
    np.testing.assert_allclose(b, _library_generator(w, mel2, rates=(2, 2)), rtol=0, atol=1e-11)
    # receptive field in frames: conv_pre 3; stage 1 (rate 2): blocks up to kernel 11: sum over pairs of
    # 5 d + 5 = 60 positions = 30 frames; plus one for the transposed convolution; stage 2 (rate 4): 60 / 4 = 15; post 1
    far = 3 + 1 + 30 + 1 + 15 + 1
    changed = np.nonzero(a != b)[0]
    assert changed.size > 0 and abs(int(np.median(changed)) - 402) < 40
    assert changed.min() >= (100 - far) * 4 and changed.max() < (100 + far + 1) * 4


def test_fade_is_equal_power():
    for n in (1, 2, 1024, 2048):
        al, be = orc.fade(n)
        np.testing.assert_allclose(al * al + be * be, 1.0, rtol=0, atol=1e-15)
        np.testing.assert_allclose(al, be[::-1], rtol=0, atol=1e-15)       # fade-in mirrors fade-out
        assert np.all(np.diff(al) > 0) if n > 1 else True
    al, be = orc.fade(2)
    np.testing.assert_allclose(al, [np.sin(np.pi / 8), np.sin(3 * np.pi / 8)], atol=1e-15)
    al, be = orc.fade(1)
    np.testing.assert_allclose([al[0], be[0]], [np.sqrt(0.5), np.sqrt(0.5)], atol=1e-15)


def test_crossfade_by_hand():
    cur = np.array([1.0, 1.0, 1.0, 1.0])
    pre = np.array([2.0, 2.0, 2.0, 2.0])
    u = (np.arange(4) + 0.5) / 4
    np.testing.assert_allclose(orc.crossfade(cur, pre), np.sin(np.pi / 2 * u) + 2 * np.cos(np.pi / 2 * u), atol=1e-15)
    # only the current chunk: fade-in; only the previous: fade-out
    np.testing.assert_allclose(orc.crossfade(cur, 0 * pre), np.sin(np.pi / 2 * u), atol=1e-15)
    np.testing.assert_allclose(orc.crossfade(0 * cur, pre), 2 * np.cos(np.pi / 2 * u), atol=1e-15)


def test_stream_tiles_the_utterance_and_follows_eq3_eq4():
    """Three chunks (8, 8, 5 frames), overlap 2, a small generator (hop 4).  The responses tile the utterance; the
    first is G(M_1) without its last overlap * hop samples; the second starts with the fade of G([tail(M_1), M_2])'s
    head against G(M_1)'s tail (Eq. 3) and the third is built on M_2's tail and S_2's tail (Eq. 4)."""
    w = synth.make_vocoder_weights(seed=9, c0=16, rates=(2, 2))
    W = orc.VocoderWeights(w, rates=(2, 2))
    rng = np.random.default_rng(6)
    m = [rng.standard_normal((n, 80)) for n in (8, 8, 5)]
    ov, hop = 2, 4
    vs = orc.VocoderStream(W, ov)
    out = [vs.chunk(m[0], False), vs.chunk(m[1], False), vs.chunk(m[2], True)]
    assert [o.shape[0] for o in out] == [(8 - ov) * hop, 8 * hop, (5 + ov) * hop]
    assert sum(o.shape[0] for o in out) == 21 * hop
    s1 = _library_generator(w, m[0], rates=(2, 2))
    np.testing.assert_allclose(out[0], s1[:-ov * hop], atol=1e-11)
    s2 = _library_generator(w, np.concatenate([m[0][-ov:], m[1]]), rates=(2, 2))
    u = (np.arange(ov * hop) + 0.5) / (ov * hop)
    head2 = np.sin(np.pi / 2 * u) * s2[:ov * hop] + np.cos(np.pi / 2 * u) * s1[-ov * hop:]
    np.testing.assert_allclose(out[1][:ov * hop], head2, atol=1e-11)
    np.testing.assert_allclose(out[1][ov * hop:], s2[ov * hop:-ov * hop], atol=1e-11)
    s3 = _library_generator(w, np.concatenate([m[1][-ov:], m[2]]), rates=(2, 2))
    head3 = np.sin(np.pi / 2 * u) * s3[:ov * hop] + np.cos(np.pi / 2 * u) * s2[-ov * hop:]
    np.testing.assert_allclose(out[2], np.concatenate([head3, s3[ov * hop:]]), atol=1e-11)


def test_stream_without_overlap_is_plain_concatenation():
    w = synth.make_vocoder_weights(seed=10, c0=16, rates=(2, 2))
    W = orc.VocoderWeights(w, rates=(2, 2))
    rng = np.random.default_rng(7)
    m = [rng.standard_normal((n, 80)) for n in (6, 3)]
    vs = orc.VocoderStream(W, 0)
    got = np.concatenate([vs.chunk(m[0], False), vs.chunk(m[1], True)])
    want = np.concatenate([orc.generator(W, m[0]), orc.generator(W, m[1])])
    np.testing.assert_allclose(got, want, atol=0)
