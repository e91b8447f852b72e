"""Pins for the encoder oracle (oracle/encoder_oracle.c; Sec. 2.1.2, Eq. 1): library routines (torch.nn.LSTM with
both directions, torch's conv1d), indexing for the embedding sum, closed forms with zero weights, and the
reversal symmetry of the two LSTM directions."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as orc
from paper_2211_13939_amd import synth


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float64))


def _small(seed=3, dim=16, hid=8, vocab=(9, 3, 3, 2)):
    return synth.make_encoder_weights(seed=seed, dim=dim, hid=hid, vocab=vocab)


def test_embedding_sum_is_indexing():
    w = _small()
    W = orc.EncoderWeights(w)
    ids = synth.encoder_ids(11, 5, vocab=(9, 3, 3, 2))
    want = sum(w["tables"][t].astype(np.float64)[ids[t]] for t in range(4))
    np.testing.assert_allclose(orc.encoder_embed(W, ids), want, rtol=0, atol=1e-15)
    # one table at a time: each id sequence picks from its own table
    for t in range(4):
        z = {**w, "tables": [a if k == t else np.zeros_like(a) for k, a in enumerate(w["tables"])]}
        np.testing.assert_allclose(orc.encoder_embed(orc.EncoderWeights(z), ids), w["tables"][t].astype(np.float64)[ids[t]], atol=1e-15)


@pytest.mark.parametrize("L", [1, 2, 5, 23])
def test_conv_relu_equals_library_routine(L):
    rng = np.random.default_rng(L)
    w = rng.standard_normal((7, 6, 5)).astype(np.float32)
    b = rng.standard_normal(7).astype(np.float32)
    x = rng.standard_normal((L, 6))
    want = F.relu(F.conv1d(_t(x).T[None], _t(w), _t(b), padding=2))[0].T.numpy()
    got = orc.encoder_conv_relu(w, b, x)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    assert (got >= 0).all() and (got == 0).any()


def test_conv_orientation_by_hand():
    """One channel, kernel (1, 2, 3, 4, 5): y[j] = 1 x[j-2] + 2 x[j-1] + 3 x[j] + 4 x[j+1] + 5 x[j+2]."""
    w = np.array([[[1.0, 2.0, 3.0, 4.0, 5.0]]], np.float32)
    x = np.zeros((7, 1)); x[3, 0] = 1.0
    np.testing.assert_allclose(orc.encoder_conv_relu(w, np.zeros(1, np.float32), x)[:, 0], [0, 5, 4, 3, 2, 1, 0])
    np.testing.assert_allclose(orc.encoder_conv_relu(-w, np.full(1, 0.5, np.float32), x)[:, 0], [0.5, 0, 0, 0, 0, 0, 0.5])


def _library_bilstm(w, x):
    dim, hid = w["w_ih_f"].shape[1], w["w_hh_f"].shape[1]
    m = torch.nn.LSTM(dim, hid, bidirectional=True).double()
    with torch.no_grad():
        m.weight_ih_l0.copy_(_t(w["w_ih_f"])); m.weight_hh_l0.copy_(_t(w["w_hh_f"]))
        m.bias_ih_l0.copy_(_t(w["b_f"])); m.bias_hh_l0.zero_()
        m.weight_ih_l0_reverse.copy_(_t(w["w_ih_b"])); m.weight_hh_l0_reverse.copy_(_t(w["w_hh_b"]))
        m.bias_ih_l0_reverse.copy_(_t(w["b_b"])); m.bias_hh_l0_reverse.zero_()
        return m(_t(x)[:, None, :])[0][:, 0, :].numpy()


@pytest.mark.parametrize("L", [1, 2, 9, 40])
def test_bilstm_equals_library_routine(L):
    w = _small(seed=4)
    rng = np.random.default_rng(L + 10)
    x = rng.standard_normal((L, 16))
    lstm = {k: w[k] for k in ("w_ih_f", "w_hh_f", "b_f", "w_ih_b", "w_hh_b", "b_b")}
    np.testing.assert_allclose(orc.bilstm(lstm, x), _library_bilstm(w, x), rtol=0, atol=1e-13)


def test_bilstm_directions_mirror_each_other():
    """Swapping the two directions' weights and reversing the input reverses the output and swaps its halves."""
    w = _small(seed=6)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((13, 16))
    a = orc.bilstm({k: w[k] for k in ("w_ih_f", "w_hh_f", "b_f", "w_ih_b", "w_hh_b", "b_b")}, x)
    sw = dict(w_ih_f=w["w_ih_b"], w_hh_f=w["w_hh_b"], b_f=w["b_b"], w_ih_b=w["w_ih_f"], w_hh_b=w["w_hh_f"], b_b=w["b_f"])
    b = orc.bilstm(sw, x[::-1])
    np.testing.assert_allclose(b[::-1, 8:], a[:, :8], atol=1e-15)
    np.testing.assert_allclose(b[::-1, :8], a[:, 8:], atol=1e-15)
    # the forward half at token j does not see later tokens, the backward half does not see earlier ones
    x2 = x.copy(); x2[7] += 1.0
    c = orc.bilstm({k: w[k] for k in ("w_ih_f", "w_hh_f", "b_f", "w_ih_b", "w_hh_b", "b_b")}, x2)
    assert np.array_equal(c[:7, :8], a[:7, :8]) and not np.array_equal(c[7:, :8], a[7:, :8])
    assert np.array_equal(c[8:, 8:], a[8:, 8:]) and not np.array_equal(c[:8, 8:], a[:8, 8:])


def test_bilstm_zero_weights_closed_form():
    """With zero matrices the gates are the biases: c_t = sig(b_f) c_{t-1} + sig(b_i) tanh(b_g), h_t = sig(b_o) tanh(c_t)."""
    hid = 4
    z = dict(w_ih_f=np.zeros((16, 6), np.float32), w_hh_f=np.zeros((16, 4), np.float32),
             w_ih_b=np.zeros((16, 6), np.float32), w_hh_b=np.zeros((16, 4), np.float32),
             b_f=np.linspace(-1, 1, 16).astype(np.float32), b_b=np.linspace(1, -1, 16).astype(np.float32))
    out = orc.bilstm(z, np.ones((5, 6)))
    sig = lambda v: 1 / (1 + np.exp(-v))
    for half, b, order in ((0, z["b_f"].astype(np.float64), range(5)), (1, z["b_b"].astype(np.float64), range(4, -1, -1))):
        c = np.zeros(hid)
        for j in order:
            c = sig(b[hid:2 * hid]) * c + sig(b[:hid]) * np.tanh(b[2 * hid:3 * hid])
            np.testing.assert_allclose(out[j, half * hid:(half + 1) * hid], sig(b[3 * hid:]) * np.tanh(c), atol=1e-15)


@pytest.mark.parametrize("L", [1, 3, 30])
def test_encoder_equals_composition_of_library_routines(L):
    w = _small(seed=7)
    W = orc.EncoderWeights(w)
    ids = synth.encoder_ids(L, 9, vocab=(9, 3, 3, 2))
    x = sum(_t(w["tables"][t])[torch.from_numpy(ids[t].astype(np.int64))] for t in range(4))
    for cw, cb in zip(w["conv_w"], w["conv_b"]):
        x = F.relu(F.conv1d(x.T[None], _t(cw), _t(cb), padding=2))[0].T
    want = _library_bilstm(w, x.numpy())
    got = orc.encoder(W, ids)
    assert got.shape == (L, 16)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_full_size_encoder_is_bounded_and_depends_on_every_id_sequence():
    w = synth.make_encoder_weights()
    W = orc.EncoderWeights(w)
    ids = synth.encoder_ids(24, 1)
    a = orc.encoder(W, ids)
    assert a.shape == (24, 512) and np.all(np.abs(a) < 1.0)
    for t in range(4):
        ids2 = ids.copy(); ids2[t, 12] = (ids2[t, 12] + 1) % synth.ENCODER["vocab"][t]
        assert np.abs(orc.encoder(W, ids2) - a).max() > 1e-3
