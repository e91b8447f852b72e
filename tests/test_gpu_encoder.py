"""Acoustic encoder on the GPU against the CPU oracle (oracle/encoder_oracle.c), through the C ABI."""
import numpy as np
import pytest

from paper_2211_13939_amd import binding, synth
from tests.helpers import TOL_BF16, TOL_F32, make_pool, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bf16", [False, True])
def test_ragged_batch_matches_oracle(bf16):
    """Six requests of 1 .. 77 tokens in one call (several column tiles, ragged ends, a one-token request; fewer
    requests than MFMA columns): F_enc of every request equals the oracle's, which encodes each request alone."""
    from oracle import oracle as orc
    w = synth.make_encoder_weights(bf16=bf16)
    W = orc.EncoderWeights(w)
    lens = [1, 5, 16, 17, 77, 33]
    ids = [synth.encoder_ids(L, 100 + i) for i, L in enumerate(lens)]
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=256, max_len=100, bf16=bf16), w)
    say(f"case encoder: requests of {lens} tokens, {'bf16' if bf16 else 'fp32'}")
    got = enc.run(ids)
    worst = 0.0
    for a, g in zip(ids, got):
        want = orc.encoder(W, a)
        assert g.shape == want.shape
        worst = max(worst, float(np.abs(g - want).max()))
    say(f"  max abs err {worst:.3e} on F_enc in (-1, 1), {enc.elapsed_ms() * 1e3:.0f} us")
    assert worst <= (TOL_BF16 if bf16 else TOL_F32)
    enc.close()


@pytest.mark.parametrize("n_tokens", [1, 2, 33, 300])
def test_a_call_of_one_request_matches_oracle_bf16(n_tokens):
    """The usual call at join time: one request (in the two-byte mode the recurrence runs on the vector units, a kernel of
    its own): one token, two tokens and a request that feeds h back 300 times."""
    from oracle import oracle as orc
    w = synth.make_encoder_weights(bf16=True)
    ids = synth.encoder_ids(n_tokens, 500 + n_tokens)
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=320, max_len=300, bf16=True), w)
    say(f"case encoder: one request of {n_tokens} tokens, bf16")
    got = enc.run([ids])[0]
    want = orc.encoder(orc.EncoderWeights(w), ids)
    assert got.shape == want.shape
    err = float(np.abs(got - want).max())
    say(f"  max abs err {err:.3e}")
    assert err <= TOL_BF16
    enc.close()


def test_more_requests_than_mfma_columns_and_long_request():
    """20 requests (more than the 16 columns of a column tile) and one of 300 tokens, bf16."""
    from oracle import oracle as orc
    w = synth.make_encoder_weights(bf16=True)
    W = orc.EncoderWeights(w)
    rng = np.random.default_rng(7)
    lens = [int(x) for x in rng.integers(3, 40, size=19)] + [300]
    ids = [synth.encoder_ids(L, 200 + i) for i, L in enumerate(lens)]
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=1024, max_len=300, bf16=True), w)
    say(f"case encoder: 20 requests, {sum(lens)} tokens, longest 300, bf16")
    got = enc.run(ids)
    worst = 0.0
    for k in (0, 7, 15, 16, 18, 19):
        worst = max(worst, float(np.abs(got[k] - orc.encoder(W, ids[k])).max()))
    say(f"  max abs err {worst:.3e}, {enc.elapsed_ms() * 1e3:.0f} us")
    assert worst <= TOL_BF16
    enc.close()


@pytest.mark.parametrize("bf16", [True, False])
def test_result_does_not_depend_on_batch_composition(bf16):
    """Bitwise, among calls that take the same kernels (the convolutions have one kernel for calls below 80 column tiles
    of tokens - all calls here - and one for larger calls, which differ in summation order only).  In the two-byte mode
    every request has workgroups of its own in the recurrence; with fp32 weights calls of up to two requests compact the
    cell update and larger calls do not, again a difference in summation order."""
    w = synth.make_encoder_weights(bf16=bf16)
    ids = [synth.encoder_ids(L, 300 + i) for i, L in enumerate((40, 9, 23, 61, 5, 33))]
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=512, max_len=100, bf16=bf16), w)
    say(f"case encoder batch composition, {'bf16' if bf16 else 'fp32'}")
    alone = enc.run([ids[2]])[0]
    np.testing.assert_array_equal(alone, enc.run([ids[2]])[0])
    pair = enc.run([ids[3], ids[2]])[1]
    np.testing.assert_array_equal(pair, enc.run([ids[2], ids[0]])[0])
    np.testing.assert_array_equal(alone, pair)
    four = enc.run([ids[0], ids[1], ids[2], ids[3]])[2]
    np.testing.assert_array_equal(four, enc.run(ids)[2])
    np.testing.assert_array_equal(four, enc.run([ids[2], ids[5], ids[4]])[0])
    if bf16:
        np.testing.assert_array_equal(four, alone)
    else:
        assert np.abs(four - alone).max() <= 1e-5       # (the two kernels agree to rounding)
    enc.close()


def test_bad_calls_are_rejected():
    w = synth.make_encoder_weights()
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=64, max_len=40), w)
    good = synth.encoder_ids(10, 1)
    bad = good.copy(); bad[1, 3] = 4                     # the prosody tables have four rows
    for case in ([bad], [synth.encoder_ids(41, 2)], [synth.encoder_ids(40, 3), synth.encoder_ids(30, 4)]):
        with pytest.raises(binding.TtsError) as e:
            enc.run(case)
        assert e.value.code == binding.TTS_E_INVAL
    neg = good.copy(); neg[0, 0] = -1
    with pytest.raises(binding.TtsError):
        enc.run([neg])
    assert enc.run([good])[0].shape == (10, 512)
    enc.close()


def test_encoder_output_feeds_the_pool_on_device(weights_fp32):
    """Eq. 1 then Eq. 2 without leaving the device: F_enc of two requests goes from the encoder's output buffer
    straight into tts_pool_add_request; the mel frames equal the oracle decoder run on the oracle encoder's F_enc."""
    import torch
    from oracle import oracle as orc
    we = synth.make_encoder_weights()
    We = orc.EncoderWeights(we)
    lens, steps = [37, 12], [14, 9]
    ids = [synth.encoder_ids(L, 400 + i) for i, L in enumerate(lens)]
    wl = synth.small_workload(2, 12, 37, 9, 14, seed=3)
    pool = make_pool(wl, weights_fp32, max_pool=2, max_enc_len=64, max_steps=16)
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=64, max_len=64), we, stream=pool.stream)
    d_f = torch.empty((sum(lens), 512), dtype=torch.float32, device=pool.device)
    starts = enc.run_device(ids, d_f)
    rids = [pool.add_request(d_f[s:s + L], n) for s, L, n in zip(starts, lens, steps)]
    pool.step_n(max(steps))
    Wd = orc.Weights(weights_fp32)
    worst = 0.0
    say(f"case encoder -> pool on device: tokens {lens}, steps {steps}")
    for rid, a, n in zip(rids, ids, steps):
        f_enc = orc.encoder(We, a).astype(np.float32)
        ref, _, _, _ = orc.pool_decode(wl.dims, Wd, [f_enc], [n], n)
        got = pool.drain_all(rid)
        assert got.shape == (n, 80)
        worst = max(worst, float(np.abs(got - ref[0]).max()))
    say(f"  max abs err {worst:.3e}")
    assert worst <= TOL_F32
    enc.close()
    pool.close()


def test_serving_loop_with_encoder_at_join_matches_oracle(weights_fp32):
    """The arrival-driven loop with module E in front: every request joins with its token ids, the encoder produces
    F_enc on the device at join time, the decoder runs on it.  Mel frames equal the oracle chain (encoder, decoder)."""
    from oracle import oracle as orc
    from paper_2211_13939_amd import stream
    n, chunk = 4, 8
    wl = synth.small_workload(n, 8, 45, 11, 30, seed=61)
    ids = [synth.encoder_ids(int(L), 700 + i) for i, L in enumerate(wl.enc_len)]
    we = synth.make_encoder_weights()
    pool = make_pool(wl, weights_fp32, chunk_frames=chunk, max_pool=3, max_enc_len=64)
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=64, max_len=64), we, stream=pool.stream)
    join = stream.EncoderAtJoin(enc, lambda i: ids[i], 64)
    got = {i: [] for i in range(n)}

    class Collect(stream.GpuBackend):
        def run(self, k):
            self.pool.step_n(k)
            chunk_ids, fin_ids = [], []
            for rid, s in self.live.items():
                s["done"] = min(s["total"], s["done"] + k)
                if s["done"] - s["drained"] >= self.chunk or s["done"] == s["total"]:
                    while True:
                        frames, fin = self.pool.drain_chunk(rid)
                        s["drained"] += frames.shape[0]
                        if frames.shape[0]:
                            got[s["index"]].append(frames.copy())
                            chunk_ids.append(rid)
                        if fin:
                            fin_ids.append(rid)
                        if fin or frames.shape[0] == 0 or s["done"] - s["drained"] < self.chunk:
                            break
            self.pool.sync()
            return None, chunk_ids, fin_ids

    be = Collect(pool, join, wl.n_steps, chunk)
    say(f"case serving loop with encoder at join: tokens {wl.enc_len.tolist()}, steps {wl.n_steps.tolist()}, pool of 3")
    res = stream.simulate(be, np.array([0.0, 0.0, 1e-4, 3e-3]), wl.n_steps, chunk, join_every=1, max_pool=3)
    assert not np.isnan(res.last_chunk_latency_s).any()
    We, Wd = orc.EncoderWeights(we), orc.Weights(weights_fp32)
    worst = 0.0
    for i in range(n):
        T = int(wl.n_steps[i])
        f_enc = orc.encoder(We, ids[i]).astype(np.float32)
        ref, _, _, _ = orc.pool_decode(wl.dims, Wd, [f_enc], [T], T)
        mel = np.concatenate(got[i])
        assert mel.shape == (T, 80)
        worst = max(worst, float(np.abs(mel - ref[0]).max()))
    say(f"  max abs err {worst:.3e}")
    assert worst <= TOL_F32
    enc.close()
    pool.close()


def test_largest_batch_and_a_very_long_request():
    """256 requests in one call (16 groups of MFMA columns per direction) and, in another call, one request of 1000
    tokens (the recurrence runs 1000 dependent steps), fp32."""
    from oracle import oracle as orc
    w = synth.make_encoder_weights()
    W = orc.EncoderWeights(w)
    rng = np.random.default_rng(29)
    lens = [int(x) for x in rng.integers(1, 12, size=256)]
    ids = [synth.encoder_ids(L, 800 + i) for i, L in enumerate(lens)]
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=4096, max_len=1000), w)
    say(f"case encoder largest batch: 256 requests, {sum(lens)} tokens; then one request of 1000 tokens")
    got = enc.run(ids)
    worst = 0.0
    for k in (0, 15, 16, 100, 255):
        worst = max(worst, float(np.abs(got[k] - orc.encoder(W, ids[k])).max()))
    long_ids = synth.encoder_ids(1000, 999)
    g = enc.run([long_ids])[0]
    worst_long = float(np.abs(g - orc.encoder(W, long_ids)).max())
    say(f"  max abs err {worst:.3e} (batch), {worst_long:.3e} (1000 tokens)")
    assert worst <= TOL_F32 and worst_long <= TOL_F32
    with pytest.raises(binding.TtsError):
        enc.run(ids + [ids[0]])                # 257 requests
    enc.close()


def test_largest_batch_bf16():
    """256 requests in one call in the two-byte mode: 512 workgroups of the recurrence, two per CU's worth of the chip."""
    from oracle import oracle as orc
    w = synth.make_encoder_weights(bf16=True)
    W = orc.EncoderWeights(w)
    rng = np.random.default_rng(31)
    lens = [int(x) for x in rng.integers(1, 40, size=256)]
    ids = [synth.encoder_ids(L, 1200 + i) for i, L in enumerate(lens)]
    enc = binding.Encoder(binding.make_encoder_config(max_tokens=256 * 40, max_len=64, bf16=True), w)
    say(f"case encoder largest batch, bf16: 256 requests, {sum(lens)} tokens")
    got = enc.run(ids)
    worst = 0.0
    for k in (0, 1, 127, 128, 200, 255):
        assert got[k].shape == (lens[k], 512)
        worst = max(worst, float(np.abs(got[k] - orc.encoder(W, ids[k])).max()))
    say(f"  max abs err {worst:.3e}, {enc.elapsed_ms() * 1e3:.0f} us")
    assert worst <= TOL_BF16
    # bit for bit what a smaller call gives that takes the same convolution kernel (from 80 column tiles up)
    np.testing.assert_array_equal(got[200], enc.run(ids[150:])[50])
    enc.close()

