"""Vocoder on the GPU against the CPU oracle (oracle/vocoder_oracle.c), through the C ABI."""
import numpy as np
import pytest

from paper_2211_13939_amd import binding, synth
from tests.helpers import TOL_BF16, TOL_F32, make_pool, say

pytestmark = pytest.mark.gpu

FIRST, LAST = binding.VOCODER_FIRST, binding.VOCODER_LAST
HOP = binding.VOCODER_HOP


def _mel(rng, n):
    # the decoder's mel frames are of order one
    return rng.standard_normal((n, 80)).astype(np.float32)


def _emulate_bf16(w, mel):
    """The generator with the two-byte path's rounding points written out with library routines (fp64 accumulate):
    every convolution's input is rounded to IEEE half (the MFMA operand type) after its activation; weights are bf16
    values already, which that type holds exactly."""
    import torch
    import torch.nn.functional as F

    def r(x):
        return torch.from_numpy(x.numpy().astype(np.float32).astype(np.float16).astype(np.float64))

    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float64))
    x = F.conv1d(r(t(mel).T[None]), t(w["pre_w"]), t(w["pre_b"]), padding=3)
    for s, u in enumerate((8, 8, 2, 2)):
        x = F.conv_transpose1d(r(F.leaky_relu(x, 0.1)), t(w["up_w"][s]), t(w["up_b"][s]), stride=u, padding=u // 2)
        acc = None
        for bk, k in enumerate((3, 7, 11)):
            y = x
            for i, d in enumerate((1, 3, 5)):
                h = F.conv1d(r(F.leaky_relu(y, 0.1)), t(w["res_w"][s][bk][2 * i]), t(w["res_b"][s][bk][2 * i]), dilation=d,
                             padding=d * (k - 1) // 2)
                h = F.conv1d(r(F.leaky_relu(h, 0.1)), t(w["res_w"][s][bk][2 * i + 1]), t(w["res_b"][s][bk][2 * i + 1]),
                             padding=(k - 1) // 2)
                y = y + h
            acc = y if acc is None else acc + y
        x = acc / 3
    x = F.conv1d(r(F.leaky_relu(x, 0.1)), t(w["post_w"]), t(w["post_b"]), padding=3)
    return torch.tanh(x)[0, 0].numpy()


@pytest.mark.parametrize("bf16", [False, True])
def test_generator_on_ragged_batch_matches_oracle(bf16):
    """Five single-chunk requests (first and last at once, so the response is G(M) itself) of 1 .. 40 frames
    in one call: several tiles per window at every stage, ragged ends, a one-frame window."""
    from oracle import oracle as orc
    w = synth.make_vocoder_weights(bf16=bf16)
    W = orc.VocoderWeights(w)
    rng = np.random.default_rng(11)
    lens = [1, 5, 17, 40, 33]
    mels = [_mel(rng, n) for n in lens]
    voc = binding.Vocoder(binding.make_vocoder_config(overlap=4, max_chunk=40, max_requests=8, max_batch=8, bf16=bf16), w)
    say(f"case vocoder generator: windows of {lens} frames, {'bf16' if bf16 else 'fp32'}")
    got = voc.run(mels, list(range(5)), [FIRST | LAST] * 5)
    worst = 0.0
    for n, m, g in zip(lens, mels, got):
        assert g.shape == (n * HOP,)
        want = orc.generator(W, m)
        worst = max(worst, float(np.abs(g - want).max()))
    say(f"  max abs err {worst:.3e} on audio in (-1, 1), {voc.elapsed_ms() * 1e3:.0f} us")
    assert worst <= (TOL_BF16 if bf16 else TOL_F32)
    voc.close()


def test_bf16_rounding_points():
    """bf16 path against the emulation of exactly its rounding points, and that emulation against the exact
    generator: the first bounds what the kernels add, the second is the price of bf16 operands."""
    from oracle import oracle as orc
    w = synth.make_vocoder_weights(bf16=True)
    W = orc.VocoderWeights(w)
    rng = np.random.default_rng(12)
    mel = _mel(rng, 24)
    voc = binding.Vocoder(binding.make_vocoder_config(overlap=0, max_chunk=24, max_requests=2, max_batch=2, bf16=True), w)
    got = voc.run([mel], [0], [FIRST | LAST])[0]
    emu = _emulate_bf16(w, mel)
    exact = orc.generator(W, mel)
    e1, e2, e3 = np.abs(got - emu).max(), np.abs(emu - exact).max(), np.abs(got - exact).max()
    say(f"case vocoder bf16 rounding points: gpu vs emulation {e1:.3e}, emulation vs exact {e2:.3e}, gpu vs exact {e3:.3e}")
    assert e1 <= 5e-3 and e3 <= TOL_BF16
    voc.close()


@pytest.mark.parametrize("overlap", [4, 8])
def test_streams_follow_eq3_eq4(overlap):
    """Three requests with different chunkings, their chunks batched as they come (different companions in every
    call, slots reused after a request's last chunk): every response equals the oracle's stream with the same
    overlap -- splice, fade against the previous tail, write-back."""
    from oracle import oracle as orc
    w = synth.make_vocoder_weights()
    W = orc.VocoderWeights(w)
    rng = np.random.default_rng(13 + overlap)
    plan = {0: [16, 16, 9], 1: [12, 3], 2: [16], 3: [10, 10, 10, 1]}       # request -> chunk sizes
    mels = {r: [_mel(rng, n) for n in sizes] for r, sizes in plan.items()}
    # call k carries chunk k of every request that has one; request 3 starts at call 1 in the slot request 2 freed
    start = {0: 0, 1: 0, 2: 0, 3: 1}
    slot = {0: 0, 1: 1, 2: 2, 3: 2}
    voc = binding.Vocoder(binding.make_vocoder_config(overlap=overlap, max_chunk=16, max_requests=3, max_batch=3), w)
    ref = {r: orc.VocoderStream(W, overlap) for r in plan}
    say(f"case vocoder streams: overlap {overlap}, chunkings {plan}")
    worst, total = 0.0, {r: 0 for r in plan}
    for call in range(5):
        items = [(r, call - start[r]) for r in plan if 0 <= call - start[r] < len(plan[r])]
        if not items:
            continue
        flags = [(FIRST if k == 0 else 0) | (LAST if k == len(plan[r]) - 1 else 0) for r, k in items]
        got = voc.run([mels[r][k] for r, k in items], [slot[r] for r, _ in items], flags)
        for (r, k), g in zip(items, got):
            want = ref[r].chunk(mels[r][k], k == len(plan[r]) - 1)
            assert g.shape == want.shape, (r, k, g.shape, want.shape)
            worst = max(worst, float(np.abs(g - want).max()))
            total[r] += g.shape[0]
    say(f"  max abs err {worst:.3e}")
    assert total == {r: sum(s) * HOP for r, s in plan.items()}
    assert worst <= TOL_F32
    voc.close()


def test_response_does_not_depend_on_batch_composition():
    w = synth.make_vocoder_weights(bf16=True)
    rng = np.random.default_rng(15)
    a = [_mel(rng, 16), _mel(rng, 16)]
    others = [_mel(rng, n) for n in (16, 7, 12)]
    cfg = binding.make_vocoder_config(overlap=4, max_chunk=16, max_requests=4, max_batch=4, bf16=True)
    voc = binding.Vocoder(cfg, w)
    alone = [voc.run([a[0]], [0], [FIRST])[0], voc.run([a[1]], [0], [LAST])[0]]
    voc.close()
    voc = binding.Vocoder(cfg, w)
    mixed = [voc.run([others[0], a[0], others[1]], [1, 3, 2], [FIRST, FIRST, FIRST | LAST])[1],
             voc.run([a[1], others[2]], [3, 1], [LAST, LAST])[0]]
    voc.close()
    for x, y in zip(alone, mixed):
        np.testing.assert_array_equal(x, y)


def test_bad_calls_are_rejected_and_change_nothing():
    w = synth.make_vocoder_weights()
    rng = np.random.default_rng(16)
    voc = binding.Vocoder(binding.make_vocoder_config(overlap=4, max_chunk=16, max_requests=2, max_batch=2), w)
    m = _mel(rng, 8)
    for chunks, slots, flags in (([m, m], [0, 0], [FIRST, FIRST]),          # a slot twice
                                 ([m], [0], [0]),                            # no previous chunk
                                 ([m], [2], [FIRST]),                        # slot out of range
                                 ([m[:3]], [0], [FIRST]),                    # shorter than the overlap, not last
                                 ([m, m, m], [0, 1, 0], [FIRST] * 3),        # more than max_batch
                                 ([m], [0], [4])):                           # unknown flag
        with pytest.raises(binding.TtsError) as e:
            voc.run(chunks, slots, flags)
        assert e.value.code == binding.TTS_E_INVAL
    first = voc.run([m], [0], [FIRST])[0]
    assert first.shape == ((8 - 4) * HOP,)
    with pytest.raises(binding.TtsError):
        voc.run([m], [1], [0])                 # slot 1 was never opened
    assert voc.run([m[:2]], [0], [LAST])[0].shape == ((4 + 2) * HOP,)
    with pytest.raises(binding.TtsError):
        voc.run([m], [0], [0])                 # closed by LAST
    voc.close()


@pytest.mark.parametrize("overlap", [False, True])
def test_serving_loop_decoder_postnet_vocoder_matches_oracle(overlap, weights_fp32):
    """Modules D and V behind each other in the arrival-driven loop: five requests arriving over time into a pool
    of three slots, chunks of 12 frames, overlap 4.  Every request's waveform (its responses in order) equals the
    oracle's: decoder alone, PostNet on the utterance so far, vocoder stream with splice, fade and write-back.
    overlap: PostNet and vocoder on a stream of their own beside the next decoder steps (more rounds out than the
    loop has staging sets: 14 chunks through 4 sets), responses taken as they reach the host."""
    import torch
    from oracle import oracle as orc
    from paper_2211_13939_amd import stream
    n, chunk, ov = 5, 12, 4
    wl = synth.small_workload(n, 10, 50, 13, 40, seed=53)
    pool = make_pool(wl, weights_fp32, chunk_frames=chunk, max_pool=3)
    ws, bs = synth.make_postnet_weights()
    wv = synth.make_vocoder_weights()
    side = torch.cuda.Stream(device=pool.device) if overlap else pool.stream
    pn = binding.Postnet(binding.make_postnet_config(max_columns=3 * (chunk + binding.POSTNET_CONTEXT)), ws, bs, stream=side)
    voc = binding.Vocoder(binding.make_vocoder_config(overlap=ov, max_chunk=chunk, max_requests=3, max_batch=3), wv, stream=side)
    audio = {i: [] for i in range(n)}
    be = stream.GpuPostnetBackend(pool, pn, lambda i: wl.encoder_outputs(i), wl.n_steps, chunk, binding.POSTNET_CONTEXT,
                                  vocoder=voc, on_audio=lambda i, a: audio[i].append(a), overlap=overlap)
    say(f"case serving loop decoder -> postnet -> vocoder{' (overlapped)' if overlap else ''}: steps {wl.n_steps.tolist()}, "
        f"pool of 3, chunks of {chunk}, overlap {ov}")
    res = stream.simulate(be, np.array([0.0, 0.0, 1e-4, 1e-4, 4e-3]), wl.n_steps, chunk, join_every=1, max_pool=3)
    assert not np.isnan(res.last_chunk_latency_s).any() and not np.isnan(res.first_chunk_latency_s).any()
    assert (res.first_chunk_latency_s <= res.last_chunk_latency_s).all() and (res.first_chunk_latency_s > 0).all()
    Wp, Wd, Wv = orc.PostnetWeights(ws, bs), orc.Weights(weights_fp32), orc.VocoderWeights(wv)
    worst = 0.0
    for i in range(n):
        T = int(wl.n_steps[i])
        mel, _, _, _ = orc.pool_decode(wl.dims, Wd, [wl.encoder_outputs(i)], [T], T)
        vs = orc.VocoderStream(Wv, ov)
        want = []
        for s0 in range(0, T, chunk):
            e0 = min(T, s0 + chunk)
            want.append(vs.chunk(orc.postnet_chunk(Wp, mel[0, :e0], s0), e0 == T))
        assert [a.shape[0] for a in audio[i]] == [w.shape[0] for w in want], i
        got = np.concatenate(audio[i])
        assert got.shape == (T * HOP,)
        worst = max(worst, float(np.abs(got - np.concatenate(want)).max()))
    say(f"  max abs err {worst:.3e}")
    # the decoder's error (<= 1e-4 per mel bin) passes through the PostNet (gain about 5) and the generator
    assert worst <= 1e-3
    voc.close()
    pn.close()
    pool.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_full_size_batch_in_the_benchmarked_launch_shape(bf16):
    """64 requests, 40-frame chunks behind 8 overlap frames: the batch `bench.py --vocoder` times, which takes the
    large tilings of the fused kernels.  Two rounds (first chunks, then middle chunks); the responses of four sampled
    requests are checked against the oracle's streams, the rest for size and range."""
    from oracle import oracle as orc
    w = synth.make_vocoder_weights(bf16=bf16)
    W = orc.VocoderWeights(w)
    rng = np.random.default_rng(21)
    n, chunk, ov = 64, 40, 8
    first = [_mel(rng, chunk) for _ in range(n)]
    second = [_mel(rng, chunk) for _ in range(n)]
    voc = binding.Vocoder(binding.make_vocoder_config(overlap=ov, max_chunk=chunk, max_requests=n, max_batch=n, bf16=bf16), w)
    say(f"case vocoder full batch: {n} requests x ({ov} + {chunk}) frames, {'bf16' if bf16 else 'fp32'}")
    r1 = voc.run(first, list(range(n)), [FIRST] * n)
    r2 = voc.run(second, list(range(n)), [0] * n)
    assert all(a.shape == ((chunk - ov) * HOP,) for a in r1) and all(a.shape == (chunk * HOP,) for a in r2)
    assert all(np.isfinite(a).all() and np.abs(a).max() < 1.0 for a in r1 + r2)
    worst = 0.0
    for k in (0, 17, 42, 63):
        vs = orc.VocoderStream(W, ov)
        worst = max(worst, float(np.abs(r1[k] - vs.chunk(first[k], False)).max()))
        worst = max(worst, float(np.abs(r2[k] - vs.chunk(second[k], False)).max()))
    say(f"  max abs err {worst:.3e} on four sampled requests, {voc.elapsed_ms() * 1e3:.0f} us for the second round")
    assert worst <= (TOL_BF16 if bf16 else TOL_F32)
    voc.close()
    # the same request alone takes the smallest tiles of every kernel: an output's sum does not depend on the tile it falls in
    solo = binding.Vocoder(binding.make_vocoder_config(overlap=ov, max_chunk=chunk, max_requests=1, max_batch=1, bf16=bf16), w)
    np.testing.assert_array_equal(solo.run([first[17]], [0], [FIRST])[0], r1[17])
    np.testing.assert_array_equal(solo.run([second[17]], [0], [0])[0], r2[17])
    solo.close()


def test_largest_batch_of_short_chunks():
    """256 chunks in one call (the most the call's batch table holds), chunks of 2 .. 5 frames with overlap 2, a mix of
    first, middle and last chunks: sizes follow the response rule and sampled responses match the oracle."""
    from oracle import oracle as orc
    w = synth.make_vocoder_weights()
    W = orc.VocoderWeights(w)
    rng = np.random.default_rng(23)
    n, ov = 256, 2
    voc = binding.Vocoder(binding.make_vocoder_config(overlap=ov, max_chunk=5, max_requests=n, max_batch=n), w)
    a = [_mel(rng, int(k)) for k in rng.integers(2, 6, size=n)]
    b = [_mel(rng, int(k)) for k in rng.integers(1, 6, size=n)]          # last chunks may be shorter than the overlap
    single = rng.random(n) < 0.25                                         # a quarter of the requests have one chunk only
    say("case vocoder largest batch: 256 chunks of 2..5 frames, overlap 2")
    r1 = voc.run(a, list(range(n)), [FIRST | (LAST if s else 0) for s in single])
    for k in range(n):
        assert r1[k].shape == ((a[k].shape[0] - (0 if single[k] else ov)) * HOP,)
    cont = [k for k in range(n) if not single[k]]
    r2 = voc.run([b[k] for k in cont], cont, [LAST] * len(cont))
    worst = 0.0
    for pos in (0, len(cont) // 2, len(cont) - 1):
        k = cont[pos]
        vs = orc.VocoderStream(W, ov)
        worst = max(worst, float(np.abs(r1[k] - vs.chunk(a[k], False)).max()))
        want = vs.chunk(b[k], True)
        assert r2[pos].shape == want.shape == ((ov + b[k].shape[0]) * HOP,)
        worst = max(worst, float(np.abs(r2[pos] - want).max()))
    k = int(np.nonzero(single)[0][0])
    worst = max(worst, float(np.abs(r1[k] - orc.generator(W, a[k])).max()))
    say(f"  max abs err {worst:.3e}")
    assert worst <= TOL_F32
    with pytest.raises(binding.TtsError):
        voc.run([a[0]] * 257, list(range(256)) + [0], [FIRST] * 257)
    voc.close()
