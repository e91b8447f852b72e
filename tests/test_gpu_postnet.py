"""PostNet on the GPU against the CPU oracle (oracle/postnet_oracle.c), through the C ABI."""
import numpy as np
import pytest

from paper_2211_13939_amd import binding, synth
from tests.helpers import TOL_BF16, TOL_F32, make_pool, say

pytestmark = pytest.mark.gpu

CTX = binding.POSTNET_CONTEXT
# The bf16-weight PostNet multiplies IEEE-half operands: the input and four layers of activations are rounded to half
# precision (2^-12 relative each) and a layer's gain with the synthetic N(0, 0.05^2) weights is about 2.5.  Every
# comparison with the oracle, on N(0, 1) mel and on the decoder's own mel alike, is held to the absolute bf16 bar of
# 2e-2 per mel bin (measured: 6e-3 on outputs of magnitude up to 11).


def _oracle_chunks(W, utterances, cuts):
    """cuts[i] = chunk boundaries of utterance i; returns the chunk-wise result of every chunk."""
    from oracle import oracle as orc
    out = []
    for mel, cut in zip(utterances, cuts):
        out.append([orc.postnet_chunk(W, mel[:e], s) for s, e in zip(cut[:-1], cut[1:])])
    return out


def _windows(utterances, cuts, k):
    """Window of chunk k of every utterance that has one: (frames [s - ctx, e), keep_from)."""
    wins, keeps, who = [], [], []
    for i, (mel, cut) in enumerate(zip(utterances, cuts)):
        if k + 1 < len(cut):
            s, e = cut[k], cut[k + 1]
            c = min(CTX, s)
            wins.append(mel[s - c:e])
            keeps.append(c)
            who.append(i)
    return wins, keeps, who


@pytest.mark.parametrize("bf16", [False, True])
def test_ragged_batch_of_chunks_matches_oracle(bf16):
    """Utterances of different lengths cut into chunks of 16 (ragged last chunk, a one-frame chunk, a
    chunk shorter than the context): every chunk, batched with the other utterances' chunks of the
    same round, equals the oracle's "stack applied to the utterance so far"."""
    from oracle import oracle as orc
    ws, bs = synth.make_postnet_weights(bf16=bf16)
    W = orc.PostnetWeights(ws, bs)
    rng = np.random.default_rng(21)
    lens = [1, 5, 16, 17, 40, 53, 33]
    utter = [rng.standard_normal((n, 80)).astype(np.float32) for n in lens]
    cuts = [list(range(0, n, 16)) + [n] for n in lens]
    say(f"case postnet: {len(lens)} utterances of {lens} frames, chunks of 16, {'bf16' if bf16 else 'fp32'}")
    ref = _oracle_chunks(W, [u.astype(np.float64) for u in utter], cuts)
    pn = binding.Postnet(binding.make_postnet_config(max_columns=7 * (16 + CTX), bf16=bf16), ws, bs)
    worst = 0.0
    for k in range(4):
        wins, keeps, who = _windows(utter, cuts, k)
        if not wins:
            break
        got = pn.run(wins, keeps)
        for g, i in zip(got, who):
            assert g.shape == ref[i][k].shape
            worst = max(worst, float(np.abs(g - ref[i][k]).max()))
    scale = max(float(np.abs(c).max()) for r in ref for c in r)
    say(f"  max abs err {worst:.3e} (largest output {scale:.2f})")
    assert worst <= (TOL_BF16 if bf16 else TOL_F32)
    pn.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_large_batch_matches_oracle(bf16):
    """A batch big enough for the large-batch kernel (84 column tiles): 26 windows of 50 frames (a 40-frame
    chunk behind 10 frames of context) and one of 31.  A window is its own utterance as far as the oracle
    is concerned: the frames in front of it are zero."""
    from oracle import oracle as orc
    ws, bs = synth.make_postnet_weights(bf16=bf16)
    W = orc.PostnetWeights(ws, bs)
    rng = np.random.default_rng(77)
    lens = [50] * 26 + [31]
    keeps = [10] * 26 + [0]
    wins = [rng.standard_normal((n, 80)).astype(np.float32) for n in lens]
    say(f"case postnet large batch: {sum(lens)} columns, {'bf16' if bf16 else 'fp32'}")
    ref = [orc.postnet_chunk(W, w.astype(np.float64), k) for w, k in zip(wins, keeps)]
    pn = binding.Postnet(binding.make_postnet_config(max_columns=2048, bf16=bf16), ws, bs)
    got = pn.run(wins, keeps)
    pn.close()
    worst = max(float(np.abs(g - r).max()) for g, r in zip(got, ref))
    scale = max(float(np.abs(r).max()) for r in ref)
    say(f"  max abs err {worst:.3e} (largest output {scale:.2f})")
    assert worst <= (TOL_BF16 if bf16 else TOL_F32)


def test_very_large_batch_matches_oracle_and_small_batches():
    """26 windows of 50 frames and a ragged one (1337 columns, 84 tiles: 21 workgroups of columns in the
    large-batch kernel, the last one partial), bf16.  Against the oracle on every window, and against the same
    windows in batches of nine (small enough for the other kernel, whose summation order differs)."""
    from oracle import oracle as orc
    ws, bs = synth.make_postnet_weights(bf16=True)
    W = orc.PostnetWeights(ws, bs)
    rng = np.random.default_rng(78)
    lens = [50] * 26 + [37]
    keeps = [10] * 26 + [3]
    wins = [rng.standard_normal((n, 80)).astype(np.float32) for n in lens]
    say(f"case postnet very large batch: {sum(lens)} columns, bf16")
    ref = [orc.postnet_chunk(W, w.astype(np.float64), k) for w, k in zip(wins, keeps)]
    pn = binding.Postnet(binding.make_postnet_config(max_columns=2048, bf16=True), ws, bs)
    got = pn.run(wins, keeps)
    small = []
    for i in range(0, len(wins), 9):
        small += pn.run(wins[i:i + 9], keeps[i:i + 9])
    pn.close()
    scale = max(float(np.abs(r).max()) for r in ref)
    worst = max(float(np.abs(g - r).max()) for g, r in zip(got, ref))
    between = max(float(np.abs(g - h).max()) for g, h in zip(got, small))
    say(f"  max abs err {worst:.3e} (largest output {scale:.2f}); against the other kernels {between:.3e}")
    assert worst <= TOL_BF16
    assert between <= TOL_BF16


def test_bf16_rounding_points():
    """The two-byte mode takes the weights as bfloat16 values, rounds the input mel and every tanh output to IEEE half
    (the MFMA operand type) and accumulates in fp32.  The same rounding points applied to the oracle's layers on the
    CPU must land within a few rounding flips of the GPU (an activation next to a rounding boundary may fall either
    way under fp32 accumulation)."""
    from oracle import oracle as orc
    ws, bs = synth.make_postnet_weights(bf16=True)
    mel = np.random.default_rng(21).standard_normal((53, 80)).astype(np.float32)
    x = mel.astype(np.float16).astype(np.float64)
    for l in range(5):
        y = orc.conv5(ws[l], bs[l], x, apply_tanh=(l < 4))
        x = y.astype(np.float32).astype(np.float16).astype(np.float64) if l < 4 else y
    emulated = mel + x
    exact = orc.postnet(orc.PostnetWeights(ws, bs), mel.astype(np.float64))
    pn = binding.Postnet(binding.make_postnet_config(max_columns=64, bf16=True), ws, bs)
    got = pn.run([mel], [0])[0]
    pn.close()
    say(f"case postnet two-byte rounding points: gpu vs emulation {np.abs(got - emulated).max():.3e}, "
        f"emulation vs exact {np.abs(emulated - exact).max():.3e}, gpu vs exact {np.abs(got - exact).max():.3e}")
    assert np.abs(got - emulated).max() <= 0.5 * np.abs(emulated - exact).max()
    assert np.abs(got - exact).max() <= TOL_BF16


def test_window_without_full_context_is_rejected_or_exact_at_start():
    """A window that starts at frame 0 needs no context: the zeros in front are the utterance's own padding."""
    from oracle import oracle as orc
    ws, bs = synth.make_postnet_weights()
    W = orc.PostnetWeights(ws, bs)
    mel = np.random.default_rng(4).standard_normal((7, 80)).astype(np.float32)
    pn = binding.Postnet(binding.make_postnet_config(max_columns=64), ws, bs)
    got = pn.run([mel], [0])[0]
    assert np.abs(got - orc.postnet(W, mel.astype(np.float64))).max() <= TOL_F32
    with pytest.raises(binding.TtsError):
        pn.run([mel], [7])                      # nothing to keep
    with pytest.raises(binding.TtsError):
        pn.run([np.zeros((65, 80), np.float32)], [0])   # more frames than max_columns
    pn.close()


def test_result_does_not_depend_on_batch_composition():
    """A chunk post-processed alone and in a batch of others: identical bits (every column only sees its own
    window).  Holds among batches that take the same kernel (below 80 column tiles here)."""
    ws, bs = synth.make_postnet_weights(bf16=True)
    rng = np.random.default_rng(8)
    wins = [rng.standard_normal((n, 80)).astype(np.float32) for n in (26, 50, 11, 37, 18)]
    keeps = [10, 10, 0, 10, 2]
    pn = binding.Postnet(binding.make_postnet_config(max_columns=256, bf16=True), ws, bs)
    together = pn.run(wins, keeps)
    for i in (0, 2, 4):
        alone = pn.run([wins[i]], [keeps[i]])[0]
        np.testing.assert_array_equal(alone, together[i])
    shuffled = pn.run(wins[::-1], keeps[::-1])[::-1]
    for a, b in zip(together, shuffled):
        np.testing.assert_array_equal(a, b)
    pn.close()


def test_decoder_chunks_through_postnet_on_device(weights_fp32):
    """The decoder's chunks handed to the PostNet on the device (tts_pool_chunk_window): three requests,
    chunks of 8 frames, each round one dynamic batch; equals the oracle decoder followed by the oracle PostNet."""
    import torch
    from oracle import oracle as orc
    wl = synth.small_workload(3, 10, 60, 20, 27, seed=31)
    chunk = 8
    pool = make_pool(wl, weights_fp32, chunk_frames=chunk)
    ws, bs = synth.make_postnet_weights()
    pn = binding.Postnet(binding.make_postnet_config(max_columns=3 * (chunk + CTX)), ws, bs, stream=pool.stream)
    W = orc.PostnetWeights(ws, bs)
    Wd = orc.Weights(weights_fp32)
    ref_mel, _, frames, _ = orc.pool_decode(wl.dims, Wd, [wl.encoder_outputs(i) for i in range(3)],
                                            [int(n) for n in wl.n_steps], int(wl.n_steps.max()))
    ids = [pool.add_request(wl.encoder_outputs(i), int(wl.n_steps[i])) for i in range(3)]
    done = [0, 0, 0]
    finished = [False] * 3
    dev = pool.device
    d_in = torch.empty((3 * (chunk + CTX), 80), dtype=torch.float32, device=dev)
    d_out = torch.empty((3 * chunk, 80), dtype=torch.float32, device=dev)
    worst = 0.0
    say(f"case decoder -> postnet on device: steps {wl.n_steps.tolist()}, chunks of {chunk}")
    while not all(finished):
        pool.step_n(chunk)
        lens, keeps, who, row = [], [], [], 0
        for i, rid in enumerate(ids):
            if finished[i]:
                continue
            c, n, fin = pool.chunk_window(rid, CTX, d_in[row:])
            if n:
                lens.append(c + n); keeps.append(c); who.append((i, n)); row += c + n
            finished[i] = fin
        if not lens:
            continue
        pn.run_device(d_in, lens, keeps, d_out)
        pool.sync()
        out = d_out.cpu().numpy()
        r = 0
        for i, n in who:
            s = done[i]
            want = orc.postnet_chunk(W, ref_mel[i, : s + n], s)
            worst = max(worst, float(np.abs(out[r:r + n] - want).max()))
            r += n
            done[i] += n
    say(f"  max abs err {worst:.3e}")
    assert done == [int(n) for n in wl.n_steps]
    assert worst <= 5 * TOL_F32      # decoder error (<= 1e-4) passes through five layers of gain
    pn.close()
    pool.close()


def test_bf16_postnet_on_the_decoders_own_bf16_mel(weights_bf16):
    """The bf16 module on the only input it ever receives: the bf16 decoder's chunks, handed over on the device
    (tts_pool_chunk_window).  Two comparisons per chunk, both at the bf16 bar of 2e-2 absolute per mel bin:
    the module alone (oracle PostNet applied to the very frames the GPU decoder produced) and the chain
    (oracle decoder followed by the oracle PostNet on its own frames)."""
    import torch
    from oracle import oracle as orc
    wl = synth.small_workload(3, 30, 120, 50, 96, seed=33, bf16=True)
    chunk = 16
    pool = make_pool(wl, weights_bf16, chunk_frames=chunk)
    ws, bs = synth.make_postnet_weights(bf16=True)
    pn = binding.Postnet(binding.make_postnet_config(max_columns=3 * (chunk + CTX), bf16=True), ws, bs, stream=pool.stream)
    W = orc.PostnetWeights(ws, bs)
    Wd = orc.Weights(weights_bf16)
    ref_mel, _, frames, _ = orc.pool_decode(wl.dims, Wd, [wl.encoder_outputs(i) for i in range(3)],
                                            [int(n) for n in wl.n_steps], int(wl.n_steps.max()), pm_round_bf16=True,
                                            n_threads=3)
    ids = [pool.add_request(wl.encoder_outputs(i), int(wl.n_steps[i])) for i in range(3)]
    done = [0, 0, 0]
    finished = [False] * 3
    gpu_mel = [np.zeros((int(n), 80), np.float64) for n in wl.n_steps]
    dev = pool.device
    d_in = torch.empty((3 * (chunk + CTX), 80), dtype=torch.float32, device=dev)
    d_out = torch.empty((3 * chunk, 80), dtype=torch.float32, device=dev)
    worst_module = worst_chain = biggest = 0.0
    say(f"case bf16 decoder -> bf16 postnet on device: L {wl.enc_len.tolist()}, steps {wl.n_steps.tolist()}, chunks of {chunk}")
    while not all(finished):
        pool.step_n(chunk)
        lens, keeps, who, row = [], [], [], 0
        for i, rid in enumerate(ids):
            if finished[i]:
                continue
            c, n, fin = pool.chunk_window(rid, CTX, d_in[row:])
            if n:
                lens.append(c + n); keeps.append(c); who.append((i, n, row + c)); row += c + n
            finished[i] = fin
        if not lens:
            continue
        pn.run_device(d_in, lens, keeps, d_out)
        pool.sync()
        out = d_out.cpu().numpy()
        win = d_in.cpu().numpy()
        r = 0
        for i, n, at in who:
            s = done[i]
            gpu_mel[i][s:s + n] = win[at:at + n]
            want_module = orc.postnet_chunk(W, gpu_mel[i][: s + n], s)
            want_chain = orc.postnet_chunk(W, ref_mel[i, : s + n], s)
            worst_module = max(worst_module, float(np.abs(out[r:r + n] - want_module).max()))
            worst_chain = max(worst_chain, float(np.abs(out[r:r + n] - want_chain).max()))
            biggest = max(biggest, float(np.abs(want_chain).max()))
            r += n
            done[i] += n
    say(f"  module alone: max abs err {worst_module:.3e}; decoder + module: {worst_chain:.3e}; largest output {biggest:.2f}")
    assert done == [int(n) for n in wl.n_steps]
    assert worst_module <= TOL_BF16
    assert worst_chain <= TOL_BF16
    pn.close()
    pool.close()


def test_serving_loop_with_postnet_matches_oracle(weights_fp32):
    """The arrival-driven loop with the PostNet behind the decoder: six requests arriving over time into a
    pool of four slots, chunks of 8 frames; every chunk handed out equals the oracle decoder followed by the
    oracle PostNet on the utterance so far, whatever the pool held when the chunk was made."""
    from oracle import oracle as orc
    from paper_2211_13939_amd import stream
    n = 6
    wl = synth.small_workload(n, 10, 60, 17, 41, seed=47)
    chunk = 8
    pool = make_pool(wl, weights_fp32, chunk_frames=chunk, max_pool=4)
    ws, bs = synth.make_postnet_weights()
    pn = binding.Postnet(binding.make_postnet_config(max_columns=4 * (chunk + CTX)), ws, bs, stream=pool.stream)
    got = {i: [] for i in range(n)}
    be = stream.GpuPostnetBackend(pool, pn, lambda i: wl.encoder_outputs(i), wl.n_steps, chunk, CTX,
                                  on_chunk=lambda i, first, fr: got[i].append((first, fr)))
    arrivals = np.array([0.0, 0.0, 1e-4, 2e-4, 2e-4, 5e-3])
    say(f"case serving loop with postnet: steps {wl.n_steps.tolist()}, pool of 4, chunks of {chunk}")
    res = stream.simulate(be, arrivals, wl.n_steps, chunk, join_every=1, max_pool=4)
    assert not np.isnan(res.first_chunk_latency_s).any() and not np.isnan(res.last_chunk_latency_s).any()
    W, Wd = orc.PostnetWeights(ws, bs), orc.Weights(weights_fp32)
    worst = 0.0
    for i in range(n):
        ref_mel, _, _, _ = orc.pool_decode(wl.dims, Wd, [wl.encoder_outputs(i)], [int(wl.n_steps[i])], int(wl.n_steps[i]))
        at = 0
        for first, fr in got[i]:
            assert first == at and fr.shape[0] == min(chunk, int(wl.n_steps[i]) - at)
            want = orc.postnet_chunk(W, ref_mel[0, : first + fr.shape[0]], first)
            worst = max(worst, float(np.abs(fr - want).max()))
            at += fr.shape[0]
        assert at == int(wl.n_steps[i])
    say(f"  max abs err {worst:.3e}")
    assert worst <= 5 * TOL_F32
    pn.close()
    pool.close()
