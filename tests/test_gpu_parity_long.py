"""bf16 parity with the CPU oracle to the LAST frame of long requests (Eq. 2 run 600 and 1200 times).

The cumulative attention weights W_acc grow with the frame count, and in the bf16 mode they are an MFMA
operand of the location convolution: any error that grows with a request's length shows up here, window
by window, and nowhere in a 50-frame comparison.  The bar is the bf16 bar (2e-2 max abs per mel bin) in
EVERY 50-frame window, not only the first."""
import numpy as np
import pytest

from paper_2211_13939_amd import synth
from tests.helpers import TOL_BF16, gpu_decode, oracle_decode, say

pytestmark = pytest.mark.gpu

WINDOW = 50


def window_errors(gpu, ref, n):
    """max |gpu - ref| over frames [w, w + WINDOW) of one request with n frames."""
    d = np.abs(gpu[:n].astype(np.float64) - ref[:n]).max(axis=-1)
    return [float(d[w:w + WINDOW].max()) for w in range(0, n, WINDOW)]


def test_c3_requests_to_their_last_frame_bf16(weights_bf16):
    """Six requests of the 64-request job, each decoded to its own end (the longest runs 600 frames, the
    longest memory has 300 positions), pooled together on the GPU; the oracle decodes each alone."""
    wl = synth.workload("c3")
    by_n, by_L = np.argsort(wl.n_steps), np.argsort(wl.enc_len)
    idx = sorted({int(by_n[-1]), int(by_n[-2]), int(by_L[-1]), int(by_L[0]), int(by_n[0]), int(by_n[32])})
    steps = int(wl.n_steps[idx].max())
    say(f"case c3 to the last frame: requests {idx}, L={wl.enc_len[idx].tolist()}, n={wl.n_steps[idx].tolist()}, bf16")
    gpu = gpu_decode(wl, weights_bf16, idx, steps)
    ref, _, frames = oracle_decode(wl, weights_bf16, idx, steps, n_threads=len(idx))
    worst = 0.0
    for k, i in enumerate(idx):
        n = int(wl.n_steps[i])
        assert int(frames[k]) == n and not np.isnan(gpu[k, :n]).any() and np.isnan(gpu[k, n:]).all()
        errs = window_errors(gpu[k], ref[k], n)
        say(f"  request {i} (L={int(wl.enc_len[i])}, n={n}): first window {errs[0]:.2e}, last {errs[-1]:.2e}, worst {max(errs):.2e}")
        worst = max(worst, max(errs))
        assert max(errs) <= TOL_BF16, (i, errs)
    say(f"  worst window {worst:.3e}")


def test_streaming_length_request_bf16(weights_bf16):
    """A request of the streaming workload's longest kind: 300 encoder positions, 4 L = 1200 frames."""
    L, n = 300, 1200
    wl = synth.Workload("long", True, np.array([L], np.int32), np.array([n], np.int32), 105)
    say(f"case streaming-length request: L={L}, n={n}, bf16")
    gpu = gpu_decode(wl, weights_bf16, [0], n)
    ref, _, frames = oracle_decode(wl, weights_bf16, [0], n, n_threads=1)
    assert int(frames[0]) == n
    errs = window_errors(gpu[0], ref[0], n)
    say("  per-window max abs err: " + " ".join(f"{e:.1e}" for e in errs))
    assert max(errs) <= TOL_BF16, errs
