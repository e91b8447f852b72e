"""Shared helpers of the GPU parity tests: run a workload through the C-ABI
pool, run the same requests through the CPU oracle, compare."""
import sys

import numpy as np

from paper_2211_13939_amd import binding, synth

TOL_F32 = 1e-4    # max abs error per mel bin, fp32 weights
TOL_BF16 = 2e-2   # bf16 weights with fp32 accumulation


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make_pool(wl, weights, max_pool=None, max_enc_len=None, max_steps=None, use_graph=True,
              memory_bf16=None, stop_threshold=-1.0, chunk_frames=None):
    cfg = binding.make_config(
        wl.dims, max_pool=max_pool or wl.n_requests,
        max_enc_len=max_enc_len or int(wl.enc_len.max()),
        max_steps=max_steps or int(wl.n_steps.max()),
        chunk_frames=chunk_frames or wl.chunk_frames, bf16=wl.bf16, memory_bf16=memory_bf16,
        use_graph=use_graph, stop_threshold=stop_threshold)
    return binding.Pool(cfg, weights)


def gpu_decode(wl, weights, idx, window, max_pool=None, **kw):
    """All requests `idx` join at step 0, `window` steps; returns mel [n, window, 80] (NaN past the end)."""
    pool = make_pool(wl, weights, max_pool=max_pool or max(len(idx), 1), **kw)
    ids = [pool.add_request(wl.encoder_outputs(i), int(min(wl.n_steps[i], window))) for i in idx]
    pool.step_n(window)
    out = np.full((len(idx), window, wl.dims["n_mel"]), np.nan, np.float32)
    for k, rid in enumerate(ids):
        m = pool.drain_all(rid)
        out[k, : m.shape[0]] = m
        pool.retire(rid)
    pool.close()
    return out


def oracle_decode(wl, weights, idx, window, memory_bf16=None, n_threads=8, stop_threshold=-1.0):
    from oracle import oracle as orc
    W = orc.Weights(weights)
    if memory_bf16 is None:
        memory_bf16 = wl.bf16
    Fs = [wl.encoder_outputs(i) for i in idx]
    ns = [int(wl.n_steps[i]) for i in idx]
    mel, stop, frames, used = orc.pool_decode(wl.dims, W, Fs, ns, window, pm_round_bf16=memory_bf16,
                                              stop_threshold=stop_threshold, n_threads=n_threads)
    return mel, stop, frames


def max_err(gpu, ref):
    """Largest |gpu - ref| over frames both sides produced; frame sets must agree."""
    g_nan, r_nan = np.isnan(gpu).any(axis=-1), np.isnan(ref).any(axis=-1)
    assert (g_nan == r_nan).all(), "GPU and oracle disagree on which frames exist"
    d = np.abs(gpu.astype(np.float64) - ref)
    return float(np.nanmax(d)) if (~g_nan).any() else 0.0
