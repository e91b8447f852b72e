"""The byte / flop model bench.py prices the step with, and its refusal of more than one GPU (CPU only)."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2211_13939_amd import synth  # noqa: E402


def test_step_bytes_is_the_stated_formula():
    """weights once (18 173 504 elements), 33 092 bias bytes, 640 memory elements + 16 bytes of attention weights per
    position, the 4 688-float carried state read and written + one 320-byte frame per request."""
    # the 64-request job at its full pool: sum of its encoder lengths, two-byte weights and memory
    wl = synth.workload("c3")
    sum_L = int(wl.enc_len.sum())
    assert (wl.n_requests, sum_L) == (64, 9405)
    assert bench.step_bytes(64, sum_L, 2, 2) == 18_173_504 * 2 + 33_092 + sum_L * (640 * 2 + 16) + 64 * (2 * 4688 * 4 + 320) == 50_989_716
    # full pools at mean lengths: c1 72.8 MB, c2 75.8 MB, c4 120.7 MB
    assert round(bench.step_bytes(1, 20, 4, 4) / 1e6, 1) == 72.8
    assert round(bench.step_bytes(16, 16 * 60, 4, 4) / 1e6, 1) == 75.8
    assert round(bench.step_bytes(256, 256 * 225, 2, 2) / 1e6, 1) == 120.7
    assert bench.step_flops(256, 256 * 225) == 256 * 2 * 18_173_504 + 13_824 * 256 * 225


def test_the_per_kernel_split_adds_up_to_the_step():
    for P, sum_L, s in ((1, 20, 4), (16, 950, 4), (64, 9405, 2), (65, 9405, 2), (256, 58719, 2), (256, 58719, 4)):
        for pre in (None, 0, 1, 2):
            parts = bench.algorithmic_bytes(P, sum_L, s, s, pre_gates=pre)
            assert set(parts) == {"k_lstm_att", "k_lsa", "k_lstm_dec", "k_proj"}
            assert sum(parts.values()) == bench.step_bytes(P, sum_L, s, s), (P, sum_L, s, pre)


def test_the_decoder_lstm_is_charged_to_the_launch_that_holds_it():
    """Two-byte pools have no decoder-LSTM kernel: its bytes move in the last kernel's launch (and, in pools of at most
    64 slots, the columns for H_att and H_dec beside the attention); fp32 pools keep the kernel."""
    small = bench.algorithmic_bytes(64, 9405, 2, 2)
    large = bench.algorithmic_bytes(256, 58719, 2, 2)
    fp32 = bench.algorithmic_bytes(16, 950, 4, 4)
    assert small["k_lstm_dec"] == 0 and large["k_lstm_dec"] == 0 and fp32["k_lstm_dec"] > 0
    w_dec = 4096 * 2560 * 2
    assert large["k_proj"] > w_dec                                    # all of the decoder LSTM's weights
    assert small["k_proj"] < w_dec and small["k_lsa"] > 4096 * 2048 * 2   # K = 512 of them there, K = 2048 beside the attention


def test_job_bytes_integrate_the_membership_trace():
    """Request i is in the pool during steps 0 .. n_i - 1: the job's bytes are the per-step bytes summed over that trace."""
    wl = synth.small_workload(5, 10, 40, 3, 9, seed=5, bf16=True)
    n, L = wl.n_steps.astype(int), wl.enc_len.astype(int)
    want = 0
    for pos in range(int(n.max())):
        act = n > pos
        want += bench.step_bytes(int(act.sum()), int(L[act].sum()), 2, 2)
    assert bench.job_roofline_bytes(wl, 2, 2) == want


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr
    assert np.isfinite(bench.HBM_PEAK_GBS)
