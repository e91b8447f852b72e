"""Parity of the HIP decoder step (through the C ABI) with the CPU oracle on the
same seeded inputs.  Bars: 1e-4 max abs error per mel bin with fp32 weights,
2e-2 with bf16 weights and fp32 accumulation, over the first 50 steps."""
import numpy as np
import pytest

from paper_2211_13939_amd import synth
from tests.helpers import TOL_BF16, TOL_F32, gpu_decode, max_err, oracle_decode, say

pytestmark = pytest.mark.gpu


def test_c1_single_request_fp32(weights_fp32):
    wl = synth.workload("c1")
    say("case c1: 1 request L=20, 10 steps, fp32")
    gpu = gpu_decode(wl, weights_fp32, [0], 10)
    ref, _, _ = oracle_decode(wl, weights_fp32, [0], 10)
    err = max_err(gpu, ref)
    say(f"  max abs err {err:.3e}")
    assert err <= TOL_F32


def test_c2_ragged_pool_fp32(weights_fp32):
    wl = synth.workload("c2")
    idx = list(range(16))
    say(f"case c2: 16 requests L={wl.enc_len.tolist()}, first 50 steps, fp32")
    gpu = gpu_decode(wl, weights_fp32, idx, 50)
    ref, _, _ = oracle_decode(wl, weights_fp32, idx, 50)
    err = max_err(gpu, ref)
    say(f"  max abs err {err:.3e}")
    assert err <= TOL_F32


def test_c3_pool64_bf16(weights_bf16):
    wl = synth.workload("c3")
    idx = list(range(64))
    say("case c3: 64 requests L in [30,300], first 50 steps, bf16 weights + bf16 memory")
    gpu = gpu_decode(wl, weights_bf16, idx, 50)
    ref, _, _ = oracle_decode(wl, weights_bf16, idx, 50, n_threads=16)
    err = max_err(gpu, ref)
    say(f"  max abs err {err:.3e}")
    assert err <= TOL_BF16


def test_bf16_weights_fp32_memory(weights_bf16):
    wl = synth.workload("c3")
    idx = [3, 17, 40, 41, 63]
    say("case c3 subset: bf16 weights, fp32 memory")
    gpu = gpu_decode(wl, weights_bf16, idx, 50, memory_bf16=False)
    ref, _, _ = oracle_decode(wl, weights_bf16, idx, 50, memory_bf16=False)
    err = max_err(gpu, ref)
    say(f"  max abs err {err:.3e}")
    assert err <= TOL_BF16
