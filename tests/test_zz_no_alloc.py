"""tts_postnet_run_static, the entry point that allocates nothing (its scratch is a static array inside the library),
against tts_postnet_run on the same inputs, through the C ABI: two calls in a row, the second with a smaller batch,
so that what the first call left in the shared array would show if the second read any of it."""
import ctypes as C

import numpy as np
import pytest

from paper_2211_13939_amd import binding, synth
from tests.helpers import say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bf16", [False, True])
def test_static_scratch_call_equals_the_arena_call_twice_in_a_row(bf16):
    import torch
    ws, bs = synth.make_postnet_weights(bf16=bf16)
    rng = np.random.default_rng(77)
    pn = binding.Postnet(binding.make_postnet_config(max_columns=2048, bf16=bf16), ws, bs)
    dev = pn.device
    # first a ragged batch that takes the wide kernels (90 column tiles; from 80 up), then a small one (the narrow kernels)
    for lens, keeps in (([50, 37, 1, 50, 64, 50, 50, 23, 50, 50, 50] * 3, [10, 10, 0, 10, 0, 10, 10, 3, 10, 10, 10] * 3),
                        ([26, 11, 5], [10, 0, 4])):
        mel = rng.standard_normal((sum(lens), 80)).astype(np.float32)
        n_out = sum(t - k for t, k in zip(lens, keeps))
        say(f"case no-alloc postnet: {len(lens)} windows, {sum(lens)} columns, {'bf16' if bf16 else 'fp32'}")
        with torch.cuda.stream(pn.stream):
            d_in = torch.from_numpy(mel).to(dev)
            want = torch.zeros((n_out, 80), dtype=torch.float32, device=dev)
            got = torch.zeros((n_out, 80), dtype=torch.float32, device=dev)
        pn.stream.synchronize()
        pn.run_device(d_in, lens, keeps, want)
        pn.run_device(d_in, lens, keeps, got, static=True)
        pn.stream.synchronize()
        w, g = want.cpu().numpy(), got.cpu().numpy()
        assert np.isfinite(w).all() and np.abs(w).max() > 0.1
        np.testing.assert_array_equal(g, w)
    # more columns than the static array holds: refused, nothing queued
    too_many = binding.TTS_POSTNET_STATIC_MAX_COLUMNS + 16
    lens = np.full(too_many // 16, 16, np.int32)
    keeps = np.zeros_like(lens)
    rc = binding.lib().tts_postnet_run_static(pn._h, C.c_void_p(d_in.data_ptr()), lens.ctypes.data_as(C.POINTER(C.c_int)),
                                              keeps.ctypes.data_as(C.POINTER(C.c_int)), int(lens.shape[0]),
                                              C.c_void_p(got.data_ptr()))
    assert rc == binding.TTS_E_INVAL and b"at most" in binding.lib().tts_last_error()
    pn.close()
