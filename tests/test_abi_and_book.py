"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, validates configurations, and its host-side pool bookkeeping
follows the pooling semantics of Sec. 2.2.2 / the timeline of Sec. 2.2.3.
No compute call is made here."""
import os
import re

import pytest

from paper_2211_13939_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in ("tts_pool.h", "tts_postnet.h", "tts_vocoder.h", "tts_encoder.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(tts_(?:pool|book|last|postnet|vocoder|encoder)_\w+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = _declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_config_validation_without_gpu():
    good = binding.make_config(synth.DIMS, max_pool=16, max_enc_len=100, max_steps=200)
    assert binding.workspace_bytes(good) > 72_000_000          # fp32 weights alone are 72.7 MB
    bf = binding.make_config(synth.DIMS, max_pool=16, max_enc_len=100, max_steps=200, bf16=True)
    assert 36_000_000 < binding.workspace_bytes(bf) < binding.workspace_bytes(good)
    for field, bad in (("max_pool", 0), ("max_pool", 257), ("max_enc_len", 0), ("max_enc_len", 1025),
                       ("max_steps", 0), ("chunk_frames", 0), ("n_mel", 81), ("att_dim", 64),
                       ("loc_in_channels", 3), ("weight_dtype", 2)):
        c = binding.make_config(synth.DIMS, max_pool=16, max_enc_len=100, max_steps=200)
        setattr(c, field, bad)
        assert binding.workspace_bytes(c) == 0, field
        assert binding.lib().tts_last_error()
    c = binding.make_config(synth.DIMS, max_pool=16, max_enc_len=100, max_steps=200, bf16=False, memory_bf16=True)
    assert binding.workspace_bytes(c) == 0


def test_timeline_membership_trace():
    """The timeline of Sec. 2.2.3: request 1 arrives before step 0; 2 and 3 arrive
    during step 1 and are first processed in step 2; 1 completes in step 3; 2 in
    step 5; 4 arrives at the end of step 5 and is batched with 3 in step 6, where
    3 completes."""
    b = binding.Book(8, 100, 100, 4)
    r1 = b.add(10, 4)                      # steps 0..3
    trace = [b.step(), b.step()]           # steps 0, 1
    r2 = b.add(10, 4)                      # arrived during step 1 -> steps 2..5
    r3 = b.add(10, 5)                      # steps 2..6
    trace += [b.step(), b.step()]          # steps 2, 3 (request 1 completes in 3)
    b.retire(r1)
    trace += [b.step(), b.step()]          # steps 4, 5 (request 2 completes in 5)
    b.retire(r2)
    r4 = b.add(10, 9)
    trace += [b.step()]                    # step 6
    ids = {1: r1, 2: r2, 3: r3, 4: r4}
    golden = []                            # the walk-through as the paper prints it
    for line in open(os.path.join(ROOT, "tests", "golden", "timeline_sec_2_2_3.txt")):
        if line.strip() and not line.startswith("#"):
            step, members = line.split(":")
            assert int(step) == len(golden)
            golden.append([ids[int(x)] for x in members.split()])
    assert len(golden) == 7 and trace == golden
    first, n, fin = b.drain(r3)
    assert (first, n, fin) == (0, 4, False)
    first, n, fin = b.drain(r3)
    assert (first, n, fin) == (4, 1, True)          # short last chunk of a finished request
    assert b.drain(r4) == (0, 0, False)             # chunk not full yet, still running


def test_book_errors_and_slot_reuse():
    b = binding.Book(2, 50, 20, 5)
    with pytest.raises(binding.TtsError) as e:
        b.add(0, 5)
    assert e.value.code == binding.TTS_E_INVAL
    with pytest.raises(binding.TtsError):
        b.add(51, 5)
    with pytest.raises(binding.TtsError):
        b.add(5, 21)
    a = b.add(5, 3)
    c = b.add(6, 20)
    with pytest.raises(binding.TtsError) as e:
        b.add(5, 5)
    assert e.value.code == binding.TTS_E_FULL
    assert b.step() == [a, c] and b.step() == [a, c] and b.step() == [a, c]
    assert b.step() == [c]                 # a reached its cap: holds its slot but no longer advances
    with pytest.raises(binding.TtsError) as e:
        b.add(5, 5)                        # still full until retired
    assert e.value.code == binding.TTS_E_FULL
    assert b.drain(a) == (0, 3, True)
    b.retire(a)
    with pytest.raises(binding.TtsError) as e:
        b.retire(a)
    assert e.value.code == binding.TTS_E_NOTFOUND
    with pytest.raises(binding.TtsError):
        b.drain(a)
    d = b.add(7, 2)
    assert d not in (a, c)                 # ids are never reused
    assert b.step() == [c, d]
    b.retire(c)                            # retiring an unfinished request is allowed
    assert b.step() == [d]
    assert b.step() == []                  # empty step is a no-op


def test_postnet_config_validation_without_gpu():
    good = binding.make_postnet_config(max_columns=100)
    assert binding.postnet_workspace_bytes(good) > 5 * 512 * 512 * 4 * 3
    bf = binding.make_postnet_config(max_columns=100, bf16=True)
    assert 0 < binding.postnet_workspace_bytes(bf) < binding.postnet_workspace_bytes(good)
    for field, bad in (("n_mel", 64), ("channels", 256), ("max_columns", 0), ("weight_dtype", 3)):
        c = binding.make_postnet_config(max_columns=100)
        setattr(c, field, bad)
        assert binding.postnet_workspace_bytes(c) == 0, field


def test_vocoder_config_validation_without_gpu():
    good = binding.make_vocoder_config(overlap=8, max_chunk=40, max_requests=16, max_batch=4)
    assert binding.vocoder_workspace_bytes(good) > 4 * 48 * 2048 * 4 * 4          # four activation buffers
    bf = binding.make_vocoder_config(overlap=8, max_chunk=40, max_requests=16, max_batch=4, bf16=True)
    assert 0 < binding.vocoder_workspace_bytes(bf) < binding.vocoder_workspace_bytes(good)
    for field, bad in (("n_mel", 64), ("c0", 512), ("overlap", -1), ("overlap", 17), ("max_chunk", 0), ("max_chunk", 7),
                       ("max_requests", 0), ("max_batch", 0), ("max_batch", 257), ("weight_dtype", 2)):
        c = binding.make_vocoder_config(overlap=8, max_chunk=40, max_requests=16, max_batch=4)
        setattr(c, field, bad)
        assert binding.vocoder_workspace_bytes(c) == 0, field
        assert binding.lib().tts_last_error()


def test_encoder_config_validation_without_gpu():
    good = binding.make_encoder_config(max_tokens=600, max_len=300)
    assert binding.encoder_workspace_bytes(good) > 3 * 512 * 512 * 5 * 4          # the three convolutions alone
    bf = binding.make_encoder_config(max_tokens=600, max_len=300, bf16=True)
    assert 0 < binding.encoder_workspace_bytes(bf) < binding.encoder_workspace_bytes(good)
    for field, bad in (("dim", 256), ("hid", 128), ("max_tokens", 10), ("max_len", 0), ("max_len", 40000), ("weight_dtype", 2)):
        c = binding.make_encoder_config(max_tokens=600, max_len=300)
        setattr(c, field, bad)
        assert binding.encoder_workspace_bytes(c) == 0, field
    c = binding.make_encoder_config(max_tokens=600, max_len=300, vocab=(128, 0, 4, 4))
    assert binding.encoder_workspace_bytes(c) == 0


def test_book_packs_running_requests_into_a_smaller_span():
    """After requests leave, the running ones move into free low slots when that brings them into a smaller
    power-of-two span; ids, frame counters and the order of the running requests go along."""
    b = binding.Book(64, 100, 50, 8)
    ids = [b.add(10, 50 if i % 3 == 0 else 3) for i in range(60)]
    assert [b.slot(r) for r in ids] == list(range(60))
    for _ in range(3):
        b.step()
    assert b.compact() == []                      # the finished requests still hold their slots
    for i, r in enumerate(ids):
        if i % 3:
            assert b.drain(r) == (0, 3, True)
            b.retire(r)
    long_ids = ids[::3]                           # 20 requests in slots 0, 3, ..., 57
    moves = b.compact()
    # 20 requests fit the class of 32: those in slots 33..57 go to the lowest free slots, in order
    assert moves == list(zip(range(33, 58, 3), [1, 2, 4, 5, 7, 8, 10, 11, 13]))
    assert [b.slot(r) for r in long_ids] == list(range(0, 33, 3)) + [1, 2, 4, 5, 7, 8, 10, 11, 13]
    assert b.compact() == []                      # nothing further to gain
    assert b.step() == long_ids                   # same requests, same order
    assert b.drain(long_ids[-1]) == (0, 0, False)  # 4 of 8 frames
    for _ in range(4):
        b.step()
    assert b.drain(long_ids[-1]) == (0, 8, False)
    # a new request takes the lowest free slot
    assert b.slot(b.add(5, 5)) == 14
    # 21 running: class 32 still; retire the nine that moved -> 12 running, class 16, everything above slot 15 moves
    for r in long_ids[11:]:
        b.retire(r)
    assert b.compact() == list(zip([18, 21, 24, 27, 30], [1, 2, 4, 5, 7]))
    assert max(b.slot(r) for r in long_ids[:11]) < 16
    # spans of `min_span` and fewer are left alone
    for r in long_ids[:4]:
        b.retire(r)                               # slots 0, 3, 6, 9 free; 8 running, the highest in slot 15
    assert b.compact() == []
    assert b.compact(min_span=2) != []
    b.close()


def test_book_does_not_move_when_free_slots_do_not_suffice():
    b = binding.Book(64, 100, 50, 8)
    ids = [b.add(10, 50 if i >= 40 else 2) for i in range(64)]
    b.step(); b.step()
    for r in ids[:10]:
        b.retire(r)                               # 24 running in slots 40..63, but only 10 free slots below 32
    assert b.compact() == []
    for r in ids[10:40]:
        b.retire(r)
    assert len(b.compact()) == 24
    assert sorted(b.slot(r) for r in ids[40:]) == list(range(24))
    b.close()
