"""Pool semantics of the HIP library (Sec. 2.2.2 / 2.2.3) and edge cases, through
the C ABI on a real GPU.  Eq. 2 never mixes two requests, so a request's frames
must not depend on who shares the pool, when it joined, or which slot it got:
those comparisons are bit-exact (same kernels, same per-column arithmetic).
Comparisons with the CPU oracle use the fp32 / bf16 bars."""
import numpy as np
import pytest

from paper_2211_13939_amd import binding, synth
from tests.helpers import TOL_BF16, TOL_F32, gpu_decode, make_pool, max_err, oracle_decode, say

pytestmark = pytest.mark.gpu


def _drain(pool, rid):
    return pool.drain_all(rid)


@pytest.fixture(scope="module")
def wl8():
    return synth.small_workload(8, 5, 90, 24, 24, seed=11)


@pytest.fixture(scope="module")
def solo_frames(wl8, weights_fp32):
    """Every request of wl8 decoded alone in a pool of one (24 frames)."""
    say("reference: 8 requests decoded alone, fp32")
    out = []
    for i in range(8):
        out.append(gpu_decode(wl8, weights_fp32, [i], 24)[0])
    return out


def test_pool_equals_solo_and_oracle(wl8, weights_fp32, solo_frames):
    say("case: pool of 8 vs each alone vs oracle")
    pooled = gpu_decode(wl8, weights_fp32, list(range(8)), 24)
    for i in range(8):
        np.testing.assert_array_equal(pooled[i], solo_frames[i])
    ref, _, _ = oracle_decode(wl8, weights_fp32, list(range(8)), 24)
    assert max_err(pooled, ref) <= TOL_F32


def test_slot_permutation(wl8, weights_fp32, solo_frames):
    say("case: join order permuted")
    order = [5, 2, 7, 0, 3, 6, 1, 4]
    pooled = gpu_decode(wl8, weights_fp32, order, 24)
    for k, i in enumerate(order):
        np.testing.assert_array_equal(pooled[k], solo_frames[i])


def test_late_join_retire_and_slot_reuse(wl8, weights_fp32, solo_frames):
    """Requests join at different steps, one is retired unfinished, its slot is
    reused by a shorter request (stale encoder rows beyond its length must not
    matter), survivors are not perturbed."""
    say("case: late join / neighbour retire / slot reuse")
    pool = make_pool(wl8, weights_fp32, max_pool=4, max_enc_len=90, max_steps=24, chunk_frames=8)
    enc = wl8.encoder_outputs
    long_i = int(np.argmax(wl8.enc_len))
    short_i = int(np.argmin(wl8.enc_len))
    others = [i for i in range(8) if i not in (long_i, short_i)][:2]
    r_long = pool.add_request(enc(long_i), 24)
    r_a = pool.add_request(enc(others[0]), 24)
    assert pool.step_n(7) == 14
    r_b = pool.add_request(enc(others[1]), 24)          # joins 7 steps late
    assert pool.step_n(5) == 15
    pool.retire(r_long)                                  # leaves unfinished after 12 frames
    r_short = pool.add_request(enc(short_i), 24)         # takes the freed slot
    assert pool.n_active() == 3 and pool.size() == 3
    total = 0
    while pool.n_active():
        total += pool.step()
    got = {others[0]: _drain(pool, r_a), others[1]: _drain(pool, r_b), short_i: _drain(pool, r_short)}
    for i, frames in got.items():
        assert frames.shape == (24, 80)
        np.testing.assert_array_equal(frames, solo_frames[i])
    assert total == (24 - 12) + (24 - 5) + 24
    pool.close()


def test_timeline_of_the_paper(wl8, weights_fp32, solo_frames):
    """The narrative of Sec. 2.2.3 with a 'step' = one chunk iteration of the
    decoder: request 1 from step 0; requests 2, 3 from step 2; request 1 done
    in step 3; request 2 done in step 5; request 4 joins for step 6 with 3."""
    say("case: timeline of Sec. 2.2.3")
    chunk = 3
    pool = make_pool(wl8, weights_fp32, max_pool=4, max_enc_len=90, max_steps=24, chunk_frames=chunk)
    enc = wl8.encoder_outputs
    frames = {}
    members = []

    def iteration(ids):
        members.append(sorted(k for k in ids))
        advanced = pool.step_n(chunk)
        assert advanced == chunk * len(ids)
        for k, rid in ids.items():
            c, fin = pool.drain_chunk(rid)
            assert c.shape[0] == chunk
            frames.setdefault(k, []).append(c.copy())

    r = {1: pool.add_request(enc(0), 4 * chunk)}
    iteration(r); iteration(r)                           # steps 0, 1
    r[2] = pool.add_request(enc(1), 4 * chunk)           # arrived during step 1
    r[3] = pool.add_request(enc(2), 5 * chunk)
    iteration(r); iteration(r)                           # steps 2, 3
    assert pool.frames(r[1]) == (4 * chunk, True)
    pool.retire(r.pop(1))
    iteration(r); iteration(r)                           # steps 4, 5
    pool.retire(r.pop(2))
    r[4] = pool.add_request(enc(3), 2 * chunk)           # arrived at the end of step 5
    iteration(r)                                         # step 6
    assert members == [[1], [1], [1, 2, 3], [1, 2, 3], [2, 3], [2, 3], [3, 4]]
    assert pool.frames(r[3]) == (5 * chunk, True)
    for k, i in ((1, 0), (2, 1), (3, 2), (4, 3)):
        got = np.concatenate(frames[k])
        np.testing.assert_array_equal(got, solo_frames[i][: got.shape[0]])
    pool.close()


def test_drain_chunks_and_errors(wl8, weights_fp32):
    say("case: drain semantics and error codes")
    pool = make_pool(wl8, weights_fp32, max_pool=2, max_enc_len=90, max_steps=24, chunk_frames=10)
    assert pool.step() == 0                               # empty pool: a no-op
    enc = wl8.encoder_outputs
    a = pool.add_request(enc(0), 23)
    b = pool.add_request(enc(1), 5)
    with pytest.raises(binding.TtsError) as e:
        pool.add_request(enc(2), 5)
    assert e.value.code == binding.TTS_E_FULL
    for bad_L, bad_n in ((0, 5), (91, 5), (10, 0), (10, 25)):
        with pytest.raises(binding.TtsError) as e:
            pool.add_request_raw(enc(2).ctypes.data, bad_L, bad_n)
        assert e.value.code == binding.TTS_E_INVAL
    assert pool.step_n(9) == 5 + 9                        # b stops after its 5 frames
    c, fin = pool.drain_chunk(a)
    assert c.shape[0] == 0 and not fin                    # 9 < 10: chunk not ready
    c, fin = pool.drain_chunk(b)
    assert c.shape[0] == 5 and fin                        # finished: short last chunk
    c, fin = pool.drain_chunk(b)
    assert c.shape[0] == 0 and fin
    pool.retire(b)
    with pytest.raises(binding.TtsError) as e:
        pool.drain_chunk(b)
    assert e.value.code == binding.TTS_E_NOTFOUND
    with pytest.raises(binding.TtsError) as e:
        pool.retire(b)
    assert e.value.code == binding.TTS_E_NOTFOUND
    assert pool.step_n(100) == 14                         # a runs to its cap, then nothing advances
    sizes = []
    while True:
        c, fin = pool.drain_chunk(a)
        sizes.append(c.shape[0])
        if fin:
            break
    assert sizes == [10, 10, 3]
    assert pool.frames(a) == (23, True)
    pool.close()


@pytest.fixture(scope="module")
def wl8_bf16():
    return synth.small_workload(8, 5, 90, 24, 24, seed=11, bf16=True)


@pytest.fixture(scope="module")
def solo_frames_bf16(wl8_bf16, weights_bf16):
    """Every request of wl8_bf16 decoded alone in a two-byte pool of one (24 frames): the step of such pools is three
    launches, with the decoder LSTM inside the last one."""
    say("reference: 8 requests decoded alone, bf16")
    return [gpu_decode(wl8_bf16, weights_bf16, [i], 24)[0] for i in range(8)]


def _mode(request, bf16):
    """(workload, weights, solo frames) of the fp32 or the two-byte flavour of the 8-request workload."""
    if bf16:
        return request.getfixturevalue("wl8_bf16"), request.getfixturevalue("weights_bf16"), request.getfixturevalue("solo_frames_bf16")
    return request.getfixturevalue("wl8"), request.getfixturevalue("weights_fp32"), request.getfixturevalue("solo_frames")


def test_snapshot_resume(wl8, weights_fp32, solo_frames):
    """The carried state set of Sec. 2.1.3 is complete: a fresh request restored
    from get_state continues on the same trajectory.  (Not bit-exact: restoring
    M_last recomputes its prenet with another summation order than the step.)"""
    say("case: snapshot / resume through get_state, set_state")
    pool = make_pool(wl8, weights_fp32, max_pool=2, max_enc_len=90, max_steps=24, chunk_frames=24)
    enc = wl8.encoder_outputs
    a = pool.add_request(enc(4), 24)
    pool.step_n(9)
    snap = {k: pool.get_state(a, k) for k in binding.STATE}
    assert snap["w_last"].shape[0] == wl8.enc_len[4] and abs(snap["w_last"].sum() - 1) < 1e-5
    assert abs(snap["w_acc"].sum() - 9) < 1e-4
    b = pool.add_request(enc(4), 15)
    for k, v in snap.items():
        pool.set_state(b, k, v)
    pool.retire(a)
    pool.step_n(15)
    got = _drain(pool, b)
    assert got.shape == (15, 80)
    assert np.abs(got - solo_frames[4][9:24]).max() <= 1e-5
    pool.close()


def test_stop_threshold(wl8):
    """sigmoid(stop logit) > threshold ends a request; the tripping frame is kept."""
    say("case: stop threshold")
    from oracle import oracle as orc
    w = synth.make_weights()
    w["stop_b"] = w["stop_b"].copy()
    w["stop_b"][:] = 0.2
    thr = 0.62          # request 0 trips at its 4th frame; every other margin is >= 5e-3
    pool = make_pool(wl8, w, max_pool=8, max_enc_len=90, max_steps=24, chunk_frames=24, stop_threshold=thr)
    ids = [pool.add_request(wl8.encoder_outputs(i), 24) for i in range(8)]
    pool.step_n(24)
    W = orc.Weights(w)
    n_early = 0
    for i, rid in enumerate(ids):
        r = orc.Request(wl8.dims, W, wl8.encoder_outputs(i), 24, stop_threshold=thr)
        ref, stops = [], []
        while True:
            o = r.step()
            if o is None:
                break
            ref.append(o[0]); stops.append(o[1])
        # the decision is only checked where the oracle's margin is clear of rounding
        margin = min(abs(1 / (1 + np.exp(-s)) - thr) for s in stops)
        n, fin = pool.frames(rid)
        assert fin
        if margin > 1e-4:
            assert n == len(ref)
            got = _drain(pool, rid)
            assert np.abs(got - np.array(ref)).max() <= TOL_F32
            assert np.abs(pool.stop_logits(rid, 0, n) - np.array(stops)).max() <= TOL_F32
            n_early += n < 24
    assert n_early >= 1
    pool.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_graph_equals_plain_launches_and_is_deterministic(wl8, bf16):
    say(f"case: graph vs plain launches, repeatability (bf16={bf16})")
    wl = synth.small_workload(8, 5, 90, 24, 24, seed=11, bf16=bf16)
    w = synth.make_weights(bf16=bf16)
    a = gpu_decode(wl, w, list(range(8)), 24, use_graph=True)
    b = gpu_decode(wl, w, list(range(8)), 24, use_graph=False)
    c = gpu_decode(wl, w, list(range(8)), 24, use_graph=True)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(a, c)


def test_device_pointer_input(wl8, weights_fp32, solo_frames):
    import torch
    say("case: encoder outputs handed over in device memory")
    pool = make_pool(wl8, weights_fp32, max_pool=2, max_enc_len=90, max_steps=24, chunk_frames=24)
    t = torch.from_numpy(wl8.encoder_outputs(6)).to(pool.device)
    rid = pool.add_request(t, 24)
    pool.step_n(24)
    np.testing.assert_array_equal(_drain(pool, rid), solo_frames[6])
    pool.close()


@pytest.mark.parametrize("L,n_steps,max_pool", [(1, 1, 1), (1, 6, 5), (16, 3, 17), (17, 3, 33), (1024, 3, 2)])
def test_edge_sizes_fp32(L, n_steps, max_pool, weights_fp32):
    say(f"case: edge sizes L={L} n_steps={n_steps} max_pool={max_pool}")
    wl = synth.small_workload(1, L, L, n_steps, n_steps, seed=100 + L)
    pool = make_pool(wl, weights_fp32, max_pool=max_pool, max_enc_len=max(L, 1), max_steps=n_steps, chunk_frames=4)
    rid = pool.add_request(wl.encoder_outputs(0), n_steps)
    pool.step_n(n_steps + 2)
    got = _drain(pool, rid)[None]
    pool.close()
    ref, _, _ = oracle_decode(wl, weights_fp32, [0], n_steps)
    assert got.shape == (1, n_steps, 80)
    assert max_err(got, ref) <= TOL_F32


def test_single_location_channel():
    say("case: location conv with one input channel (W_acc only)")
    dims = dict(synth.DIMS, loc_in_channels=1)
    w = synth.make_weights(dims=dims)
    wl = synth.small_workload(3, 20, 60, 12, 12, seed=21)
    wl.dims = dims
    got = gpu_decode(wl, w, [0, 1, 2], 12)
    ref, _, _ = oracle_decode(wl, w, [0, 1, 2], 12)
    assert max_err(got, ref) <= TOL_F32


def test_c4_full_pool_bf16(weights_bf16):
    """256 requests at the full c4 shape (bench launch configuration: graphs,
    bf16 memory): oracle on a 16-request sample over 50 steps; the other
    requests are covered by the pool-composition invariance."""
    wl = synth.workload("c4")
    say("case c4: 256 requests L in [50,400], first 50 steps, bf16; oracle on 16 of them")
    gpu = gpu_decode(wl, weights_bf16, list(range(256)), 50)
    assert np.isfinite(gpu).all()
    sample = list(range(0, 256, 16))
    ref, _, _ = oracle_decode(wl, weights_bf16, sample, 50, n_threads=16)
    err = max_err(gpu[sample], ref)
    say(f"  max abs err {err:.3e}")
    assert err <= TOL_BF16
    # alone in a pool of the same capacity (the capacity fixes how the attention query is computed)
    solo = gpu_decode(wl, weights_bf16, [37], 50, max_pool=256)
    np.testing.assert_array_equal(solo[0], gpu[37])


def test_small_and_large_capacity_pools_agree(wl8, weights_fp32, solo_frames):
    """Pools of at most 64 slots form part of the next step's gates beside the projection and
    hand the attention query over as partial products, larger ones contract all of K in the
    LSTM kernels and compute the query in the attention kernel: the same numbers up to
    summation order."""
    say("case capacity: max_pool 8 vs 80, fp32")
    big = gpu_decode(wl8, weights_fp32, list(range(8)), 24, max_pool=80)
    for i in range(8):
        n = solo_frames[i].shape[0]
        assert np.abs(big[i, :n] - solo_frames[i]).max() <= 1e-5


@pytest.mark.parametrize("bf16,max_pool,n_req", [(True, 32, 24), (True, 48, 40), (False, 48, 36), (False, 64, 52),
                                                  (True, 80, 70), (True, 96, 90), (True, 112, 100), (True, 128, 120), (True, 160, 150),
                                                  (True, 176, 170), (True, 208, 200)])
def test_pools_of_several_tiles_with_gate_presums(bf16, max_pool, n_req, weights_bf16, weights_fp32):
    """Pools of two to four tiles: the pre-sum workgroups split by pool tiles (one group up to two
    tiles, two groups of 2 + 1 or 2 + 2 tiles above) and take one to three row tiles each.  bf16 pools of
    more tiles pre-sum the attention LSTM's late columns only, in groups of at most four tiles walked one
    at a time (5 to 8 tiles: two groups; 10 and 11: three, with two idle workgroups per XCD; 13: four, the last of
    one tile), and their
    projection runs as three or two workgroups per tile.  Against the oracle on a sample, and a request's
    bits do not depend on the pool's composition (alone in slot 0 vs among all, vs among 5 joining in
    another order: the same sums whether the pool spans one tile or eleven)."""
    weights = weights_bf16 if bf16 else weights_fp32
    wl = synth.small_workload(n_req, 10, 120, 30, 30, seed=71, bf16=bf16)
    say(f"case capacity {max_pool}, {'bf16' if bf16 else 'fp32'}: {n_req} requests, 30 steps")
    full = gpu_decode(wl, weights, list(range(n_req)), 30, max_pool=max_pool)
    sample = [0, 7, 16, n_req - 1]
    ref, _, _ = oracle_decode(wl, weights, sample, 30, n_threads=4)
    for k, i in enumerate(sample):
        assert np.abs(full[i] - ref[k]).max() <= (TOL_BF16 if bf16 else TOL_F32)
    alone = gpu_decode(wl, weights, [7], 30, max_pool=max_pool)[0]
    np.testing.assert_array_equal(alone, full[7])
    few = gpu_decode(wl, weights, [20, 3, 7, 11, 0], 30, max_pool=max_pool)
    np.testing.assert_array_equal(few[2], full[7])
    np.testing.assert_array_equal(few[4], full[0])


@pytest.mark.parametrize("bf16,max_pool", [(False, 20), (True, 20), (True, 200)])
def test_state_overwrite_refreshes_the_gate_presums(bf16, max_pool, weights_bf16, weights_fp32):
    """A request's H_att, A and H_dec are overwritten between steps with another request's: the
    pre-sums formed from the old state during the last projection must not reach the next step.
    Two pools run the same request; in the second its recurrent state is first replaced by
    garbage, then by the first pool's: the following frames are identical.  (Capacity 200, bf16: the
    pool keeps pre-sums of the attention LSTM only.  Capacity 20, bf16: the decoder LSTM's pre-sums are formed inside
    the step that uses them.)"""
    say(f"case: set_state between steps in a pool with gate pre-sums, capacity {max_pool}")
    wl8 = synth.small_workload(8, 5, 90, 24, 24, seed=11, bf16=bf16)
    weights_fp32 = weights_bf16 if bf16 else weights_fp32
    pools, rids = [], []
    for k in range(2):
        pool = make_pool(wl8, weights_fp32, max_pool=max_pool, max_enc_len=int(wl8.enc_len.max()), max_steps=24, chunk_frames=24)
        # the neighbour in the same tile keeps its own state (its pre-sums are formed again with the tile's)
        ids = [pool.add_request(wl8.encoder_outputs(i), 24) for i in (2, 5)]
        pool.step_n(7)
        pools.append(pool)
        rids.append(ids)
    a, b = pools
    rng = np.random.default_rng(5)
    for name in ("h_att", "a", "h_dec"):
        good = a.get_state(rids[0][0], name)
        b.set_state(rids[1][0], name, rng.standard_normal(good.shape).astype(np.float32))
        b.set_state(rids[1][0], name, good)
    for pool in pools:
        pool.step_n(17)
    for k in range(2):
        np.testing.assert_array_equal(_drain(a, rids[0][k]), _drain(b, rids[1][k]))
    for pool in pools:
        pool.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_wait_bound_zero_loses_only_the_step_in_flight_and_the_pool_goes_on(bf16, request):
    """In pools of at most 64 slots workgroups wait, a bounded number of polls, for words other workgroups hand
    them.  With the bound set to zero (forced from the host: every kernel still runs through) every such wait gives
    up at once.  The requests whose words were missing are frozen at the frames they have -- nothing invalid is ever
    stored -- and reported once; after that the same pool serves new requests with exactly the solo frames again.
    (Two-byte pools: the waits of the three-launch step too -- the projection's workers for the decoder LSTM's words,
    their leader for the workers' sums.)"""
    wl8, weights_fp32, solo_frames = _mode(request, bf16)
    from paper_2211_13939_amd import binding
    from paper_2211_13939_amd.binding import TtsError
    say("case: wait bound 0 (give-up path, forced from the host), then the same pool again")
    pool = make_pool(wl8, weights_fp32, max_pool=8, max_enc_len=90, max_steps=24, chunk_frames=24)
    rids = [pool.add_request(wl8.encoder_outputs(i), 24) for i in (1, 2)]
    pool.step_n(3)
    pool.sync()                      # fine so far
    assert not pool.lost(rids[0])
    pool.set_wait_polls(0)
    pool.step_n(2)                   # returns: nothing hangs
    with pytest.raises(TtsError) as info:
        pool.sync()
    assert info.value.code == binding.TTS_E_LOST and str(rids[0]) in str(info.value)
    pool.sync()                      # said once; the pool is usable
    for k, i in enumerate((1, 2)):
        assert pool.lost(rids[k])
        assert pool.frames(rids[k]) == (3, True)
        got = _drain(pool, rids[k])  # the frames made before the give-up are valid and complete
        np.testing.assert_array_equal(got, solo_frames[i][:3])
        pool.retire(rids[k])
    # with the bound still at zero a new request is lost at its first step, and says so
    rid = pool.add_request(wl8.encoder_outputs(3), 24)
    pool.step_n(4)
    with pytest.raises(TtsError):
        pool.sync()
    assert pool.lost(rid) and pool.frames(rid) == (0, True)
    pool.retire(rid)
    # the default bound again: the same pool, the same slots, the solo frames bit for bit
    pool.set_wait_polls(1 << 18)
    again = [pool.add_request(wl8.encoder_outputs(i), 24) for i in (1, 2, 3)]
    pool.step_n(24)
    pool.sync()
    for k, i in enumerate((1, 2, 3)):
        assert not pool.lost(again[k])
        np.testing.assert_array_equal(_drain(pool, again[k]), solo_frames[i])
    pool.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_steps_beside_other_work_on_the_gpu(bf16, request):
    """The kernels of a step wait for words of partner workgroups (bounded).  With another stream keeping the CUs
    busy a partner may start late: the frames must not change and no wait may run out."""
    import torch
    wl8, weights_fp32, solo_frames = _mode(request, bf16)
    say("case: decoder steps while a second stream runs large matrix products")
    pool = make_pool(wl8, weights_fp32, max_pool=8, max_enc_len=90, max_steps=24, chunk_frames=24)
    rids = [pool.add_request(wl8.encoder_outputs(i), 24) for i in range(8)]
    side = torch.cuda.Stream(device=pool.device)
    a = torch.randn(4096, 4096, device=pool.device)
    with torch.cuda.stream(side):
        for _ in range(40):
            a = (a @ a) * 1e-4
    for _ in range(6):
        pool.step_n(4)
    pool.sync()                      # raises if a wait ran out
    side.synchronize()
    for i, rid in enumerate(rids):
        np.testing.assert_array_equal(_drain(pool, rid), solo_frames[i])
    pool.close()


def test_c3_shrinking_pool_full_job(weights_bf16):
    """The whole c3 job as the benchmark runs it (all requests join in one call, requests retire at
    their own end, the running ones are packed into fewer tiles as the pool shrinks): every request
    produces exactly its frame count, sampled requests match the oracle over their first 50 frames
    and, to their last frame, the bits of the same request decoded alone (which never moves)."""
    wl = synth.workload("c3")
    say("case c3: full job, 64 requests, pool shrinks")
    pool = make_pool(wl, weights_bf16)
    ids = pool.add_requests([wl.encoder_outputs(i) for i in range(64)], [int(x) for x in wl.n_steps])
    longest = int(np.argmax(wl.n_steps))
    sample = sorted({3, 30, 59, longest})
    total = 0
    while pool.n_active():
        total += pool.step_n(40)
        for i, rid in enumerate(ids):
            if rid is not None and pool.frames(rid)[1] and i not in sample:
                pool.retire(rid)
                ids[i] = None
    assert total == int(wl.n_steps.sum())
    assert pool.moves() > 0
    ref, _, _ = oracle_decode(wl, weights_bf16, sample, 50, n_threads=4)
    for k, i in enumerate(sample):
        got = _drain(pool, ids[i])
        assert got.shape[0] == wl.n_steps[i] and np.isfinite(got).all()
        assert np.abs(got[:50] - ref[k]).max() <= TOL_BF16
        alone = gpu_decode(wl, weights_bf16, [i], int(wl.n_steps[i]), max_pool=64)[0]
        np.testing.assert_array_equal(got, alone)
    pool.close()


def test_large_attention_vector_takes_the_two_pass_softmax(weights_fp32):
    """With sum |v| <= 30 the attention kernel subtracts that bound instead of the maximum energy and
    forms the softmax in one pass; a model with a larger v takes the maximum-subtracting passes.
    Both must match the oracle: v scaled up eight-fold (sum |v| about 40) here, the default elsewhere."""
    w = dict(weights_fp32)
    w["v"] = (w["v"] * 8.0).astype(np.float32)
    assert np.abs(w["v"]).sum() > 30.0 > np.abs(weights_fp32["v"]).sum()
    wl = synth.small_workload(5, 10, 120, 12, 12, seed=41)
    say("case large v: 5 requests, 12 steps, fp32, sum|v| = %.1f" % np.abs(w["v"]).sum())
    gpu = gpu_decode(wl, w, list(range(5)), 12)
    ref, _, _ = oracle_decode(wl, w, list(range(5)), 12, n_threads=5)
    err = max_err(gpu, ref)
    say(f"  max abs err {err:.3e}")
    assert err <= TOL_F32


@pytest.mark.parametrize("bf16,max_pool,n_req", [(True, 64, 60), (False, 64, 44), (True, 160, 150), (False, 100, 90)])
def test_requests_move_to_lower_slots_when_the_pool_shrinks(bf16, max_pool, n_req, weights_bf16, weights_fp32):
    """Two of every three requests end after 6 steps and are retired; the others, scattered over all
    tiles, are moved into the freed low slots before the next step (first into half the span or
    less, later, after more of them left, further down) and carry on: their frames, those produced
    before a move but handed out after it included, are bit for bit the frames of a pool in which
    nobody leaves or moves, and their recurrent state reads back the same."""
    weights = weights_bf16 if bf16 else weights_fp32
    wl = synth.small_workload(n_req, 10, 120, 30, 30, seed=83, bf16=bf16)
    say(f"case capacity {max_pool}, {'bf16' if bf16 else 'fp32'}: {n_req} requests, two of three leave after 6 steps")
    stay = list(range(0, n_req, 3))
    ref = gpu_decode(wl, weights, list(range(n_req)), 30, max_pool=max_pool, chunk_frames=8)
    still = make_pool(wl, weights, max_pool=max_pool, max_steps=30, chunk_frames=8)
    still_ids = [still.add_request(wl.encoder_outputs(i), 30) for i in range(n_req)]
    still.step_n(10)
    assert still.moves() == 0 and still.span() == n_req

    pool = make_pool(wl, weights, max_pool=max_pool, max_steps=30, chunk_frames=8)
    ids = [pool.add_request(wl.encoder_outputs(i), 30 if i in stay else 6) for i in range(n_req)]
    pool.step_n(6)
    for i, rid in enumerate(ids):
        if i not in stay:
            np.testing.assert_array_equal(_drain(pool, rid), ref[i, :6])
            pool.retire(rid)
    assert pool.moves() == 0 and pool.span() == stay[-1] + 1
    pool.step_n(4)                                # the move happens here, with 6 frames waiting in each ring
    small = 1 << (len(stay) - 1).bit_length()
    assert pool.moves() > 0 and pool.span() <= small < n_req
    got = {i: [pool.drain_chunk(ids[i])[0].copy()] for i in stay}      # frames 0..7
    for name in ("m", "a", "w_last", "w_acc", "h_att", "c_att", "h_dec", "c_dec"):
        for i in (stay[0], stay[-1]):
            np.testing.assert_array_equal(pool.get_state(ids[i], name), still.get_state(still_ids[i], name))
    still.close()
    # a second round of leaving: only every fourth of the rest stays
    moves = pool.moves()
    for k, i in enumerate(stay):
        if k % 4:
            pool.retire(ids[i])
    last = stay[::4]
    pool.step_n(20)
    if small > 16:
        assert pool.moves() > moves and pool.span() <= max(16, small // 4)
    for i in last:
        got[i].append(_drain(pool, ids[i]))
        np.testing.assert_array_equal(np.concatenate(got[i]), ref[i])
    for i in stay:
        if i not in last:
            np.testing.assert_array_equal(got[i][0], ref[i, :8])
    pool.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_joining_together_equals_joining_one_by_one(bf16, weights_bf16, weights_fp32):
    """tts_pool_add_requests: 70 requests at once (two launches; encoder outputs in device memory, every
    seventh in host memory, lengths 1, 7, 8, 9 and the maximum among them) against the same requests
    added one call at a time: identical frames and attention state.  Nothing is added when one of the
    requests is invalid or the pool lacks room."""
    import torch
    weights = weights_bf16 if bf16 else weights_fp32
    wl = synth.small_workload(70, 10, 200, 12, 12, seed=91, bf16=bf16)
    wl.enc_len[:5] = [1, 7, 8, 9, 200]
    say(f"case: 70 requests join in one call, {'bf16' if bf16 else 'fp32'}")
    encs = [wl.encoder_outputs(i) for i in range(70)]
    mixed = [e if i % 7 == 3 else torch.from_numpy(e).cuda() for i, e in enumerate(encs)]
    kw = dict(max_pool=80, max_enc_len=200, max_steps=12, chunk_frames=12)
    one = make_pool(wl, weights, **kw)
    ids_one = [one.add_request(e, 12) for e in mixed]
    many = make_pool(wl, weights, **kw)
    with pytest.raises(binding.TtsError) as ei:
        many.add_requests(mixed + mixed[:11], [12] * 81)
    assert ei.value.code == binding.TTS_E_FULL and many.size() == 0
    with pytest.raises(binding.TtsError) as ei:
        many.add_requests(mixed[:3], [12, 13, 12])
    assert ei.value.code == binding.TTS_E_INVAL and many.size() == 0
    assert many.add_requests([], []) == []
    ids_many = many.add_requests(mixed, [12] * 70)
    assert many.size() == 70 and len(set(ids_many)) == 70
    for pool in (one, many):
        pool.step_n(12)
    for a, b in zip(ids_one, ids_many):
        np.testing.assert_array_equal(_drain(one, a), _drain(many, b))
    for i in (0, 3, 4, 69):
        np.testing.assert_array_equal(one.get_state(ids_one[i], "w_acc"), many.get_state(ids_many[i], "w_acc"))
    ref, _, _ = oracle_decode(wl, weights, [0, 2, 3, 4, 66], 12, n_threads=5)
    many2 = make_pool(wl, weights, **kw)
    ids2 = many2.add_requests(mixed, [12] * 70)
    many2.step_n(12)
    for k, i in enumerate([0, 2, 3, 4, 66]):
        assert np.abs(_drain(many2, ids2[i]) - ref[k]).max() <= (TOL_BF16 if bf16 else TOL_F32)
    for pool in (one, many, many2):
        pool.close()


def test_moves_with_a_stop_threshold():
    """With a stop threshold a request may have ended on the device before the host knows (its frame
    counter is then the host's upper bound, its done flag is set): moved or not, every request keeps
    its frames, its frame count and its stop logits."""
    say("case: slot moves in a pool with a stop threshold")
    w = synth.make_weights()
    w["stop_b"] = w["stop_b"].copy()
    w["stop_b"][:] = 0.2
    thr = 0.62
    wl = synth.small_workload(40, 5, 90, 24, 24, seed=11)
    kw = dict(max_pool=48, max_enc_len=90, max_steps=24, chunk_frames=24, stop_threshold=thr)
    still, moved = make_pool(wl, w, **kw), make_pool(wl, w, **kw)
    encs = [wl.encoder_outputs(i) for i in range(40)]
    ids_s = still.add_requests(encs, [24] * 40)
    ids_m = moved.add_requests(encs, [24] * 40)
    leave = [i for i in range(32) if i % 2]
    still.step_n(24)
    moved.step_n(6)
    for i in leave:
        moved.retire(ids_m[i])
    moved.step_n(18)
    assert still.moves() == 0 and moved.moves() == 8 and moved.span() <= 32
    n_early = 0
    for i in range(40):
        if i in leave:
            continue
        n_s, fin_s = still.frames(ids_s[i])
        n_m, fin_m = moved.frames(ids_m[i])
        assert (n_s, fin_s) == (n_m, fin_m) and fin_s
        n_early += n_s < 24
        np.testing.assert_array_equal(moved.stop_logits(ids_m[i], 0, n_m), still.stop_logits(ids_s[i], 0, n_s))
        np.testing.assert_array_equal(_drain(moved, ids_m[i]), _drain(still, ids_s[i]))
    assert n_early >= 1
    still.close()
    moved.close()


@pytest.mark.parametrize("n_req", [20, 40, 70, 100, 140, 180, 230])
def test_large_capacity_pool_at_partial_occupancy(n_req, weights_bf16):
    """A pool of capacity 256 (bf16: pre-sums of the attention LSTM only, two projection workgroups per
    tile) that holds fewer requests launches over the tiles they span (2, 3, 5, 7, 9, 12, 15 here): a
    request's frames are those it produces alone in such a pool, and a sample matches the oracle."""
    wl = synth.small_workload(n_req, 10, 120, 20, 20, seed=97, bf16=True)
    say(f"case capacity 256, bf16: {n_req} requests, 20 steps")
    full = gpu_decode(wl, weights_bf16, list(range(n_req)), 20, max_pool=256)
    sample = [0, 17, n_req - 1]
    ref, _, _ = oracle_decode(wl, weights_bf16, sample, 20, n_threads=3)
    for k, i in enumerate(sample):
        assert np.abs(full[i] - ref[k]).max() <= TOL_BF16
    alone = gpu_decode(wl, weights_bf16, [17], 20, max_pool=256)[0]
    np.testing.assert_array_equal(alone, full[17])
    np.testing.assert_array_equal(gpu_decode(wl, weights_bf16, [n_req - 1], 20, max_pool=256)[0], full[n_req - 1])


@pytest.mark.parametrize("bf16,seed", [(True, 5), (False, 6)])
def test_random_arrivals_and_departures(bf16, seed, weights_bf16, weights_fp32):
    """150 requests arrive in random groups, run for 8 to 40 steps each and leave at their end, in a pool of
    48 slots that is stepped 1 to 8 steps at a time and drained in chunks of 8: slots are reused, the pool is
    packed again and again, and every request's frames are bit for bit those of a pool in which nobody leaves
    or moves."""
    weights = weights_bf16 if bf16 else weights_fp32
    rng = np.random.default_rng(seed)
    wl = synth.small_workload(150, 5, 60, 8, 40, seed=200 + seed, bf16=bf16)
    say(f"case: random arrivals and departures, {'bf16' if bf16 else 'fp32'}")
    kw = dict(max_pool=48, max_enc_len=60, max_steps=40, chunk_frames=8)
    ref = {}
    for b0 in range(0, 150, 48):
        idx = list(range(b0, min(150, b0 + 48)))
        out = gpu_decode(wl, weights, idx, 40, **kw)
        for k, i in enumerate(idx):
            ref[i] = out[k, : wl.n_steps[i]]
    pool = make_pool(wl, weights, **kw)
    nxt, live, got, moves_seen = 0, {}, {i: [] for i in range(150)}, 0
    while nxt < 150 or live:
        room = 48 - pool.size()
        n_new = int(min(room, 150 - nxt, rng.integers(0, 12)))
        if n_new:
            idx = list(range(nxt, nxt + n_new))
            for i, rid in zip(idx, pool.add_requests([wl.encoder_outputs(i) for i in idx], [int(wl.n_steps[i]) for i in idx])):
                live[rid] = i
            nxt += n_new
        if not live:
            continue
        pool.step_n(int(rng.integers(1, 9)))
        for rid in list(live):
            while True:
                frames, fin = pool.drain_chunk(rid)
                if frames.shape[0]:
                    got[live[rid]].append(frames.copy())
                if fin or frames.shape[0] == 0:
                    break
            if fin:
                pool.retire(rid)
                del live[rid]
    assert pool.moves() > 0 and pool.size() == 0
    for i in range(150):
        np.testing.assert_array_equal(np.concatenate(got[i]), ref[i])
    pool.close()


@pytest.mark.parametrize("stop_threshold,n_req,max_pool", [(-1.0, 20, 20), (0.62, 20, 20), (-1.0, 90, 150), (0.62, 40, 256)])
def test_steps_of_one_call_equal_one_call_per_step_to_the_state(stop_threshold, n_req, max_pool):
    """Two-byte pools of at most 64 slots form the attention LSTM of step t + 1 inside the last launch of step t when
    both steps belong to one call; the first step of a call launches its own.  Both forms must leave the same bits:
    frames, stop values and every piece of the carried state, also for requests that end inside a call (by their
    frame count or by the stop threshold), whose state must stay where their last step left it.  (Capacities 150
    and 256: larger pools, whose steps are the same four launches either way, at six and three tiles.)"""
    say(f"case: steps of one call vs one call per step, frames and state (stop threshold {stop_threshold}, "
        f"{n_req} requests, capacity {max_pool})")
    wl = synth.small_workload(n_req, 5, 90, 24, 24, seed=23, bf16=True)
    w = synth.make_weights(bf16=True)
    w["stop_b"] = w["stop_b"].copy()
    w["stop_b"][:] = 0.2
    n_steps = [3 + (5 * i) % 20 for i in range(n_req)]     # 3 .. 22 frames: most end inside the one call
    pools, ids = [], []
    for _ in range(2):
        p = make_pool(wl, w, max_pool=max_pool, max_enc_len=90, max_steps=24, chunk_frames=24, stop_threshold=stop_threshold)
        ids.append([p.add_request(wl.encoder_outputs(i), n_steps[i]) for i in range(n_req)])
        pools.append(p)
    pools[0].step_n(24)
    for _ in range(24):
        pools[1].step()
    for p in pools:
        p.sync()
    ended_early = 0
    for a, b in zip(*ids):
        fa, fb = pools[0].frames(a), pools[1].frames(b)
        assert fa == fb and fa[1]
        ended_early += fa[0] < 24
        np.testing.assert_array_equal(pools[0].stop_logits(a, 0, fa[0]), pools[1].stop_logits(b, 0, fb[0]))
        for name in ("m", "a", "w_last", "w_acc", "h_att", "c_att", "h_dec", "c_dec"):
            np.testing.assert_array_equal(pools[0].get_state(a, name), pools[1].get_state(b, name), err_msg=name)
        np.testing.assert_array_equal(_drain(pools[0], a), _drain(pools[1], b))
    assert ended_early >= 3 * n_req // 4
    for p in pools:
        p.close()


def test_wait_bound_zero_in_a_pool_above_64_slots(weights_bf16):
    """Pools of more than 64 slots with two-byte weights form the decoder LSTM inside the last kernel's launch once
    they span more than 16 slots, and the projection's workgroups wait (a bounded number of polls) for the words it
    hands them.  With the bound at zero, forced from the host, every such wait gives up at once and every kernel still
    runs through: the requests are reported lost with the frames they had, and the same pool then decodes new requests
    to the frames a pool of the same capacity yields with the default bound."""
    from paper_2211_13939_amd import binding
    from paper_2211_13939_amd.binding import TtsError
    say("case: wait bound 0 in a capacity-100 pool of 20 requests (two tiles), then the same pool again")
    wl = synth.small_workload(20, 5, 90, 12, 12, seed=31, bf16=True)

    def decode(pool):
        ids = [pool.add_request(wl.encoder_outputs(i), 12) for i in range(20)]
        pool.step_n(12)
        pool.sync()
        out = [_drain(pool, rid) for rid in ids]
        for rid in ids:
            pool.retire(rid)
        return out

    ref_pool = make_pool(wl, weights_bf16, max_pool=100, max_enc_len=90, max_steps=12, chunk_frames=12)
    want = decode(ref_pool)
    ref_pool.close()
    pool = make_pool(wl, weights_bf16, max_pool=100, max_enc_len=90, max_steps=12, chunk_frames=12)
    ids = [pool.add_request(wl.encoder_outputs(i), 12) for i in range(20)]
    pool.step_n(3)
    pool.sync()
    pool.set_wait_polls(0)
    pool.step_n(2)                   # returns: nothing hangs
    with pytest.raises(TtsError) as info:
        pool.sync()
    assert info.value.code == binding.TTS_E_LOST
    pool.sync()                      # said once
    for k, rid in enumerate(ids):
        assert pool.lost(rid) and pool.frames(rid) == (3, True)
        np.testing.assert_array_equal(_drain(pool, rid), want[k][:3])
        pool.retire(rid)
    pool.set_wait_polls(1 << 18)
    got = decode(pool)
    for a, b in zip(got, want):
        np.testing.assert_array_equal(a, b)
    pool.close()


@pytest.mark.parametrize("max_pool,n_req", [(16, 10), (200, 120)])
def test_kernel_times_follow_the_form_of_a_call(max_pool, n_req, weights_bf16):
    """tts_pool_kernel_times launches its steps as one call launches them and reports per kernel: a pool of at most 64
    slots has an attention-LSTM launch only in the call's first step and a last kernel that differs in the call's last
    step; neither that pool nor one of more than 64 slots (two-byte weights) has a decoder-LSTM kernel.  The timed steps
    are real steps: the frames equal those of a pool stepped without timing."""
    say(f"case: kernel times, capacity {max_pool}, {n_req} requests")
    wl = synth.small_workload(n_req, 5, 90, 12, 12, seed=41, bf16=True)
    a = make_pool(wl, weights_bf16, max_pool=max_pool, max_enc_len=90, max_steps=12, chunk_frames=12)
    b = make_pool(wl, weights_bf16, max_pool=max_pool, max_enc_len=90, max_steps=12, chunk_frames=12)
    ia = [a.add_request(wl.encoder_outputs(i), 12) for i in range(n_req)]
    ib = [b.add_request(wl.encoder_outputs(i), 12) for i in range(n_req)]
    a.step_n(2)
    us = a.kernel_times_us(8)
    a.step_n(2)
    b.step_n(12)
    assert us["k_lstm_att"] > 0 and us["k_lsa"] > 0 and us["k_proj"] > 0 and us["k_lstm_dec"] == 0
    assert ("k_proj_last_step" in us) == (max_pool <= 64)
    for x, y in zip(ia, ib):
        np.testing.assert_array_equal(_drain(a, x), _drain(b, y))
    a.close()
    b.close()


def test_steps_of_a_pool_above_64_slots_beside_other_work_on_the_gpu(weights_bf16):
    """As test_steps_beside_other_work_on_the_gpu, for a pool whose last launch holds the decoder LSTM and whose
    projection workgroups wait for its words: with another stream keeping the CUs busy the frames must not change
    and no wait may run out."""
    import torch
    say("case: capacity-100 pool of 40 requests while a second stream runs large matrix products")
    wl = synth.small_workload(40, 5, 90, 24, 24, seed=43, bf16=True)

    def decode(busy):
        pool = make_pool(wl, weights_bf16, max_pool=100, max_enc_len=90, max_steps=24, chunk_frames=24)
        rids = [pool.add_request(wl.encoder_outputs(i), 24) for i in range(40)]
        side = torch.cuda.Stream(device=pool.device)
        if busy:
            a = torch.randn(4096, 4096, device=pool.device)
            with torch.cuda.stream(side):
                for _ in range(40):
                    a = (a @ a) * 1e-4
        for _ in range(6):
            pool.step_n(4)
        pool.sync()                      # raises if a wait ran out
        side.synchronize()
        out = [_drain(pool, rid) for rid in rids]
        pool.close()
        return out

    quiet, busy = decode(False), decode(True)
    for a, b in zip(quiet, busy):
        np.testing.assert_array_equal(a, b)
