"""Host logic of the arrival-driven serving loop (Sec. 2.2.2) against the
latency closed form of Sec. 2.2.3, with a model backend of constant step time."""
import os

import numpy as np

from paper_2211_13939_amd import stream

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "first_chunk_latency_sec_2_2_3.txt")


def _paper_bounds():
    """name -> (coefficient of T_t, coefficient of T_{t+1}) as the paper states them."""
    out = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            name, a, b = line.split()
            out[name] = (float(a), float(b))
    return out


class ModelBackend(stream.PoolBackend):
    """Every step takes `t_step` seconds whatever the pool holds."""

    def __init__(self, n_steps, chunk, t_step):
        self.n_steps, self.chunk, self.t_step = n_steps, chunk, t_step
        self.live = {}
        self.next_id = 1
        self.membership = []

    def add(self, index):
        rid = self.next_id
        self.next_id += 1
        self.live[rid] = dict(index=index, done=0, total=int(self.n_steps[index]), drained=0)
        return rid

    def run(self, k):
        self.membership.append((k, sorted(s["index"] for s in self.live.values())))
        chunks, fins = [], []
        for rid, s in self.live.items():
            s["done"] = min(s["total"], s["done"] + k)
            while s["done"] - s["drained"] >= self.chunk:
                s["drained"] += self.chunk
                chunks.append(rid)
            if s["done"] == s["total"]:
                if s["drained"] < s["done"]:
                    s["drained"] = s["done"]
                    chunks.append(rid)
                fins.append(rid)
        return k * self.t_step, chunks, fins

    def retire(self, rid):
        self.live.pop(rid)


def test_first_chunk_latency_closed_form():
    """One iteration = one chunk for every pooled request, constant time T.  A
    request arriving during iteration t waits for its end, then needs T_{t+1}:
    latency in [T, 2T], mean T/2 + T for uniform arrival phase."""
    chunk, t_step = 8, 1e-3
    T = chunk * t_step
    rng = np.random.default_rng(0)
    n_probe = 4000
    # request 0 keeps the loop busy for the whole experiment
    arrivals = np.concatenate([[0.0], np.sort(rng.uniform(T, 2000 * T, n_probe))])
    n_steps = np.concatenate([[2100 * chunk], np.full(n_probe, chunk)])
    be = ModelBackend(n_steps, chunk, t_step)
    res = stream.simulate(be, arrivals, n_steps, chunk, join_every=chunk)
    fcl = res.first_chunk_latency_s[1:]
    assert np.isfinite(fcl).all()
    b = _paper_bounds()
    t_max, t_mean, t_min = (sum(b[k]) * T for k in ("maximum", "expectation", "minimum_equal_iterations"))
    assert (t_max, t_mean, t_min) == (2 * T, 1.5 * T, T)
    assert fcl.min() >= t_min - 1e-12 and fcl.max() <= t_max + 1e-12
    assert abs(fcl.mean() - t_mean) < 0.02 * T
    assert abs(res.first_chunk_latency_s[0] - t_min) < 1e-12  # arrived right before an iteration: the minimum


def test_idle_server_serves_immediately_and_clock_jumps():
    chunk, t_step = 4, 1e-3
    arrivals = np.array([0.0, 1.0, 5.0])
    n_steps = np.array([10, 4, 9])
    be = ModelBackend(n_steps, chunk, t_step)
    res = stream.simulate(be, arrivals, n_steps, chunk, join_every=1)
    np.testing.assert_allclose(res.first_chunk_latency_s, [4e-3, 4e-3, 4e-3], atol=1e-12)
    np.testing.assert_allclose(res.last_chunk_latency_s, [10e-3, 4e-3, 9e-3], atol=1e-12)
    assert abs(res.busy_s - 23e-3) < 1e-12 and res.n_steps == 23
    assert abs(res.end_clock_s - 5.009) < 1e-9
    assert all(m == [0] or m == [1] or m == [2] for _, m in be.membership)


def test_per_step_join_batches_overlapping_requests():
    """With per-step joins a request arriving while another runs is in the batch
    of the next step; nobody queues behind the running request."""
    chunk, t_step = 4, 1e-3
    arrivals = np.array([0.0, 2.5e-3])
    n_steps = np.array([12, 8])
    be = ModelBackend(n_steps, chunk, t_step)
    res = stream.simulate(be, arrivals, n_steps, chunk, join_every=1, step_time_guess_s=t_step)
    # request 1 arrives during step 2 (t in [2,3) ms), joins at t = 3 ms, first chunk after 4 more steps
    assert abs(res.first_chunk_latency_s[1] - (3e-3 + 4e-3 - 2.5e-3)) < 1e-9
    assert abs(res.first_chunk_latency_s[0] - 4e-3) < 1e-9
    both = [k for k, m in be.membership if m == [0, 1]]
    assert sum(both) == 8


class LateBackend(ModelBackend):
    """The modules behind the decoder take `t_late` seconds and run beside it: a chunk is handed out that long
    after the segment that completed it (the fourth element of run's result)."""

    def __init__(self, n_steps, chunk, t_step, t_late):
        super().__init__(n_steps, chunk, t_step)
        self.t_late = t_late
        self.out = []            # (due time on the backend's own clock, index, last)
        self.now = 0.0

    def _due(self, until):
        got = [(i, t, last) for t, i, last in self.out if t <= until]
        self.out = [(t, i, last) for t, i, last in self.out if t > until]
        return got

    def run(self, k):
        elapsed, chunks, fins = super().run(k)
        start, end = self.now, self.now + elapsed
        for rid in chunks:
            s = self.live[rid]
            self.out.append((end + self.t_late, s["index"], s["drained"] == s["total"]))
        self.now = end
        # deliveries are reported as seconds from the start of the segment that hears of them
        got = [(i, max(0.0, t - start), last) for i, t, last in self._due(end)]
        return elapsed, [], fins, got

    def pending(self):
        return bool(self.out)

    def flush(self):
        start = self.now
        end = max(t for t, _, _ in self.out)
        self.now = end
        return end - start, [(i, t - start, last) for i, t, last in self._due(end)]


def test_late_deliveries_are_counted_when_they_arrive():
    """A backend whose later modules run beside the decoder: every chunk is handed out t_late after the segment
    that completed it, also when the request has left the pool or the pool has run empty meanwhile."""
    chunk, t_step, t_late = 4, 1e-3, 2.5e-3
    n_steps = np.array([8, 5, 4])
    arrivals = np.array([0.0, 0.0, 0.1])              # the third arrives long after the first two are through
    be = LateBackend(n_steps, chunk, t_step, t_late)
    res = stream.simulate(be, arrivals, n_steps, chunk, join_every=1, step_time_guess_s=t_step)
    # first chunks complete after 4 steps; request 1's last (one frame) after 5, request 0's after 8; request 2 runs alone
    np.testing.assert_allclose(res.first_chunk_latency_s, [4e-3 + t_late, 4e-3 + t_late, 4e-3 + t_late], rtol=0, atol=1e-9)
    np.testing.assert_allclose(res.last_chunk_latency_s, [8e-3 + t_late, 5e-3 + t_late, 4e-3 + t_late], rtol=0, atol=1e-9)
    assert not be.pending() and not be.live


class ModelRoundBackend(stream.RoundBackend):
    """A round takes (the longest request's steps) x t_step seconds whatever the batch holds."""

    def __init__(self, n_steps, t_step):
        self.n_steps, self.t_step = n_steps, t_step
        self.batches = []

    def round(self, indices):
        self.batches.append(list(indices))
        return max(int(self.n_steps[i]) for i in indices) * self.t_step


def test_non_incremental_twin_two_rounds_closed_form():
    """Sec. 3.1's non-incremental twin with a constant step time t: the batch is fixed for a round, a round lasts as
    long as its longest request, arrivals during a round queue for the next one, and the response is the whole
    utterance at the end of the round.  Requests 0, 1 are there at time 0 (100 and 40 steps); 2 and 3 arrive during
    the first round (30 and 70 steps); 4 arrives long after everything is done (25 steps)."""
    t = 1e-3
    n_steps = np.array([100, 40, 30, 70, 25])
    arrivals = np.array([0.0, 0.0, 10 * t, 50 * t, 500 * t])
    be = ModelRoundBackend(n_steps, t)
    res = stream.simulate_twin(be, arrivals, n_steps)
    assert be.batches == [[0, 1], [2, 3], [4]]
    want = np.array([100 * t, 100 * t, 170 * t - 10 * t, 170 * t - 50 * t, 25 * t])
    np.testing.assert_allclose(res.latency_s, want, rtol=0, atol=1e-12)
    assert [r["steps"] for r in res.rounds] == [100, 70, 25]
    assert abs(res.rounds[1]["start"] - 100 * t) < 1e-12 and abs(res.rounds[2]["start"] - 500 * t) < 1e-12
    # frames computed: 2 x 100 + 2 x 70 + 25; frames asked for: 265
    assert abs(res.padding_waste() - (365 - 265) / 365) < 1e-12
    assert abs(res.busy_s - 195 * t) < 1e-12 and abs(res.end_clock_s - 525 * t) < 1e-12


def test_twin_batch_limit_and_mixed_lengths_wait_for_the_longest():
    """With a batch limit the overflow waits a whole round; in a mixed batch the short request's latency is the long
    one's (the padding the paper blames for Mixed being as slow as Long), while the incremental loop lets it go after
    its own steps."""
    t = 1e-3
    n_steps = np.array([400, 40, 40])
    arrivals = np.zeros(3)
    res = stream.simulate_twin(ModelRoundBackend(n_steps, t), arrivals, n_steps, max_batch=2)
    np.testing.assert_allclose(res.latency_s, [400 * t, 400 * t, 440 * t], atol=1e-12)
    inc = stream.simulate(ModelBackend(n_steps, 40, t), arrivals, n_steps, 40, join_every=1)
    np.testing.assert_allclose(inc.last_chunk_latency_s, [400 * t, 40 * t, 40 * t], atol=1e-12)
