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
