"""Arrival-driven serving loop over a request pool (Sec. 2.2.2, 2.2.3).

The loop is the paper's "infinite loop": requests that have arrived join the
pool, every pooled request is advanced, full chunks are handed out, finished
requests leave.  Time is simulated: the clock advances by the *measured* wall
time of each segment of work, and jumps to the next arrival when the pool is
empty, so a 10 s arrival trace does not need 10 s of wall time.

Two join policies:
  join_every = chunk   the paper's iteration: module D produces one chunk for
                       every pooled request per iteration, arrivals wait for
                       the next iteration (first-chunk latency between T and
                       2T for constant iteration time T, mean 1.5 T).
  join_every = 1       a request joins before the next decoder step.

The non-incremental twin the paper compares with (Sec. 3.1) is here too, as a second loop over the same pool:
`simulate_twin` builds a batch from the requests received so far, keeps that batch unchanged for the whole round
(every request is decoded for as many steps as the round's longest needs, and is padded to the round's longest
encoder length), hands each request its complete result when the round ends, and lets later arrivals queue for the
next round.

This module is host logic only; the backend does the work.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np


class PoolBackend:
    """What the loop needs from a pool.  `run(k)` advances every pooled request
    by k steps, hands out every chunk that became ready and returns
    (elapsed seconds, ids whose chunk was handed out, ids that finished).

    A backend whose later modules run beside the decoder (on another stream)
    hands chunks out after the segment that produced them.  It returns a fourth
    element, a list of deliveries (request index, when, is the request's last):
    `when` is a time.perf_counter() value if the backend is timed by the loop
    (elapsed is None), else seconds from the start of the segment.  Its second
    element is then empty and its third names the requests that have finished
    DECODING (they leave the pool); `pending()` says whether deliveries are
    still out and `flush()` waits for them and returns (elapsed, deliveries)."""

    def pending(self) -> bool:
        return False

    def flush(self):
        return 0.0, []

    def add(self, index: int) -> int:
        raise NotImplementedError

    def run(self, k: int):
        raise NotImplementedError

    def retire(self, rid: int) -> None:
        raise NotImplementedError


@dataclass
class StreamResult:
    first_chunk_latency_s: np.ndarray
    last_chunk_latency_s: np.ndarray
    pool_size_hist: Dict[int, int]
    n_segments: int
    n_steps: int
    busy_s: float
    end_clock_s: float

    def percentiles(self, which="first"):
        x = self.first_chunk_latency_s if which == "first" else self.last_chunk_latency_s
        return {f"p{p}": float(np.percentile(x, p)) for p in (50, 95, 99)}


def simulate(backend: PoolBackend, arrival_s: Sequence[float], n_steps: Sequence[int], chunk: int,
             join_every: int = 1, step_time_guess_s: float = 30e-6, max_pool: Optional[int] = None) -> StreamResult:
    arrival_s = np.asarray(arrival_s, np.float64)
    n_steps = np.asarray(n_steps, np.int64)
    n = arrival_s.shape[0]
    order = np.argsort(arrival_s, kind="stable")
    nxt = 0                                  # next arrival (position in `order`) not yet admitted
    clock = 0.0
    live: Dict[int, dict] = {}               # rid -> {index, done_steps, first_seen}
    fcl = np.full(n, np.nan)
    lcl = np.full(n, np.nan)
    hist: Dict[int, int] = {}
    n_seg = 0
    total_steps = 0
    busy = 0.0
    step_est = step_time_guess_s

    def deliver(items, clock0, t0, timed_by_loop):
        for index, when, last in items:
            t = clock0 + ((when - t0) if timed_by_loop else when)
            if np.isnan(fcl[index]):
                fcl[index] = t - arrival_s[index]
            if last:
                lcl[index] = t - arrival_s[index]

    t_end = None                             # perf_counter at the end of the last timed stretch, while the pool stays busy
    while nxt < n or live or backend.pending():
        if not live and backend.pending():
            # nothing left to decode: wait for the chunks that the later modules still hold
            t0 = t_end if t_end is not None else time.perf_counter()
            elapsed, items = backend.flush()
            t_end = time.perf_counter()
            dt = (t_end - t0) if elapsed is None else float(elapsed)
            deliver(items, clock, t0, elapsed is None)
            clock += dt
            busy += dt
            if nxt >= n:
                continue
        if not live and nxt < n and arrival_s[order[nxt]] > clock:
            clock = float(arrival_s[order[nxt]])          # idle until the next arrival
            t_end = None
        # admit everything that has arrived (bounded by the pool's capacity); while the pool stays busy the clock
        # runs on from the end of the last segment, so that the loop's own bookkeeping is inside the measured time
        t0 = t_end if t_end is not None else time.perf_counter()
        while nxt < n and arrival_s[order[nxt]] <= clock and (max_pool is None or len(live) < max_pool):
            i = int(order[nxt])
            rid = backend.add(i)
            live[rid] = dict(index=i, done=0, total=int(n_steps[i]), first=False)
            nxt += 1
        if not live:
            continue
        # how many steps until something must happen on the host
        if join_every > 1:
            k = join_every
        else:
            k = min(_steps_to_event(s, chunk) for s in live.values())
            if nxt < n and (max_pool is None or len(live) < max_pool):
                gap = arrival_s[order[nxt]] - clock
                k = max(1, min(k, int(np.ceil(gap / max(step_est, 1e-9)))))
        hist[len(live)] = hist.get(len(live), 0) + k
        out = backend.run(k)
        elapsed, chunk_ids, fin_ids = out[0], out[1], out[2]
        # a real backend is timed here (joins, steps, drains); a model backend reports its own time
        t_end = time.perf_counter()
        dt = (t_end - t0) if elapsed is None else float(elapsed)
        if len(out) > 3:
            deliver(out[3], clock, t0, elapsed is None)
        clock += dt
        busy += dt
        n_seg += 1
        total_steps += k
        step_est = 0.8 * step_est + 0.2 * (dt / k)
        for s in live.values():
            s["done"] = min(s["total"], s["done"] + k)
        for rid in chunk_ids:
            s = live[rid]
            if not s["first"]:
                s["first"] = True
                fcl[s["index"]] = clock - arrival_s[s["index"]]
        for rid in fin_ids:
            s = live.pop(rid)
            if len(out) <= 3:
                if not s["first"]:
                    fcl[s["index"]] = clock - arrival_s[s["index"]]
                lcl[s["index"]] = clock - arrival_s[s["index"]]
            backend.retire(rid)
    return StreamResult(fcl, lcl, hist, n_seg, total_steps, busy, clock)


class RoundBackend:
    """What the non-incremental loop needs: `round(indices)` decodes the batch to its end and returns the elapsed
    seconds (None: the loop times it)."""

    def round(self, indices: Sequence[int]):
        raise NotImplementedError


@dataclass
class TwinResult:
    latency_s: np.ndarray            # per request: end of its round - arrival (the whole utterance is the response)
    rounds: List[dict]               # per round: start, duration, indices, steps, padded_frames, useful_frames
    busy_s: float
    end_clock_s: float

    def percentiles(self):
        return {f"p{p}": float(np.percentile(self.latency_s, p)) for p in (50, 95, 99)}

    def padding_waste(self) -> float:
        """Share of the decoder frames computed that no request asked for."""
        pad = sum(r["padded_frames"] for r in self.rounds)
        use = sum(r["useful_frames"] for r in self.rounds)
        return (pad - use) / max(1, pad)


def simulate_twin(backend: RoundBackend, arrival_s: Sequence[float], n_steps: Sequence[int],
                  max_batch: Optional[int] = None) -> TwinResult:
    """The non-incremental twin (Sec. 3.1): the requests received so far form a batch whose size stays unchanged for
    the whole inference round; requests that arrive during a round wait in the queue for the next one; a request's
    response is its whole utterance, at the end of its round."""
    arrival_s = np.asarray(arrival_s, np.float64)
    n_steps = np.asarray(n_steps, np.int64)
    n = arrival_s.shape[0]
    order = np.argsort(arrival_s, kind="stable")
    nxt, clock, busy = 0, 0.0, 0.0
    lat = np.full(n, np.nan)
    rounds: List[dict] = []
    while nxt < n:
        if arrival_s[order[nxt]] > clock:
            clock = float(arrival_s[order[nxt]])          # idle until the next request is received
        batch = []
        while nxt < n and arrival_s[order[nxt]] <= clock and (max_batch is None or len(batch) < max_batch):
            batch.append(int(order[nxt]))
            nxt += 1
        t0 = time.perf_counter()
        elapsed = backend.round(batch)
        dt = (time.perf_counter() - t0) if elapsed is None else float(elapsed)
        steps = int(n_steps[batch].max())
        rounds.append(dict(start=clock, duration=dt, indices=batch, steps=steps, padded_frames=steps * len(batch),
                           useful_frames=int(n_steps[batch].sum())))
        clock += dt
        busy += dt
        for i in batch:
            lat[i] = clock - arrival_s[i]
    return TwinResult(lat, rounds, busy, clock)


class GpuTwinBackend(RoundBackend):
    """A round on a binding.Pool: every request of the batch joins at once and is advanced for the round's longest
    step count (the padding steps are real decoder steps: the pool's step kernels run on all of the batch until the
    last request ends), then each utterance is copied to the host and the batch leaves.

    pad_memory: the encoder outputs are also padded with zero rows to the round's longest, as a batch tensor would be
    (the padded positions then take part in the attention like any other: this kernel set has no mask to give them
    zero weight with, since its own pool never pads); the frames are then a timing vehicle only.  Without it every
    request keeps its own length and its first n_i frames are exactly those of the incremental pool."""

    def __init__(self, pool, enc, n_steps, pad_memory: bool = True, on_result=None):
        self.pool, self.enc, self.n_steps, self.pad_memory, self.on_result = pool, enc, n_steps, pad_memory, on_result

    def round(self, indices):
        torch = self.pool._torch
        steps = int(max(self.n_steps[i] for i in indices))
        encs = [self.enc(i) for i in indices]
        if self.pad_memory:
            Lmax = max(int(e.shape[0]) for e in encs)
            padded = []
            for e in encs:
                t = e if torch.is_tensor(e) else torch.from_numpy(np.ascontiguousarray(e, np.float32))
                t = t.to(self.pool.device)
                if int(t.shape[0]) < Lmax:
                    with torch.cuda.stream(self.pool.stream):
                        t = torch.cat([t, torch.zeros((Lmax - int(t.shape[0]), t.shape[1]), dtype=t.dtype, device=t.device)])
                padded.append(t)
            self.pool.stream.synchronize()
            encs = padded
        ids = self.pool.add_requests(encs, [steps] * len(indices))
        self.pool.step_n(steps)
        for i, rid in zip(indices, ids):
            mel = self.pool.drain_all(rid)
            if self.on_result is not None:
                self.on_result(i, mel[: int(self.n_steps[i])])
            self.pool.retire(rid)
        return None


def _steps_to_event(s: dict, chunk: int) -> int:
    """Steps until this request completes its next chunk or finishes."""
    to_chunk = chunk - (s["done"] % chunk)
    to_end = s["total"] - s["done"]
    return max(1, min(to_chunk, to_end))


class GpuBackend(PoolBackend):
    """Drives a binding.Pool; encoder outputs are taken from `enc(i)` (host
    numpy or device tensor)."""

    def __init__(self, pool, enc, n_steps, chunk: int):
        self.pool, self.enc, self.n_steps, self.chunk = pool, enc, n_steps, chunk
        self.live: Dict[int, dict] = {}

    def add(self, index: int) -> int:
        rid = self.pool.add_request(self.enc(index), int(self.n_steps[index]))
        self.live[rid] = dict(index=index, done=0, total=int(self.n_steps[index]), drained=0)
        return rid

    def run(self, k: int):
        self.pool.step_n(k)
        chunk_ids, fin_ids = [], []
        for rid, s in self.live.items():
            s["done"] = min(s["total"], s["done"] + k)
            ready = s["done"] - s["drained"] >= self.chunk or s["done"] == s["total"]
            if ready:
                while True:
                    frames, fin = self.pool.drain_chunk(rid)
                    s["drained"] += frames.shape[0]
                    if frames.shape[0]:
                        chunk_ids.append(rid)
                    if fin:
                        fin_ids.append(rid)
                    if fin or frames.shape[0] == 0 or s["done"] - s["drained"] < self.chunk:
                        break
        if not chunk_ids and not fin_ids:
            self.pool.sync()
        return None, chunk_ids, fin_ids

    def retire(self, rid: int) -> None:
        self.pool.retire(rid)
        self.live.pop(rid, None)


class GpuPostnetBackend(GpuBackend):
    """Module D complete: the decoder step followed by the chunk-level PostNet.  Every chunk that
    becomes ready in a segment is handed over on the device (with its context frames) and all of
    them go through the PostNet as one dynamic batch (Sec. 2.2.2: each module batches the pool
    items it has to process), then one copy brings the post-processed chunks to the host."""

    N_SETS = 4      # staging buffer sets of the overlapped form: rounds that may be out at one time

    def __init__(self, pool, postnet, enc, n_steps, chunk: int, context: int, on_chunk=None, vocoder=None, on_audio=None,
                 overlap: bool = False):
        """on_chunk(request index, first frame, frames [n, n_mel]) is called for every chunk handed out.
        With a vocoder (module V) the post-processed chunks of a round go on, still on the device, through
        tts_vocoder_run as one dynamic batch (Eq. 3, Eq. 4: splice, generator, fade, state write-back) and the
        responses are the waveform pieces: on_audio(request index, samples [m]).

        overlap: the modules behind the decoder run on their own stream (the one `postnet` and `vocoder` were
        created on, which must not be the pool's) beside the next decoder steps: a round only waits for the copy of
        its chunks out of the pool, and the loop hears of a chunk when its response has reached the host (the
        deliveries of PoolBackend); the callbacks are made then."""
        super().__init__(pool, enc, n_steps, chunk)
        import torch
        self.postnet, self.context, self.on_chunk = postnet, context, on_chunk
        self.vocoder, self.on_audio = vocoder, on_audio
        self.overlap = overlap
        if overlap:
            assert postnet.stream.cuda_stream != pool.stream.cuda_stream, "the later modules need a stream of their own"
            assert vocoder is None or vocoder.stream.cuda_stream == postnet.stream.cuda_stream
            self._out = []          # rounds on the side stream: dict(ev, items, set)
        if vocoder is not None:
            cap_v = int(pool.cfg.max_pool)
            assert vocoder.cfg.max_requests >= cap_v and vocoder.cfg.max_batch >= cap_v and vocoder.cfg.max_chunk >= chunk
            self._free_slots = list(range(cap_v))[::-1]
            hop = 256
            self._d_audio = torch.empty(cap_v * (chunk + vocoder.cfg.overlap) * hop, dtype=torch.float32, device=pool.device)
            self._h_audio = torch.empty(cap_v * (chunk + vocoder.cfg.overlap) * hop, dtype=torch.float32).pin_memory()
        cap = int(pool.cfg.max_pool)
        self._d_in = torch.empty((cap * (chunk + context), pool.n_mel), dtype=torch.float32, device=pool.device)
        self._d_out = torch.empty((cap * chunk, pool.n_mel), dtype=torch.float32, device=pool.device)
        self._h_out = torch.empty((cap * chunk, pool.n_mel), dtype=torch.float32).pin_memory()
        if overlap:
            def one_set(first):
                d = dict(d_in=self._d_in if first else torch.empty_like(self._d_in),
                         d_out=self._d_out if first else torch.empty_like(self._d_out),
                         h_out=self._h_out if first else torch.empty_like(self._h_out).pin_memory(), ev=None)
                if vocoder is not None:
                    d["d_audio"] = self._d_audio if first else torch.empty_like(self._d_audio)
                    d["h_audio"] = self._h_audio if first else torch.empty_like(self._h_audio).pin_memory()
                return d
            self._sets = [one_set(i == 0) for i in range(self.N_SETS)]
            self._next_set = 0

    # ---- the overlapped form
    def _harvest(self):
        """Rounds whose responses have reached the host, oldest first: [(request index, perf_counter, last)]."""
        got = []
        while self._out and self._out[0]["ev"].query():
            r = self._out.pop(0)
            t = time.perf_counter()
            got += [(index, t, last) for index, last in r["items"]]
            st = r["set"]                   # its host buffers stay as they are until N_SETS - 1 more rounds have gone out
            if self.on_audio is not None and "n_out" in r:
                host, at = st["h_audio"].numpy(), 0
                for (index, _), m in zip(r["items"], r["n_out"]):
                    self.on_audio(index, host[at:at + m].copy())
                    at += m
            if self.on_chunk is not None:
                host = st["h_out"].numpy()
                for index, first, r0, n in r["handed"]:
                    self.on_chunk(index, first, host[r0:r0 + n].copy())
        return got

    def pending(self) -> bool:
        return self.overlap and bool(self._out)

    def flush(self):
        got = []
        while self._out:
            got += self._harvest()
        return None, got

    def _run_overlapped(self, k: int):
        torch = self.pool._torch
        main, side = self.pool.stream, self.postnet.stream
        self.pool.step_n(k)
        for s in self.live.values():
            s["done"] = min(s["total"], s["done"] + k)
        fin_ids, span = [], self.chunk + self.context
        while True:                         # a request that ends may hand out a full chunk and then its rest
            st = self._sets[self._next_set]
            if st["ev"] is not None:
                st["ev"].synchronize()      # the round that used this set last (N_SETS rounds ago) is through
            lens, keeps, row, out_rows, items, voc, handed = [], [], 0, 0, [], [], []
            for rid, s in self.live.items():
                ready = s["done"] - s["drained"] >= self.chunk or s["done"] == s["total"]
                if not ready or rid in fin_ids or row + span > st["d_in"].shape[0]:
                    continue
                c, n, fin = self.pool.chunk_window(rid, self.context, st["d_in"][row:])
                if n:
                    lens.append(c + n)
                    keeps.append(c)
                    row += c + n
                    items.append((s["index"], bool(fin)))
                    handed.append((s["index"], s["drained"], out_rows, n))
                    if self.vocoder is not None:
                        first = 0
                        if "vslot" not in s:
                            s["vslot"] = self._free_slots.pop()
                            first = 1
                        voc.append((n, s["vslot"], first | (2 if fin else 0)))
                    out_rows += n
                    s["drained"] += n
                if fin:
                    assert n > 0 or self.vocoder is None or "vslot" not in s
                    fin_ids.append(rid)
            if not lens:
                break
            copied = torch.cuda.Event()
            copied.record(main)             # the chunks are out of the pool's ring: the decoder may go on
            side.wait_event(copied)
            self.postnet.run_device(st["d_in"], lens, keeps, st["d_out"])
            rnd = dict(items=items, set=st, handed=handed)
            with torch.cuda.stream(side):
                if self.vocoder is not None:
                    rnd["n_out"] = self.vocoder.run_device(st["d_out"], [v[0] for v in voc], [v[1] for v in voc],
                                                           [v[2] for v in voc], st["d_audio"])
                    total = sum(rnd["n_out"])
                    st["h_audio"][:total].copy_(st["d_audio"][:total], non_blocking=True)
                if self.vocoder is None or self.on_chunk is not None:
                    st["h_out"][:out_rows].copy_(st["d_out"][:out_rows], non_blocking=True)
                st["ev"] = torch.cuda.Event()
                st["ev"].record(side)
            rnd["ev"] = st["ev"]
            self._out.append(rnd)
            self._next_set = (self._next_set + 1) % self.N_SETS
        # the segment ends when the decoder's steps (and the copies out of its ring) are through; responses that
        # arrive meanwhile are taken as they come
        stepped = torch.cuda.Event()
        stepped.record(main)
        got = []
        while not stepped.query():
            got += self._harvest()
        got += self._harvest()
        return None, [], fin_ids, got

    def run(self, k: int):
        if self.overlap:
            return self._run_overlapped(k)
        self.pool.step_n(k)
        for s in self.live.values():
            s["done"] = min(s["total"], s["done"] + k)
        chunk_ids, fin_ids = [], []
        span = self.chunk + self.context
        while True:                         # a request that ends may hand out a full chunk and then its rest
            lens, keeps, row, out_rows, handed, voc = [], [], 0, 0, [], []
            for rid, s in self.live.items():
                ready = s["done"] - s["drained"] >= self.chunk or s["done"] == s["total"]
                if not ready or rid in fin_ids or row + span > self._d_in.shape[0]:
                    continue
                c, n, fin = self.pool.chunk_window(rid, self.context, self._d_in[row:])
                if n:
                    lens.append(c + n)
                    keeps.append(c)
                    row += c + n
                    handed.append((s["index"], s["drained"], out_rows, n))
                    if self.vocoder is not None:
                        if "vslot" not in s:
                            s["vslot"] = self._free_slots.pop()
                            first = 1
                        else:
                            first = 0
                        voc.append((n, s["vslot"], first | (2 if fin else 0), s["index"]))
                    out_rows += n
                    s["drained"] += n
                    if rid not in chunk_ids:
                        chunk_ids.append(rid)
                if fin:
                    # the request's last frames always leave with a chunk of their own: the vocoder's LAST flag rides on it
                    assert n > 0 or self.vocoder is None or "vslot" not in s
                    fin_ids.append(rid)
            if not lens:
                break
            self.postnet.run_device(self._d_in, lens, keeps, self._d_out)
            if self.vocoder is not None:
                n_out = self.vocoder.run_device(self._d_out, [v[0] for v in voc], [v[1] for v in voc], [v[2] for v in voc],
                                                self._d_audio)
                total = sum(n_out)
                with self.pool._torch.cuda.stream(self.pool.stream):
                    self._h_audio[:total].copy_(self._d_audio[:total], non_blocking=True)
                if self.on_audio is not None:
                    self.pool.sync()
                    host, at = self._h_audio.numpy(), 0
                    for (_, _, _, index), m in zip(voc, n_out):
                        self.on_audio(index, host[at:at + m].copy())
                        at += m
            if self.vocoder is None or self.on_chunk is not None:
                with self.pool._torch.cuda.stream(self.pool.stream):
                    self._h_out[:out_rows].copy_(self._d_out[:out_rows], non_blocking=True)
            if self.on_chunk is not None:
                self.pool.sync()
                host = self._h_out.numpy()
                for index, first, r0, n in handed:
                    self.on_chunk(index, first, host[r0:r0 + n].copy())
        self.pool.sync()
        return None, chunk_ids, fin_ids

    def retire(self, rid: int) -> None:
        s = self.live.get(rid)
        if s is not None and "vslot" in s:
            self._free_slots.append(s["vslot"])
        super().retire(rid)


class EncoderAtJoin:
    """Module E for the serving loop (Eq. 1; Sec. 2.2.1: once per request): `enc(i)` for a GpuBackend.  The request's
    id sequences go through tts_encoder_run on the pool's stream and F_enc stays on the device; the pool copies it
    into its own memory when the request is added, so one output buffer serves every join."""

    def __init__(self, encoder, ids_of, max_len: int):
        import torch
        self.encoder, self.ids_of = encoder, ids_of
        self._d_f = torch.empty((max_len, 2 * encoder.cfg.hid), dtype=torch.float32, device=encoder.device)

    def __call__(self, index: int):
        ids = self.ids_of(index)
        self.encoder.run_device([ids], self._d_f)
        return self._d_f[: ids.shape[1]]
