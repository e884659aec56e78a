"""The library's batching rule (prep_policy_*, host only) against the oracle's simulation of
PREBA section 4.3 on seeded traces: the same batches at the same times.  The consumers are
simulated here with a virtual clock; the library decides when a batch is due and who is in it."""
import numpy as np
import pytest

import paper_2411_19114_amd as prep
from oracle import batching

INF = (1 << 63) - 1


def drive(arrivals, n_consumers, batch_max, time_queue, service_time):
    policy = prep.BatchPolicy(batch_max, time_queue)
    try:
        free = [0] * n_consumers
        nxt, n = 0, len(arrivals)
        batches = []
        while nxt < n or policy.pending():
            consumer = min(range(n_consumers), key=lambda c: (free[c], c))
            due = policy.deadline()
            t_take = max(free[consumer], due) if due != INF else None
            if nxt < n and (t_take is None or arrivals[nxt] <= t_take):
                policy.arrive(nxt, arrivals[nxt])
                nxt += 1
                continue
            ids = policy.take(t_take)
            assert ids, "the rule released nothing at its own deadline"
            batches.append((t_take, consumer, ids))
            free[consumer] = t_take + service_time(len(ids))
        return batches
    finally:
        policy.close()


@pytest.mark.parametrize("seed", range(12))
def test_same_batches_as_the_oracle_on_poisson_traces(seed):
    rng = np.random.default_rng(100 + seed)
    n = 600
    consumers, bmax = int(rng.integers(1, 8)), int(rng.integers(1, 17))
    tq = int(rng.integers(0, 3000))
    mean_gap = float(rng.integers(10, 500))
    arrivals = np.cumsum(rng.exponential(mean_gap, size=n).astype(np.int64)).tolist()
    base, per = int(rng.integers(50, 500)), int(rng.integers(0, 80))
    service = lambda k: base + per * k
    assert drive(arrivals, consumers, bmax, tq, service) == batching.simulate(arrivals, consumers, bmax, tq, service)


def test_bursts_ties_and_idle_gaps():
    arrivals = [0] * 9 + [5, 5, 5, 1000, 1000, 5000, 5001, 5002, 5003, 9000]
    for consumers in (1, 2, 7):
        for bmax in (1, 4, 8):
            for tq in (0, 3, 700):
                service = lambda k: 40 + 3 * k
                assert drive(arrivals, consumers, bmax, tq, service) == \
                    batching.simulate(arrivals, consumers, bmax, tq, service)


def test_take_before_the_deadline_returns_nothing_and_keeps_the_queue():
    p = prep.BatchPolicy(4, 100)
    try:
        assert p.deadline() == INF and p.take(10**9) == []
        p.arrive(7, 50)
        p.arrive(8, 60)
        assert p.deadline() == 150 and p.take(149) == [] and p.pending() == 2
        assert p.take(150) == [7, 8] and p.pending() == 0
        for i in range(5):
            p.arrive(i, 200 + i)
        assert p.deadline() == 203          # the arrival that filled the batch
        assert p.take(203) == [0, 1, 2, 3] and p.deadline() == 304
        with pytest.raises(prep.PrepError):
            p.arrive(9, 100)                # time runs backwards
    finally:
        p.close()


def test_argument_errors():
    with pytest.raises(prep.PrepError):
        prep.BatchPolicy(0, 10)
    with pytest.raises(prep.PrepError):
        prep.BatchPolicy(4, -1)
