"""Pins of the batching oracle (oracle/batching.py): cases whose outcome the rule of PREBA
section 4.3 fixes without any simulation, and invariants that hold for every trace."""
import os

import numpy as np
import pytest

from oracle import batching

HERE = os.path.dirname(os.path.abspath(__file__))


def test_time_queue_is_tail_knee_over_consumers():
    for line in open(os.path.join(HERE, "golden", "time_queue_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        knee, n, want = (int(x) for x in line.split())
        assert batching.time_queue_for(knee * 1000000, n) == want * 1000000


def test_burst_on_one_consumer_runs_full_batches_back_to_back():
    b = batching.simulate([0] * 12, 1, 4, 1000, lambda k: 100)
    assert b == [(0, 0, [0, 1, 2, 3]), (100, 0, [4, 5, 6, 7]), (200, 0, [8, 9, 10, 11])]


def test_burst_is_spread_over_the_consumers():
    b = batching.simulate([0] * 16, 2, 4, 1000, lambda k: 100)
    assert [(s, c) for s, c, _ in b] == [(0, 0), (0, 1), (100, 0), (100, 1)]
    assert [r for _, _, ids in b for r in ids] == list(range(16))


def test_sparse_requests_wait_exactly_time_queue_and_go_alone():
    arrivals = [0, 10000, 20000, 30000]
    b = batching.simulate(arrivals, 3, 8, 700, lambda k: 50)
    assert [(s, ids) for s, _, ids in b] == [(a + 700, [i]) for i, a in enumerate(arrivals)]
    assert [c for _, c, _ in b] == [0, 1, 2, 0]  # the consumer that has been free the longest


def test_partial_batch_leaves_when_the_oldest_has_waited_time_queue():
    assert batching.simulate([0, 1, 2], 1, 4, 10, lambda k: 5) == [(10, 0, [0, 1, 2])]


def test_batch_leaves_the_moment_it_is_full():
    assert batching.simulate([0, 1, 2, 3, 4], 1, 4, 100, lambda k: 5) == [(3, 0, [0, 1, 2, 3]), (104, 0, [4])]


def test_requests_that_arrive_while_all_consumers_are_busy_join_the_waiting_batch():
    # the consumer is busy until 50; the batch due at 10 starts at 50 with everything that came
    b = batching.simulate([0, 0, 5, 20, 40, 60], 1, 8, 10, lambda k: 50)
    assert b[0] == (0 + 10, 0, [0, 1, 2])
    assert b[1] == (60, 0, [3, 4, 5])


@pytest.mark.parametrize("seed", range(6))
def test_invariants_on_poisson_traces(seed):
    rng = np.random.default_rng(seed)
    n, consumers, bmax, tq = 400, int(rng.integers(1, 8)), int(rng.integers(1, 17)), int(rng.integers(1, 2000))
    arrivals = np.cumsum(rng.exponential(float(rng.integers(20, 400)), size=n).astype(np.int64)).tolist()
    service = lambda k: 300 + 40 * k
    batches = batching.simulate(arrivals, consumers, bmax, tq, service)
    # every request is served once, in arrival order
    assert [r for _, _, ids in batches for r in ids] == list(range(n))
    busy_until = [0] * consumers
    for start, c, ids in batches:
        assert 1 <= len(ids) <= bmax
        assert start >= arrivals[ids[-1]]                # nobody is served before arriving
        assert start >= busy_until[c]                    # a consumer runs one batch at a time
        # a batch that starts later than the rule released it was waiting for a consumer
        released = min(arrivals[ids[0]] + tq, arrivals[ids[bmax - 1]] if len(ids) == bmax else 1 << 62)
        if start > released:
            assert start == min(busy_until)
        # the batch never starts before the rule releases it
        assert start >= released or len(ids) == bmax and start >= arrivals[ids[-1]]
        busy_until[c] = start + service(len(ids))
