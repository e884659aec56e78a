"""The batching server (prep_server_*) on the GPU: every request comes back once, with the
tensor the oracle computes for its file, in batches that obey Batch_max and Time_queue."""
import time

import numpy as np
import pytest

import oracle
import synth
from helpers import MEAN, STD, TENSOR_ABS_TOL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def prep():
    import paper_2411_19114_amd as p
    return p


def _params(prep, dtype="f32"):
    from paper_2411_19114_amd.binding import make_params
    return make_params(256, 224, 224, dtype, MEAN, STD)


def _collect(server, n, timeout_s=60.0):
    got, t0 = [], time.time()
    while len(got) < n and time.time() - t0 < timeout_s:
        r = server.next(200000)
        if r is not None:
            got.append((r, server.copy_tensor(r) if r.status == 0 else None))
            server.release(r)
    return got


def test_burst_of_requests_is_served_in_full_batches_with_the_right_tensors(prep):
    streams = synth.make_batch(1, 6) + synth.make_batch(5, 9)
    corrupt = streams[2][:len(streams[2]) // 2]
    requests = (streams + [corrupt]) * 3          # 48 requests
    server = prep.Server(n_consumers=3, batch_max=8, time_queue_us=20000, params=_params(prep),
                         max_width=256, max_height=256, max_request_bytes=1 << 17, queue_capacity=64)
    try:
        for tag, s in enumerate(requests):
            assert server.submit(s, 1000 + tag) == 0
        got = _collect(server, len(requests))
        assert sorted(r.tag for r, _ in got) == [1000 + i for i in range(len(requests))]
        ref = {}
        for r, ten in got:
            i = (r.tag - 1000) % (len(streams) + 1)
            assert 1 <= r.batch_size <= 8 and 0 <= r.consumer < 3
            assert r.arrival_ns <= r.start_ns <= r.done_ns
            if i == len(streams):
                assert r.status == prep.E_CORRUPT
                continue
            assert r.status == 0
            if i not in ref:
                ref[i] = oracle.decode_preprocess(streams[i], 256, 224, 224, MEAN, STD)
            assert np.abs(ten.astype(np.float64) - ref[i]).max() <= TENSOR_ABS_TOL
        # 48 requests submitted at once, three consumers: most batches are full
        assert sum(1 for r, _ in got if r.batch_size == 8) >= 16
    finally:
        server.close()


def test_a_lone_request_waits_time_queue_and_no_longer_than_needed(prep):
    s = synth.make_batch(1, 1)[0]
    server = prep.Server(n_consumers=2, batch_max=16, time_queue_us=150000, params=_params(prep, "f16"),
                         max_width=256, max_height=256, max_request_bytes=1 << 17, queue_capacity=32)
    try:
        for rep in range(3):
            assert server.submit(s, rep) == 0
            (r, ten), = _collect(server, 1)
            assert r.status == 0 and r.batch_size == 1 and r.tag == rep
            waited_ms = (r.start_ns - r.arrival_ns) / 1e6
            assert 150.0 <= waited_ms < 400.0, waited_ms
            ref = oracle.decode_preprocess(s, 256, 224, 224, MEAN, STD)
            assert np.abs(ten.astype(np.float64) - ref).max() <= TENSOR_ABS_TOL
        # a full batch does not wait
        for tag in range(16):
            assert server.submit(s, 100 + tag) == 0
        got = _collect(server, 16)
        assert len(got) == 16 and all(r.batch_size == 16 for r, _ in got)
        assert max(r.start_ns - r.arrival_ns for r, _ in got) / 1e6 < 100.0
    finally:
        server.close()


def test_refusals(prep):
    s = synth.make_batch(1, 1)[0]
    server = prep.Server(n_consumers=1, batch_max=2, time_queue_us=200000, params=_params(prep),
                         max_width=256, max_height=256, max_request_bytes=len(s), queue_capacity=2)
    try:
        assert server.submit(s + b"\x00", 1) == prep.E_TOO_LARGE          # larger than max_request_bytes
        assert server.submit(s, 2) == 0
        # the first request waits for Time_queue; the queue holds two
        rc = [server.submit(s, 3 + k) for k in range(8)]
        assert prep.E_TOO_LARGE in rc
        n_ok = 1 + rc.count(0)
        got = _collect(server, n_ok)
        assert len(got) == n_ok and all(r.status == 0 for r, _ in got)
        assert server.next(1000) is None
    finally:
        server.close()
    with pytest.raises(prep.PrepError):
        prep.Server(n_consumers=0, batch_max=2, time_queue_us=0, params=_params(prep), max_width=16,
                    max_height=16, max_request_bytes=100, queue_capacity=2)
