"""The threaded host baseline of the benchmark (oracle/host_threads.c) against the sequential oracle loop:
bit-exact for every thread count, with chunks that hold no flag, chunks that start with one, more threads
than elements, and wrap-around."""
import numpy as np
import pytest

import oracle
from paper_2506_23906_amd import workloads as W


@pytest.mark.parametrize("threads", [1, 2, 3, 8, 61])
def test_threads_equal_the_sequential_loop(threads):
    rng = np.random.default_rng(2390650 + threads)
    for n, density in [(1, 0.5), (7, 0.0), (60, 0.1), (1000, 0.0), (1000, 1.0), (4099, 0.002), (100_003, 0.0005),
                       (100_003, 0.3)]:
        x = rng.integers(-128, 128, size=n, dtype=np.int8)
        f = (rng.random(n) < density).astype(np.uint8)
        assert np.array_equal(oracle.host_threads_segscan(x, f, threads), oracle.segscan(x, f)), (n, density)


def test_flags_on_chunk_boundaries_and_long_open_runs():
    n, threads = 8000, 8                       # chunks of 1000
    x = np.full(n, 127, dtype=np.int8)
    for starts in [(), (1000,), (999,), (1001,), (1000, 2000, 3000), (3500,), (7999,), (1, 7000)]:
        f = np.zeros(n, dtype=np.uint8)
        f[list(starts)] = 1
        assert np.array_equal(oracle.host_threads_segscan(x, f, threads), oracle.segscan(x, f)), starts


def test_wraps_like_the_loop_and_workload_twin():
    x = np.full(1 << 25, 127, dtype=np.int8)   # 2^25 * 127 > 2^31: the running sum wraps
    f = np.zeros(1 << 25, dtype=np.uint8)
    z = oracle.host_threads_segscan(x, f, 8)
    assert np.array_equal(z, oracle.segscan(x, f)) and z.min() < 0
    x, f = W.segscan_i8_uniform_len(1 << 20)
    assert np.array_equal(oracle.host_threads_segscan(x, f, 8), oracle.segscan(x, f))


def test_bad_thread_counts_are_errors():
    x = np.zeros(4, dtype=np.int8)
    f = np.zeros(4, dtype=np.uint8)
    for threads in (0, -1, 257):
        with pytest.raises(RuntimeError):
            oracle.host_threads_segscan(x, f, threads)
    assert oracle.host_threads_segscan(np.zeros(0, dtype=np.int8), np.zeros(0, dtype=np.uint8), 4).shape == (0,)
