"""Plumbing shared by the benchmark and the GPU tests: host array -> device tensor, the error ratio of the
acceptance criterion, and the three ways a call is timed (HIP events around back-to-back launches; replays of a
HIP graph for calls shorter than the host can issue them; a cycle through enough distinct buffers that nothing is
served from the 256 MB last-level cache).  No GEMM arithmetic here."""
import time

import numpy as np

LAST_LEVEL_CACHE_BYTES = 256 << 20


def to_gpu(arr):
    import torch
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def rel_error(got, c_ref, d_ref):
    """max |got - ref| / D over entries with D > 0; entries with D == 0 must be exactly 0"""
    got = got.astype(np.float64)
    zero = d_ref == 0
    assert np.all(got[zero] == 0), "entries with zero denominator must be exactly zero"
    if np.all(zero):
        return 0.0
    err = np.abs(got[~zero] - c_ref[~zero]) / d_ref[~zero]
    assert not np.any(np.isnan(err)), "NaN in result"
    return float(err.max())


def ramp(fn, seconds=0.05, calls_at_least=3):
    """untimed launches for at least `seconds` of device time: after an idle spell (host-side input generation) the
    part needs some ten milliseconds of load before it holds its steady clock.  The first call is left out of the
    count (it carries one-time costs: code upload, attribute calls), the rest is measured batch by batch until the
    device has been busy that long."""
    import torch
    fn()
    torch.cuda.synchronize()
    busy, batch = 0.0, calls_at_least
    while busy < seconds:
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(batch):
            fn()
        stop.record()
        torch.cuda.synchronize()
        spent = max(start.elapsed_time(stop) * 1e-3, 1e-6)
        busy += spent
        batch = min(2000, max(calls_at_least, int((seconds - busy) / (spent / batch)) + 1))


def timed(fn, steps, warmup):
    """(device seconds per call from HIP events on the stream the launches go to, host seconds per call)"""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - wall0) / steps
    return start.elapsed_time(stop) * 1e-3 / steps, wall


def timed_each(fn, before, steps, warmup):
    """device seconds per call of `fn`, each call between its own pair of events, with `before()` run untimed in
    front of every call (an in-place routine gets its operand back that way: called over and over on its own
    result, the values would overflow or die out within a few calls and the launches be timed on other data)"""
    import torch
    for _ in range(warmup):
        before()
        fn()
    torch.cuda.synchronize()
    pairs = []
    for _ in range(steps):
        before()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        fn()
        stop.record()
        pairs.append((start, stop))
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in pairs) * 1e-3 / steps


def fastest_single(fn, calls=20):
    """device seconds of the fastest of `calls` launches, each between its own pair of events"""
    import torch
    best = float("inf")
    for _ in range(calls):
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        fn()
        stop.record()
        torch.cuda.synchronize()
        best = min(best, start.elapsed_time(stop) * 1e-3)
    return best


def _capture(calls):
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls[0]()                                   # warm-up on a capture-capable stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for call in calls:
            call()
    return graph


def graph_timed(call, c_buffer, steps, warmup, per_graph=20):
    """Device time per call of a microsecond-scale launch: shorter than the host can issue launches (about 8 us per
    call from Python), so the call is captured once into a HIP graph of `per_graph` launches and the graph is
    replayed; the events then bracket back-to-back kernels.  Every replay of a one-launch graph is first checked
    against the eager result.  Returns (seconds per call from replays, from eager launches)."""
    import torch
    c0 = c_buffer.clone()
    call()
    eager = c_buffer.clone()
    graph = _capture([call] * per_graph)
    one = _capture([call])
    for _ in range(3):
        c_buffer.copy_(c0)
        one.replay()
        torch.cuda.synchronize()
        as_bits = {1: torch.uint8, 2: torch.int16, 4: torch.int32, 8: torch.int64}[c_buffer.element_size()]
        if not torch.equal(c_buffer.view(as_bits), eager.view(as_bits)):          # bit for bit (padding may hold NaN)
            differ = (c_buffer.view(as_bits) != eager.view(as_bits))
            raise AssertionError(f"graph replay differs from the eager call in {int(differ.sum())} of {eager.numel()} elements "
                                 f"(first at {int(differ.nonzero()[0])})")
    dev, _ = timed(graph.replay, max(1, steps // 2), max(1, warmup // 4))
    dev_eager, _ = timed(call, steps, warmup)
    return dev / per_graph, dev_eager


def cold_timed(make_call, bytes_per_set, steps=3, min_total=4 * LAST_LEVEL_CACHE_BYTES, max_sets=512):
    """Device time per call when every call finds its operands in HBM: make_call(i) returns the call on the i-th
    of `sets` distinct copies of the operands (sets * bytes_per_set >= four times the last-level cache, so a copy
    has been evicted before its turn comes again); one cycle over all copies is captured in a HIP graph and
    replayed.  Returns (seconds per call, sets)."""
    sets = int(min(max_sets, max(2, -(-min_total // max(1, bytes_per_set)))))
    calls = [make_call(i) for i in range(sets)]
    graph = _capture(calls)
    dev, _ = timed(graph.replay, steps, 1)
    return dev / sets, sets
