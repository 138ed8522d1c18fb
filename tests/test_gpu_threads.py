"""Two host threads, each issuing forward + backward calls on a stream of its own, get the results
of the same calls issued from one thread (the library serialises the enqueue of concurrent calls;
helper stream, events and per-device flags are shared state behind one lock)."""
import threading

import numpy as np
import pytest

from paper_2605_08123_amd.workloads import Workload, make_inputs

pytestmark = pytest.mark.gpu


def _run(w, arrays, stream, reps, out, key):
    import torch

    import paper_2605_08123_amd as ska
    dev = torch.device("cuda:0")
    td = torch.float32 if w.dtype == "f32" else torch.bfloat16
    try:
        with torch.cuda.stream(stream):
            Q, K, V, G = (torch.from_numpy(x).to(dev).to(td) for x in arrays)
            for _ in range(reps):
                O, UV = ska.sinkhorn_attn_fwd(Q, K, V, w.W, w.T, w.R, w.eps)
                dQ, dK, dV = ska.sinkhorn_attn_bwd(Q, K, V, O, G, UV, w.W, w.T, w.R, w.eps)
            stream.synchronize()
        out[key] = [t.float().cpu().numpy() for t in (O, UV, dQ, dK, dV)]
    except Exception as e:   # noqa: BLE001 - reported by the asserting thread
        out[key] = e


@pytest.mark.parametrize("split", [False, True])
def test_two_threads_two_streams(split):
    import torch

    import paper_2605_08123_amd as ska
    ska.sinkhorn_attn_set_split_min_edges(0.0 if split else 5e7)   # True: both threads share the helper stream
    try:
        wa = Workload("thr_a", 11, 1, 2, 700, 64, 40, 5, 2, 0.5, "bf16")
        wb = Workload("thr_b", 12, 2, 2, 450, 32, 17, 4, 2, 1.0, "f32")
        arrs = {"a": make_inputs(wa), "b": make_inputs(wb)}
        single, multi = {}, {}
        for key, w in (("a", wa), ("b", wb)):
            _run(w, arrs[key], torch.cuda.Stream(), 1, single, key)
        threads = [threading.Thread(target=_run, args=(w, arrs[key], torch.cuda.Stream(), 6, multi, key))
                   for key, w in (("a", wa), ("b", wb))]
        for t in threads:
            t.start()
        for t in threads:
            t.join(timeout=100)
        torch.cuda.synchronize()
        for key in ("a", "b"):
            assert not isinstance(single[key], Exception), single[key]
            assert not isinstance(multi[key], Exception), multi[key]
            for x, y in zip(single[key], multi[key]):
                assert np.array_equal(x, y, equal_nan=True)   # the same kernels on the same inputs: bit for bit
    finally:
        ska.sinkhorn_attn_set_split_min_edges(5e7)
