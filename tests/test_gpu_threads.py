"""Concurrent callers: several host threads, each on its own stream, launch different shapes at once.  The library
keeps per-device launch facts in caches that any thread may be the first to fill; results must not depend on that."""
import threading

import numpy as np
import pytest
import torch

from paper_2410_09426_amd import binding as fq
from paper_2410_09426_amd import synth
from gpu_util import dev

pytestmark = pytest.mark.gpu


def test_four_threads_four_streams():
    shapes = [(301, 64, 64), (77, 32, 96), (150, 64, 128), (40, 86, 128)]
    cases = [synth.generic(900 + i, T, n1, n2) for i, (T, n1, n2) in enumerate(shapes)]
    # reference results: the same calls, one after the other, on the default stream
    ref = []
    bufs = []
    for c in cases:
        x, P1, P2, clip = dev(c.x), dev(c.P1), dev(c.P2), dev(c.clip)
        codes = torch.empty((c.T, c.n // 2), dtype=torch.uint8, device="cuda")
        scales = torch.empty((c.T,), dtype=torch.float16, device="cuda")
        fq.flatquant_transform_quant(x, P1, P2, clip, c.clip_mode, c.T, c.n1, c.n2, c.n, codes, scales, stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
        ref.append((codes.cpu().numpy().copy(), scales.cpu().view(torch.int16).numpy().copy()))
        bufs.append((x, P1, P2, clip))
    errors = []

    def worker(i):
        try:
            c = cases[i]
            x, P1, P2, clip = bufs[i]
            st = torch.cuda.Stream()
            codes = torch.empty((c.T, c.n // 2), dtype=torch.uint8, device="cuda")
            scales = torch.empty((c.T,), dtype=torch.float16, device="cuda")
            for rep in range(25):
                codes.fill_(0xCD)
                st.wait_stream(torch.cuda.current_stream())
                fq.flatquant_transform_quant(x, P1, P2, clip, c.clip_mode, c.T, c.n1, c.n2, c.n, codes, scales, stream=st)
                st.synchronize()
                if not (np.array_equal(codes.cpu().numpy(), ref[i][0]) and np.array_equal(scales.cpu().view(torch.int16).numpy(), ref[i][1])):
                    errors.append(f"thread {i} rep {rep}: result differs from the single-threaded one")
                    return
        except Exception as e:   # noqa: BLE001 - reported below, in the main thread
            errors.append(f"thread {i}: {e!r}")

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(len(cases))]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a worker did not finish"
    assert not errors, errors
