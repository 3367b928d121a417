"""Entry points called from several host threads at once, each on a stream of its own (default priority): the per-device
set-up is done once under a lock and the launch paths share no mutable state, so every thread gets the serial result."""
import threading

import numpy as np
import pytest
import torch

from paper_2506_04985_amd import binding as fptq

pytestmark = pytest.mark.gpu


def test_concurrent_callers_get_the_serial_results():
    fptq.fptq_init()
    rng = np.random.default_rng(3)
    cases = []
    for i, (M, N, K) in enumerate([(300, 1500, 1024), (8, 4096, 2048), (640, 512, 4096), (1100, 2304, 512)]):
        x = (torch.randn((M, K), device="cuda") * 2).to(torch.bfloat16)
        wq = fptq.fptq_pack_weights(torch.from_numpy(rng.integers(-8, 8, (N, K), dtype=np.int8)).cuda())
        s_w = torch.from_numpy(rng.uniform(0.005, 0.02, N).astype(np.float32)).cuda()
        xq, _ = fptq.fptq_quantize_act(x, 0.4, 1, 1e-5)
        y = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.4, s_w)
        cases.append((M, N, K, x, wq, s_w, y))
    torch.cuda.synchronize()
    errors = []

    def worker(idx):
        try:
            M, N, K, x, wq, s_w, want = cases[idx]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for _ in range(40):
                    fptq.fptq_init()
                    xq, _ = fptq.fptq_quantize_act(x, 0.4, 1, 1e-5)
                    y = fptq.fptq_w4a4_linear(xq, wq, M, N, K, 0.4, s_w)
                    stream.synchronize()
                    if not torch.equal(y.view(torch.int16), want.view(torch.int16)):
                        errors.append((idx, "mismatch"))
                        return
        except Exception as e:          # noqa: BLE001  (reported to the main thread)
            errors.append((idx, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(len(cases))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert errors == []
