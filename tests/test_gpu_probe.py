"""The measurement aids: the MFMA-only loop is deterministic and the streaming read really reads every byte."""
import numpy as np
import pytest
import torch

from paper_2506_04985_amd import probe

pytestmark = pytest.mark.gpu


def test_mfma_probe_counts_and_is_deterministic():
    ops, out0 = probe.mfma_rate(3, 0)
    assert ops == 256 * 4 * 3 * 64 * 65536
    assert int(out0.abs().max()) == 0                       # zero operands: zero accumulators
    _, a = probe.mfma_rate(5, 1)
    _, b = probe.mfma_rate(5, 1)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and int((a != 0).sum()) > 60000
    # the explicit form: fresh operands give a deterministic, non-trivial checksum; the same stream on zeros gives zeros
    out = torch.empty(131072, dtype=torch.int32, device="cuda")
    assert probe.mfma_rate_ex(4, 2, 2, out) == 512 * 4 * 4 * 64 * 65536
    first = out.clone()
    probe.mfma_rate_ex(4, 2, 2, out)
    assert torch.equal(first, out) and int((out != 0).sum()) > 120000
    probe.mfma_rate_ex(4, 3, 1, out)
    assert int(out[:65536].abs().max()) == 0
    for bad_args in ((0, 1, 1), (4, 4, 1), (4, 1, 3)):
        with pytest.raises(probe.ProbeError):
            probe.mfma_rate_ex(*bad_args, out)
    for bad in (0, -1, (1 << 20) + 1):
        with pytest.raises(probe.ProbeError) as e:
            probe.mfma_rate(bad, 1)
        assert e.value.code == -6


@pytest.mark.parametrize("nbytes", [16, 48, 16 * 2047, 16 * 2048, 16 * 2049, 16 * 1000003])
def test_read_probe_sees_every_word(nbytes):
    rng = np.random.default_rng(nbytes)
    host = rng.integers(-2**31, 2**31 - 1, nbytes // 4, dtype=np.int64).astype(np.int32)
    x = probe.read(torch.from_numpy(host).cuda()).cpu().numpy()
    assert np.array_equal(x, np.bitwise_xor.reduce(host.reshape(-1, 4), axis=0))


def test_read_probe_rejects_bad_sizes():
    buf = torch.zeros(40, dtype=torch.uint8, device="cuda")
    with pytest.raises(probe.ProbeError) as e:
        probe.read(buf)                            # 40 is not a multiple of 16
    assert e.value.code == -2


@pytest.mark.parametrize("threads,loads", [(256, 1), (256, 8), (1024, 2), (1024, 4)])
@pytest.mark.parametrize("nbytes", [16, 16 * 4097, 16 * 1000003])
def test_burst_read_sees_every_word(nbytes, threads, loads):
    rng = np.random.default_rng(nbytes + threads + loads)
    host = rng.integers(-2**31, 2**31 - 1, nbytes // 4, dtype=np.int64).astype(np.int32)
    slots = torch.zeros(1024, dtype=torch.int32, device="cuda")
    probe.read_burst(torch.from_numpy(host).cuda(), slots, threads, loads)
    got = np.bitwise_xor.reduce(slots.cpu().numpy().reshape(256, 4), axis=0)
    assert np.array_equal(got, np.bitwise_xor.reduce(host.reshape(-1, 4), axis=0))
    with pytest.raises(probe.ProbeError):
        probe.read_burst(torch.from_numpy(host).cuda(), slots, 512, 3)
