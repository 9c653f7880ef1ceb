"""The measurement aids of the C ABI: ddp_stream_probe (a read/write reference kernel) computes what its header says, and
the CU-range stream helpers validate their arguments and give streams that run kernels."""
import pytest
import torch

from paper_2502_11058_amd import binding as B

pytestmark = pytest.mark.gpu


def _expect(code, fn, *a, **k):
    with pytest.raises(B.DdpError) as e:
        fn(*a, **k)
    assert e.value.code == code, str(e.value)


@pytest.mark.parametrize("nr,nw", [(1, 1), (3, 2), (8, 1), (16, 4), (0, 2), (4, 0)])
def test_probe_writes_one_plus_the_sum_of_the_reads(nr, nw):
    assert torch.cuda.is_available(), "no GPU visible"
    n = 3 * 2048 + 1024 + 4                       # several workgroups and a ragged last one (bytes stay a multiple of 16)
    dev = torch.device("cuda", 0)
    rd = [torch.full((n,), float(k + 1), dtype=torch.float32, device=dev) for k in range(nr)]
    wr = [torch.full((n + 8,), -7.0, dtype=torch.float32, device=dev) for _ in range(nw)]
    B.ddp_stream_probe(rd, wr, 4 * n, 8192, 0)
    torch.cuda.synchronize()
    want = 1.0 + sum(range(1, nr + 1))
    for t in wr:
        assert float(t[:n].min()) == want and float(t[:n].max()) == want
        assert float(t[n:].min()) == -7.0 and float(t[n:].max()) == -7.0      # nothing past the stated bytes
    for k, t in enumerate(rd):
        assert float(t.min()) == float(k + 1) == float(t.max())               # inputs untouched


def test_probe_and_stream_arguments_are_checked():
    assert torch.cuda.is_available(), "no GPU visible"
    dev = torch.device("cuda", 0)
    a, b = torch.zeros(4096, device=dev), torch.zeros(4096, device=dev)
    _expect(1, B.ddp_stream_probe, [], [], 4096)                               # no stream at all
    _expect(1, B.ddp_stream_probe, [a] * 5, [b], 4096)                         # 5 read streams is not offered
    _expect(1, B.ddp_stream_probe, [a], [b] * 5, 4096)
    _expect(1, B.ddp_stream_probe, [a], [b], 4096 + 8)                         # bytes not a multiple of 16
    _expect(1, B.ddp_stream_probe, [a], [b], 4096, 1000)                       # chunk not a multiple of 4096
    _expect(1, B.ddp_stream_probe, [a], [b], 4096, 8192, 70000)                # LDS request too large
    _expect(3, B.ddp_stream_probe, [a[1:]], [b], 4096)                         # misaligned
    ncu = B.ddp_device_cu_count(0)
    assert ncu >= 64
    _expect(1, B.ddp_stream_create_cu_range, 0, 0, 0)
    _expect(1, B.ddp_stream_create_cu_range, 0, ncu - 1, 2)
    _expect(1, B.ddp_stream_create_cu_range, 0, -1, 4)
    h = B.ddp_stream_create_cu_range(0, 0, 16)
    s = torch.cuda.ExternalStream(h)
    B.ddp_stream_probe([a], [b], 4096 * 4, 8192, 0, stream=s)                  # a kernel runs on the confined stream
    s.synchronize()
    assert float(b.min()) == 1.0 == float(b.max())
    B.ddp_stream_destroy(h)
    B.ddp_stream_destroy(0)                                                    # NULL is a no-op
