"""The plain streaming kernels that bench.py times beside the path (a measurement aid): they
move what they say they move, and refuse what they cannot do."""
import pytest
import torch

from paper_2205_12268_amd import probe

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nt", [False, True])
def test_probe_kernels_move_what_they_say(nt):
    n = (3 << 20) + 52          # floats: several grid strides and a ragged tail of 16-byte words
    g = torch.Generator(device="cuda").manual_seed(7)
    src = torch.rand(n, device="cuda", generator=g)
    keep = src.clone()
    dst = torch.full((n + 8,), -1.0, device="cuda")
    probe.wcc_probe_stream(probe.COPY, src, dst, n * 4, nt, 100)   # a long grid stride
    assert torch.equal(dst[:n], keep) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    probe.wcc_probe_stream(probe.COPY, src, dst, n * 4, nt)
    assert torch.equal(dst[:n], keep) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    probe.wcc_probe_stream(probe.WRITE, None, dst, n * 4, nt)
    want = torch.tensor([1.0, 2.0, 3.0, 4.0], device="cuda").repeat(n // 4)
    assert torch.equal(dst[:n], want) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    probe.wcc_probe_stream(probe.WRITE8, None, dst, n * 4, nt)
    assert torch.equal(dst[:n], want) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    probe.wcc_probe_stream(probe.READ, src, dst, n * 4, nt)
    torch.cuda.synchronize()
    assert torch.equal(src, keep) and bool((dst == -1.0).all())


def test_probe_errors():
    a = torch.zeros(64, device="cuda")
    b = torch.zeros(64, device="cuda")
    for args, status in (((probe.COPY, None, b, 256), 1), ((probe.COPY, a, None, 256), 1),
                         ((probe.READ, None, b, 256), 1), ((7, a, b, 256), 3), ((-1, a, b, 256), 3),
                         ((probe.COPY, a, b, 0), 2), ((probe.COPY, a, b, 100), 2),
                         ((probe.COPY, a, b, 256, False, -1), 2)):
        with pytest.raises(probe.ProbeError) as e:
            probe.wcc_probe_stream(*args)
        assert e.value.status == status, args
    torch.cuda.synchronize()
    assert bool((b == 0).all())
