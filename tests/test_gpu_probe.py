"""The plain streaming kernels that bench.py times beside the path (a measurement aid): they
move what they say they move, and refuse what they cannot do."""
import pytest
import torch

from paper_2205_12268_amd import wcc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nt", [False, True])
def test_probe_kernels_move_what_they_say(nt):
    ctx = wcc.Context(0)
    n = (3 << 20) + 52          # floats: several grid strides and a ragged tail of 16-byte words
    g = torch.Generator(device="cuda").manual_seed(7)
    src = torch.rand(n, device="cuda", generator=g)
    keep = src.clone()
    dst = torch.full((n + 8,), -1.0, device="cuda")
    ctx.wcc_probe_stream(wcc.PROBE_COPY, src, dst, n * 4, nt, 100)   # a long grid stride
    assert torch.equal(dst[:n], keep) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    ctx.wcc_probe_stream(wcc.PROBE_COPY, src, dst, n * 4, nt)
    assert torch.equal(dst[:n], keep) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    ctx.wcc_probe_stream(wcc.PROBE_WRITE, None, dst, n * 4, nt)
    want = torch.tensor([1.0, 2.0, 3.0, 4.0], device="cuda").repeat(n // 4)
    assert torch.equal(dst[:n], want) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    ctx.wcc_probe_stream(wcc.PROBE_WRITE8, None, dst, n * 4, nt)
    assert torch.equal(dst[:n], want) and bool((dst[n:] == -1.0).all())
    dst.fill_(-1.0)
    ctx.wcc_probe_stream(wcc.PROBE_READ, src, dst, n * 4, nt)
    torch.cuda.synchronize()
    assert torch.equal(src, keep) and bool((dst == -1.0).all())
    ctx.close()


def test_probe_errors():
    ctx = wcc.Context(0)
    a = torch.zeros(64, device="cuda")
    b = torch.zeros(64, device="cuda")
    for args, status in (((wcc.PROBE_COPY, None, b, 256), 1), ((wcc.PROBE_COPY, a, None, 256), 1),
                         ((wcc.PROBE_READ, None, b, 256), 1), ((7, a, b, 256), 3), ((-1, a, b, 256), 3),
                         ((wcc.PROBE_COPY, a, b, 0), 2), ((wcc.PROBE_COPY, a, b, 100), 2),
                         ((wcc.PROBE_COPY, a, b, 256, False, -1), 2)):
        with pytest.raises(wcc.WccError) as e:
            ctx.wcc_probe_stream(*args)
        assert e.value.status == status, args
    torch.cuda.synchronize()
    assert bool((b == 0).all())
    ctx.close()
