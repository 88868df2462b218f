"""The streaming probes the bench uses for its measured ceilings: the copy kinds copy, the read kinds
leave their sink alone, odd sizes (tails of the unrolled loop) included."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes", [16, 4096 + 16, (1 << 20) + 48, 64 << 20])
def test_probe_kinds(nbytes):
    import torch
    from paper_2604_18002_amd import binding as ngc
    g = torch.Generator(device="cuda")
    g.manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    for kind in (ngc.PROBE_COPY, ngc.PROBE_COPY_NT):
        dst = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
        ngc.ngc_probe_stream(kind, src, dst, nbytes)
        torch.cuda.synchronize()
        assert torch.equal(dst[:nbytes], src) and not bool(dst[nbytes:].any())
    for kind in (ngc.PROBE_READ, ngc.PROBE_READ_NT):
        sink = torch.full((64,), 7, dtype=torch.uint8, device="cuda")
        ngc.ngc_probe_stream(kind, src, sink, nbytes)
        torch.cuda.synchronize()
        assert bool((sink == 7).all())
    with pytest.raises(ngc.NgcError):
        ngc.ngc_probe_stream(ngc.PROBE_COPY, src, src, 24)          # not a multiple of 16
    with pytest.raises(ngc.NgcError):
        ngc.ngc_probe_stream(9, src, src, 16)
