"""The streaming probes the bench uses for its measured ceilings (libngc_probe.so): the copy kinds copy, the read
kinds leave their sink alone, odd sizes (tails of the unrolled loops) included; the compaction probe moves the
rows a compaction moves."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes", [16, 4096 + 16, (1 << 20) + 48, 64 << 20])
def test_probe_kinds(nbytes):
    import torch
    from paper_2604_18002_amd import probe
    g = torch.Generator(device="cuda")
    g.manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    for kind in (probe.COPY, probe.COPY_NT):
        dst = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
        probe.ngc_probe_stream(kind, src, dst, nbytes)
        torch.cuda.synchronize()
        assert torch.equal(dst[:nbytes], src) and not bool(dst[nbytes:].any())
    for kind in (probe.READ, probe.READ_NT):
        sink = torch.full((64,), 7, dtype=torch.uint8, device="cuda")
        probe.ngc_probe_stream(kind, src, sink, nbytes)
        torch.cuda.synchronize()
        assert bool((sink == 7).all())
    dst = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
    probe.ngc_probe_stream(probe.FILL_NT, None, dst, nbytes)
    torch.cuda.synchronize()
    assert bool((dst[:nbytes] != 0).all()) and not bool(dst[nbytes:].any())
    with pytest.raises(probe.ProbeError):
        probe.ngc_probe_stream(probe.COPY, src, src, 24)          # not a multiple of 16
    with pytest.raises(probe.ProbeError):
        probe.ngc_probe_stream(9, src, src, 16)


def test_read_ceiling_at_a_launch_size():
    # trains of small launches over successive regions of a small buffer: sizes are rounded down to 4 KB, the
    # regions stay inside the buffer, and the figure is a positive rate below the vendor's peak
    from paper_2604_18002_amd import probe
    r = probe.read_ceiling_at((3 << 20) + 1234, launches=5, span=16 << 20, trains=2)
    assert r["bytes_per_launch"] == (3 << 20) and r["launches_per_train"] == 5
    assert 0 < r["GBs"] < 8000 and r["us_per_launch"] > 0
    r = probe.read_ceiling_at(100, launches=2, span=1 << 20, trains=1)       # below one page: 4 KB
    assert r["bytes_per_launch"] == 4096


@pytest.mark.parametrize("threads,unroll,pipelined", [(256, 4, False), (256, 16, False), (512, 8, True), (1024, 4, True),
                                                      (1024, 8, False), (1024, 16, False)])
def test_copy_shapes_copy(threads, unroll, pipelined):
    import torch
    from paper_2604_18002_amd import probe
    for nbytes, grid in (((3 << 20) + 16 * 7, 5), (16 * 100, 3), (40 << 20, 64)):   # tails, tiny, several strides
        src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda")
        dst = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
        probe.ngc_probe_copy_shape(src, dst, nbytes, threads, unroll, grid, pipelined)
        torch.cuda.synchronize()
        assert torch.equal(dst[:nbytes], src) and not bool(dst[nbytes:].any()), (nbytes, grid)
    with pytest.raises(probe.ProbeError):
        probe.ngc_probe_copy_shape(src, dst, nbytes, 384, 4, 8, False)


@pytest.mark.parametrize("threads,unroll", [(256, 4), (512, 2), (1024, 4)])
def test_compaction_probe_moves_the_kept_rows(threads, unroll):
    import torch
    from paper_2604_18002_amd import probe
    nseg, cap = 7, 1500
    kept_h, keep_h, moved = probe.compaction_case(nseg, cap, 300, 1500, 2, 5, seed=threads)
    keep_h[3] = 0                                              # an empty segment
    k = torch.randint(0, 256, (nseg, cap, 256), dtype=torch.uint8, device="cuda")
    v = torch.randint(0, 256, (nseg, cap, 256), dtype=torch.uint8, device="cuda")
    k0, v0 = k.clone(), v.clone()
    kept, keep = torch.from_numpy(kept_h).cuda(), torch.from_numpy(keep_h).cuda()
    probe.ngc_probe_compact(k, v, kept, keep, nseg, cap, kept.shape[1], threads, unroll, 0)
    torch.cuda.synchronize()
    for s in range(nseg):
        K = int(keep_h[s])
        idx = torch.from_numpy(kept_h[s, :K].astype(np.int64)).cuda()
        assert torch.equal(k[s, :K], k0[s, idx]) and torch.equal(v[s, :K], v0[s, idx]), s
    # the read-only mode leaves the buffers alone
    k1 = k.clone()
    probe.ngc_probe_compact(k, v, kept, keep, nseg, cap, kept.shape[1], threads, unroll, 1)
    torch.cuda.synchronize()
    assert torch.equal(k, k1)
