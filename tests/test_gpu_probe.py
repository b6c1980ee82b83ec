"""The streaming probe kernels (measurement aid) do what their description says."""
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("blocks_per_cu", [0, 2])
def test_probe_kernels_move_the_bytes_they_claim(blocks_per_cu):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2105_09080_amd import binding as B
    n = (1 << 20) + 4 * 37                       # a ragged number of 16-byte words
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        src = torch.randn(n, device="cuda")
        src2 = torch.randn(n, device="cuda")
        inout = torch.randn(n, device="cuda")
        dst = torch.zeros(n + 8, device="cuda")
        sink = torch.full((4,), 7.0, device="cuda")
        m0 = inout.clone()
        stream.synchronize()
        h = stream.cuda_stream
        B.gpga_probe_stream(2, src, dst, 4 * n, h, blocks_per_cu=blocks_per_cu)
        stream.synchronize()
        assert torch.equal(dst[:n], src) and float(dst[n:].abs().max()) == 0.0     # nothing past the end
        B.gpga_probe_stream(1, None, dst, 4 * n, h, blocks_per_cu=blocks_per_cu)
        stream.synchronize()
        assert bool((dst[:n] == 1.0).all()) and float(dst[n:].abs().max()) == 0.0
        B.gpga_probe_stream(0, src, sink, 4 * n, h, blocks_per_cu=blocks_per_cu)
        stream.synchronize()
        assert bool((sink == 7.0).all())                                         # the read probe writes nothing
        B.gpga_probe_stream(3, src, dst, 4 * n, h, src2=src2, inout=inout, blocks_per_cu=blocks_per_cu)
        stream.synchronize()
        mom = 0.9 * m0 + src2
        assert torch.allclose(inout, mom, rtol=1e-6, atol=1e-6)
        assert torch.allclose(dst[:n], src - 0.1 * mom, rtol=1e-6, atol=1e-6)
    for bad in (dict(kind=4), dict(nbytes=24), dict(kind=2, src=None)):
        kw = dict(kind=2, src=src, dst=dst, nbytes=4 * n)
        kw.update(bad)
        with pytest.raises(B.GpgaError):
            B.gpga_probe_stream(kw["kind"], kw["src"], kw["dst"], kw["nbytes"], h)
