"""The benchmark's measurement aids (libwush_probes.so): they must report what they claim to."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def Q():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2512_00956_amd import probes
    probes.lib()
    return probes


def _rate_checks(t, iters):
    per_mfma = t[:, 0] / (iters * 64)
    assert np.all((per_mfma > 31.5) & (per_mfma < 36.0)), per_mfma
    ghz = t[:, 0] / (t[:, 1] * 10.0)
    assert np.all((ghz > 0.5) & (ghz < 3.0)), ghz


def test_fp4_mfma_probe_reports_the_instruction_rate(Q):
    """One block-scaled 32x32x64 FP4 MFMA issues every 32 shader cycles (8 passes), whatever the
    operand bits; only the clock depends on them."""
    import torch
    bits = torch.randint(0, 256, (16384,), dtype=torch.uint8, device="cuda")
    out = torch.zeros((8, 2), dtype=torch.int64, device="cuda")
    Q.mfma_fp4(bits, 200, 8, out)
    torch.cuda.synchronize()
    _rate_checks(out.cpu().numpy().astype(np.float64), 200)


def test_f16_mfma_probe_reports_the_instruction_rate(Q):
    """One 32x32x16 FP16 MFMA issues every 32 shader cycles per wave."""
    import torch
    vals = (torch.randn(8192, device="cuda") * 3).half()
    out = torch.zeros((8, 2), dtype=torch.int64, device="cuda")
    Q.mfma_f16(vals, 200, 8, out)
    torch.cuda.synchronize()
    _rate_checks(out.cpu().numpy().astype(np.float64), 200)


@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4, 5, 6, 10, 11, 13, 20, 21, 23, 30, 40])
def test_stream_probe_touches_what_it_claims(Q, mode):
    """Every output byte the probe is priced for is written (rows * row_bytes * 17 / 64 for the tile
    modes 1 and 2, rows * row_bytes / 4 for the linear one and for the read-pattern modes), none beyond,
    and the result depends on the input (xor of the data read)."""
    import torch
    rows, row_bytes = 256, 4096
    g = torch.Generator(device="cuda").manual_seed(3)
    src = torch.randint(0, 256, (rows * row_bytes,), dtype=torch.uint8, device="cuda", generator=g)
    n_out = rows * row_bytes // 4 + (rows * row_bytes // 64 if mode in (1, 2, 3, 4, 6) else 0)
    dst = torch.full((n_out + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
    Q.stream(src, rows, row_bytes, dst, mode, 16)
    torch.cuda.synchronize()
    d = dst.cpu().numpy()
    assert (d[n_out:] == 0xA5).all()
    if mode in (0, 30):
        s = src.cpu().numpy().reshape(-1, 4, 1024)
        ref = s[:, 0] ^ s[:, 1] ^ s[:, 2] ^ s[:, 3]
        assert np.array_equal(d[:n_out].reshape(-1, 1024), ref)
    else:
        first = d.copy()
        src2 = src.clone()
        src2[12345] ^= 0xFF
        Q.stream(src2, rows, row_bytes, dst, mode, 16)
        torch.cuda.synchronize()
        assert (dst.cpu().numpy() != first).any()


def test_read_only_stream_reads_everything(Q):
    """Mode 50 stores, per wave, the xor of all it read: the xor over all waves must be the xor of the source, and
    flipping any byte must change it."""
    import torch
    rows, row_bytes, blocks = 512, 4096, 16
    g = torch.Generator(device="cuda").manual_seed(5)
    src = torch.randint(0, 256, (rows * row_bytes,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.zeros(blocks * 8 * 1024 + 4096, dtype=torch.uint8, device="cuda")
    dst[blocks * 8 * 1024:] = 0xA5
    Q.stream(src, rows, row_bytes, dst, 50, blocks)
    torch.cuda.synchronize()
    d = dst.cpu().numpy()
    assert (d[blocks * 8 * 1024:] == 0xA5).all()
    got = np.bitwise_xor.reduce(d[:blocks * 8 * 1024].reshape(-1, 16), axis=0)     # per wave 64 lanes x 16 B
    want = np.bitwise_xor.reduce(src.cpu().numpy().reshape(-1, 16), axis=0)
    assert np.array_equal(got, want)
