"""The machine-peak probes of the C ABI (GPU): they must copy correctly and return sane rates."""
import pytest
import torch

import paper_1904_07421_amd as J

pytestmark = pytest.mark.gpu


def test_copy_probe_copies_and_reports_a_rate():
    src = torch.arange(1 << 22, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    print("probe copy 16 MiB", flush=True)
    gbs = J.jitdb_probe_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert 10.0 < gbs < 16000.0     # between a PCIe-class rate and twice the HBM data-sheet peak


@pytest.mark.parametrize("dtype,peak", [(J.JITDB_BF16, 2500.0), (J.JITDB_F32, 157.3)])
def test_mfma_probe_stays_under_the_data_sheet_peak(dtype, peak):
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    print(f"probe mfma dtype={dtype}", flush=True)
    tf = J.jitdb_probe_mfma(dtype, sink)
    torch.cuda.synchronize()
    assert float(sink[0]) == 0.0
    assert 0.05 * peak < tf < 1.05 * peak


def test_probe_bad_arguments():
    src = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(J.JitdbError):
        J.jitdb_probe_copy(src[:3], src[4:7])          # 12 bytes: not a multiple of 16
    with pytest.raises(J.JitdbError):
        J.jitdb_probe_mfma(7, src)


@pytest.mark.parametrize("kind,name", [(0, "copy"), (1, "read"), (2, "write"), (3, "copy-nt"), (4, "copy-chunk")])
def test_stream_probe_kinds(kind, name):
    src = torch.arange(1 << 22, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    print(f"probe stream {name} 16 MiB", flush=True)
    gbs = J.jitdb_probe_stream(kind, src, dst)
    torch.cuda.synchronize()
    assert 10.0 < gbs < 16000.0
    if kind in (0, 3, 4):
        assert torch.equal(src, dst)
    if kind == 1:
        assert not bool(dst.any())          # a read-only stream writes nothing
    with pytest.raises(J.JitdbError):
        J.jitdb_probe_stream(9, src, dst)
