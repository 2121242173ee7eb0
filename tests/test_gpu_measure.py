"""The measurement kernels behind bench.py's ceilings: the copy really copies (whole pieces and a ragged tail),
the read and MFMA loops run and report their work, bad arguments come back as statuses."""
import pytest
import torch

from paper_2502_08141_amd import lowra

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes", [16, 16 * 1024, 16 * 1024 + 48, 3 * 1024 * 1024 + 16])
def test_measure_copy_copies(nbytes):
    print(f"[measure copy {nbytes} bytes]", flush=True)
    g = torch.Generator(device="cuda"); g.manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
    lowra.lowra_measure_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:nbytes], src) and not dst[nbytes:].any()      # nothing past the end is written


def test_measure_read_and_mfma_run():
    src = torch.zeros(5 * 1024 * 1024 + 32, dtype=torch.uint8, device="cuda")
    out4 = torch.zeros(16, dtype=torch.uint8, device="cuda")
    lowra.lowra_measure_read(src, out4)
    for random_operands in (False, True):
        flops = lowra.lowra_measure_mfma(64, 8, out4, random_operands=random_operands)
        assert flops == 64 * 4 * 8 * 4 * 2.0 * 32 * 32 * 16
    torch.cuda.synchronize()
    assert not out4.any()


def test_measure_rejects_bad_arguments():
    out4 = torch.zeros(16, dtype=torch.uint8, device="cuda")
    src = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(lowra.LowraError):
        lowra.lowra_measure_copy(src, src[:24])           # not a multiple of 16 bytes
    with pytest.raises(lowra.LowraError):
        lowra.lowra_measure_copy(src[8:], src[8:24])      # misaligned
    with pytest.raises(lowra.LowraError):
        lowra.lowra_measure_mfma(0, 8, out4)
    with pytest.raises(lowra.LowraError):
        lowra.lowra_measure_mfma(4, 6, out4, random_operands=True)        # iterations % 4 != 0
