"""The measured-peak probes behind the benchmark's `measured_peak`: they must return figures that are physically
possible on the chip (below the datasheet peaks the roofline is quoted against) and not absurdly low, reject
bad arguments, and leave the first half of the scratch buffer untouched."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_probes_return_plausible_peaks_and_check_arguments():
    import paper_2408_05676_amd as laser
    buf = torch.full((1 << 29,), 7, dtype=torch.uint8, device="cuda")        # 512 MiB: above the last-level cache
    read_gbs, copy_gbs = laser.probe_hbm(buf, reps=5)
    tflops = laser.probe_mfma_f16(buf, reps=3)
    torch.cuda.synchronize()
    print(f"[probes] read {read_gbs:.0f} GB/s, copy {copy_gbs:.0f} GB/s, fp16 matrix loop {tflops:.0f} TFLOP/s")
    assert 1500.0 < read_gbs < 8000.0 and 1500.0 < copy_gbs < 8000.0
    assert 800.0 < tflops < 2600.0
    assert int(buf[: 1 << 28].min()) == 7 and int(buf.max()) == 7          # the copy wrote the same bytes; nothing else was written
    with pytest.raises(laser.LaserError):
        laser.probe_hbm(torch.zeros(1024, dtype=torch.uint8, device="cuda"))
    with pytest.raises(laser.LaserError):
        laser.probe_mfma_f16(buf, reps=0)
