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


def test_exchange_probe_reads_no_stale_value():
    """The write-once exchange the persistent kernel relies on (write-through stores, grid barrier, plain cached loads of
    lines nobody has read before): 300 rounds between all compute units without a stale value or an expired wait."""
    import paper_2408_05676_amd as laser
    scratch = torch.empty(4096 + 300 * 2048 * 304, dtype=torch.uint8, device="cuda")
    us, errs = laser.probe_exchange(scratch, 300)
    print(f"[probe] one all-to-all exchange: {us:.2f} us")
    assert errs == 0 and 0.5 < us < 100.0
