"""Measurement helpers of the library on the GPU: the calibration kernels run, copy correctly and report sane rates."""
import pytest

pytestmark = pytest.mark.gpu


def test_calibration_copy_read_and_mfma():
    import torch
    import paper_2602_24174_amd as T
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    T.tasc_calibration_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    rate = T.tasc_calibration_mfma(200)
    print(f"MFMA loop: {rate:.0f} TFLOP/s", flush=True)
    assert 200.0 < rate < 2600.0            # above any vector-ALU rate, below the published dense bf16 peak
    buf = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
    small, large = T.tasc_calibration_read(buf[:2 << 20], 512), T.tasc_calibration_read(buf, 8)
    print(f"read stream: 2 MiB {small:.0f} GB/s, 64 MiB {large:.0f} GB/s", flush=True)
    assert 500.0 < large < 40000.0 and small > large      # the L2-resident stream is the faster one
    local, chip = T.tasc_calibration_handover(32, 8, 1024), T.tasc_calibration_handover(64, 1, 1024)
    flags = T.tasc_calibration_handover(64, 1, 1024, True)
    print(f"hand-over of 1 KB: 32 workgroups on one XCD {local:.2f} us, 64 over the chip {chip:.2f} us (with flags {flags:.2f} us)", flush=True)
    assert 0.1 < local < 20.0 and 0.1 < chip < 50.0 and 0.1 < flags < 100.0
    with pytest.raises(T.TascError):
        T.tasc_calibration_handover(1, 1, 1024)            # needs two workgroups
    t_store, t_swiglu, t_part = T.tasc_calibration_gemm(224, 1152, 896, 0), T.tasc_calibration_gemm(224, 9728, 896, 2), \
        T.tasc_calibration_gemm(224, 896, 4864, 4, 6)
    print(f"tiled GEMM at the 0.5B verify shapes: qkv {t_store:.1f} us, gate/up {t_swiglu:.1f} us, down in 6 slices {t_part:.1f} us", flush=True)
    assert 1.0 < t_store < 200.0 and 1.0 < t_swiglu < 400.0 and 1.0 < t_part < 400.0
    for bad in ((224, 1000, 896, 0, 1), (224, 1152, 900, 0, 1), (224, 1152, 896, 3, 1), (224, 1152, 896, 0, 2), (0, 1152, 896, 0, 1)):
        with pytest.raises(T.TascError):
            T.tasc_calibration_gemm(*bad)                  # N not a multiple of 128, K not of 64, LM-head epilogue, slices without partial sums, no rows
    with pytest.raises(T.TascError):
        T.tasc_calibration_read(buf[:1000], 1)             # not a multiple of 64 KB
    with pytest.raises(T.TascError):
        T.tasc_calibration_mfma(0)
    with pytest.raises(T.TascError):
        T.tasc_calibration_copy(dst[1:], src[1:])     # 4-byte offset: not 16-byte aligned


def test_position_rates_from_a_real_run():
    """The sweep helper on a live generate: rates are non-increasing in the position and consistent with the mean."""
    import workload as W
    from paper_2602_24174_amd.acceptance_sweeps import SweepRig
    cfg = W.get_config("cfg1").scaled(gen_len=40)
    rig = SweepRig(cfg)
    r = rig.run(k=6, lam=0.5)
    assert r["equals_greedy"]
    assert all(a >= b for a, b in zip(r["rate"], r["rate"][1:]))
    assert abs(sum(r["rate"]) - r["mean_accept"]) < 1e-9
    assert sum(r["hist"]) == r["steps"] * cfg.batch
