"""Attainable rates of the device beside the published peaks: a plain copy kernel and a read stream (HBM, L2) and a
register-only MFMA loop.

    python -m paper_2602_24174_amd.calibrate

Prints the copy kernel's rate over 1 GiB (read + write, best of 5), the read rates of tasc_calibration_read over 1 GiB
(HBM), 128 MiB (memory-side cache) and 2 MiB (the L2 of every XCD), the bf16 MFMA rate of tasc_calibration_mfma, and
the latency of one hand-over among resident workgroups (tasc_calibration_handover): polled data against arrival flags,
on one XCD and across the chip, for the sizes the small-batch verify step hands from phase to phase.
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    import torch
    import paper_2602_24174_amd as T
    n = 1 << 30
    src = torch.zeros(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream().cuda_stream
    best = 0.0
    for _ in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        T.tasc_calibration_copy(dst, src, stream)
        e1.record()
        torch.cuda.synchronize()
        best = max(best, 2 * n / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    print(f"copy kernel, 1 GiB read + 1 GiB written: {best:.2f} TB/s of HBM traffic (published peak 8 TB/s)")
    for label, nbytes, passes in (("1 GiB (HBM)", 1 << 30, 8), ("128 MiB (memory-side cache)", 128 << 20, 64), ("2 MiB (L2 of every XCD)", 2 << 20, 4096)):
        rate = max(T.tasc_calibration_read(src[:nbytes], passes, stream) for _ in range(3))
        print(f"read stream over {label}, 8 independent 16-byte loads per lane: {rate / 1e3:.2f} TB/s "
              f"({rate / torch.cuda.get_device_properties(0).multi_processor_count:.0f} GB/s per compute unit)")
    rates = [T.tasc_calibration_mfma(2000, stream) for _ in range(3)]
    print(f"MFMA loop, v_mfma_f32_32x32x16_bf16 on register operands, 8 waves per compute unit: {max(rates):.0f} TFLOP/s "
          f"(published dense bf16 peak 2500 TFLOP/s)")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    print("hand-over among resident workgroups, microseconds per hand-over (polled data | arrival flags, then loads):")
    for label, n, stride in (("32 workgroups on one XCD", 32, 8), ("32 workgroups over all XCDs", 32, 1), ("96 workgroups over all XCDs", 96, 1),
                             (f"all {cus} workgroups", cus, 1)):
        if (n - 1) * stride >= cus:
            continue
        cells = []
        for nbytes in (1024, 10240, 20480):
            a = T.tasc_calibration_handover(n, stride, nbytes, False, stream)
            b = T.tasc_calibration_handover(n, stride, nbytes, True, stream)
            cells.append(f"{nbytes // 1024:2d} KB {a:5.2f} | {b:5.2f}")
        print(f"  {label:32s} " + "   ".join(cells))


if __name__ == "__main__":
    main()
