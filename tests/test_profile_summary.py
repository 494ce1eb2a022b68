"""Host logic of the rocprofv3 summariser: parsing of the kernel-trace CSV and the launch window that is
compared with bench.py's own kernel events, and the copy calibration of the byte counters (CPU only)."""
import os

import pytest

from paper_2603_02188_amd import profile_summary as ps

KNAME = "void mlra::(anonymous namespace)::decode_mfma_kernel<6, 0>(mlra::MfmaParams)"


def _write_trace(root, durations_ns, other_every=2):
    os.makedirs(os.path.join(root, "host"), exist_ok=True)
    path = os.path.join(root, "host", "1_kernel_trace.csv")
    t = 1000
    rows = ['"Kind","Kernel_Name","Start_Timestamp","End_Timestamp"']
    for i, d in enumerate(durations_ns):
        if i % other_every == 0:      # another kernel in between, which the window must not count
            rows.append(f'"KERNEL_DISPATCH","void mlra::absorb_q_mfma_kernel(int)",{t},{t + 7})')
            t += 10
        rows.append(f'"KERNEL_DISPATCH","{KNAME}",{t},{t + d}')
        t += d + 5
    # rows out of start order on disk: the summariser sorts by start time
    rows = [rows[0]] + rows[1:][::-1]
    with open(path, "w") as f:
        f.write("\n".join(rows) + "\n")


def test_window_mean_takes_the_named_kernels_launches_in_start_order(tmp_path):
    durs = [1000 * (i + 1) for i in range(10)]          # 1 us, 2 us, ... 10 us
    _write_trace(str(tmp_path), durs)
    line = ps.window_mean(str(tmp_path), "decode_mfma_kernel", 3, 4)    # launches 3..6: 4, 5, 6, 7 us
    assert "launches 3..6 of 10 of decode_mfma_kernel<6, 0>" in line
    assert "mean 5.5 us (min 4.0, max 7.0)" in line


def test_window_mean_refuses_a_window_past_the_end(tmp_path):
    _write_trace(str(tmp_path), [1000] * 5)
    with pytest.raises(SystemExit):
        ps.window_mean(str(tmp_path), "decode_mfma_kernel", 3, 4)


def test_copy_scale_uses_the_largest_copies():
    acc = {ps.COPY_KERNEL: {"FETCH_SIZE": [10.0, 524288.0, 524290.0, 524286.0]}}
    # 2^20 KiB per copy over a reading of 2^19: 2 KiB per counter unit
    assert ps._copy_scale(acc, "FETCH_SIZE") == pytest.approx(2.0, rel=1e-5)
    assert ps._copy_scale({}, "FETCH_SIZE") is None


def test_short_kernel_names():
    assert ps._short(KNAME) == "decode_mfma_kernel<6, 0>"


def test_mfma_busy_fraction_from_the_two_counters():
    # a kernel of 281,600 cycles: every one of the 32 shader engines counts them; the 1024 SIMDs' matrix pipes
    # are busy 172,800 cycles each -> 0.61 (the figures of the C3 counter profile)
    assert ps.mfma_busy_fraction(172800.0 * 1024, 281600.0 * 32) == pytest.approx(0.6136, abs=1e-3)
    assert ps.mfma_busy_fraction(1.769e8, 9.011e6) == pytest.approx(0.61, abs=0.01)
    assert ps.mfma_busy_fraction(1.0, 0.0) == 0.0
