"""The library's measurement aids run and return on the GPU (they compute nothing that could be compared: the
benchmark times them)."""
import pytest
import torch

import paper_2505_20776_amd as sx

pytestmark = pytest.mark.gpu


def test_issue_mix_modes_run():
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    for n in (0, 4, 8):
        for mode in (1, 2, 3, 4):
            print(f"[case] calib_issue_mix mode={mode} vector_per_matrix={n}", flush=True)
            assert sx.calib_issue_mix(mode, n, 50, 8, sink=sink) == 0
    torch.cuda.synchronize()
    assert float(sink.item()) == 0.0            # the sink is never written for real data


def test_stream_and_matrix_calibration_run():
    buf = torch.ones(1 << 20, dtype=torch.uint8, device="cuda")
    print("[case] calib_stream_read 1 MiB, calib_mfma both tiles", flush=True)
    assert sx.calib_stream_read(buf, buf.numel()) == 0
    assert sx.calib_mfma(10, 32, 8) == 8 * 4 * 10 * 16 * 2 * 32 * 32 * 16
    assert sx.calib_mfma(10, 16, 8) == 8 * 4 * 10 * 16 * 2 * 16 * 16 * 32
    torch.cuda.synchronize()
