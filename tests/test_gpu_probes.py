"""The hardware probes run and report plausible rates (they are measurement helpers: only their sanity is tested)."""
import pytest
import torch

import paper_2602_12957_amd.binding as B

pytestmark = pytest.mark.gpu


def _time(kind, n_wg, iters, arg, scratch):
    stream = torch.cuda.current_stream().cuda_stream
    B.hsd_probe_launch(stream, kind, n_wg, 2, arg, scratch.data_ptr(), scratch.numel())
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    B.hsd_probe_launch(stream, kind, n_wg, iters, arg, scratch.data_ptr(), scratch.numel())
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3


def test_probes_run_and_report_plausible_rates():
    scratch = torch.zeros(8 * 65536, dtype=torch.uint8, device="cuda:0")
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    iters = 2000
    dt = _time(B.HSD_PROBE_MFMA, n_cu, iters, 0, scratch)
    tflops = n_cu * 4 * iters * 16 * 32768 / dt / 1e12
    assert 500 < tflops < 2600, tflops                       # between a fifth of and the datasheet's dense bf16 peak
    for kind in (B.HSD_PROBE_LOAD_REG, B.HSD_PROBE_LOAD_LDS):
        dt = _time(kind, n_cu, 500, 0, scratch)
        per_cu = 500 * 32768 / (dt * 1e9)
        assert 20 < per_cu < 400, per_cu                     # bytes per ns and compute unit
    dt = _time(B.HSD_PROBE_LDS_READ, n_cu, 1000, 8, scratch)
    per_cu = 1000 * 8192 * 8 / (dt * 1e9)
    assert 100 < per_cu < 1500, per_cu
    assert int(scratch[4:].max()) == 0                       # the probes only ever write the first four bytes
