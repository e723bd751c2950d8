"""The measurement helpers of the library (jup_diag_*): argument validation on the CPU, and on the GPU that they run,
end, and report figures of the right order (they feed bench.py's calibration legs, not the method)."""
import ctypes

import pytest

from paper_2504_08242_amd import binding as jb

FAKE = ctypes.c_void_p(0x7000_0000_0000)  # never dereferenced by host logic


def test_diag_entry_points_reject_bad_arguments_before_any_launch():
    L = jb.lib()
    nbytes = ctypes.c_double()
    bad_fill = [
        (None, 16 << 20, 256, 8, 4096),          # no buffer
        (FAKE, 1 << 19, 256, 8, 4096),           # window below 1 MiB
        (FAKE, (16 << 20) + 1024, 256, 8, 4096), # not a power of two
        (FAKE, 3 << 20, 256, 8, 4096),           # not a power of two
        (FAKE, 16 << 20, 0, 8, 4096),            # no workgroups
        (FAKE, 16 << 20, 256, 3, 4096),          # depth not offered
        (FAKE, 16 << 20, 256, 8, 100),           # pieces not a multiple of 16
    ]
    for buf, window, wgs, depth, pieces in bad_fill:
        rc = L.jup_diag_fill_probe(buf, window, wgs, depth, pieces, None, ctypes.byref(nbytes))
        assert rc == jb.JUP_EINVAL and jb.last_error(), (window, wgs, depth, pieces)
    bad_stream = [
        (None, 1 << 30, 256, 4, 16, 1),     # no buffer
        (FAKE, 1 << 20, 256, 4, 16, 1),     # buffer shorter than 256 regions of 128 KiB
        (FAKE, 1 << 30, 0, 4, 16, 1),       # no workgroups
        (FAKE, 1 << 30, 256, 3, 15, 1),     # depth not offered
        (FAKE, 1 << 30, 256, 4, 18, 1),     # pieces not a multiple of the depth
        (FAKE, 1 << 30, 256, 4, 16, 0),     # no launches
    ]
    for buf, nbuf, wgs, depth, pieces, launches in bad_stream:
        rc = L.jup_diag_stream_probe(buf, nbuf, wgs, depth, pieces, launches, None, ctypes.byref(nbytes))
        assert rc == jb.JUP_EINVAL and jb.last_error(), (nbuf, wgs, depth, pieces, launches)
    for wgs, threads, trips, ticks, sink in [(256, 512, 100, None, FAKE), (256, 500, 100, FAKE, FAKE),
                                             (256, 2048, 100, FAKE, FAKE), (0, 512, 100, FAKE, FAKE),
                                             (256, 512, 0, FAKE, FAKE)]:
        rc = L.jup_diag_lds_read_probe(wgs, threads, trips, ticks, sink, None, ctypes.byref(nbytes))
        assert rc == jb.JUP_EINVAL and jb.last_error(), (wgs, threads, trips)
    assert L.jup_diag_clock_probe(0, FAKE, None) == jb.JUP_EINVAL
    assert L.jup_diag_clock_probe(1 << 31, FAKE, None) == jb.JUP_EINVAL
    assert L.jup_diag_mfma_loop(FAKE, 16, 256, 10, FAKE, FAKE, None, ctypes.byref(nbytes)) == jb.JUP_EINVAL  # operands too small


@pytest.mark.gpu
def test_diag_probes_run_and_report_plausible_rates():
    import torch
    window = torch.ones(4 << 20, dtype=torch.uint8, device="cuda:0")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    rates = {}
    for depth in (1, 8):
        for _ in range(2):
            ev[0].record()
            nbytes = jb.diag_fill_probe(window, 256, depth, 1024)
            ev[1].record()
            torch.cuda.synchronize()
        assert nbytes == 256 * 8 * 1024 * 1024
        rates[depth] = nbytes / ev[0].elapsed_time(ev[1]) / 1e9   # TB/s
    assert 1.0 < rates[1] < 64.0 and 1.0 < rates[8] < 64.0, rates       # an L2 -> LDS rate, not a no-op and not nonsense
    assert rates[8] > rates[1], rates                                    # more in flight is faster
    big = torch.ones(256 << 20, dtype=torch.uint8, device="cuda:0")
    for _ in range(2):
        ev[0].record()
        nbytes = jb.diag_stream_probe(big, 256, 4, 32, 4)   # four launches of 64 MiB over the four quarters of the buffer
        ev[1].record()
        torch.cuda.synchronize()
    assert nbytes == 4 * 256 * 32 * 8192
    assert 0.5 < nbytes / ev[0].elapsed_time(ev[1]) / 1e9 < 8.0    # TB/s out of HBM: below the published peak
    del big
    ticks = torch.zeros(64, dtype=torch.int64, device="cuda:0")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    per_wg = jb.diag_lds_read_probe(64, 1024, 500, ticks, sink)
    torch.cuda.synchronize()
    t = ticks.cpu().numpy().astype("float64")
    assert (t > 0).all() and int(sink.item()) == 0
    assert 32.0 < per_wg / t.mean() < 2048.0, per_wg / t.mean()         # bytes per clock and CU
    clk = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    jb.diag_clock_probe(100_000, clk)                                    # one millisecond of the 100 MHz reference
    torch.cuda.synchronize()
    shader, ref = clk.cpu().tolist()
    assert ref >= 100_000 and 300.0 < 100.0 * shader / ref < 3000.0      # MHz


@pytest.mark.gpu
def test_kernel_name_reports_the_documented_tile_policy():
    """jup_diag_kernel_name names the instantiation a projection of n tokens runs as (what ties a counter reading on file
    to the tiling that runs today).  The shapes the design document gives for the 7B-shaped stage, alone on the chip and
    inside an overlapped call: a change of the policy has to show up here and there."""
    from paper_2504_08242_amd import synth_inputs as si
    cfg = dict(si.LLAMA7B_STAGE, n_layers=1)
    layers = si.make_layers(cfg, seed=5, bf16=True)
    stage = jb.Stage(cfg, "bf16", jb.upload_layers(layers, "bf16"), 2048)
    K = jb.KERNEL_IDS
    want = {   # (kernel, rows, overlapped): <row blocks, column blocks, waves along M, waves along N, epilogue>
        ("gemm_gate_up", 512, False): "gemm_bf16<8,6,4,2,2>", ("gemm_qkv", 512, False): "gemm_bf16<4,6,4,2,0>",
        ("gemm_o", 512, False): "gemm_bf16<4,4,4,2,1>", ("gemm_down", 512, False): "gemm_bf16<8,4,4,2,1>",
        ("gemm_gate_up", 512, True): "gemm_bf16<8,8,4,2,2>", ("gemm_qkv", 512, True): "gemm_bf16<8,6,4,2,0>",
        ("gemm_qkv", 256, False): "gemm_bf16<4,3,4,1,0>", ("gemm_gate_up", 256, False): "gemm_bf16<8,3,4,1,2>",
        ("gemm_o", 256, False): "gemm_bf16<4,4,4,2,1>", ("gemm_down", 256, False): "gemm_bf16<4,4,4,2,1>",
        ("gemm_qkv", 128, False): "gemm_bf16<4,2,4,1,0>", ("gemm_gate_up", 128, False): "gemm_bf16<4,3,4,1,2>",
        ("gemm_qkv", 64, False): "gemm_bf16<2,2,2,2,0>", ("gemm_gate_up", 64, False): "gemm_bf16<2,3,2,3,2>",
        ("gemm_gate_up", 5, False): "gemm_bf16<1,3,1,3,2>", ("gemm_qkv", 5, False): "gemm_bf16<2,2,2,2,0>",
        ("gemm_gate_up", 1024, False): "gemm_bf16<8,6,4,2,2>", ("gemm_qkv", 1024, False): "gemm_bf16<8,3,8,1,0>",
    }
    got = {k: stage.kernel_name(K[k[0]], k[1], k[2]) for k in want}
    assert got == want, {k: (got[k], want[k]) for k in want if got[k] != want[k]}
    stage.destroy()
