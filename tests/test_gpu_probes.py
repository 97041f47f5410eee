"""The library's measurement probes (attainable rates, issue cycles, tile loads) run and report
plausible figures; their results are context for the roofline fractions, not parity."""
import pytest

pytestmark = pytest.mark.gpu


def test_issue_and_tile_load_probes_report_cycles():
    import torch
    import paper_2601_07353_amd as T
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    iters = 200
    for waves in (4, 8):
        for mode in range(5):
            cyc = torch.zeros(8, dtype=torch.int64, device="cuda")
            T.talon_probe_issue(mode, waves, iters, cyc, sink)
            torch.cuda.synchronize()
            c = cyc.cpu().numpy()
            assert (c[:waves] > 0).all() and not c[waves:].any()
            if mode in (2, 3):       # sixteen 32x32x16 bf16 matrix instructions per round: 32 cycles each at best
                per = c[:waves].min() / iters / 16.0
                assert 30.0 < per < 80.0, per
    window = torch.zeros(16 << 20, dtype=torch.uint8, device="cuda")
    for loads in (4, 8):
        for with_mfma in (False, True):
            cyc = torch.zeros(2048, dtype=torch.int64, device="cuda")
            T.talon_probe_tile_loads(window, loads, with_mfma, 4, iters, cyc, sink)
            torch.cuda.synchronize()
            c = cyc.cpu().numpy().reshape(256, 8)
            assert (c[:, :4] > 0).all() and not c[:, 4:].any()
            rate = 4 * loads * 1024.0 / (c[:, :4].mean() / iters)      # bytes per cycle and compute unit
            assert 4.0 < rate < 256.0, rate
    assert int(sink.item()) == 0


def test_probe_arguments_are_checked():
    import torch
    import paper_2601_07353_amd as T
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    cyc = torch.zeros(2048, dtype=torch.int64, device="cuda")
    small = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(T.TalonError):
        T.talon_probe_tile_loads(small, 4, False, 4, 10, cyc, sink)      # window too small
    with pytest.raises(T.TalonError):
        T.talon_probe_issue(7, 4, 10, cyc, sink)                         # no such mix
    with pytest.raises(T.TalonError):
        T.talon_probe_issue(0, 5, 10, cyc, sink)                         # 4 or 8 wavefronts
