"""ef_measure_peak: the measured ceilings the benchmark prints beside the published peaks.  The figures must be
plausible for the part (a streaming read between a third of and the whole published HBM rate, the matrix-core loop
between 40 % and 105 % of the published dense 16-bit rate), repeatable, and bad arguments must be refused."""
import pytest
import torch

from paper_2510_26730_amd import binding as ef
from paper_2510_26730_amd import synth

pytestmark = pytest.mark.gpu


def test_measured_peaks_are_plausible_and_bad_arguments_refused():
    cfg = synth.CONFIGS["tiny"]
    ctx = ef.ef_create(n_layers=1, d_model=cfg.d, n_experts=cfg.E, top_k=cfg.k, d_ff=cfg.F, slots_total=1, max_tokens=32)
    try:
        n = 1 << 30
        buf = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
        s = torch.cuda.current_stream()
        hbm = [ef.ef_measure_peak(ctx, ef.EF_PEAK_HBM_READ, buf, n, 4, s) for _ in range(2)]
        mfma = [ef.ef_measure_peak(ctx, ef.EF_PEAK_MFMA_16BIT, None, 0, 2, s) for _ in range(2)]
        print(f"  streaming read {hbm[0]:.0f} / {hbm[1]:.0f} GB/s, matrix cores {mfma[0]:.0f} / {mfma[1]:.0f} TFLOP/s", flush=True)
        assert all(2600.0 < x < 8000.0 for x in hbm)
        assert all(1000.0 < x < 2625.0 for x in mfma)
        assert abs(hbm[0] - hbm[1]) < 0.3 * hbm[0] and abs(mfma[0] - mfma[1]) < 0.3 * mfma[0]   # clocks move between runs
        for bad in (dict(what=ef.EF_PEAK_HBM_READ, buf=buf, nbytes=(8 << 20) + 16, reps=1),      # not a multiple of 8 MiB
                    dict(what=ef.EF_PEAK_HBM_READ, buf=None, nbytes=8 << 20, reps=1),
                    dict(what=ef.EF_PEAK_HBM_READ, buf=buf, nbytes=8 << 20, reps=0),
                    dict(what=7, buf=buf, nbytes=8 << 20, reps=1)):
            with pytest.raises(ef.EfError):
                ef.ef_measure_peak(ctx, bad["what"], bad["buf"], bad["nbytes"], bad["reps"], s)
        del buf
    finally:
        ef.ef_destroy(ctx)
