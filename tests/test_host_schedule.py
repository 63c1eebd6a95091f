"""The library's host-side schedule logic (Sec. 5.6) against the oracle's, on random accuracy curves (no GPU)."""
import numpy as np

from oracle import schedule as osch


def test_schedules_host_logic_matches_the_oracle():
    from paper_1507_01239_amd import schedule as S
    rng = np.random.default_rng(0)
    for trial in range(50):
        accs = np.cumsum(np.abs(rng.standard_normal(12)) * rng.choice([0.05, 0.3, 2.0], 12)) + 30
        ref_rates, ref_stop = osch.newbob(0.32, list(accs))
        nb, rates, stop = S.Newbob(0.32), [], None
        lr = 0.32
        for e, a in enumerate(accs):
            rates.append(lr)
            lr = nb.after_epoch(float(a))
            if lr is None:
                stop = e
                break
        assert rates == ref_rates and stop == ref_stop
    assert np.allclose(S.exponential_rates(0.32, 15, 0.01), osch.exponential(0.32, 15, 0.01), rtol=1e-12)
    assert S.scaled_initial_rate(0.008, 8) == osch.scaled_initial_rate(0.008, 8)
