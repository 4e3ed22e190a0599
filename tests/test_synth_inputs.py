"""Host-side checks of the seeded input generators (no CADA arithmetic here)."""
import numpy as np

from cada_synth import configs, generators, philox


def test_philox4x32_10_known_answers():
    """Known-answer vectors published with the Philox reference distribution
    (counter, key -> output): all-zero, all-ones and the digits-of-pi case."""
    kat = [((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
           ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
           ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
            (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1))]
    for ctr, key, out in kat:
        got = tuple(int(x) for x in philox.philox4x32_10(*ctr, *key))
        assert got == out


def test_counter_rows_statistics_and_reproducibility():
    cfg = configs.CFG3.scaled(layer_dims=(4096,), M=3, N_m=64, B=8)
    prob = generators.make_problem(cfg)
    X, y = prob.rows(1, np.arange(64))
    X2, y2 = prob.rows(1, np.array([5, 63]))
    assert np.array_equal(X[[5, 63]], X2) and np.array_equal(y[[5, 63]], y2)
    assert X.dtype == np.float32 and set(np.unique(y)) <= {-1.0, 1.0}
    resid = (X - prob.shift[1]).astype(np.float64)
    assert abs(resid.mean()) < 5e-4 and abs(resid.var() * cfg.p - 1.0) < 0.02
    assert 0.25 < (y > 0).mean() < 0.75
    Xo, _ = prob.rows(2, np.arange(4))
    assert not np.array_equal(Xo, X[:4])


def test_schedule_rows_distinct_and_in_range():
    for cfg in (configs.CFG1, configs.CFG2.scaled(K=50)):
        s = generators.make_schedule(cfg)
        assert s.shape == (cfg.K, cfg.M, cfg.B) and s.dtype == np.int32
        assert s.min() >= 0 and s.max() < cfg.N_m
        srt = np.sort(s, axis=2)
        assert (np.diff(srt, axis=2) > 0).all()
        assert np.array_equal(s, generators.make_schedule(cfg))


def test_small_recipes_shapes():
    p1 = generators.make_problem(configs.CFG1)
    assert p1.X.shape == (10000, 54) and p1.y.shape == (10000,) and p1.theta0.shape == (54,)
    c4 = configs.CFG4.scaled(layer_dims=(20, 16, 10), M=3, N_m=50)
    p4 = generators.make_problem(c4)
    assert p4.X.shape == (150, 20) and p4.y.dtype == np.int32 and p4.theta0.size == c4.p
    c5 = configs.CFG5.scaled(layer_dims=(24, 16, 16, 10), M=3, N_m=40)
    p5 = generators.make_problem(c5)
    assert p5.X.shape == (120, 24) and p5.y.min() >= 0 and p5.y.max() < 10
    c2 = configs.CFG2.scaled(M=2, N_m=100)
    p2 = generators.make_problem(c2)
    assert 0.75 < (p2.X == 0).mean() < 0.85
    assert configs.CFG4.p == 407050 and configs.CFG5.p == 4206602
