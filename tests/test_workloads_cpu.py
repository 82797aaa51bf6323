"""CPU-only checks of the synthetic input generator and the workload table."""
import numpy as np

from paper_2507_11683_amd import workloads as W


def test_workload_table_matches_the_benchmark_configurations():
    t, m, mw, s, sb = (W.WORKLOADS[k] for k in ("tiny", "medium", "medium_wide", "statewide",
                                                  "statewide_bf16_rank3of16"))
    assert (t.T, t.N, t.F, t.P, t.Q, t.B, t.n_windows) == (2000, 207, 2, 12, 12, 64, 1977)
    assert (m.T, m.N, m.n_windows) == (34272, 207, 34249)
    assert (mw.T, mw.N, mw.n_windows) == (52116, 325, 52093)
    assert (s.T, s.N, s.B, s.n_windows) == (105120, 11160, 32, 105097)
    assert s.series_bytes_f32 == 9385113600
    assert (sb.storage, sb.world, sb.rank, sb.seed, sb.epochs) == ("bf16", 16, 3, 7, (0, 1, 2))
    assert t.bytes_per_snapshot() == 79488 and mw.bytes_per_snapshot() == 124800
    assert s.bytes_per_snapshot() == 4285440 and sb.bytes_per_snapshot() == 3214080


def test_generator_is_counter_based_and_traffic_shaped():
    w = W.WORKLOADS["medium"]
    a = W.make_series(w)
    b = W.make_series(w)
    assert np.array_equal(a, b)
    # slab generation gives the same bits as one pass
    c = np.zeros_like(a)
    W.traffic_series(w.T, w.N, w.data_seed, w.gen_flags, out=c, t_begin=0, t_end=1000)
    W.traffic_series(w.T, w.N, w.data_seed, w.gen_flags, out=c, t_begin=1000, t_end=w.T)
    assert np.array_equal(a, c)
    speed, tod = a[..., 0], a[..., 1]
    assert speed.min() == 0.0 and speed.max() <= 80.0
    assert 0.005 < float((speed == 0).mean()) < 0.015          # ~1 % dropout
    assert 55 < float(speed[speed > 0].mean()) < 65
    assert np.array_equal(tod[:, 0], ((np.arange(w.T) % 288) / np.float32(288.0)).astype(np.float32))
    assert np.all(tod == tod[:, :1])
    assert np.isfinite(a).all()
    assert not np.array_equal(a[:100], W.traffic_series(100, w.N, w.data_seed + 1, w.gen_flags))
