"""The C ABI used from plain C (tests/abi_consumer/abi_consumer.c: pgti.h + the HIP runtime, no Python and
no torch in that process): its share and its batches, written to a file, against the CPU oracle."""
import os
import subprocess
import sys

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_consumer"))


def _series(T, N, F):
    t = np.arange(T, dtype=np.int64)[:, None, None]
    n = np.arange(N, dtype=np.int64)[None, :, None]
    f = np.arange(F, dtype=np.int64)[None, None, :]
    return (((t * 131 + n * 17 + f * 7) % 1009).astype(np.float32) * np.float32(0.125) - np.float32(40.0)).astype(np.float32)


@pytest.mark.parametrize("bf16", [0, 1], ids=["f32", "bf16"])
@pytest.mark.parametrize("geom", [(300, 207, 2, 12, 12, 64, 5, 3, 1, 2), (97, 33, 3, 5, 2, 8, 0, 0, 0, 1),
                                  (2500, 8, 1, 3, 3, 4, 9, 1, 2, 5)],
                         ids=lambda g: "T%d_N%d_F%d_P%d_Q%d_B%d_seed%d_epoch%d_rank%dof%d" % g)
def test_plain_c_consumer_matches_the_oracle(tmp_path, geom, bf16):
    import build_consumer as consumer_build  # tests/abi_consumer/build_consumer.py: compiles in a second if missing or stale
    exe = consumer_build.build()
    T, N, F, P, Q, B, seed, epoch, rank, world = geom
    out = tmp_path / "consumer.bin"
    run = subprocess.run([exe, str(out)] + [str(v) for v in (T, N, F, P, Q, B, seed, epoch, rank, world, bf16)],
                         capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    raw = out.read_bytes()
    n_share, nb = np.frombuffer(raw, np.int64, 2, 0)
    first_count, last_count = np.frombuffer(raw, np.int32, 2, 16)
    share = np.frombuffer(raw, np.int32, n_share, 24)
    series = _series(T, N, F)
    mean = (20.0 + np.arange(F)).astype(np.float32)
    std = (7.5 + 0.25 * np.arange(F)).astype(np.float32)
    n = T - P - Q + 1
    want_share = oracle.epoch_indices(seed, epoch, rank, world, n)
    assert n_share == len(want_share) and nb == -(-n_share // B)
    assert np.array_equal(share, want_share)
    storage = oracle.BF16 if bf16 else oracle.F32
    ser = oracle.store_bf16(series) if bf16 else series
    xe, ye = B * P * N * F, B * Q * N * F
    off = 24 + 4 * n_share
    for b, count in ((0, first_count), (nb - 1, last_count)):
        x = np.frombuffer(raw, np.float32, xe, off).reshape(B, P, N, F)
        y = np.frombuffer(raw, np.float32, ye, off + 4 * xe).reshape(B, Q, N, F)
        off += 4 * (xe + ye)
        starts = want_share[b * B:(b + 1) * B]
        assert count == len(starts)
        wx, wy = oracle.build_batch(ser, storage, P, Q, mean, std, starts)
        assert np.array_equal(x[:count].view(np.uint32), wx.view(np.uint32)), b
        assert np.array_equal(y[:count].view(np.uint32), wy.view(np.uint32)), b
        assert not x[count:].any() and not y[count:].any()  # rows past a short batch keep the zeros they had
    assert off == len(raw)
