"""GPU check of pgti_epoch_indices_static, the epoch-order call for callers that cannot allocate:
its share must equal, bit for bit, what pgti_epoch_indices (the call it is a variant of) produces for
the same arguments, and what the CPU oracle defines, on two calls in a row through the C ABI, the
second with a smaller input (the file-scope scratch array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2507_11683_amd import pgti
else:  # collected on a CPU machine only to be deselected
    pgti = None

P = Q = 12


def _share_of_existing_entry_point(n_windows, seed, epoch, rank, world):
    """pgti_epoch_indices on a context whose series has n_windows valid starts."""
    T = n_windows + P + Q - 1
    series = np.zeros((T, 1, 1), dtype=np.float32)
    with pgti.Context(0) as ctx:
        ctx.load_series(series, P, Q, 8, pgti.PGTI_F32, np.zeros(1, np.float32), np.ones(1, np.float32))
        n_share = ctx.epoch_indices(seed, epoch, rank, world)
        share = ctx.get_indices()
    assert n_share == len(share)
    return share


def test_static_epoch_order_matches_the_allocating_call_twice_in_a_row():
    # (n_windows, seed, epoch, rank, world): the largest size the call accepts, then ever smaller
    # inputs: Statewide's window count (512 buckets), one rank of 16 of it, Tiny's count (16 buckets),
    # a single-workgroup size, one start
    cases = [(1 << 20, 3, 0, 0, 1), (105097, 0, 0, 0, 1), (105097, 7, 2, 3, 16), (1977, 0, 0, 0, 1),
             (1000, 5, 1, 1, 3), (1, 0, 0, 0, 1)]
    wants = [_share_of_existing_entry_point(*c) for c in cases]
    out = torch.empty((1 << 20) + 64, dtype=torch.int32, device="cuda")
    canary = -7
    stream = torch.cuda.current_stream()
    for (n, seed, epoch, rank, world), want in zip(cases, wants):
        print("static epoch order:", n, seed, epoch, rank, world, flush=True)
        out.fill_(canary)
        got_len = pgti.epoch_indices_static(n, seed, epoch, rank, world, out, stream)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert got_len == len(want)
        assert np.array_equal(got[:got_len], want), "differs from pgti_epoch_indices"
        assert np.array_equal(want, oracle.epoch_indices(seed, epoch, rank, world, n)), "differs from the oracle"
        assert np.all(got[got_len:] == canary), "wrote past the share"


def test_static_epoch_order_back_to_back_on_one_stream_without_host_sync():
    # two calls enqueued back to back (larger, then smaller) into two buffers: stream order alone
    # must keep the second from seeing the first's leftovers
    a = torch.empty(52093, dtype=torch.int32, device="cuda")
    b = torch.empty(34249, dtype=torch.int32, device="cuda")
    la = pgti.epoch_indices_static(52093, 11, 4, 0, 1, a)
    lb = pgti.epoch_indices_static(34249, 11, 5, 0, 1, b)
    torch.cuda.synchronize()
    assert la == 52093 and lb == 34249
    assert np.array_equal(a.cpu().numpy(), oracle.epoch_indices(11, 4, 0, 1, 52093))
    assert np.array_equal(b.cpu().numpy(), oracle.epoch_indices(11, 5, 0, 1, 34249))


def test_static_epoch_order_can_be_captured_and_replayed():
    # the call enqueues kernels only (no allocation, no memset node), so it can sit in a HIP graph;
    # every replay, with eager work and synchronisations in between, must give the same share
    n, seed, epoch = 34249, 21, 2
    want = oracle.epoch_indices(seed, epoch, 1, 3, n)
    out = torch.empty(len(want) + 8, dtype=torch.int32, device="cuda")
    s = torch.cuda.Stream()
    with pgti.Context(0):  # resolves the scratch address on this device before any capture
        pass
    with torch.cuda.stream(s):
        assert pgti.epoch_indices_static(n, seed, epoch, 1, 3, out, s) == len(want)  # eager once
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        got = pgti.epoch_indices_static(n, seed, epoch, 1, 3, out, torch.cuda.current_stream())
    assert got == len(want)
    for rep in range(4):
        out.fill_(-5)
        other = pgti.epoch_indices_static(1977, 1, rep, 0, 1, torch.empty(1977, dtype=torch.int32, device="cuda"))  # dirties the scratch
        torch.cuda.synchronize()
        assert other == 1977
        with torch.cuda.stream(s):
            g.replay()
        s.synchronize()
        res = out.cpu().numpy()
        assert np.array_equal(res[:len(want)], want), rep
        assert np.all(res[len(want):] == -5)


def test_static_epoch_order_rejects_what_it_cannot_hold():
    out = torch.empty(16, dtype=torch.int32, device="cuda")
    lib = pgti.load_library()
    sh = torch.cuda.current_stream().cuda_stream
    assert lib.pgti_epoch_indices_static(0, pgti.PGTI_STATIC_MAX_WINDOWS + 1, 0, 0, 0, 1, out.data_ptr(), 16, sh) \
        == pgti.PGTI_ERR_RANGE
    assert b"exceed" in lib.pgti_last_error()
    assert lib.pgti_epoch_indices_static(0, 100, 0, 0, 0, 1, out.data_ptr(), 16, sh) == pgti.PGTI_ERR_ARG  # capacity
    assert lib.pgti_epoch_indices_static(0, 100, 0, 0, 4, 4, out.data_ptr(), 16, sh) == pgti.PGTI_ERR_RANGE  # rank
    assert lib.pgti_epoch_indices_static(0, 0, 0, 0, 0, 1, out.data_ptr(), 16, sh) == pgti.PGTI_ERR_ARG
    assert lib.pgti_epoch_indices_static(0, 16, 0, 0, 0, 1, None, 16, sh) == pgti.PGTI_ERR_ARG
