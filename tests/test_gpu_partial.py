"""GPU parity tests of partial IKJTs (windows into shared storage) against the CPU oracle: all integer
outputs bit-exact; the pooled lookup on the windows against the oracle and, bit for bit, against the
lookup on the IKJT of the same batch."""
import numpy as np
import pytest
import torch

from oracle import recd_oracle as orc
from paper_2211_05239_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def recd():
    from paper_2211_05239_amd import recd as mod
    return mod


@pytest.fixture(scope="module")
def ctx(recd):
    c = recd.Context(0)
    yield c
    c.close()


class DevicePartial:
    def __init__(self, F, B, N):
        L = F * B
        i64 = dict(dtype=torch.int64, device="cuda")
        self.p_values = torch.full((max(N, 1),), -7, **i64)
        self.win_start = torch.full((max(L, 1),), -7, **i64)
        self.win_len = torch.full((max(L, 1),), -7, **i64)
        self.inverse = torch.full((max(L, 1),), -7, dtype=torch.int32, device="cuda")
        self.feat_uoff = torch.full((F + 1,), -7, **i64)
        self.feat_poff = torch.full((F + 1,), -7, **i64)
        self.row_window = torch.full((max(L, 1), 2), -7, **i64)


def gpu_build_partial(ctx, batch, rows=True):
    values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
    if values.numel() == 0:
        values = torch.zeros(1, dtype=torch.int64, device="cuda")[:0]
    pk = DevicePartial(batch.F, batch.B, batch.N)
    pk.U, pk.P, pk.M = ctx.build_partial_ikjt(batch.F, batch.B, values, offsets, pk.p_values, pk.win_start,
                                              pk.win_len, pk.inverse, pk.feat_uoff, pk.feat_poff,
                                              pk.row_window if rows else None, want_counts=True)
    return values, offsets, pk


def _check_partial(pk, batch):
    F, B = batch.F, batch.B
    pv, ws, wl, inv, fu, fp = orc.build_partial_ikjt(F, B, batch.values, batch.offsets)
    assert (pk.U, pk.P) == (len(ws), len(pv))
    assert pk.M == int(wl.sum())
    assert np.array_equal(pk.p_values[:pk.P].cpu().numpy(), pv)
    assert np.array_equal(pk.win_start[:pk.U].cpu().numpy(), ws)
    assert np.array_equal(pk.win_len[:pk.U].cpu().numpy(), wl)
    assert np.array_equal(pk.inverse[:F * B].cpu().numpy(), inv)
    assert np.array_equal(pk.feat_uoff.cpu().numpy(), fu) and np.array_equal(pk.feat_poff.cpu().numpy(), fp)
    assert np.array_equal(pk.row_window[:F * B].cpu().numpy(), orc.partial_row_windows(F, B, ws, wl, inv, fu))
    assert (pk.p_values[pk.P:] == -7).all() and (pk.win_start[pk.U:] == -7).all()
    return pv, ws, wl, inv, fu, fp


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("weak", [0, 1])
def test_partial_build_small(ctx, recd, seed, weak):
    rng = np.random.default_rng(9500 + seed)
    F, B = int(rng.integers(1, 5)), int(rng.integers(1, 400))
    if seed % 2:
        batch = synth.tiny_batch(rng, F, B, int(rng.integers(2, 4)), int(rng.integers(0, 6)))
    else:
        w = synth.scaled(synth.WORKLOADS["cfg1"], F=F, B=B, S=6, rows=8, shift=0.5, len_max=int(rng.integers(1, 9)))
        batch = synth.make_batch(w, seed)
    ctx.set_option(recd.RECD_OPT_WEAK_HASH, weak)
    try:
        _, _, pk = gpu_build_partial(ctx, batch)
    finally:
        ctx.set_option(recd.RECD_OPT_WEAK_HASH, 0)
    _check_partial(pk, batch)


def test_partial_build_paper_example_and_hand_cases(ctx):
    kjt = synth.batch_from_lists([[[3, 4, 5], [4, 5, 6], [3, 4, 5]]])
    _, _, pk = gpu_build_partial(ctx, kjt)
    assert pk.p_values[:pk.P].tolist() == [3, 4, 5, 6]
    assert pk.row_window[:3].tolist() == [[0, 3], [1, 3], [0, 3]]
    _check_partial(pk, kjt)
    A = list(range(10, 15))
    sh = lambda k: list(range(10 + k, 15 + k))
    for rows in ([A, A, sh(1), sh(1), sh(1), sh(2), sh(3), sh(3)], [A, [50, 51], sh(1)], [A, [50, 51], A, sh(1)],
                 [A, A[2:], A[2:] + [99, 98]], [[], [1], [], [1, 2]], [[7] * 200, [7] * 199 + [8], [7] * 150]):
        kjt = synth.batch_from_lists([rows, rows[::-1]])
        _, _, pk = gpu_build_partial(ctx, kjt)
        _check_partial(pk, kjt)
    # B = 0
    _, _, pk = gpu_build_partial(ctx, synth.batch_from_lists([[], []]))
    assert (pk.U, pk.P, pk.M) == (0, 0, 0) and pk.feat_poff.tolist() == [0, 0, 0]


@pytest.mark.parametrize("shift", [0.0, 0.3, 0.9])
def test_partial_long_lists_and_lookup(ctx, shift):
    """Zipf lengths up to 256 (overlap search over several 64-id sweeps), then the pooled lookup on the
    windows: oracle parity and bit equality with the lookup on the IKJT."""
    w = synth.scaled(synth.WORKLOADS["cfg5"], F=4, B=3000, rows=20_000, D=64, shift=shift)
    batch = synth.make_batch(w, 0)
    tabs = synth.make_tables(w)
    d_tabs = gu.tables_to_dev(tabs, "f32")
    values, offsets, pk = gpu_build_partial(ctx, batch, rows=True)
    pv, ws, wl, inv, fu, fp = _check_partial(pk, batch)
    if shift > 0:
        assert pk.P < pk.M
    F, B, D = w.F, w.B, w.D
    pooled = torch.full((F * B, D), float("nan"), device="cuda")
    ctx.pooled_lookup_partial(d_tabs, pk.p_values, pk.win_start, pk.win_len, pk.feat_uoff, F * B, pooled)
    _, _, ik = gu.gpu_build(ctx, batch)
    ref_dev = torch.full((F * B, D), float("nan"), device="cuda")
    ctx.pooled_lookup_unique(d_tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, F * B, ref_dev)
    assert torch.equal(pooled[:pk.U], ref_dev[:ik.U]) and pk.U == ik.U
    assert torch.isnan(pooled[pk.U:]).all()
    uv, uo, _, _ = orc.build_ikjt(F, B, batch.values, batch.offsets)
    gu.assert_close_f32(gu.out_to_f64(pooled[:pk.U]), orc.pooled_lookup(tabs, "f32", uv, uo, fu), "pooled windows")
    out = torch.zeros(F, B, D, device="cuda")
    kjt = torch.zeros(F, B, D, device="cuda")
    ctx.expand_inverse(F, B, pooled, pk.feat_uoff, pk.inverse, out)
    ctx.kjt_pooled_lookup(d_tabs, B, values, offsets, kjt)
    assert torch.equal(out, kjt)


def test_partial_validation(ctx, recd):
    tab = [torch.zeros(10, 8, device="cuda")]
    pv = torch.tensor([1, 2, 3, 4], dtype=torch.int64, device="cuda")
    fu = torch.tensor([0, 2], dtype=torch.int64, device="cuda")
    pooled = torch.zeros(2, 8, device="cuda")
    i64 = lambda x: torch.tensor(x, dtype=torch.int64, device="cuda")
    ctx.set_option(recd.RECD_OPT_VALIDATE, 1)
    try:
        ctx.pooled_lookup_partial(tab, pv, i64([0, 1]), i64([3, 3]), fu, 2, pooled)
        for ws, wl in (([0, 2], [3, 3]), ([-1, 0], [2, 2]), ([0, 0], [2, -1])):
            with pytest.raises(recd.RecdError) as e:
                ctx.pooled_lookup_partial(tab, pv, i64(ws), i64(wl), fu, 2, pooled)
            assert e.value.status == recd.RECD_EBOUNDS
        with pytest.raises(recd.RecdError) as e:  # id 12 outside the table
            ctx.pooled_lookup_partial(tab, i64([1, 12, 3, 4]), i64([0, 1]), i64([3, 3]), fu, 2, pooled)
        assert e.value.status == recd.RECD_EBOUNDS
    finally:
        ctx.set_option(recd.RECD_OPT_VALIDATE, 0)
