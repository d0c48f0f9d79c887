"""The allocation-free builder entry point (recd_build_ikjt_noalloc) against recd_build_ikjt, through
the C ABI: identical integer outputs on two calls in a row, the second on a smaller batch (the static
scratch array keeps the first call's contents), then an oversized request."""
import numpy as np
import pytest
import torch

from paper_2211_05239_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def recd():
    from paper_2211_05239_amd import recd as mod
    return mod


def _both(ctx, batch):
    F, B = batch.F, batch.B
    values, offsets, ref = gu.gpu_build(ctx, batch)
    ik = gu.DeviceIKJT(F, B, batch.N)
    ctx.build_ikjt_noalloc(F, B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse, ik.feat_uoff)
    torch.cuda.synchronize()
    fu = ik.feat_uoff.cpu().numpy()
    ik.U = int(fu[F])
    ik.M = int(ik.u_offsets[ik.U].item())
    assert (ik.U, ik.M) == (ref.U, ref.M)
    for a, b in zip(ik.numpy(), ref.numpy()):
        assert np.array_equal(a, b)
    # entries beyond U + 1 / M are left untouched, as by the allocating call
    assert torch.equal(ik.u_offsets[ik.U + 1:], ref.u_offsets[ref.U + 1:])
    assert torch.equal(ik.u_values[ik.M:], ref.u_values[ref.M:])
    return ik


def test_noalloc_build_equals_build_twice_in_a_row(recd):
    ctx = recd.Context(0)
    try:
        big = synth.make_batch(synth.scaled(synth.WORKLOADS["cfg2"], F=16, B=4096, rows=1_000_000), 0)
        small = synth.make_batch(synth.scaled(synth.WORKLOADS["cfg1"], F=3, B=301, rows=5000), 1)
        assert big.F * big.B == recd.RECD_NOALLOC_MAX_LISTS
        _both(ctx, big)       # several scan blocks, ragged lists, the largest size the entry point takes
        _both(ctx, small)     # right behind it, smaller: stale scratch contents must not leak
        _both(ctx, synth.batch_from_lists([[[], [], []]]))    # a single empty slot
        _both(ctx, synth.batch_from_lists([[] for _ in range(3)]))  # B = 0
        _both(ctx, big)
    finally:
        ctx.close()


def test_noalloc_build_weak_hash_and_second_context(recd):
    """All contexts of a GPU share the one array; sequential use from two contexts on one stream."""
    c1, c2 = recd.Context(0), recd.Context(0)
    try:
        c2.set_option(recd.RECD_OPT_WEAK_HASH, 1)
        b = synth.make_batch(synth.scaled(synth.WORKLOADS["cfg5"], F=8, B=2048, rows=30_000), 2)
        _both(c1, b)
        _both(c2, b)
        _both(c1, b)
    finally:
        c1.close()
        c2.close()


def test_noalloc_build_rejects_oversize(recd):
    ctx = recd.Context(0)
    try:
        z = torch.zeros(8, dtype=torch.int64, device="cuda")
        zi = torch.zeros(8, dtype=torch.int32, device="cuda")
        with pytest.raises(recd.RecdError) as e:
            ctx.build_ikjt_noalloc(1, recd.RECD_NOALLOC_MAX_LISTS + 1, z, z, z, z, zi, z)
        assert e.value.status == recd.RECD_ECAPACITY
        with pytest.raises(recd.RecdError) as e:
            ctx.build_ikjt_noalloc(1024, 65, z, z, z, z, zi, z)
        assert e.value.status == recd.RECD_ECAPACITY
    finally:
        ctx.close()
