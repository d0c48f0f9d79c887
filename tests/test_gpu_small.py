"""The one-launch builder of small batches (at most 1024 rows per feature: a block per feature, hash
table in LDS, the blocks exchange their counts once) against the CPU oracle (Sec. 4.2: unique lists in
first-occurrence order, offsets, inverse) and against the general builder, through the C ABI; and the
form of the one-pass forward in which every run sums its list."""
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


def _check(ik, batch):
    ref = orc.build_ikjt(batch.F, batch.B, batch.values, batch.offsets)
    assert ik.U == int(ref[3][-1]) and ik.M == len(ref[0])
    for name, g, r in zip(("u_values", "u_offsets", "inverse", "feat_uoff"), ik.numpy(), ref):
        assert g.dtype == r.dtype and np.array_equal(g, r), name
    return ref


@pytest.mark.parametrize("B", [1, 2, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 1000, 1023, 1024])
def test_rows_per_feature(ctx, B):
    """Every lanes-per-row variant (8, 4, 2, 1) and the sizes around its limits."""
    rng = np.random.default_rng(900 + B)
    for F in (1, 3):
        batch = synth.tiny_batch(rng, F, B, int(rng.integers(2, 9)), int(rng.integers(0, 12)))
        _, _, ik = gu.gpu_build(ctx, batch)   # also compares with the general builder
        _check(ik, batch)


@pytest.mark.parametrize("F", [2, 63, 64, 65, 128, 200, 256])
def test_many_features(ctx, F):
    """More blocks than a wave has lanes: the sums over the features before a block take several rounds."""
    w = synth.scaled(synth.WORKLOADS["cfg1"], F=F, B=37, rows=50)
    batch = synth.make_batch(w, F)
    _, _, ik = gu.gpu_build(ctx, batch)
    _check(ik, batch)


def test_workloads_and_weak_hash(ctx, recd):
    for name, kw in (("cfg1", {}), ("cfg2", dict(F=5, B=1024)), ("cfg3", dict(F=3, B=700))):
        w = synth.scaled(synth.WORKLOADS[name], **kw)
        batch = synth.make_batch(w, 3)
        for weak in (0, 1):
            ctx.set_option(recd.RECD_OPT_WEAK_HASH, weak)
            try:
                _, _, ik = gu.gpu_build(ctx, batch)
            finally:
                ctx.set_option(recd.RECD_OPT_WEAK_HASH, 0)
            _check(ik, batch)


def test_repeated_calls_and_deferred_counts(ctx):
    """The words the blocks exchange are left clear by every launch: calls in a row, of changing sizes,
    with the counts read afterwards from the build's own publication."""
    rng = np.random.default_rng(77)
    for it in range(12):
        F, B = int(rng.integers(1, 40)), int(rng.integers(1, 600))
        batch = synth.tiny_batch(rng, F, B, 4, 6)
        values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
        if values.numel() == 0:
            values = torch.zeros(1, dtype=torch.int64, device="cuda")[:0]
        ik = gu.DeviceIKJT(F, B, batch.N)
        ctx.build_ikjt(F, B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse, ik.feat_uoff)
        ik.U, ik.M = ctx.last_ikjt_counts()
        _check(ik, batch)


def test_run_index(ctx):
    for seed, (F, B) in enumerate(((1, 1), (4, 512), (7, 300), (130, 20))):
        w = synth.scaled(synth.WORKLOADS["cfg2"], F=F, B=B, rows=300)
        batch = synth.make_batch(w, seed)
        values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
        ik = gu.DeviceIKJT(F, B, batch.N)
        runs = torch.full((3 * (F * B + 2),), -7, dtype=torch.int64, device="cuda")
        ik.U, ik.M = ctx.build_ikjt_runs(F, B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse,
                                         ik.feat_uoff, runs, want_counts=True)
        uv, uo, inv, fu = _check(ik, batch)
        ref = orc.pack_run_index(*orc.run_index(F, B, inv, fu, uo), ik.U, ik.M)
        got = runs.cpu().numpy()
        assert np.array_equal(got[:len(ref)], ref)
        assert (got[len(ref):] == -7).all()
        assert ctx.last_ikjt_run_count() == int(ref[0])


def test_expired_wait_is_reported(ctx, recd):
    """With every wait between the blocks made to expire the build fails with an error, the kernel ends
    normally, and the next build is right again."""
    w = synth.scaled(synth.WORKLOADS["cfg1"], F=6, B=200)
    batch = synth.make_batch(w, 0)
    values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
    ik = gu.DeviceIKJT(w.F, w.B, batch.N)
    ctx.set_option(recd._OPT_INTERNAL_SMALL_PATH, 2)
    try:
        with pytest.raises(recd.RecdError) as e:
            ctx.build_ikjt(w.F, w.B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse, ik.feat_uoff,
                           want_counts=True)
        assert e.value.status == recd.RECD_EHIP
        ctx.build_ikjt(w.F, w.B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse, ik.feat_uoff)
        with pytest.raises(recd.RecdError):
            ctx.last_ikjt_counts()
    finally:
        ctx.set_option(recd._OPT_INTERNAL_SMALL_PATH, 1)
    _, _, ik = gu.gpu_build(ctx, batch)
    _check(ik, batch)


def test_one_pass_forward_every_run_sums(ctx, recd):
    """Small batches: no copy pass; a list that comes back later in the batch is summed again by the
    run that names it.  Same bits as the two calls and as the KJT lookup."""
    w = synth.scaled(synth.WORKLOADS["cfg2"], F=5, B=700, rows=4000, D=64)   # redraws: lists come back
    batch = synth.make_batch(w, 5)
    tabs = synth.make_tables(w)
    d_tabs = gu.tables_to_dev(tabs, "f32")
    F, B, D = w.F, w.B, w.D
    values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
    ik = gu.DeviceIKJT(F, B, batch.N)
    runs = torch.zeros(3 * (F * B + 2), dtype=torch.int64, device="cuda")
    ik.U, ik.M = ctx.build_ikjt_runs(F, B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse, ik.feat_uoff,
                                     runs, want_counts=True)
    n_runs = ctx.last_ikjt_run_count()
    assert n_runs > ik.U   # some list does come back
    outs = []
    for small in (1, 0):
        ctx.set_option(recd._OPT_INTERNAL_SMALL_PATH, small)
        pooled = torch.full((F * B, D), float("nan"), device="cuda")
        out = torch.full((F, B, D), float("nan"), device="cuda")
        ctx.pooled_lookup_expand(d_tabs, B, ik.u_values, runs, n_runs, pooled, out)
        outs.append((pooled, out))
    ctx.set_option(recd._OPT_INTERNAL_SMALL_PATH, 1)
    kjt = torch.full((F, B, D), float("nan"), device="cuda")
    ctx.kjt_pooled_lookup(d_tabs, B, values, offsets, kjt)
    torch.cuda.synchronize()
    bits = lambda t: t.view(torch.int32)
    assert torch.equal(bits(outs[0][0]), bits(outs[1][0]))
    assert torch.equal(bits(outs[0][1]), bits(outs[1][1]))
    assert torch.equal(bits(outs[0][1]), bits(kjt))
    uv, uo, inv, fu = orc.build_ikjt(F, B, batch.values, batch.offsets)
    ref = orc.expand_inverse(F, B, orc.pooled_lookup(tabs, "f32", uv, uo, fu), fu, inv)
    gu.assert_close_f32(gu.out_to_f64(outs[0][1]), ref, "one-pass forward, small batch")
