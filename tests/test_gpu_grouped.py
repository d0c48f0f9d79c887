"""GPU parity tests of grouped IKJTs (one shared inverse per feature group) against the CPU oracle:
integer outputs bit-exact; the lookups, the group-sum module and the backward pass on a grouped
IKJT within the float bars of the ungrouped path."""
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


class DeviceGroupedIKJT:
    def __init__(self, F, B, G, N):
        L = F * B
        self.F, self.B, self.G = F, B, G
        self.u_values = torch.full((max(N, 1),), -7, dtype=torch.int64, device="cuda")
        self.u_offsets = torch.full((L + 1,), -7, dtype=torch.int64, device="cuda")
        self.inverse_g = torch.full((max(G * B, 1),), -7, dtype=torch.int32, device="cuda")
        self.group_uoff = torch.full((G + 1,), -7, dtype=torch.int64, device="cuda")
        self.feat_uoff = torch.full((F + 1,), -7, dtype=torch.int64, device="cuda")
        self.inverse_f = torch.full((max(L, 1),), -7, dtype=torch.int32, device="cuda")
        self.U = self.M = self.UG = None


def gpu_build_grouped(ctx, batch, group_off):
    values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
    if values.numel() == 0:
        values = torch.zeros(1, dtype=torch.int64, device="cuda")[:0]
    ik = DeviceGroupedIKJT(batch.F, batch.B, len(group_off) - 1, batch.N)
    ik.U, ik.M, ik.UG = ctx.build_ikjt_grouped(batch.F, batch.B, group_off, values, offsets, ik.u_values,
                                               ik.u_offsets, ik.inverse_g, ik.group_uoff, ik.feat_uoff,
                                               ik.inverse_f, want_counts=True)
    return values, offsets, ik


def _per_feature_inverse(inv_g, group_off, B):
    sizes = np.diff(np.asarray(group_off))
    return np.concatenate([np.tile(inv_g[g * B:(g + 1) * B], int(n)) for g, n in enumerate(sizes)])


def _check_grouped(ik, batch, group_off):
    uv, uo, inv_g, gu_, fu = orc.build_ikjt_grouped(batch.F, batch.B, group_off, batch.values, batch.offsets)
    G, B = len(group_off) - 1, batch.B
    assert (ik.U, ik.M, ik.UG) == (int(fu[-1]), len(uv), int(gu_[-1]))
    assert np.array_equal(ik.u_values[:ik.M].cpu().numpy(), uv)
    assert np.array_equal(ik.u_offsets[:ik.U + 1].cpu().numpy(), uo)
    assert np.array_equal(ik.inverse_g[:G * B].cpu().numpy(), inv_g)
    assert np.array_equal(ik.group_uoff.cpu().numpy(), gu_)
    assert np.array_equal(ik.feat_uoff.cpu().numpy(), fu)
    assert np.array_equal(ik.inverse_f[:batch.F * B].cpu().numpy(), _per_feature_inverse(inv_g, group_off, B))
    assert (ik.u_values[ik.M:] == -7).all() and (ik.u_offsets[ik.U + 1:] == -7).all()
    return uv, uo, inv_g, gu_, fu


def _random_groups(rng, F):
    cuts = sorted(set(rng.integers(1, F + 1, size=int(rng.integers(0, 4))).tolist()) | {F})
    return [0] + cuts


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("weak", [0, 1])
def test_grouped_build_tiny_random(ctx, recd, seed, weak):
    rng = np.random.default_rng(8000 + seed)
    F, B = int(rng.integers(1, 7)), int(rng.integers(1, 300))
    batch = synth.tiny_batch(rng, F, B, int(rng.integers(2, 4)), int(rng.integers(0, 4)))
    group_off = _random_groups(rng, F)
    ctx.set_option(recd.RECD_OPT_WEAK_HASH, weak)
    try:
        _, _, ik = gpu_build_grouped(ctx, batch, group_off)
    finally:
        ctx.set_option(recd.RECD_OPT_WEAK_HASH, 0)
    _check_grouped(ik, batch, group_off)


def test_grouped_build_paper_example_and_special_cases(ctx):
    # Sec. 4.2: c and d as a group, rows 0 and 1 duplicates, common inverse [0, 0, 1]
    kjt = synth.batch_from_lists([[[7, 8], [7, 8], [10]], [[9], [9], [11]]])
    _, _, ik = gpu_build_grouped(ctx, kjt, [0, 2])
    assert ik.inverse_g[:3].tolist() == [0, 0, 1] and ik.feat_uoff.tolist() == [0, 2, 4]
    assert ik.u_values[:ik.M].tolist() == [7, 8, 10, 9, 11]
    _check_grouped(ik, kjt, [0, 2])
    # unsynchronised: x constant, y always new -> nothing is deduplicated, x stored once per slot
    kjt = synth.batch_from_lists([[[5, 6]] * 7, [[i] for i in range(7)]])
    _, _, ik = gpu_build_grouped(ctx, kjt, [0, 2])
    assert ik.inverse_g[:7].tolist() == list(range(7)) and ik.M == 21
    _check_grouped(ik, kjt, [0, 2])
    # all rows empty in all features
    kjt = synth.batch_from_lists([[[]] * 5, [[]] * 5, [[]] * 5])
    _, _, ik = gpu_build_grouped(ctx, kjt, [0, 1, 3])
    assert ik.M == 0 and ik.UG == 2 and ik.U == 3
    _check_grouped(ik, kjt, [0, 1, 3])


def test_grouped_singletons_equal_ungrouped(ctx):
    w = synth.scaled(synth.WORKLOADS["cfg2"], F=5, B=1500, rows=20_000)
    batch = synth.make_batch(w, 0)
    _, _, ik = gpu_build_grouped(ctx, batch, list(range(6)))
    _, _, ref = gu.gpu_build(ctx, batch)
    assert (ik.U, ik.M) == (ref.U, ref.M) and ik.UG == ref.U
    assert torch.equal(ik.u_values[:ik.M], ref.u_values[:ref.M])
    assert torch.equal(ik.u_offsets[:ik.U + 1], ref.u_offsets[:ref.U + 1])
    assert torch.equal(ik.inverse_g[:5 * 1500], ref.inverse[:5 * 1500])
    assert torch.equal(ik.feat_uoff, ref.feat_uoff) and torch.equal(ik.group_uoff, ref.feat_uoff)


def test_grouped_empty_sizes_and_errors(ctx, recd):
    kjt = synth.batch_from_lists([[], []])  # F = 2, B = 0
    _, _, ik = gpu_build_grouped(ctx, kjt, [0, 2])
    assert (ik.U, ik.M, ik.UG) == (0, 0, 0) and ik.feat_uoff.tolist() == [0, 0, 0]
    assert ik.group_uoff.tolist() == [0, 0]
    kjt = synth.batch_from_lists([[[1]], [[2]]])
    for bad in ([0, 1], [1, 2], [0, 1, 1, 2], [0, 2, 1, 2]):
        with pytest.raises(recd.RecdError) as e:
            gpu_build_grouped(ctx, kjt, bad)
        assert e.value.status == recd.RECD_EINVAL


@pytest.mark.parametrize("name,F,B,groups", [("cfg2", 8, 2048, [0, 3, 4, 8]), ("cfg4", 6, 1000, [0, 6]),
                                             ("cfg1", 131, 67, [0, 1, 64, 130, 131])])
def test_grouped_forward_backward(ctx, name, F, B, groups):
    """Everything downstream runs unchanged on a grouped IKJT: the pooled and the unpooled lookups, both
    expands (with the per-feature copy of the shared inverse), the group-sum module expanded once per
    group, and the backward pass."""
    w = synth.scaled(synth.WORKLOADS[name], F=F, B=B, rows=3000, D=32)
    batch = synth.make_batch(w, 0)
    tabs = synth.make_tables(w)
    d_tabs = gu.tables_to_dev(tabs, "f32")
    values, offsets, ik = gpu_build_grouped(ctx, batch, groups)
    uv, uo, inv_g, gu_, fu = _check_grouped(ik, batch, groups)
    G, D, N = len(groups) - 1, w.D, batch.N
    pooled = torch.full((F * B, D), float("nan"), device="cuda")
    ctx.pooled_lookup_unique(d_tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, F * B, pooled)
    out = torch.zeros(F, B, D, device="cuda")
    ctx.expand_inverse(F, B, pooled, ik.feat_uoff, ik.inverse_f, out)
    kjt = torch.zeros(F, B, D, device="cuda")
    ctx.kjt_pooled_lookup(d_tabs, B, values, offsets, kjt)
    assert torch.equal(out, kjt)
    ref_pooled = orc.pooled_lookup(tabs, "f32", uv, uo, fu)
    gu.assert_close_f32(gu.out_to_f64(pooled[:ik.U]), ref_pooled, "pooled on grouped IKJT")
    # deduplicated compute on the group, expanded once through the shared inverse
    comb = torch.full((G * B, D), float("nan"), device="cuda")
    ctx.group_sum_unique(F, groups, pooled, ik.feat_uoff, ik.group_uoff, comb)
    gout = torch.zeros(G, B, D, device="cuda")
    ctx.expand_inverse(G, B, comb, ik.group_uoff, ik.inverse_g, gout)
    ref_comb = orc.group_sum(groups, ref_pooled, fu, gu_)
    gu.assert_close_f32(gu.out_to_f64(comb[:ik.UG]), ref_comb, "group sum")
    assert torch.isnan(comb[ik.UG:]).all()
    gu.assert_close_f32(gu.out_to_f64(gout), orc.expand_inverse(G, B, ref_comb, gu_, inv_g), "group expand")
    full = orc.kjt_pooled_lookup(tabs, "f32", B, batch.values, batch.offsets)
    ref_g = np.stack([full[groups[g]:groups[g + 1]].sum(axis=0) for g in range(G)])
    gu.assert_close_f32(gu.out_to_f64(gout), ref_g, "group sum vs per-feature KJT lookups")
    # sequence path
    emb = torch.zeros(max(ik.M, 1), D, device="cuda")
    seq = torch.zeros(max(N, 1), D, device="cuda")[:N]
    kseq = torch.zeros(max(N, 1), D, device="cuda")[:N]
    ctx.sequence_lookup_unique(d_tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, ik.U, emb)
    ctx.jagged_expand_inverse(F, B, emb, ik.u_offsets, ik.feat_uoff, ik.inverse_f, offsets, seq)
    ctx.kjt_sequence_lookup(d_tabs, B, values, offsets, kseq)
    assert torch.equal(seq, kseq)
    # backward: the gradient of the table rows is that of the non-deduplicated definition
    grad_out = synth.make_grad_out(w, 0)
    touched = torch.zeros(max(ik.M, 1), dtype=torch.int64, device="cuda")
    feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    grad_rows = torch.zeros(max(ik.M, 1), D, device="cuda")
    R = ctx.backward_dedup(F, B, gu.to_dev(grad_out), ik.inverse_f, ik.feat_uoff, ik.u_values, ik.u_offsets,
                           [w.rows] * F, ik.U, ik.M, touched, feat_roff, grad_rows, want_count=True)
    tr, fr, gr = orc.backward_kjt(F, B, grad_out, batch.values, batch.offsets)
    assert R == len(tr) and np.array_equal(touched[:R].cpu().numpy(), tr)
    assert np.array_equal(feat_roff.cpu().numpy(), fr)
    gu.assert_close_f32(gu.out_to_f64(grad_rows[:R]), gr, "row gradients on a grouped IKJT")
