"""Randomised differential test: every entry point on randomly drawn shapes, dtypes, duplication
patterns and groupings, against the CPU oracle (same bars as the fixed-shape parity tests)."""
import os

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


def _bits(t):
    return t.view(torch.int32 if t.element_size() == 4 else torch.int16)


def _draw(seed):
    rng = np.random.default_rng(31000 + seed)
    F = int(rng.integers(1, 9))
    B = int(rng.integers(1, 700))
    dt = ["f32", "f32", "f16", "bf16"][int(rng.integers(4))]
    D = int(rng.choice([4, 8, 16, 24, 32, 64, 128, 192, 256] if dt == "f32" else [8, 16, 64, 128, 256, 512]))
    rows = int(rng.integers(3, 400))
    kind = int(rng.integers(3))
    if kind == 0:    # few distinct short lists: duplicates everywhere, adjacent or not
        batch = synth.tiny_batch(rng, F, B, int(rng.integers(2, min(rows, 6) + 1)), int(rng.integers(0, 7)))
    elif kind == 1:  # sessions, lists sliding inside a session
        w = synth.scaled(synth.WORKLOADS["cfg1"], F=F, B=B, S=float(rng.integers(1, 20)), rows=rows,
                         len_max=int(rng.integers(0, 90)), shift=float(rng.choice([0.0, 0.3])))
        batch = synth.make_batch(w, seed)
    else:            # sessions with long zipf lists and redraws
        w = synth.scaled(synth.WORKLOADS["cfg2"], F=F, B=B, S=float(rng.integers(1, 12)), rows=rows,
                         len_max=int(rng.integers(1, 200)), redraw=float(rng.choice([0.0, 0.2])))
        batch = synth.make_batch(w, seed)
    wt = synth.scaled(synth.WORKLOADS["cfg1"], F=F, B=B, rows=rows, D=D, table_dtype=dt)
    tabs = synth.make_tables(wt, seed=seed)
    cuts = sorted(set(rng.integers(1, F + 1, size=int(rng.integers(0, 3))).tolist()) | {F})
    return rng, F, B, D, dt, rows, batch, tabs, [0] + cuts


# RECD_RANDOM_SEEDS=<n> draws more configurations for a longer run
@pytest.mark.parametrize("seed", range(int(os.environ.get("RECD_RANDOM_SEEDS", "24"))))
def test_random_configuration(ctx, recd, seed):
    rng, F, B, D, dt, rows, batch, tabs, groups = _draw(seed)
    N = batch.N
    d_tabs = gu.tables_to_dev(tabs, dt)
    odt = gu.TORCH_DT[dt] if rng.random() < 0.5 else torch.float32
    close = gu.assert_close_f32 if odt == torch.float32 else gu.assert_close_16
    lo_kjt = np.arange(F + 1, dtype=np.int64) * B

    # builder, pooled lookups in a random mode, expand
    values, offsets, ik = gu.gpu_build(ctx, batch)
    uv, uo, inv, fu = orc.build_ikjt(F, B, batch.values, batch.offsets)
    for name, g, r in zip(("u_values", "u_offsets", "inverse", "feat_uoff"), ik.numpy(), (uv, uo, inv, fu)):
        assert np.array_equal(g, r), name
    mode = ["sum", "mean", "max"][int(rng.integers(3))]
    pooled = torch.full((F * B, D), float("nan"), dtype=odt, device="cuda")
    out = torch.full((F, B, D), float("nan"), dtype=odt, device="cuda")
    kjt = torch.full((F, B, D), float("nan"), dtype=odt, device="cuda")
    ctx.pooled_lookup_unique(d_tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, F * B, pooled, mode=mode)
    ctx.expand_inverse(F, B, pooled, ik.feat_uoff, ik.inverse, out)
    ctx.kjt_pooled_lookup(d_tabs, B, values, offsets, kjt, mode=mode)
    assert torch.equal(_bits(out), _bits(kjt))
    close(gu.out_to_f64(pooled[:ik.U]), orc.pooled_lookup_mode(mode, tabs, dt, uv, uo, fu), f"{mode} pooled")
    close(gu.out_to_f64(kjt).reshape(F * B, D),
          orc.pooled_lookup_mode(mode, tabs, dt, batch.values, batch.offsets, lo_kjt), f"{mode} kjt")

    # sequence path
    emb = torch.full((max(ik.M, 1), D), float("nan"), dtype=odt, device="cuda")
    seq = torch.full((max(N, 1), D), float("nan"), dtype=odt, device="cuda")[:N]
    kseq = torch.full((max(N, 1), D), float("nan"), dtype=odt, device="cuda")[:N]
    ctx.sequence_lookup_unique(d_tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, ik.U, emb)
    ctx.jagged_expand_inverse(F, B, emb, ik.u_offsets, ik.feat_uoff, ik.inverse, offsets, seq)
    ctx.kjt_sequence_lookup(d_tabs, B, values, offsets, kseq)
    assert torch.equal(_bits(seq), _bits(kseq))
    assert np.array_equal(gu.out_to_f64(kseq), orc.sequence_lookup(tabs, dt, batch.values, batch.offsets, lo_kjt))

    # grouped and partial builders
    gik_u = torch.full((max(N, 1),), -7, dtype=torch.int64, device="cuda")
    gik_o = torch.full((F * B + 1,), -7, dtype=torch.int64, device="cuda")
    G = len(groups) - 1
    inv_g = torch.zeros(max(G * B, 1), dtype=torch.int32, device="cuda")
    g_uoff = torch.zeros(G + 1, dtype=torch.int64, device="cuda")
    f_uoff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    inv_f = torch.zeros(max(F * B, 1), dtype=torch.int32, device="cuda")
    cU, cM, cG = ctx.build_ikjt_grouped(F, B, groups, values, offsets, gik_u, gik_o, inv_g, g_uoff, f_uoff, inv_f,
                                        want_counts=True)
    r_uv, r_uo, r_inv, r_gu, r_fu = orc.build_ikjt_grouped(F, B, groups, batch.values, batch.offsets)
    assert (cU, cM, cG) == (int(r_fu[-1]), len(r_uv), int(r_gu[-1]))
    assert np.array_equal(gik_u[:cM].cpu().numpy(), r_uv) and np.array_equal(gik_o[:cU + 1].cpu().numpy(), r_uo)
    assert np.array_equal(inv_g[:G * B].cpu().numpy(), r_inv)
    assert np.array_equal(g_uoff.cpu().numpy(), r_gu) and np.array_equal(f_uoff.cpu().numpy(), r_fu)
    p_values = torch.full((max(N, 1),), -7, dtype=torch.int64, device="cuda")
    ws = torch.zeros(max(F * B, 1), dtype=torch.int64, device="cuda")
    wl = torch.zeros(max(F * B, 1), dtype=torch.int64, device="cuda")
    p_inv = torch.zeros(max(F * B, 1), dtype=torch.int32, device="cuda")
    p_fu = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    p_fp = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    pU, pP, pM = ctx.build_partial_ikjt(F, B, values, offsets, p_values, ws, wl, p_inv, p_fu, p_fp, None,
                                        want_counts=True)
    o_pv, o_ws, o_wl, o_inv, o_fu, o_fp = orc.build_partial_ikjt(F, B, batch.values, batch.offsets)
    assert (pU, pP) == (len(o_ws), len(o_pv))
    assert np.array_equal(p_values[:pP].cpu().numpy(), o_pv) and np.array_equal(ws[:pU].cpu().numpy(), o_ws)
    assert np.array_equal(wl[:pU].cpu().numpy(), o_wl) and np.array_equal(p_fp.cpu().numpy(), o_fp)
    pooled_p = torch.full((F * B, D), float("nan"), dtype=odt, device="cuda")
    pooled_s = torch.full((F * B, D), float("nan"), dtype=odt, device="cuda")
    ctx.pooled_lookup_partial(d_tabs, p_values, ws, wl, p_fu, F * B, pooled_p)
    ctx.pooled_lookup_unique(d_tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, F * B, pooled_s)
    assert torch.equal(_bits(pooled_p[:pU]), _bits(pooled_s[:ik.U]))

    # per-id weights: builder, both lookups, backward
    weights = synth.make_weights(batch, seed, perturb=float(rng.choice([0.0, 0.3])))
    d_w = gu.to_dev(weights) if N else torch.zeros(1, device="cuda")[:0]
    wik = gu.DeviceIKJT(F, B, N)
    u_w = torch.full((max(N, 1),), float("nan"), device="cuda")
    wik.U, wik.M = ctx.build_ikjt_weighted(F, B, values, d_w, offsets, wik.u_values, u_w, wik.u_offsets,
                                           wik.inverse, wik.feat_uoff, want_counts=True)
    w_uv, w_uw, w_uo, w_inv, w_fu = orc.build_ikjt_weighted(F, B, batch.values, weights, batch.offsets)
    for name, g, r in zip(("u_values", "u_offsets", "inverse", "feat_uoff"), wik.numpy(), (w_uv, w_uo, w_inv, w_fu)):
        assert np.array_equal(g, r), "weighted " + name
    assert np.array_equal(u_w[:wik.M].cpu().numpy().view(np.uint32), w_uw.view(np.uint32))
    ctx.pooled_lookup_unique_weighted(d_tabs, wik.u_values, u_w, wik.u_offsets, wik.feat_uoff, F * B, pooled)
    ctx.expand_inverse(F, B, pooled, wik.feat_uoff, wik.inverse, out)
    ctx.kjt_pooled_lookup_weighted(d_tabs, B, values, d_w, offsets, kjt)
    assert torch.equal(_bits(out), _bits(kjt))
    close(gu.out_to_f64(kjt).reshape(F * B, D),
          orc.pooled_lookup_weighted(tabs, dt, batch.values, weights, batch.offsets, lo_kjt), "weighted kjt")

    # backward of both paths (fp32 tables)
    if dt == "f32":
        gout = (rng.standard_normal((F, B, D), dtype=np.float32) * np.float32(0.01))
        touched = torch.full((max(ik.M, 1),), -1, dtype=torch.int64, device="cuda")
        feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
        grad_rows = torch.zeros(max(ik.M, 1), D, device="cuda")
        bmode = "mean" if rng.random() < 0.5 else "sum"
        R = ctx.backward_dedup(F, B, gu.to_dev(gout), ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets,
                               [rows] * F, ik.U, ik.M, touched, feat_roff, grad_rows, want_count=True, mode=bmode)
        tr, fr, gr = orc.backward_kjt(F, B, gout, batch.values, batch.offsets, mode=bmode)
        assert R == len(tr) and np.array_equal(touched[:R].cpu().numpy(), tr)
        gu.assert_close_f32(gu.out_to_f64(grad_rows[:R]), gr, f"row gradients ({bmode})")
        Rm = ctx.backward_dedup_max(F, B, gu.to_dev(gout), ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets,
                                    [rows] * F, ik.U, ik.M, d_tabs, touched, feat_roff, grad_rows, want_count=True)
        trm, frm, grm = orc.backward_kjt_max(F, B, gout, batch.values, batch.offsets, tabs)
        assert Rm == len(trm) and np.array_equal(touched[:Rm].cpu().numpy(), trm)
        gu.assert_close_f32(gu.out_to_f64(grad_rows[:Rm]), grm, "max-pooling row gradients")
        Rw = ctx.backward_dedup_weighted(F, B, gu.to_dev(gout), wik.inverse, wik.feat_uoff, wik.u_values, u_w,
                                         wik.u_offsets, [rows] * F, wik.U, wik.M, touched, feat_roff, grad_rows,
                                         want_count=True)
        trw, frw, grw = orc.backward_kjt_weighted(F, B, gout, batch.values, weights, batch.offsets)
        assert Rw == len(trw) and np.array_equal(touched[:Rw].cpu().numpy(), trw)
        gu.assert_close_f32(gu.out_to_f64(grad_rows[:Rw]), grw, "weighted row gradients")
        sg = (rng.standard_normal((max(N, 1), D), dtype=np.float32) * np.float32(0.01))[:N]
        grad_emb = torch.zeros(max(ik.M, 1), D, device="cuda")
        d_sg = gu.to_dev(sg) if N else torch.zeros(1, D, device="cuda")[:0]
        R2 = ctx.backward_sequence_dedup(F, B, d_sg, offsets, ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets,
                                         [rows] * F, ik.U, ik.M, grad_emb, touched, feat_roff, grad_rows,
                                         want_count=True)
        tr2, fr2, gr2 = orc.backward_sequence_kjt(F, B, sg, batch.values, batch.offsets)
        assert R2 == len(tr2) and np.array_equal(touched[:R2].cpu().numpy(), tr2)
        assert np.array_equal(feat_roff.cpu().numpy(), fr2)
        gu.assert_close_f32(gu.out_to_f64(grad_rows[:R2]), gr2, "row gradients of the sequence path")
