"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (default
context options, U and M handed from the builder to the later calls).

Integer outputs (unique lists, offsets, inverse, touched rows) are compared with the oracle in
full.  Floating-point outputs are compared on sampled features: features are independent, so the
oracle runs on one feature's slice of the batch with that feature's table copied to the host.
Tables are drawn on the device with torch's seeded generator (input generation only)."""
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


def _device_tables(w, dtype):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 1000 * w.index + 777)
    tabs = []
    for _ in range(w.F):
        t = torch.empty(w.rows, w.D, dtype=torch.float32, device="cuda")
        t.normal_(0.0, 0.01, generator=gen)
        tabs.append(t if dtype == torch.float32 else t.to(dtype))
    return tabs


def _host_table(t, table_dtype):
    if table_dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _feature_slice(batch, f):
    B = batch.B
    lo, hi = int(batch.offsets[f * B]), int(batch.offsets[(f + 1) * B])
    return batch.values[lo:hi], batch.offsets[f * B:(f + 1) * B + 1] - lo


# eight features, one for each of the eight block queues (feature mod 8) of the lookup kernels
SPREAD_64 = (0, 9, 18, 27, 36, 45, 54, 63)


def _run_forward(recd, w, batch_index, sample_features):
    batch = synth.make_batch(w, batch_index)
    F, B, D = w.F, w.B, w.D
    tdt = gu.TORCH_DT[w.table_dtype]
    tabs = _device_tables(w, tdt)
    ctx = recd.Context(0)
    values, offsets, ik = gu.gpu_build(ctx, batch)
    pooled = torch.zeros(ik.U, D, dtype=tdt, device="cuda")
    out = torch.zeros(F, B, D, dtype=tdt, device="cuda")
    kjt = torch.zeros(F, B, D, dtype=tdt, device="cuda")
    ctx.pooled_lookup_unique(tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, ik.U, pooled)
    ctx.expand_inverse(F, B, pooled, ik.feat_uoff, ik.inverse, out)
    ctx.kjt_pooled_lookup(tabs, B, values, offsets, kjt)
    torch.cuda.synchronize()

    # integers: everything, exactly
    ref = orc.build_ikjt(F, B, batch.values, batch.offsets)
    got = ik.numpy()
    for name, g, r in zip(("u_values", "u_offsets", "inverse", "feat_uoff"), got, ref):
        assert np.array_equal(g, r), name
    uv, uo, inv, fu = ref
    # properties that hold at any size
    assert torch.equal(out.view(torch.int32 if tdt == torch.float32 else torch.int16),
                       kjt.view(torch.int32 if tdt == torch.float32 else torch.int16))
    idx = torch.from_numpy(fu[:-1]).cuda().repeat_interleave(B) + ik.inverse.long()
    assert torch.equal(out.view(F * B, D), pooled[idx])
    # the one-pass call on the builder's run index: the same bits in pooled and out
    runs = torch.zeros(3 * (F * B + 2), dtype=torch.int64, device="cuda")
    ik2 = gu.DeviceIKJT(F, B, batch.N)
    ctx.build_ikjt_runs(F, B, values, offsets, ik2.u_values, ik2.u_offsets, ik2.inverse, ik2.feat_uoff, runs)
    n_runs = ctx.last_ikjt_run_count()
    assert torch.equal(ik2.inverse, ik.inverse) and torch.equal(ik2.u_values[:ik.M], ik.u_values[:ik.M])
    ref_runs = orc.pack_run_index(*orc.run_index(F, B, inv, fu, uo), ik.U, ik.M)
    assert n_runs == int(ref_runs[0]) and np.array_equal(runs[:len(ref_runs)].cpu().numpy(), ref_runs)
    pooled2, out2 = torch.zeros_like(pooled), torch.zeros_like(out)
    ctx.pooled_lookup_expand(tabs, B, ik2.u_values, runs, n_runs, pooled2, out2)
    bits = torch.int32 if tdt == torch.float32 else torch.int16
    assert torch.equal(out2.view(bits), out.view(bits)) and torch.equal(pooled2.view(bits), pooled.view(bits))
    del pooled2, out2, runs

    close = gu.assert_close_f32 if w.table_dtype == "f32" else gu.assert_close_16
    for f in sample_features:
        v_f, o_f = _feature_slice(batch, f)
        host = _host_table(tabs[f], w.table_dtype)
        ref_kjt = orc.kjt_pooled_lookup([host], w.table_dtype, B, v_f, o_f)[0]
        close(gu.out_to_f64(kjt[f]), ref_kjt, f"kjt lookup feature {f}")
        close(gu.out_to_f64(out[f]), ref_kjt, f"expanded feature {f}")
        uv_f, uo_f, inv_f, fu_f = orc.build_ikjt(1, B, v_f, o_f)
        ref_pooled = orc.pooled_lookup([host], w.table_dtype, uv_f, uo_f, fu_f)
        close(gu.out_to_f64(pooled[fu[f]:fu[f + 1]]), ref_pooled, f"pooled feature {f}")
    ctx.close()
    return batch, ik


def test_cfg2_full(recd):
    _run_forward(recd, synth.WORKLOADS["cfg2"], 0, sample_features=(0, 1, 2, 3, 12, 13, 14, 15))


def test_cfg3_full_fp16(recd):
    _run_forward(recd, synth.WORKLOADS["cfg3"], 0, sample_features=SPREAD_64)


def test_cfg4_sweep_member_full(recd):
    _run_forward(recd, synth.sweep_workload(8), 0, sample_features=(0, 9, 18, 27, 4, 13, 22, 31))


def test_cfg5_training_step_full(recd):
    w = synth.WORKLOADS["cfg5"]
    F, B, D = w.F, w.B, w.D
    batch = synth.make_batch(w, 1)
    tabs = _device_tables(w, torch.float32)
    sample = SPREAD_64
    before = {f: tabs[f].cpu().numpy() for f in sample}
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    grad_out = torch.empty(F, B, D, dtype=torch.float32, device="cuda")
    grad_out.normal_(0.0, 0.01, generator=g)
    state = [torch.zeros(w.rows, device="cuda") for _ in range(F)]
    ctx = recd.Context(0)
    values, offsets, ik = gu.gpu_build(ctx, batch)
    ref = orc.build_ikjt(F, B, batch.values, batch.offsets)
    for name, got, r in zip(("u_values", "u_offsets", "inverse", "feat_uoff"), ik.numpy(), ref):
        assert np.array_equal(got, r), name
    uv, uo, inv, fu = ref
    touched = torch.full((ik.M,), -1, dtype=torch.int64, device="cuda")
    feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    grad_rows = torch.zeros(ik.M, D, device="cuda")
    R = ctx.backward_dedup(F, B, grad_out, ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets,
                           [w.rows] * F, ik.U, ik.M, touched, feat_roff, grad_rows, tables=tabs,
                           adagrad_state=state, lr=0.01, eps=1e-8, want_count=True)
    torch.cuda.synchronize()
    fr = feat_roff.cpu().numpy()
    tr = touched[:R].cpu().numpy()
    assert fr[0] == 0 and fr[-1] == R
    # touched rows of every feature: exactly the distinct ids, ascending
    for f in range(F):
        lo, hi = batch.offsets[f * B], batch.offsets[(f + 1) * B]
        assert np.array_equal(tr[fr[f]:fr[f + 1]], np.unique(batch.values[lo:hi])), f
    for f in sample:
        v_f, o_f = _feature_slice(batch, f)
        uv_f, uo_f, inv_f, fu_f = orc.build_ikjt(1, B, v_f, o_f)
        gout_f = grad_out[f:f + 1].cpu().numpy()
        tr_f, _, gr_f = orc.backward_dedup(1, B, gout_f, inv_f, fu_f, uv_f, uo_f)
        assert np.array_equal(tr_f, tr[fr[f]:fr[f + 1]])
        gu.assert_close_f32(grad_rows[fr[f]:fr[f + 1]].double().cpu().numpy(), gr_f, f"grad rows {f}")
        w_new, m_new = orc.rowwise_adagrad(gr_f, before[f][tr_f].astype(np.float64),
                                           np.zeros(len(tr_f)), 0.01, 1e-8)
        after = tabs[f].cpu().numpy()
        gu.assert_close_f32(after[tr_f].astype(np.float64), w_new, f"updated rows {f}")
        gu.assert_close_f32(state[f].cpu().numpy()[tr_f].astype(np.float64), m_new, f"state {f}")
        untouched = np.ones(w.rows, bool)
        untouched[tr_f] = False
        assert np.array_equal(after[untouched], before[f][untouched])
    ctx.close()


def test_cfg5_bench_step_full(recd):
    """Two consecutive steps exactly as bench.py issues them: build without a host count, lookup
    sized by the previous step's U, expand, U and M read back while those run, planned backward
    with the fused update and no stored gradient rows; the second step in bench.py's other form
    (run index, one-pass lookup + expand, plan from the runs).  Integer outputs in full; the expanded rows
    and the tables after both steps on sampled features, where the oracle runs both steps too (the
    second step looks up the rows the first one updated)."""
    w = synth.WORKLOADS["cfg5"]
    F, B, D = w.F, w.B, w.D
    batches = [synth.make_batch(w, i) for i in (1, 2)]
    tabs = _device_tables(w, torch.float32)
    sample = SPREAD_64
    host_tab = {f: tabs[f].cpu().numpy().copy() for f in sample}   # the oracle's own fp32 copy, updated by the oracle
    host_state = {f: np.zeros(w.rows) for f in sample}
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    grad_out = torch.empty(F, B, D, dtype=torch.float32, device="cuda")
    grad_out.normal_(0.0, 0.01, generator=g)
    gout_host = {f: grad_out[f:f + 1].cpu().numpy() for f in sample}
    state = [torch.zeros(w.rows, device="cuda") for _ in range(F)]
    Nmax = max(b.N for b in batches)
    ctx = recd.Context(0, workspace_hint_bytes=recd.workspace_bytes(F, B, Nmax, D))
    pooled = torch.zeros(F * B, D, device="cuda")
    out = torch.zeros(F, B, D, device="cuda")
    touched = torch.zeros(Nmax, dtype=torch.int64, device="cuda")
    feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    u_hint = F * B
    runs = torch.zeros(3 * (F * B + 2), dtype=torch.int64, device="cuda")
    for step, batch in enumerate(batches):
        values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
        ik = gu.DeviceIKJT(F, B, batch.N)
        if step == 0:   # the default step of bench.py
            ctx.build_ikjt(F, B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse, ik.feat_uoff)
            ctx.pooled_lookup_unique(tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, u_hint, pooled)
            ctx.expand_inverse(F, B, pooled, ik.feat_uoff, ik.inverse, out)
            U, M = ctx.last_ikjt_counts()
            ctx.backward_plan(F, B, D, ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets, [w.rows] * F, U, M,
                              touched, feat_roff)
        else:           # --one-pass-forward --plan-from-runs
            ctx.build_ikjt_runs(F, B, values, offsets, ik.u_values, ik.u_offsets, ik.inverse, ik.feat_uoff, runs)
            ctx.pooled_lookup_expand(tabs, B, ik.u_values, runs, u_hint + u_hint // 16, pooled, out)
            U, M = ctx.last_ikjt_counts()
            ctx.backward_plan_runs(F, B, D, ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets, [w.rows] * F, U, M,
                                   runs, ctx.last_ikjt_run_count(), touched, feat_roff)
        u_hint = max(U, 1)
        ctx.backward_apply(grad_out, None, tables=tabs, adagrad_state=state, lr=0.01, eps=1e-8)
        torch.cuda.synchronize()
        ik.U, ik.M = U, M
        ref = orc.build_ikjt(F, B, batch.values, batch.offsets)
        assert (U, M) == (int(ref[3][-1]), len(ref[0]))
        for name, got, r in zip(("u_values", "u_offsets", "inverse", "feat_uoff"), ik.numpy(), ref):
            assert np.array_equal(got, r), (step, name)
        fr = feat_roff.cpu().numpy()
        tr = touched[:fr[-1]].cpu().numpy()
        for f in sample:
            v_f, o_f = _feature_slice(batch, f)
            uv_f, uo_f, inv_f, fu_f = orc.build_ikjt(1, B, v_f, o_f)
            # forward of this step on the table as the previous step left it
            ref_out = orc.expand_inverse(1, B, orc.pooled_lookup([host_tab[f]], "f32", uv_f, uo_f, fu_f), fu_f, inv_f)
            gu.assert_close_f32(gu.out_to_f64(out[f:f + 1]), ref_out, f"step {step}: expanded feature {f}")
            tr_f, _, gr_f = orc.backward_dedup(1, B, gout_host[f], inv_f, fu_f, uv_f, uo_f)
            assert np.array_equal(tr_f, tr[fr[f]:fr[f + 1]]), (step, f)
            w_new, m_new = orc.rowwise_adagrad(gr_f, host_tab[f][tr_f].astype(np.float64), host_state[f][tr_f],
                                               0.01, 1e-8)
            host_tab[f][tr_f] = w_new.astype(np.float32)   # stored as fp32, as the tables are
            host_state[f][tr_f] = m_new
            gu.assert_close_f32(tabs[f].cpu().numpy().astype(np.float64), host_tab[f].astype(np.float64),
                                f"step {step}: table {f}")
            gu.assert_close_f32(state[f].cpu().numpy().astype(np.float64), host_state[f], f"step {step}: state {f}")
    ctx.close()


def _run_sequence(recd, w, batch_index, sample_features):
    """Unpooled path at full size: every output row against the non-deduplicated lookup (bit for
    bit), sampled features against the oracle (exact: the path only copies)."""
    batch = synth.make_batch(w, batch_index)
    F, B, D, N = w.F, w.B, w.D, batch.N
    tdt = gu.TORCH_DT[w.table_dtype]
    tabs = _device_tables(w, tdt)
    ctx = recd.Context(0)
    values, offsets, ik = gu.gpu_build(ctx, batch)
    emb = torch.zeros(ik.M, D, dtype=tdt, device="cuda")
    out = torch.zeros(N, D, dtype=tdt, device="cuda")
    kjt = torch.zeros(N, D, dtype=tdt, device="cuda")
    ctx.sequence_lookup_unique(tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, ik.U, emb)
    ctx.jagged_expand_inverse(F, B, emb, ik.u_offsets, ik.feat_uoff, ik.inverse, offsets, out)
    ctx.kjt_sequence_lookup(tabs, B, values, offsets, kjt)
    torch.cuda.synchronize()
    bits = torch.int32 if tdt == torch.float32 else torch.int16
    assert torch.equal(out.view(bits), kjt.view(bits))
    del kjt
    uv, uo, inv, fu = orc.build_ikjt(F, B, batch.values, batch.offsets)
    assert ik.M == len(uv)
    for f in sample_features:
        host = _host_table(tabs[f], w.table_dtype)
        v_f, o_f = _feature_slice(batch, f)
        lo, hi = int(batch.offsets[f * B]), int(batch.offsets[(f + 1) * B])
        ref = orc.sequence_lookup([host], w.table_dtype, v_f, o_f, np.array([0, B], dtype=np.int64))
        assert np.array_equal(gu.out_to_f64(out[lo:hi]), ref), f"expanded activations of feature {f}"
        ulo, uhi = int(uo[fu[f]]), int(uo[fu[f + 1]])
        uo_f = uo[fu[f]:fu[f + 1] + 1] - ulo
        ref_emb = orc.sequence_lookup([host], w.table_dtype, uv[ulo:uhi], uo_f,
                                      np.array([0, fu[f + 1] - fu[f]], dtype=np.int64))
        assert np.array_equal(gu.out_to_f64(emb[ulo:uhi]), ref_emb), f"unique activations of feature {f}"
        ref_out = orc.jagged_expand(1, B, ref_emb, uo_f, np.array([0, fu[f + 1] - fu[f]], dtype=np.int64),
                                    inv[f * B:(f + 1) * B], o_f)
        assert np.array_equal(ref_out, ref)
    ctx.close()


def test_cfg2_sequence_full(recd):
    _run_sequence(recd, synth.WORKLOADS["cfg2"], 0, sample_features=(0, 9, 15))


def test_cfg3_sequence_full_fp16(recd):
    _run_sequence(recd, synth.WORKLOADS["cfg3"], 0, sample_features=(5, 63))


def test_cfg5_sequence_full(recd):
    _run_sequence(recd, synth.WORKLOADS["cfg5"], 2, sample_features=(0, 33, 63))


def test_cfg5_grouped_full(recd):
    """Configuration 5 with its 64 features in 8 groups of 8: integers against the oracle in full, the
    group-sum module expanded through the shared inverse against the oracle on sampled groups."""
    w = synth.WORKLOADS["cfg5"]
    F, B, D = w.F, w.B, w.D
    groups = list(range(0, F + 1, 8))
    G = len(groups) - 1
    batch = synth.make_batch(w, 3)
    tabs = _device_tables(w, torch.float32)
    ctx = recd.Context(0)
    values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
    u_values = torch.zeros(batch.N, dtype=torch.int64, device="cuda")
    u_offsets = torch.zeros(F * B + 1, dtype=torch.int64, device="cuda")
    inverse_g = torch.zeros(G * B, dtype=torch.int32, device="cuda")
    group_uoff = torch.zeros(G + 1, dtype=torch.int64, device="cuda")
    feat_uoff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    inverse_f = torch.zeros(F * B, dtype=torch.int32, device="cuda")
    U, M, UG = ctx.build_ikjt_grouped(F, B, groups, values, offsets, u_values, u_offsets, inverse_g,
                                      group_uoff, feat_uoff, inverse_f, want_counts=True)
    uv, uo, inv_g, gu_, fu = orc.build_ikjt_grouped(F, B, groups, batch.values, batch.offsets)
    assert (U, M, UG) == (int(fu[-1]), len(uv), int(gu_[-1]))
    assert np.array_equal(u_values[:M].cpu().numpy(), uv)
    assert np.array_equal(u_offsets[:U + 1].cpu().numpy(), uo)
    assert np.array_equal(inverse_g.cpu().numpy(), inv_g)
    assert np.array_equal(group_uoff.cpu().numpy(), gu_) and np.array_equal(feat_uoff.cpu().numpy(), fu)
    assert torch.equal(inverse_f.view(G, 8, B), inverse_g.view(G, 1, B).expand(G, 8, B))
    pooled = torch.zeros(U, D, device="cuda")
    ctx.pooled_lookup_unique(tabs, u_values, u_offsets, feat_uoff, U, pooled)
    out = torch.zeros(F, B, D, device="cuda")
    kjt = torch.zeros(F, B, D, device="cuda")
    ctx.expand_inverse(F, B, pooled, feat_uoff, inverse_f, out)
    ctx.kjt_pooled_lookup(tabs, B, values, offsets, kjt)
    assert torch.equal(out, kjt)
    comb = torch.zeros(UG, D, device="cuda")
    ctx.group_sum_unique(F, groups, pooled, feat_uoff, group_uoff, comb)
    gout = torch.zeros(G, B, D, device="cuda")
    ctx.expand_inverse(G, B, comb, group_uoff, inverse_g, gout)
    torch.cuda.synchronize()
    for g in (0, 5):
        ref = np.zeros((B, D))
        for f in range(groups[g], groups[g + 1]):
            v_f, o_f = _feature_slice(batch, f)
            ref += orc.kjt_pooled_lookup([_host_table(tabs[f], "f32")], "f32", B, v_f, o_f)[0]
        gu.assert_close_f32(gu.out_to_f64(gout[g]), ref, f"group {g} sum")
    ctx.close()


def test_cfg5_partial_full(recd):
    """Configuration 5 with lists that slide within a session (a quarter of the samples shift by one
    id): every integer output of the partial builder against the oracle, the pooled lookup on the
    windows bit for bit against the lookup on the IKJT."""
    w = synth.scaled(synth.WORKLOADS["cfg5"], shift=0.25)
    F, B, D = w.F, w.B, w.D
    batch = synth.make_batch(w, 0)
    tabs = _device_tables(w, torch.float32)
    ctx = recd.Context(0)
    values, offsets = gu.to_dev(batch.values), gu.to_dev(batch.offsets)
    i64 = dict(dtype=torch.int64, device="cuda")
    p_values = torch.zeros(batch.N, **i64)
    win_start, win_len = torch.zeros(F * B, **i64), torch.zeros(F * B, **i64)
    inverse = torch.zeros(F * B, dtype=torch.int32, device="cuda")
    feat_uoff, feat_poff = torch.zeros(F + 1, **i64), torch.zeros(F + 1, **i64)
    row_window = torch.zeros(F * B, 2, **i64)
    U, P, M = ctx.build_partial_ikjt(F, B, values, offsets, p_values, win_start, win_len, inverse,
                                     feat_uoff, feat_poff, row_window, want_counts=True)
    pv, ws, wl, inv, fu, fp = orc.build_partial_ikjt(F, B, batch.values, batch.offsets)
    assert (U, P, M) == (len(ws), len(pv), int(wl.sum())) and P < M
    assert np.array_equal(p_values[:P].cpu().numpy(), pv)
    assert np.array_equal(win_start[:U].cpu().numpy(), ws) and np.array_equal(win_len[:U].cpu().numpy(), wl)
    assert np.array_equal(inverse.cpu().numpy(), inv)
    assert np.array_equal(feat_uoff.cpu().numpy(), fu) and np.array_equal(feat_poff.cpu().numpy(), fp)
    assert np.array_equal(row_window.cpu().numpy(), orc.partial_row_windows(F, B, ws, wl, inv, fu))
    # lossless: every row's window spells the row's list
    rw = row_window.cpu().numpy()
    lens = np.diff(batch.offsets)
    assert np.array_equal(rw[:, 1], lens)
    idx = np.repeat(rw[:, 0] - batch.offsets[:-1], lens) + np.arange(batch.N)
    assert np.array_equal(pv[idx], batch.values)
    pooled = torch.zeros(U, D, device="cuda")
    ctx.pooled_lookup_partial(tabs, p_values, win_start, win_len, feat_uoff, U, pooled)
    _, _, ik = gu.gpu_build(ctx, batch)
    ref = torch.zeros(ik.U, D, device="cuda")
    ctx.pooled_lookup_unique(tabs, ik.u_values, ik.u_offsets, ik.feat_uoff, ik.U, ref)
    assert U == ik.U and torch.equal(pooled, ref)
    ctx.close()


def test_cfg5_sequence_backward_full(recd):
    """Backward of the sequence path at configuration 5's size (35 M gradient rows): touched rows of
    every feature exactly, row gradients, the gradient of the unique activations and the Adagrad update
    of sampled features against the oracle."""
    w = synth.WORKLOADS["cfg5"]
    F, B, D = w.F, w.B, w.D
    batch = synth.make_batch(w, 1)
    N = batch.N
    tabs = _device_tables(w, torch.float32)
    sample = (7, 50)
    before = {f: tabs[f].cpu().numpy() for f in sample}
    g = torch.Generator(device="cuda")
    g.manual_seed(4242)
    grad_out = torch.empty(N, D, dtype=torch.float32, device="cuda")
    grad_out.normal_(0.0, 0.01, generator=g)
    state = [torch.zeros(w.rows, device="cuda") for _ in range(F)]
    ctx = recd.Context(0)
    values, offsets, ik = gu.gpu_build(ctx, batch)
    grad_emb = torch.zeros(ik.M, D, device="cuda")
    touched = torch.full((ik.M,), -1, dtype=torch.int64, device="cuda")
    feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    grad_rows = torch.zeros(ik.M, D, device="cuda")
    R = ctx.backward_sequence_dedup(F, B, grad_out, offsets, ik.inverse, ik.feat_uoff, ik.u_values,
                                    ik.u_offsets, [w.rows] * F, ik.U, ik.M, grad_emb, touched, feat_roff,
                                    grad_rows, tables=tabs, adagrad_state=state, lr=0.01, eps=1e-8,
                                    want_count=True)
    torch.cuda.synchronize()
    fr = feat_roff.cpu().numpy()
    tr = touched[:R].cpu().numpy()
    assert fr[0] == 0 and fr[-1] == R
    for f in range(F):
        lo, hi = batch.offsets[f * B], batch.offsets[(f + 1) * B]
        assert np.array_equal(tr[fr[f]:fr[f + 1]], np.unique(batch.values[lo:hi])), f
    uo = ik.u_offsets[:ik.U + 1].cpu().numpy()
    fu = ik.feat_uoff.cpu().numpy()
    for f in sample:
        v_f, o_f = _feature_slice(batch, f)
        lo, hi = int(batch.offsets[f * B]), int(batch.offsets[(f + 1) * B])
        gout_f = grad_out[lo:hi].cpu().numpy()
        tr_f, _, gr_f = orc.backward_sequence_kjt(1, B, gout_f, v_f, o_f)
        assert np.array_equal(tr_f, tr[fr[f]:fr[f + 1]])
        gu.assert_close_f32(grad_rows[fr[f]:fr[f + 1]].double().cpu().numpy(), gr_f, f"grad rows {f}")
        uv_f, uo_f, inv_f, fu_f = orc.build_ikjt(1, B, v_f, o_f)
        ref_emb = np.zeros((len(uv_f), D))
        for b in range(B):
            n = o_f[b + 1] - o_f[b]
            u = inv_f[b]
            ref_emb[uo_f[u]:uo_f[u] + n] += gout_f[o_f[b]:o_f[b] + n].astype(np.float64)
        ulo, uhi = int(uo[fu[f]]), int(uo[fu[f + 1]])
        gu.assert_close_f32(grad_emb[ulo:uhi].double().cpu().numpy(), ref_emb, f"grad_emb {f}")
        w_new, m_new = orc.rowwise_adagrad(gr_f, before[f][tr_f].astype(np.float64), np.zeros(len(tr_f)),
                                           0.01, 1e-8)
        after = tabs[f].cpu().numpy()
        gu.assert_close_f32(after[tr_f].astype(np.float64), w_new, f"updated rows {f}")
        untouched = np.ones(w.rows, bool)
        untouched[tr_f] = False
        assert np.array_equal(after[untouched], before[f][untouched])
    ctx.close()


def test_cfg5_weighted_full(recd):
    """Per-id weights at the benchmark size: the weighted builder in full, the weighted lookup on both
    paths bit for bit and on sampled features against the oracle, the weighted backward with the
    fused update on sampled features."""
    w = synth.WORKLOADS["cfg5"]
    F, B, D = w.F, w.B, w.D
    batch = synth.make_batch(w, 2)
    weights = synth.make_weights(batch, 2, perturb=0.05)
    tabs = _device_tables(w, torch.float32)
    sample = (3, 57)
    before = {f: tabs[f].cpu().numpy() for f in sample}
    ctx = recd.Context(0)
    values, offsets, d_w = gu.to_dev(batch.values), gu.to_dev(batch.offsets), gu.to_dev(weights)
    ik = gu.DeviceIKJT(F, B, batch.N)
    u_weights = torch.zeros(batch.N, device="cuda")
    ik.U, ik.M = ctx.build_ikjt_weighted(F, B, values, d_w, offsets, ik.u_values, u_weights, ik.u_offsets,
                                         ik.inverse, ik.feat_uoff, want_counts=True)
    uv, uw, uo, inv, fu = orc.build_ikjt_weighted(F, B, batch.values, weights, batch.offsets)
    for name, got, r in zip(("u_values", "u_offsets", "inverse", "feat_uoff"), ik.numpy(), (uv, uo, inv, fu)):
        assert np.array_equal(got, r), name
    assert np.array_equal(u_weights[:ik.M].cpu().numpy().view(np.uint32), uw.view(np.uint32))
    pooled = torch.zeros(ik.U, D, device="cuda")
    out = torch.zeros(F, B, D, device="cuda")
    kjt = torch.zeros(F, B, D, device="cuda")
    ctx.pooled_lookup_unique_weighted(tabs, ik.u_values, u_weights, ik.u_offsets, ik.feat_uoff, ik.U, pooled)
    ctx.expand_inverse(F, B, pooled, ik.feat_uoff, ik.inverse, out)
    ctx.kjt_pooled_lookup_weighted(tabs, B, values, d_w, offsets, kjt)
    assert torch.equal(out, kjt)
    g = torch.Generator(device="cuda")
    g.manual_seed(101)
    grad_out = torch.empty(F, B, D, dtype=torch.float32, device="cuda")
    grad_out.normal_(0.0, 0.01, generator=g)
    state = [torch.zeros(w.rows, device="cuda") for _ in range(F)]
    touched = torch.full((ik.M,), -1, dtype=torch.int64, device="cuda")
    feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    grad_rows = torch.zeros(ik.M, D, device="cuda")
    out_host = {f: gu.out_to_f64(out[f]) for f in sample}  # before the update changes the tables
    R = ctx.backward_dedup_weighted(F, B, grad_out, ik.inverse, ik.feat_uoff, ik.u_values, u_weights,
                                    ik.u_offsets, [w.rows] * F, ik.U, ik.M, touched, feat_roff, grad_rows,
                                    tables=tabs, adagrad_state=state, lr=0.01, eps=1e-8, want_count=True)
    fr = feat_roff.cpu().numpy()
    tr = touched[:R].cpu().numpy()
    for f in sample:
        v_f, o_f = _feature_slice(batch, f)
        lo, hi = int(batch.offsets[f * B]), int(batch.offsets[(f + 1) * B])
        ref = orc.pooled_lookup_weighted([before[f]], "f32", v_f, weights[lo:hi], o_f, np.array([0, B]))
        gu.assert_close_f32(out_host[f], ref, f"weighted lookup of feature {f}")
        tr_f, _, gr_f = orc.backward_kjt_weighted(1, B, grad_out[f:f + 1].cpu().numpy(), v_f, weights[lo:hi], o_f)
        assert np.array_equal(tr_f, tr[fr[f]:fr[f + 1]])
        gu.assert_close_f32(grad_rows[fr[f]:fr[f + 1]].double().cpu().numpy(), gr_f, f"grad rows {f}")
        w_new, m_new = orc.rowwise_adagrad(gr_f, before[f][tr_f].astype(np.float64), np.zeros(len(tr_f)),
                                           0.01, 1e-8)
        gu.assert_close_f32(tabs[f].cpu().numpy()[tr_f].astype(np.float64), w_new, f"updated rows {f}")
        gu.assert_close_f32(state[f].cpu().numpy()[tr_f].astype(np.float64), m_new, f"state {f}")
    ctx.close()


def test_cfg5_mean_backward_full(recd):
    w = synth.WORKLOADS["cfg5"]
    F, B, D = w.F, w.B, w.D
    batch = synth.make_batch(w, 3)
    ctx = recd.Context(0)
    values, offsets, ik = gu.gpu_build(ctx, batch)
    g = torch.Generator(device="cuda")
    g.manual_seed(102)
    grad_out = torch.empty(F, B, D, dtype=torch.float32, device="cuda")
    grad_out.normal_(0.0, 0.01, generator=g)
    touched = torch.full((ik.M,), -1, dtype=torch.int64, device="cuda")
    feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    grad_rows = torch.zeros(ik.M, D, device="cuda")
    R = ctx.backward_dedup(F, B, grad_out, ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets, [w.rows] * F,
                           ik.U, ik.M, touched, feat_roff, grad_rows, want_count=True, mode="mean")
    fr = feat_roff.cpu().numpy()
    tr = touched[:R].cpu().numpy()
    for f in (5, 62):
        v_f, o_f = _feature_slice(batch, f)
        tr_f, _, gr_f = orc.backward_kjt(1, B, grad_out[f:f + 1].cpu().numpy(), v_f, o_f, mode="mean")
        assert np.array_equal(tr_f, tr[fr[f]:fr[f + 1]])
        gu.assert_close_f32(grad_rows[fr[f]:fr[f + 1]].double().cpu().numpy(), gr_f, f"mean grad rows {f}")
    ctx.close()


def test_cfg5_max_backward_full(recd):
    w = synth.WORKLOADS["cfg5"]
    F, B, D = w.F, w.B, w.D
    batch = synth.make_batch(w, 1)
    tabs = _device_tables(w, torch.float32)
    ctx = recd.Context(0)
    values, offsets, ik = gu.gpu_build(ctx, batch)
    g = torch.Generator(device="cuda")
    g.manual_seed(103)
    grad_out = torch.empty(F, B, D, dtype=torch.float32, device="cuda")
    grad_out.normal_(0.0, 0.01, generator=g)
    touched = torch.full((ik.M,), -1, dtype=torch.int64, device="cuda")
    feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
    grad_rows = torch.zeros(ik.M, D, device="cuda")
    R = ctx.backward_dedup_max(F, B, grad_out, ik.inverse, ik.feat_uoff, ik.u_values, ik.u_offsets, [w.rows] * F,
                               ik.U, ik.M, tabs, touched, feat_roff, grad_rows, want_count=True)
    fr = feat_roff.cpu().numpy()
    tr = touched[:R].cpu().numpy()
    for f in (7, 33):
        v_f, o_f = _feature_slice(batch, f)
        tr_f, _, gr_f = orc.backward_kjt_max(1, B, grad_out[f:f + 1].cpu().numpy(), v_f, o_f, [tabs[f].cpu().numpy()])
        assert np.array_equal(tr_f, tr[fr[f]:fr[f + 1]])
        gu.assert_close_f32(grad_rows[fr[f]:fr[f + 1]].double().cpu().numpy(), gr_f, f"max grad rows {f}")
    ctx.close()


def test_more_than_2_31_ids(recd):
    """Positions beyond 2^31 in `values` and in `u_values` (the interface takes int64 positions; F*B and
    the ids themselves stay below 2^31): 54 lists of about 5e7 ids each, 2.7e9 ids in all, almost all
    lists distinct, a few repeated next to and far from their first occurrence.  Integer outputs against
    the oracle; the lookups against each other bit for bit and, for three lists, against an exact sum
    (table entries are -1, 0 or 1 and the partial sums stay far below 2^24, so fp32 adds exactly)."""
    F, B, D, rows = 2, 27, 4, 1_000_003
    rng = np.random.default_rng(20231)
    lens = rng.integers(49_000_000, 51_000_000, size=F * B)
    # which earlier row of the same feature a row repeats (-1: its own content)
    src = np.full(F * B, -1)
    for f in range(F):
        src[f * B + 5] = f * B + 4      # adjacent
        src[f * B + 17] = f * B + 2     # far apart
        src[f * B + 23] = f * B + 17    # a repeat of a repeat
    for l in range(F * B):
        if src[l] >= 0:
            lens[l] = lens[src[l]]
    offsets = np.zeros(F * B + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    N = int(offsets[-1])
    assert N > 2**31 + 2**27
    values = np.empty(N, dtype=np.int64)
    for l in range(F * B):
        a, b = offsets[l], offsets[l + 1]
        if src[l] >= 0:
            values[a:b] = values[offsets[src[l]]:offsets[src[l] + 1]]
        else:   # cheap, position-dependent, different for every list
            values[a:b] = (np.arange(b - a, dtype=np.int64) * (2 * l + 3) + 7 * l * l) % rows
    print(f"  {N} ids generated", flush=True)   # progress lines: the stages take tens of seconds each
    d_values, d_offsets = torch.from_numpy(values).cuda(), torch.from_numpy(offsets).cuda()
    ctx = recd.Context(0)
    u_values = torch.full((N,), -7, dtype=torch.int64, device="cuda")
    u_offsets = torch.full((F * B + 1,), -7, dtype=torch.int64, device="cuda")
    inverse = torch.full((F * B,), -7, dtype=torch.int32, device="cuda")
    feat_uoff = torch.full((F + 1,), -7, dtype=torch.int64, device="cuda")
    U, M = ctx.build_ikjt(F, B, d_values, d_offsets, u_values, u_offsets, inverse, feat_uoff, want_counts=True)
    assert U == F * (B - 3) and M > 2**31
    print(f"  built on the GPU: U={U} M={M}", flush=True)
    uv, uo, inv, fu = orc.build_ikjt(F, B, values, offsets)
    print("  built by the oracle", flush=True)
    assert (U, M) == (int(fu[-1]), len(uv))
    assert np.array_equal(u_offsets[:U + 1].cpu().numpy(), uo)
    assert np.array_equal(inverse.cpu().numpy(), inv)
    assert np.array_equal(feat_uoff.cpu().numpy(), fu)
    got = u_values[:M].cpu().numpy()
    assert np.array_equal(got, uv)
    del got, uv
    print("  unique lists compared", flush=True)
    # lookups: tables of -1 / 0 / 1
    tabs = [((np.arange(rows * D, dtype=np.int64).reshape(rows, D) * (f + 2) // 3) % 3 - 1).astype(np.float32)
            for f in range(F)]
    d_tabs = [torch.from_numpy(t).cuda() for t in tabs]
    pooled = torch.full((F * B, D), float("nan"), device="cuda")
    out = torch.full((F, B, D), float("nan"), device="cuda")
    kjt = torch.full((F, B, D), float("nan"), device="cuda")
    ctx.pooled_lookup_unique(d_tabs, u_values, u_offsets, feat_uoff, U, pooled)
    ctx.expand_inverse(F, B, pooled, feat_uoff, inverse, out)
    ctx.kjt_pooled_lookup(d_tabs, B, d_values, d_offsets, kjt)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), kjt.view(torch.int32))
    for l in (0, B + 17, F * B - 1):   # the last one lies beyond position 2^31
        f = l // B
        exact = tabs[f][values[offsets[l]:offsets[l + 1]]].astype(np.float64).sum(axis=0)
        assert np.abs(exact).max() < 2**22
        assert np.array_equal(kjt[f, l - f * B].double().cpu().numpy(), exact), l
    assert offsets[F * B - 1] > 2**31
    ctx.close()
