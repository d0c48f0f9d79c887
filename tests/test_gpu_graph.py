"""A whole step (build, unique lookup, expand, backward with the fused update) captured once into a
HIP graph and replayed on other batches: with host upper bounds in the place of U and M no call
synchronises, allocates or clears memory with a memset node, so the step is capturable as it is.
Every replay is checked against the eager calls on the same inputs (bit for bit) and against the
oracle; eager work and synchronisations run between the replays."""
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


class _Step:
    """Static buffers of one step at worst-case sizes, and the calls in step order."""

    def __init__(self, recd, w, n_max, stream):
        F, B, D = w.F, w.B, w.D
        self.w, self.n_max = w, n_max
        with torch.cuda.stream(stream):
            self.ctx = recd.Context(0, workspace_hint_bytes=recd.workspace_bytes(F, B, n_max, D))
            z = lambda *shape, dt=torch.int64: torch.zeros(*shape, dtype=dt, device="cuda")
            self.values, self.offsets = z(n_max), z(F * B + 1)
            self.u_values, self.u_offsets = z(n_max), z(F * B + 1)
            self.inverse, self.feat_uoff = z(F * B, dt=torch.int32), z(F + 1)
            self.pooled = z(F * B, D, dt=torch.float32)
            self.out = z(F, B, D, dt=torch.float32)
            self.grad_out = z(F, B, D, dt=torch.float32)
            self.touched, self.feat_roff = z(n_max), z(F + 1)
            self.grad_rows = z(n_max, D, dt=torch.float32)
            self.tables = [z(w.rows, D, dt=torch.float32) for _ in range(F)]
            self.state = [z(w.rows, dt=torch.float32) for _ in range(F)]

    def load(self, batch, gout, tabs):
        self.values[:batch.N].copy_(torch.from_numpy(batch.values))
        self.offsets.copy_(torch.from_numpy(batch.offsets))
        self.grad_out.copy_(torch.from_numpy(gout))
        for t, s, src in zip(self.tables, self.state, tabs):
            t.copy_(torch.from_numpy(src))
            s.zero_()

    def run(self):
        w, c = self.w, self.ctx
        F, B = w.F, w.B
        c.build_ikjt(F, B, self.values, self.offsets, self.u_values, self.u_offsets, self.inverse, self.feat_uoff)
        c.pooled_lookup_unique(self.tables, self.u_values, self.u_offsets, self.feat_uoff, F * B, self.pooled)
        c.expand_inverse(F, B, self.pooled, self.feat_uoff, self.inverse, self.out)
        c.backward_dedup(F, B, self.grad_out, self.inverse, self.feat_uoff, self.u_values, self.u_offsets,
                         [w.rows] * F, F * B, self.n_max, self.touched, self.feat_roff, self.grad_rows,
                         tables=self.tables, adagrad_state=self.state, lr=0.01, eps=1e-8)

    def results(self):
        torch.cuda.synchronize()
        return [x.clone() for x in (self.out, self.feat_roff, self.inverse, self.feat_uoff, *self.tables, *self.state)]


@pytest.mark.parametrize("B", [1024, 1536], ids=["one-launch-builder", "general-builder"])
def test_step_replays_as_a_graph(recd, B):
    w = synth.scaled(synth.WORKLOADS["cfg2"], F=4, B=B, rows=20_000, D=64)
    batches = [synth.make_batch(w, i) for i in range(4)]
    gouts = [synth.make_grad_out(w, i) for i in range(4)]
    tabs = synth.make_tables(w)
    n_max = max(b.N for b in batches)
    stream = torch.cuda.Stream()
    step = _Step(recd, w, n_max, stream)
    F, B, D = w.F, w.B, w.D

    # eager results of every batch first (they also warm the library up before the capture)
    eager = []
    with torch.cuda.stream(stream):
        for b, g in zip(batches, gouts):
            step.load(b, g, tabs)
            step.run()
            eager.append(step.results())

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        step.load(batches[0], gouts[0], tabs)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            step.run()

    for rnd in range(2):
        for i in (2, 0, 3, 1):
            with torch.cuda.stream(stream):
                step.load(batches[i], gouts[i], tabs)   # eager copies between the replays
                graph.replay()
                got = step.results()
            for a, e in zip(got, eager[i]):
                assert torch.equal(a, e), f"replay of batch {i} (round {rnd}) differs from the eager step"
            # and the oracle: expanded output and the updated rows of feature 1
            uv, uo, inv, fu = orc.build_ikjt(F, B, batches[i].values, batches[i].offsets)
            ref = orc.expand_inverse(F, B, orc.pooled_lookup(tabs, "f32", uv, uo, fu), fu, inv)
            gu.assert_close_f32(gu.out_to_f64(got[0]), ref, "expanded output")
            tr, fr, gr = orc.backward_dedup(F, B, gouts[i], inv, fu, uv, uo)
            assert np.array_equal(got[1].cpu().numpy(), fr)
            rows1 = tr[fr[1]:fr[2]]
            w_new, _ = orc.rowwise_adagrad(gr[fr[1]:fr[2]], tabs[1][rows1].astype(np.float64),
                                           np.zeros(len(rows1)), 0.01, 1e-8)
            gu.assert_close_f32(got[4 + 1].cpu().numpy()[rows1].astype(np.float64), w_new, "updated rows")
    step.ctx.close()
