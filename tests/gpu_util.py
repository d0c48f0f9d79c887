"""Helpers of the GPU parity tests: upload a seeded batch, run the HIP path through the C ABI,
bring results back as numpy.  No arithmetic of the method lives here."""
import numpy as np
import torch

TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def tables_to_dev(tabs, dtype):
    out = []
    for t in tabs:
        if dtype == "bf16":
            out.append(torch.from_numpy(t.astype(np.int16)).view(torch.bfloat16).cuda())
        else:
            out.append(torch.from_numpy(t).cuda())
    return out


def out_to_f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


class DeviceIKJT:
    def __init__(self, F, B, N):
        L = F * B
        self.F, self.B = F, B
        self.u_values = torch.full((max(N, 1),), -7, dtype=torch.int64, device="cuda")
        self.u_offsets = torch.full((L + 1,), -7, dtype=torch.int64, device="cuda")
        self.inverse = torch.full((max(L, 1),), -7, dtype=torch.int32, device="cuda")
        self.feat_uoff = torch.full((F + 1,), -7, dtype=torch.int64, device="cuda")
        self.U = self.M = None

    def numpy(self):
        U, M = self.U, self.M
        return (self.u_values[:M].cpu().numpy(), self.u_offsets[:U + 1].cpu().numpy(),
                self.inverse[:self.F * self.B].cpu().numpy(), self.feat_uoff.cpu().numpy())


def gpu_build(ctx, batch):
    values, offsets = to_dev(batch.values), to_dev(batch.offsets)
    if values.numel() == 0:
        values = torch.zeros(1, dtype=torch.int64, device="cuda")[:0]
    ik = DeviceIKJT(batch.F, batch.B, batch.N)
    ik.U, ik.M = ctx.build_ikjt(batch.F, batch.B, values, offsets, ik.u_values, ik.u_offsets,
                                ik.inverse, ik.feat_uoff, want_counts=True)
    from paper_2211_05239_amd import recd as mod
    small = ctx.options.get(mod._OPT_INTERNAL_SMALL_PATH, 1)
    if 0 < batch.B <= 1024 and batch.F > 0 and small != 0:
        # a batch this small is built by the one-launch builder: the general one must give the same arrays
        ik2 = DeviceIKJT(batch.F, batch.B, batch.N)
        ctx.set_option(mod._OPT_INTERNAL_SMALL_PATH, 0)
        try:
            ik2.U, ik2.M = ctx.build_ikjt(batch.F, batch.B, values, offsets, ik2.u_values, ik2.u_offsets,
                                          ik2.inverse, ik2.feat_uoff, want_counts=True)
        finally:
            ctx.set_option(mod._OPT_INTERNAL_SMALL_PATH, small)
        assert (ik.U, ik.M) == (ik2.U, ik2.M)
        for name in ("u_values", "u_offsets", "inverse", "feat_uoff"):
            assert torch.equal(getattr(ik, name), getattr(ik2, name)), name
    return values, offsets, ik


def gpu_forward(ctx, batch, dev_tables, out_dtype):
    """Returns (ikjt, pooled[U,D], expanded[F,B,D], kjt_out[F,B,D]) as device tensors."""
    F, B = batch.F, batch.B
    D = dev_tables[0].shape[1]
    values, offsets, ik = gpu_build(ctx, batch)
    pooled = torch.full((max(F * B, 1), D), float("nan"), dtype=out_dtype, device="cuda")
    ctx.pooled_lookup_unique(dev_tables, ik.u_values, ik.u_offsets, ik.feat_uoff, F * B, pooled)
    out = torch.full((F, B, D), float("nan"), dtype=out_dtype, device="cuda")
    ctx.expand_inverse(F, B, pooled, ik.feat_uoff, ik.inverse, out)
    kjt = torch.full((F, B, D), float("nan"), dtype=out_dtype, device="cuda")
    ctx.kjt_pooled_lookup(dev_tables, B, values, offsets, kjt)
    torch.cuda.synchronize()
    return ik, pooled, out, kjt


def assert_close_f32(got, ref, what=""):
    """fp32 bar: |err| <= 1e-5 * (1 + |ref|)."""
    err = np.abs(got - ref)
    bound = 1e-5 * (1.0 + np.abs(ref))
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond 1e-5*(1+|ref|), max err {err.max()}"


def assert_close_16(got, ref, what=""):
    """fp16/bf16 bar: 1e-2 relative, with an absolute floor of 1e-6 for sums that cancel to ~0."""
    err = np.abs(got - ref)
    bound = 1e-2 * np.abs(ref) + 1e-6
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond 1e-2 relative, max err {err.max()}"


def long_sum_depth(n, lane_groups, cut=32):
    """Largest number of fp32 additions any one term of a table row's gradient passes through when
    the row has n > cut entries (the backward's chunked two-level sum): the entries are cut into
    chunks of ch = 256 entries (ceil(n/64) if that would give more than 64 chunks); a chunk is
    summed by a four-wave block, wave w taking the 64-entry pieces w, w+4, ... and lane group g
    of `lane_groups` adding the piece's entries g, g+G, ... into one accumulator; then a butterfly
    over the lane groups, the four wave partials in wave order, and the chunk partials in chunk
    order."""
    assert n > cut
    ch = 256 if (n + 255) // 256 <= 64 else (n + 63) // 64
    nch = (n + ch - 1) // ch
    pieces = (ch + 63) // 64
    per_wave = (pieces + 3) // 4
    return per_wave * (64 // lane_groups) + int(np.log2(lane_groups)) + 3 + nch


def assert_long_sum(got, ref, abs_terms, depth, what=""):
    """Bar of a long fp32 sum: the stated 1e-5 * (1 + |ref|) or, where it is larger, the first-order
    worst-case bound of the summation tree, depth * 2^-24 * sum |terms|."""
    err = np.abs(got - ref)
    bound = np.maximum(1e-5 * (1.0 + np.abs(ref)), depth * 2.0 ** -24 * abs_terms)
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond the bound, max err {err.max()}, bound {bound.min()}"
