"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Tolerances (written out here; each follows from the forward-error bound of an fp32 or bf16 sum):
  fp32 aggregation, GCN ... |gpu - ref| <= 1e-6 + 1e-4 |ref|
  fp32 aggregation, GIN ... |gpu - ref| <= 1e-6 max(1, sum|x_u|) + 1e-4 |ref|   (unnormalised sums:
                            the absolute term has to follow the magnitude of what is added up)
  bf16-input aggregation .. |gpu - ref| <= 2e-2 |ref| + 1e-2 max|ref|   (and, tighter, the fp32
                            accumulation bound 1e-5 * sum|w x| since bf16 inputs are exact in fp32)
  fp32 Update ............. |gpu - ref| <= 1e-4 |ref| + 2 K 2^-24 (|a| @ |w|)
  bf16 Update ............. |gpu - ref| <= 2e-2 |ref| + 2^-7 (|a| @ |w|)
  bf16 layers ............. |gpu - ref| <= 2e-2 |ref| + 2^-8 (|agg| @ |w1| (@ |w2|))
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_06800_amd import binding, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# ----------------------------------------------------------------------------- helpers
def to_dev(a: np.ndarray):
    """numpy fp32 / bf16-bit array -> torch tensor on the GPU (bf16 bits are reinterpreted)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_close(got, ref, rtol, atol, what=""):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r} err {err[i]:.3e} bound {np.broadcast_to(bound, err.shape)[i]:.3e}")
    return float(np.max(err / np.maximum(bound, 1e-300))) if err.size else 0.0


def agg_tolerances(dtype):
    return (1e-4, 1e-6) if dtype == "f32" else (2e-2, None)


def report_ratio(what, ratio):
    """Worst error over its bound, printed for the tolerance table (run pytest with -s to see it)."""
    print(f"\nRATIO {what}: max err / bound = {ratio:.4f}", flush=True)


def check_aggregate(w_row_ptr, w_col, parts, part_id, bounds, x, mode, eps=0.0, build=None, ld_pad=0,
                    misalign=0, rows=None, what="", report=None, options=None):
    """Run mgg_aggregate on one share and compare every (or the sampled) output row."""
    build = build or {}
    ref_part = oracle.build_partition(w_row_ptr, w_col, parts, part_id, bounds)
    lb, ub, hg = ref_part["lb"], ref_part["ub"], ref_part["halo_gid"]
    part = binding.mgg_build_partition(w_row_ptr, w_col, parts, part_id, bounds, **build)
    for key, value in (options or {}).items():
        part.set_option(key, value)
    x_local_np, x_halo_np = x[lb:ub], x[hg]
    dim = x.shape[1]

    def place(a):
        """Device copy with optional row padding and a base pointer that is not 16-byte aligned."""
        t = to_dev(a)
        if ld_pad or misalign:
            # NaN in the padding: the kernel may read it (rows are read in whole 16-byte vectors when
            # the leading dimension leaves room) but nothing of it may reach the output
            buf = torch.full((a.shape[0] * (dim + ld_pad) + misalign,), float("nan"), dtype=t.dtype, device=DEV)
            view = buf[misalign:].view(a.shape[0], dim + ld_pad)[:, :dim]
            view.copy_(t)
            return view
        return t

    xl, xh = place(x_local_np), (place(x_halo_np) if hg.size else None)
    out = torch.full((ub - lb, dim + ld_pad), float("nan"), dtype=torch.float32, device=DEV)[:, :dim]
    binding.mgg_aggregate(part, mode, xl, xh, eps=eps, out=out)
    torch.cuda.synchronize()
    got = to_host64(out)
    ref = oracle.aggregate(w_row_ptr, w_col, mode, x_local_np, lb=lb, ub=ub, x_halo=x_halo_np, halo_gid=hg,
                           eps=eps, rows=rows)
    if rows is not None:
        got = got[np.asarray(rows)]
    is_bf16 = x.dtype == np.uint16
    # sum |w x| per output element: the scale of the rounding error of any fp32 summation
    xa_l = np.abs(inputs.bf16_bits_to_f32(x_local_np)) if is_bf16 else np.abs(x_local_np)
    xa_h = np.abs(inputs.bf16_bits_to_f32(x_halo_np)) if is_bf16 else np.abs(x_halo_np)
    scale = oracle.aggregate(w_row_ptr, w_col, mode, xa_l, lb=lb, ub=ub, x_halo=xa_h, halo_gid=hg,
                             eps=abs(eps), rows=rows)
    if is_bf16:
        assert_close(got, ref, 2e-2, 1e-2 * max(np.abs(ref).max(), 1e-30), what)
        # tighter: bf16 inputs are exact in fp32, so only the fp32 accumulation error remains
        assert np.all(np.abs(got - ref) <= 1e-5 * scale + 1e-30), f"{what}: beyond the fp32 accumulation bound"
        ratio = float(np.max(np.abs(got - ref) / (1e-5 * scale + 1e-30)))
    elif mode == "gcn":
        ratio = assert_close(got, ref, 1e-4, 1e-6, what)
    else:
        ratio = assert_close(got, ref, 1e-4, 1e-6 * np.maximum(1.0, scale), what)
    part.destroy()
    if report is not None:
        report(what, ratio)
    return got


def small_rmat(scale=12, draws=60000, seed=0):
    rng = np.random.default_rng(seed)
    row_ptr, col = inputs.rmat_graph(scale, draws, 0.57, 0.19, 0.19, 0.05, rng)
    return row_ptr, col, rng


# ----------------------------------------------------------------------------- aggregation
@pytest.mark.parametrize("dim", [1, 3, 4, 16, 20, 47, 64, 100, 128, 256, 260, 602, 608, 1024, 2052, 4100, 601 * 3])
@pytest.mark.parametrize("mode", ["gcn", "gin"])
def test_aggregate_fp32_dims(dim, mode):
    row_ptr, col, rng = small_rmat(seed=dim)
    n = row_ptr.size - 1
    x = rng.standard_normal((n, dim)).astype(np.float32)
    bounds = inputs.equal_node_bounds(n, 4)
    check_aggregate(row_ptr, col, 4, 0, bounds, x, mode, eps=0.25, what=f"f32 dim {dim} {mode}")


@pytest.mark.parametrize("dim", [1, 2, 8, 24, 30, 64, 128, 129, 136, 520])
def test_aggregate_bf16_dims(dim):
    row_ptr, col, rng = small_rmat(seed=1000 + dim)
    n = row_ptr.size - 1
    x = inputs.to_bf16_bits(rng.standard_normal((n, dim)).astype(np.float32))
    bounds = inputs.equal_node_bounds(n, 8)
    check_aggregate(row_ptr, col, 8, 0, bounds, x, "gin", what=f"bf16 dim {dim} gin")
    check_aggregate(row_ptr, col, 8, 3, bounds, x, "gcn", what=f"bf16 dim {dim} gcn")


@pytest.mark.parametrize("build", [dict(ps=1, dist=1), dict(ps=2, dist=3), dict(ps=7, dist=2), dict(ps=32, dist=1),
                                   dict(ps=64, dist=4), dict(ps=32, dist=1024), dict(short_max=-1),
                                   dict(short_max=4096), dict(ps=5, dist=5, short_max=3),
                                   dict(xcd_min_deg=1, short_max=-1), dict(xcd_min_deg=40), dict(xcd_min_deg=500, dist=2),
                                   dict(wpb=1), dict(wpb=2, xcd_min_deg=40), dict(wpb=8), dict(wpb=16, ps=16, dist=2),
                                   dict(hot_phases=4, xcd_min_deg=40), dict(hot_phases=1, hot_rows=64, min_piece=1, xcd_min_deg=1),
                                   dict(hot_phases=31, hot_rows=16, min_piece=4, hot_min_count=2, xcd_min_deg=20, ps=8, dist=1),
                                   dict(hot_phases=2, hot_row_bytes=1024, min_piece=64, xcd_min_deg=100),
                                   dict(hot_phases=-2, xcd_min_deg=40), dict(hot_phases=-16, xcd_min_deg=20, min_piece=2)])
def test_every_schedule_gives_the_same_answer(build):
    """Neighbour-partition size, pairs per work item and the short-row bin change only the
    schedule (section 4.1 Step-3, section 5.1), never the value."""
    row_ptr, col, rng = small_rmat(seed=77)
    n = row_ptr.size - 1
    x = rng.standard_normal((n, 64)).astype(np.float32)
    bounds = inputs.equal_node_bounds(n, 4)
    for p in (0, 2):
        check_aggregate(row_ptr, col, 4, p, bounds, x, "gcn", build=build, what=f"{build} part {p}")
    xb = inputs.to_bf16_bits(x[:, :40])
    check_aggregate(row_ptr, col, 4, 1, bounds, xb, "gin", eps=-0.5, build=build, what=f"{build} bf16")


@pytest.mark.parametrize("ld_pad,misalign", [(0, 1), (3, 0), (4, 0), (5, 2), (8, 4)])
def test_padded_rows_and_unaligned_base(ld_pad, misalign):
    row_ptr, col, rng = small_rmat(scale=11, draws=30000, seed=5)
    n = row_ptr.size - 1
    bounds = inputs.equal_node_bounds(n, 2)
    for dim in (64, 100):
        x = rng.standard_normal((n, dim)).astype(np.float32)
        check_aggregate(row_ptr, col, 2, 1, bounds, x, "gcn", ld_pad=ld_pad, misalign=misalign,
                        what=f"dim {dim} pad {ld_pad} misalign {misalign}")
    xb = inputs.to_bf16_bits(rng.standard_normal((n, 128)).astype(np.float32))
    check_aggregate(row_ptr, col, 2, 0, bounds, xb, "gin", ld_pad=ld_pad, misalign=misalign, what="bf16 padded")


def test_tables_beyond_4gb_take_64_bit_row_offsets():
    """Row offsets inside a table are 32-bit unless a table reaches beyond 4 GB; rows spaced 2.1 MB apart
    put a 2048-row table there (work items, short rows and the self term all use the wide path)."""
    row_ptr, col, rng = small_rmat(seed=41)
    n = row_ptr.size - 1
    x = rng.standard_normal((n, 64)).astype(np.float32)
    bounds = inputs.equal_node_bounds(n, 2)
    ld = (1 << 32) // (4 * (n // 2)) + 1024                  # rows * ld * 4 bytes just beyond 2^32
    assert (n // 2) * ld * 4 >= 1 << 32
    for mode in ("gcn", "gin"):
        check_aggregate(row_ptr, col, 2, 1, bounds, x, mode, eps=0.5, ld_pad=ld - 64, what=f"wide offsets {mode}")
    torch.cuda.empty_cache()


def test_degenerate_graphs():
    rng = np.random.default_rng(3)
    # no edges at all: every row is its own embedding (times 1 + eps for GIN)
    n = 300
    row_ptr, col = np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32)
    x = rng.standard_normal((n, 64)).astype(np.float32)
    got = check_aggregate(row_ptr, col, 1, 0, np.array([0, n]), x, "gcn", what="edgeless gcn")
    assert np.array_equal(got.astype(np.float32), x)
    check_aggregate(row_ptr, col, 1, 0, np.array([0, n]), x, "gin", eps=0.5, what="edgeless gin")
    # star: one row with n-1 neighbours (cut into many items), n-1 rows with one
    n = 5000
    adj = [list(range(1, n))] + [[0]] * (n - 1)
    row_ptr, col = inputs.csr_from_adjacency_lists(adj)
    x = rng.standard_normal((n, 32)).astype(np.float32)
    check_aggregate(row_ptr, col, 1, 0, np.array([0, n]), x, "gcn", what="star")
    check_aggregate(row_ptr, col, 2, 0, np.array([0, 1, n]), x, "gin", what="star centre, all remote")
    check_aggregate(row_ptr, col, 2, 1, np.array([0, 1, n]), x, "gcn", what="star leaves, one halo row")
    # an empty node range is a no-op
    part = binding.mgg_build_partition(row_ptr, col, 3, 1, [0, 10, 10, n])
    out = binding.mgg_aggregate(part, "gcn", torch.zeros((0, 32), device=DEV), torch.zeros((4, 32), device=DEV))
    assert out.shape == (0, 32)
    # self-loops and duplicate neighbours in the input
    row_ptr, col = inputs.csr_from_adjacency_lists([[0, 1, 1, 2], [0], [0, 2]])
    x = rng.standard_normal((3, 16)).astype(np.float32)
    check_aggregate(row_ptr, col, 1, 0, np.array([0, 3]), x, "gcn", what="self-loops gcn")
    check_aggregate(row_ptr, col, 1, 0, np.array([0, 3]), x, "gin", what="self-loops gin")


def test_partition_consistency_on_the_gpu():
    """All shares, one after another, reproduce the single-partition result (whole-graph degrees)."""
    row_ptr, col, rng = small_rmat(seed=9)
    n = row_ptr.size - 1
    x = rng.standard_normal((n, 48)).astype(np.float32)
    whole = check_aggregate(row_ptr, col, 1, 0, np.array([0, n]), x, "gcn")
    for parts in (3, 8):
        bounds = inputs.equal_node_bounds(n, parts)
        pieces = [check_aggregate(row_ptr, col, parts, p, bounds, x, "gcn") for p in range(parts)]
        np.testing.assert_allclose(np.concatenate(pieces), whole, rtol=2e-4, atol=2e-6)


def test_results_do_not_depend_on_scheduling():
    """Partial sums of split rows are combined in a fixed order: two runs agree bit for bit."""
    w = inputs.config(2, shrink=6)
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    ref_part = oracle.build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    xl, xh = to_dev(w.x[w.lb:w.ub]), to_dev(w.x[ref_part["halo_gid"]])
    a = binding.mgg_aggregate(part, "gcn", xl, xh).clone()
    for _ in range(3):
        b = binding.mgg_aggregate(part, "gcn", xl, xh)
        assert torch.equal(a, b)


@pytest.fixture
def lds_halo():
    binding.mgg_set_option("lds_halo", 1)
    yield
    binding.mgg_set_option("lds_halo", 0)


@pytest.mark.parametrize("dim,bf16", [(16, False), (64, False), (100, False), (256, False), (128, True), (8, True), (512, True)])
@pytest.mark.parametrize("build", [dict(), dict(ps=7, dist=2), dict(ps=64, dist=4), dict(ps=1, dist=40, short_max=-1)])
def test_lds_staged_halo_rows_give_the_same_answer(lds_halo, dim, bf16, build):
    """Halo rows staged through LDS ahead of their accumulation (section 5.2) change the
    schedule only; shapes the staged path does not cover fall back to register loads."""
    row_ptr, col, rng = small_rmat(seed=300 + dim)
    n = row_ptr.size - 1
    x = rng.standard_normal((n, dim)).astype(np.float32)
    if bf16:
        x = inputs.to_bf16_bits(x)
    bounds = inputs.equal_node_bounds(n, 4)
    for p, mode in ((0, "gcn"), (3, "gin")):
        check_aggregate(row_ptr, col, 4, p, bounds, x, mode, build=build, what=f"lds dim {dim} {build} part {p}")


@pytest.mark.parametrize("slab_bytes", [64, 128, 256, 1024])
@pytest.mark.parametrize("dim,bf16", [(64, False), (100, False), (602, False), (608, False), (47, False), (128, True), (520, True), (130, True)])
def test_column_slab_passes_give_the_same_answer(slab_bytes, dim, bf16):
    """Walking the feature dimension slab by slab changes which bytes sit in L2, not the value."""
    binding.mgg_set_option("col_slab_bytes", slab_bytes)
    try:
        row_ptr, col, rng = small_rmat(seed=500 + dim)
        n = row_ptr.size - 1
        x = rng.standard_normal((n, dim)).astype(np.float32)
        if bf16:
            x = inputs.to_bf16_bits(x)
        bounds = inputs.equal_node_bounds(n, 4)
        check_aggregate(row_ptr, col, 4, 0, bounds, x, "gcn", build=dict(xcd_min_deg=64), what=f"slab {slab_bytes} dim {dim}")
        check_aggregate(row_ptr, col, 4, 2, bounds, x, "gin", build=dict(xcd_min_deg=-1, dist=2), what=f"slab {slab_bytes} dim {dim} gin")
        binding.mgg_set_option("lds_halo", 1)
        check_aggregate(row_ptr, col, 4, 1, bounds, x, "gcn", what=f"slab {slab_bytes} dim {dim} lds")
    finally:
        binding.mgg_set_option("col_slab_bytes", 0)
        binding.mgg_set_option("lds_halo", 0)


@pytest.mark.parametrize("slab_bytes", [1, 2048, 4096])
@pytest.mark.parametrize("dim,bf16", [(300, False), (602, False), (1000, False), (1027, False), (1040, True), (2048, True), (2100, True)])
def test_rows_wider_than_a_wavefront_without_narrow_slabs(slab_bytes, dim, bf16):
    """With column slabs off (1) or wider than 1 KB a lane holds 2 to 4 chunks of a row (rows beyond 4 KB are
    still walked 4 KB at a time): the kernel variants the automatic slab rule never picks."""
    row_ptr, col, rng = small_rmat(seed=900 + dim)
    n = row_ptr.size - 1
    x = rng.standard_normal((n, dim)).astype(np.float32)
    if bf16:
        x = inputs.to_bf16_bits(x)
    bounds = inputs.equal_node_bounds(n, 4)
    for p, mode, build in ((0, "gcn", dict(xcd_min_deg=64)), (2, "gin", dict(dist=2))):
        check_aggregate(row_ptr, col, 4, p, bounds, x, mode, eps=0.125, build=build, options={"col_slab_bytes": slab_bytes},
                        what=f"wide rows, slab option {slab_bytes}, dim {dim} {mode}")


@pytest.mark.parametrize("dim,bf16,mode", [(64, False, "gcn"), (100, False, "gin"), (602, False, "gcn"), (128, True, "gin")])
def test_local_and_remote_in_two_launches_give_the_same_answer(dim, bf16, mode):
    """Ablation of interleaving (section 5.1): local lists first, remote lists added by a second launch."""
    binding.mgg_set_option("split_phases", 1)
    try:
        row_ptr, col, rng = small_rmat(seed=700 + dim)
        n = row_ptr.size - 1
        x = rng.standard_normal((n, dim)).astype(np.float32)
        if bf16:
            x = inputs.to_bf16_bits(x)
        bounds = inputs.equal_node_bounds(n, 4)
        for p, build in ((0, dict()), (3, dict(ps=8, dist=2, xcd_min_deg=30)), (1, dict(xcd_min_deg=-1, short_max=-1))):
            check_aggregate(row_ptr, col, 4, p, bounds, x, mode, eps=0.5, build=build, what=f"two launches dim {dim} part {p}")
        check_aggregate(row_ptr, col, 1, 0, np.array([0, n]), x, mode, what="two launches, no halo")
    finally:
        binding.mgg_set_option("split_phases", 0)


@pytest.mark.parametrize("dim,bf16_in,mode,build", [(64, False, "gcn", {}), (128, True, "gin", {}), (47, False, "gcn", dict(ps=7, dist=2)),
                                                     (602, False, "gcn", dict(xcd_min_deg=30)), (130, True, "gin", dict(short_max=-1)),
                                                     (8, True, "gcn", dict(hot_phases=2))])
def test_aggregate_bf16_output_is_the_rounded_fp32_output(dim, bf16_in, mode, build):
    """mgg_aggregate_to with bf16 output rounds the same fp32 sums (nearest even) as they are written:
    bit for bit what rounding the fp32 output gives, so a bf16 MFMA fed either way sees the same input."""
    row_ptr, col, rng = small_rmat(seed=31)
    n = row_ptr.size - 1
    bounds = inputs.equal_node_bounds(n, 3)
    x = rng.standard_normal((n, dim)).astype(np.float32)
    if bf16_in:
        x = inputs.to_bf16_bits(x)
    for p in range(3):
        part = binding.mgg_build_partition(row_ptr, col, 3, p, bounds, **build)
        hg = part.export()["halo_gid"]
        xl, xh = to_dev(x[bounds[p]:bounds[p + 1]]), (to_dev(x[hg]) if hg.size else None)
        f32 = binding.mgg_aggregate(part, mode, xl, xh, eps=0.5)
        buf = torch.full((int(part.info.n_own), dim + 5), float("nan"), dtype=torch.bfloat16, device=DEV)
        b16 = binding.mgg_aggregate(part, mode, xl, xh, eps=0.5, out=buf[:, :dim])
        aligned = binding.mgg_aggregate(part, mode, xl, xh, eps=0.5, out_dtype=torch.bfloat16)
        torch.cuda.synchronize()
        assert torch.isnan(buf[:, dim:]).all()
        assert torch.equal(b16, f32.to(torch.bfloat16)) and torch.equal(aligned, b16)
        part.destroy()


# ----------------------------------------------------------------------------- update
def update_bound(a64, w64, k, bf16):
    s = np.abs(a64) @ np.abs(w64)
    return (2.0 ** -7) * s if bf16 else 2.0 * k * 2.0 ** -24 * s


@pytest.mark.parametrize("n_rows,d_in,d_out", [(1, 1, 1), (127, 16, 16), (129, 64, 64), (1000, 100, 256),
                                               (333, 602, 256), (4096, 256, 47), (77, 33, 300), (500, 5, 513), (300, 96, 512),
                                               (257, 40, 256),
                                               # more row tiles than resident workgroups: each walks over several tiles
                                               (70001, 100, 256), (66000, 36, 512), (66000, 20, 256)])
@pytest.mark.parametrize("act", ["none", "relu"])
def test_update_fp32(n_rows, d_in, d_out, act):
    rng = np.random.default_rng(n_rows + d_in)
    a = rng.standard_normal((n_rows, d_in)).astype(np.float32)
    w = (0.1 * rng.standard_normal((d_in, d_out))).astype(np.float32)
    b = rng.standard_normal(d_out).astype(np.float32)
    for bias in (None, b):
        got = binding.mgg_update(to_dev(a), to_dev(w), None if bias is None else to_dev(bias), act)
        torch.cuda.synchronize()
        ref = oracle.update(a, w, bias, act)
        bound = update_bound(a.astype(np.float64), w.astype(np.float64), d_in, False)
        assert_close(to_host64(got), ref, 1e-4, bound, f"update f32 {n_rows}x{d_in}x{d_out} {act}")


def test_update_fp32_padded_and_unaligned_input():
    rng = np.random.default_rng(12)
    a = rng.standard_normal((300, 602)).astype(np.float32)
    w = (0.1 * rng.standard_normal((602, 64))).astype(np.float32)
    buf = torch.zeros(300 * 603 + 1, device=DEV)
    av = buf[1:].view(300, 603)[:, :602]
    av.copy_(to_dev(a))
    out = torch.full((300, 70), float("nan"), device=DEV)[:, :64]
    binding.mgg_update(av, to_dev(w), None, "relu", out=out)
    ref = oracle.update(a, w, None, "relu")
    assert_close(to_host64(out), ref, 1e-4, update_bound(a.astype(np.float64), w.astype(np.float64), 602, False), "padded update")


@pytest.mark.parametrize("n_rows,d_in,d_out", [(1, 8, 8), (200, 128, 128), (1025, 64, 47), (300, 100, 130), (64, 7, 5)])
@pytest.mark.parametrize("a_is_bf16", [False, True])
def test_update_bf16(n_rows, d_in, d_out, a_is_bf16):
    rng = np.random.default_rng(n_rows * 7 + d_out)
    a32 = rng.standard_normal((n_rows, d_in)).astype(np.float32)
    wb = inputs.to_bf16_bits((0.1 * rng.standard_normal((d_in, d_out))).astype(np.float32))
    a_in = inputs.to_bf16_bits(a32) if a_is_bf16 else a32
    ref = oracle.update(a_in, wb, None, "relu")
    s_bound = update_bound(oracle.to_f64(a_in), oracle.to_f64(wb), d_in, True)
    for out_dtype in (torch.float32, torch.bfloat16):
        got = binding.mgg_update(to_dev(a_in), to_dev(wb), None, "relu", out_dtype=out_dtype)
        torch.cuda.synchronize()
        assert_close(to_host64(got), ref, 2e-2, s_bound, f"update bf16 {n_rows}x{d_in}x{d_out} a_bf16={a_is_bf16}")


@pytest.mark.parametrize("n_rows,d_in,d_out,w_bf16,a_bf16,out_bf16", [
    (1000, 64, 64, False, False, False), (33, 32, 128, False, False, False), (4097, 256, 47, False, False, False),
    (70000, 128, 100, False, False, False), (515, 128, 128, True, False, True), (515, 128, 128, True, True, False),
    (31, 64, 40, True, True, True), (2049, 256, 96, True, False, False), (300, 64, 128, True, True, True)])
def test_update_whole_line_kernels(n_rows, d_in, d_out, w_bf16, a_bf16, out_bf16):
    """Shapes the whole-line kernels cover (whole K slabs, 33..128 output columns): against the
    oracle, and bit for bit against the register-resident kernels, which contract in the same order;
    the output view has padded rows so that a store past the last column would be seen."""
    rng = np.random.default_rng(n_rows + d_in)
    a = rng.standard_normal((n_rows, d_in)).astype(np.float32)
    w = (0.1 * rng.standard_normal((d_in, d_out))).astype(np.float32)
    b = rng.standard_normal(d_out).astype(np.float32)
    a_in = inputs.to_bf16_bits(a) if a_bf16 else a
    w_in = inputs.to_bf16_bits(w) if w_bf16 else w
    ref = oracle.update(a_in, w_in, b, "relu")         # the oracle takes the inputs as given and rounds nothing
    s_bound = np.abs(oracle.to_f64(a_in)) @ np.abs(oracle.to_f64(w_in)) + np.abs(b)
    got = {}
    for stream in (1, 0):
        binding.mgg_set_option("update_stream", stream)
        try:
            pad = 8 if out_bf16 else 4
            buf = torch.full((n_rows, d_out + pad), float("nan"), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=DEV)
            out = binding.mgg_update(to_dev(a_in), to_dev(w_in), to_dev(b), "relu", out=buf[:, :d_out])
            torch.cuda.synchronize()
        finally:
            binding.mgg_set_option("update_stream", 1)
        assert torch.isnan(buf[:, d_out:]).all()
        got[stream] = out
        if w_bf16:
            assert_close(to_host64(out), ref, 2e-2, 2.0 ** -7 * s_bound, f"stream={stream}")
        else:
            assert_close(to_host64(out), ref, 1e-4, 2.0 * d_in * 2.0 ** -24 * s_bound, f"stream={stream}")
    assert torch.equal(got[0], got[1])


@pytest.mark.parametrize("n_rows,d_in,d_out,bf16", [(1000, 256, 47, False), (77, 64, 64, False), (513, 100, 130, False),
                                                   (300, 128, 300, False), (5, 8, 1, False), (400, 128, 47, True)])
def test_update_softmax(n_rows, d_in, d_out, bf16):
    """Row softmax after the product (the last step of the 2-layer GCN of section 7).  A softmax
    moves by at most half the change of its logits, so the bound is that of the logits plus the
    rounding of expf and of the division."""
    rng = np.random.default_rng(d_out)
    a = rng.standard_normal((n_rows, d_in)).astype(np.float32)
    w = (0.3 * rng.standard_normal((d_in, d_out))).astype(np.float32)
    b = rng.standard_normal(d_out).astype(np.float32)
    a_in, w_in = (inputs.to_bf16_bits(a), inputs.to_bf16_bits(w)) if bf16 else (a, w)
    ref = oracle.update(a_in, w_in, b, "softmax")
    s_bound = np.abs(oracle.to_f64(a_in)) @ np.abs(oracle.to_f64(w_in)) + np.abs(b)
    logit_err = (2.0 ** -7 if bf16 else 2.0 * d_in * 2.0 ** -24) * s_bound.max(axis=1, keepdims=True)
    buf = torch.full((n_rows, d_out + 3), float("nan"), dtype=torch.float32, device=DEV)
    out = binding.mgg_update(to_dev(a_in), to_dev(w_in), to_dev(b), "softmax", out=buf[:, :d_out])
    torch.cuda.synchronize()
    assert torch.isnan(buf[:, d_out:]).all()
    got = to_host64(out)
    assert_close(got, ref, 1e-5, 1e-6 + logit_err, "softmax")
    np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-5)


@pytest.mark.parametrize("n_rows,dims,acts,with_bias,out_bf16", [
    (1000, (128, 128, 128), ("relu", "none"), False, False), (70001, (128, 128, 128), ("relu", "relu"), True, True),
    (333, (64, 100, 47), ("relu", "none"), True, False), (31, (128, 40, 128), ("none", "relu"), True, False),
    (515, (64, 128, 64), ("relu", "none"), False, True),
    (200, (96, 128, 128), ("relu", "none"), True, False), (200, (128, 300, 64), ("relu", "none"), False, False)])
def test_update_mlp(n_rows, dims, acts, with_bias, out_bf16):
    """Two chained Updates with bf16 weights and fp32 input (GIN's MLP after the aggregation): the
    one-kernel form where the shape allows (the last two shapes fall back to two launches), against the
    oracle and against two separate mgg_update calls with a bf16 hidden buffer."""
    rng = np.random.default_rng(sum(dims) + n_rows)
    a = rng.standard_normal((n_rows, dims[0])).astype(np.float32)
    w = [inputs.to_bf16_bits((0.1 * rng.standard_normal((dims[i], dims[i + 1]))).astype(np.float32)) for i in range(2)]
    b = [rng.standard_normal(dims[i + 1]).astype(np.float32) if with_bias else None for i in range(2)]
    hid_ref = oracle.update(a, w[0], b[0], acts[0])
    ref = oracle.update(hid_ref, w[1], b[1], acts[1])
    s = np.abs(a).astype(np.float64) @ np.abs(oracle.to_f64(w[0])) + (0 if b[0] is None else np.abs(b[0]))
    s = s @ np.abs(oracle.to_f64(w[1])) + (0 if b[1] is None else np.abs(b[1]))
    d_b = [None if x is None else to_dev(x) for x in b]
    odt = torch.bfloat16 if out_bf16 else torch.float32
    pad = 8 if out_bf16 else 4
    buf = torch.full((n_rows, dims[2] + pad), float("nan"), dtype=odt, device=DEV)
    hidden = torch.empty((n_rows, dims[1]), dtype=torch.bfloat16, device=DEV)
    got = binding.mgg_update_mlp(to_dev(a), to_dev(w[0]), to_dev(w[1]), acts, d_b, hidden=hidden, out=buf[:, :dims[2]])
    two = binding.mgg_update(binding.mgg_update(to_dev(a), to_dev(w[0]), d_b[0], acts[0], out_dtype=torch.bfloat16),
                             to_dev(w[1]), d_b[1], acts[1], out_dtype=odt)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:, dims[2]:]).all()
    assert_close(to_host64(got), ref, 2e-2, BF16_LAYER_ATOL * s, f"mlp {dims}")
    # same roundings as the two-call form, another summation order in the second product
    assert_close(to_host64(got), to_host64(two), 2e-2 if out_bf16 else 1e-3, 2.0 ** (-7 if out_bf16 else -12) * s, f"mlp vs two calls {dims}")
    covered = dims[0] in (64, 128) and 32 < dims[1] <= 128 and 32 < dims[2] <= 128
    if covered:                                           # the one-kernel form needs no hidden buffer
        again = binding.mgg_update_mlp(to_dev(a), to_dev(w[0]), to_dev(w[1]), acts, d_b, out_dtype=odt)
        # input already rounded to bf16: the bits the kernel makes of the fp32 input itself
        from_bf16 = binding.mgg_update_mlp(to_dev(a).to(torch.bfloat16), to_dev(w[0]), to_dev(w[1]), acts, d_b, out_dtype=odt)
        torch.cuda.synchronize()
        assert torch.equal(again, got) and torch.equal(from_bf16, got)
    else:
        with pytest.raises(binding.MggError):
            binding.mgg_update_mlp(to_dev(a), to_dev(w[0]), to_dev(w[1]), acts, d_b, out_dtype=odt)


# ----------------------------------------------------------------------------- whole layers on the five configs
SHRINK = {1: 0, 2: 5, 3: 7, 4: 4, 5: 6}
# absolute term of the bf16 layers, in units of |agg| @ |W1| (@ |W2|): every operand of the bf16 MFMA
# carries one rounding of 2^-9 relative, so a product carries 2^-8, and the hidden activations of the
# two-linear MLP are rounded once more (measured worst error: 2 % of this bound)
BF16_LAYER_ATOL = 2.0 ** -8


def run_config_layers(w: inputs.Workload, rows=None, order="agg_first", report=None):
    """Forward of every layer of a workload on the GPU and in the oracle, every output row (or `rows`)."""
    ref_part = oracle.build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    lb, ub, hg = ref_part["lb"], ref_part["ub"], ref_part["halo_gid"]
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    assert part.info.num_halo == hg.size and part.info.n_own == ub - lb
    x_local, x_halo = w.x[lb:ub], w.x[hg]
    bf16 = w.dtype == "bf16"
    d_x_local, d_x_halo = to_dev(x_local), (to_dev(x_halo) if hg.size else None)
    for li, layer in enumerate(w.layers):
        if li == 1:
            # second layer of the 2-layer config: owned rows = layer-1 output; halo rows = seeded stand-in
            x_halo = inputs.layer2_halo_table(w.notes["layer2_halo_seed"], hg.size, layer.dims[0])
            x_local = h_gpu_np                                   # what the GPU produced for layer 1
            d_x_local, d_x_halo = h_gpu, to_dev(x_halo)
        dw = [to_dev(m) for m in layer.weights]
        h_gpu = binding.mgg_layer_forward(part, layer.mode, d_x_local, d_x_halo, dw, layer.acts, eps=layer.eps, order=order)
        torch.cuda.synchronize()
        h_gpu_np = h_gpu.float().cpu().numpy()
        # the oracle's layer, step by step (oracle.layer_forward is this composition): the aggregation is kept
        # for the error scale |agg| @ |W| chained through the linears
        agg = oracle.aggregate(w.row_ptr, w.col, layer.mode, x_local, lb=lb, ub=ub, x_halo=x_halo, halo_gid=hg,
                               eps=layer.eps, rows=rows)
        ref = agg
        for i, m in enumerate(layer.weights):
            ref = oracle.update(ref, m, None, layer.acts[i])
        s = np.abs(agg)
        del agg
        if order != "agg_first":
            # the product with the first matrix may run before the aggregation: rounding errors then scale
            # with sum_u |w_uv| (|x_u| @ |W|) instead of |sum_u w_uv x_u| @ |W|
            xa_l = np.abs(inputs.bf16_bits_to_f32(x_local)) if x_local.dtype == np.uint16 else np.abs(x_local)
            xa_h = np.abs(inputs.bf16_bits_to_f32(x_halo)) if x_halo.dtype == np.uint16 else np.abs(x_halo)
            s = oracle.aggregate(w.row_ptr, w.col, layer.mode, xa_l, lb=lb, ub=ub, x_halo=xa_h, halo_gid=hg,
                                 eps=abs(layer.eps), rows=rows)
        for m in layer.weights:
            s = s @ np.abs(oracle.to_f64(m))
        k = max(layer.dims[:-1])
        bound = BF16_LAYER_ATOL * s if bf16 else 2e-6 * s + 2.0 * k * 2.0 ** -24 * s
        got = h_gpu_np.astype(np.float64)
        if rows is not None:
            got = got[np.asarray(rows)]
        ratio = assert_close(got, ref, 2e-2 if bf16 else 1e-4, bound, f"{w.name} layer {li}")
        if report is not None:
            report(f"{w.name} layer {li} ({order})", ratio)
        del ref, s, got
    part.destroy()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_layers_of_the_five_configs_scaled(cfg):
    run_config_layers(inputs.config(cfg, shrink=SHRINK[cfg]))


def test_aggregate_cfg2_full_size_every_row():
    """Config 2 at full size, in the launch configuration bench.py times: every owned row against the oracle."""
    w = inputs.config(2)
    check_aggregate(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, w.x, "gcn", what="cfg2 full aggregation", report=report_ratio)
    run_config_layers(w, report=report_ratio)


# ----------------------------------------------------------------------------- run-time search
def test_tune_aggregate_runs_the_search_on_the_gpu():
    """mgg_tune_aggregate drives the propose / report search with measured latencies: every
    trial is a legal configuration measured once, the winner is the table's minimum, and a
    partition built with the winning knobs still matches the oracle."""
    w = inputs.config(2, shrink=4)
    ref_part = oracle.build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    lb, ub, hg = ref_part["lb"], ref_part["ub"], ref_part["halo_gid"]
    xl, xh = to_dev(w.x[lb:ub]), to_dev(w.x[hg])
    out = torch.empty((ub - lb, w.dim), dtype=torch.float32, device=DEV)
    tuner = binding.Tuner(32, 16, 16)
    best, best_ms = binding.mgg_tune_aggregate(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, "gcn", xl, xh, out,
                                               tuner, iters=3)
    table = tuner.table()
    assert tuner.next() is None                                     # the search has ended
    assert table[0][0] == (1, 1, 1) and table[1][0] == (2, 1, 1)    # all knobs start at 1, ps moves first
    assert len({k for k, _ in table}) == len(table) <= 6 + 5 + 5 + 30
    assert all(ps in (1, 2, 4, 8, 16, 32) and d in (1, 2, 4, 8, 16) and b in (1, 2, 4, 8, 16) for (ps, d, b), _ in table)
    assert all(ms > 0 for _, ms in table)
    assert (best, best_ms) == min(table, key=lambda kv: kv[1])
    assert best_ms < table[0][1]                                    # better than the starting point
    tuner.destroy()
    check_aggregate(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, w.x, "gcn",
                    build=dict(ps=best[0], dist=best[1], wpb=best[2]), what=f"tuned {best}")


# ----------------------------------------------------------------------------- full-size workloads
def _column_sum_check(w, out, mode, eps, rtol):
    """Property that holds at any size: summing the output over the owned rows gives
    sum_u c_u x_u with c_u = sum over owned rows v that list u of the edge weight (plus the self
    term); computed here with numpy reductions over the edge list, not with the oracle's row loop."""
    lb, ub = w.lb, w.ub
    rp, col = w.row_ptr, w.col
    n = rp.size - 1
    x = inputs.bf16_bits_to_f32(w.x).astype(np.float64) if w.x.dtype == np.uint16 else w.x.astype(np.float64)
    deg = np.diff(rp).astype(np.float64)
    src = col[rp[lb]:rp[ub]]
    dst = np.repeat(np.arange(lb, ub), np.diff(rp)[lb:ub])
    if mode == "gcn":
        dinv = 1.0 / np.sqrt(deg + 1.0)
        c = np.bincount(src, weights=dinv[src] * dinv[dst], minlength=n)
        c[lb:ub] += dinv[lb:ub] ** 2
    else:
        c = np.bincount(src, minlength=n).astype(np.float64)
        c[lb:ub] += 1.0 + eps
    want = c @ x
    scale = np.abs(c) @ np.abs(x)
    got = out.double().sum(dim=0).cpu().numpy()
    assert np.all(np.abs(got - want) <= rtol * scale), f"{w.name}: column-sum checksum off by {np.abs(got - want).max():.3e}"


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_full_size_aggregation_every_row_and_checksum(cfg):
    """Configs 3-5 at full size in the layout bench.py times (rows padded to 16-byte multiples where
    needed): every owned row of the aggregation against the oracle, and the column sums of the whole
    output in closed form (computed from the edge list with numpy reductions, not by the oracle's loop)."""
    w = inputs.config(cfg)
    layer = w.layers[0]
    esz = 2 if w.dtype == "bf16" else 4
    ld_pad = (-w.dim) % (128 // esz) if (w.dim * esz) % 16 else 0
    got = check_aggregate(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, w.x, layer.mode, eps=layer.eps, ld_pad=ld_pad,
                          what=f"cfg{cfg} full aggregation", report=report_ratio)
    _column_sum_check(w, torch.from_numpy(got), layer.mode, layer.eps, 1e-5)


@pytest.mark.parametrize("cfg,order", [(3, "agg_first"), (4, "agg_first"), (4, "update_first"), (5, "agg_first"), (5, "update_first")])
def test_full_size_layers_every_row(cfg, order):
    """Every row of every layer's output of configs 3-5 at full size, in both orders of aggregation and
    first product for the two configs whose weights narrow the rows."""
    run_config_layers(inputs.config(cfg), order=order, report=report_ratio)


def test_edge_balanced_shares_on_the_gpu():
    """The node ranges of Algorithm 1 (about E / P edges each) as partition bounds: every share of a
    shrunken config 2 against the oracle, and the shares together against the one-partition result."""
    w = inputs.config(2, shrink=4)
    n = w.row_ptr.size - 1
    bounds = binding.mgg_split_edge_balanced(w.row_ptr, 4)
    assert np.array_equal(bounds, oracle.split_edge_balanced(w.row_ptr, 4))
    edges = np.diff(w.row_ptr[bounds])
    assert edges.max() < 2 * edges.mean()                 # against 57 % of all edges in share 0 of the equal-node split
    whole = check_aggregate(w.row_ptr, w.col, 1, 0, np.array([0, n]), w.x, "gcn")
    pieces = [check_aggregate(w.row_ptr, w.col, 4, p, bounds, w.x, "gcn", what=f"edge-balanced share {p}") for p in range(4)]
    np.testing.assert_allclose(np.concatenate(pieces), whole, rtol=2e-4, atol=2e-6)


# ----------------------------------------------------------------------------- Update before Aggregate
@pytest.mark.parametrize("cfg", [4, 5])
@pytest.mark.parametrize("order", ["update_first", "auto"])
def test_update_first_order_on_the_narrowing_configs(cfg, order):
    """Aggregate(X) W = Aggregate(X W) (section 7 writes the layer as one product A-hat X W):
    configs 4 (602 -> 256) and 5 (100 -> 256 -> 47) through the reordered path."""
    run_config_layers(inputs.config(cfg, shrink=SHRINK[cfg]), order=order)


@pytest.mark.parametrize("mode,bf16,dims,acts,with_bias", [
    ("gcn", False, (64, 47), ("relu",), True), ("gcn", False, (100, 5), ("none",), True),
    ("gin", False, (96, 32, 17), ("relu", "none"), True), ("gin", True, (128, 64, 130), ("relu", "relu"), False),
    ("gcn", True, (136, 24), ("relu",), False), ("gcn", False, (33, 64), ("relu",), True),
    ("gcn", False, (64, 47), ("softmax",), True), ("gin", False, (96, 32, 10), ("relu", "softmax"), True)])
def test_update_first_matches_the_oracle(mode, bf16, dims, acts, with_bias):
    row_ptr, col, rng = small_rmat(seed=5)
    n = row_ptr.size - 1
    bounds = inputs.equal_node_bounds(n, 3)
    x = rng.standard_normal((n, dims[0])).astype(np.float32)
    weights = [(0.1 * rng.standard_normal((dims[i], dims[i + 1]))).astype(np.float32) for i in range(len(dims) - 1)]
    biases = [rng.standard_normal(dims[i + 1]).astype(np.float32) if with_bias else None for i in range(len(dims) - 1)]
    if bf16:
        x, weights = inputs.to_bf16_bits(x), [inputs.to_bf16_bits(m) for m in weights]
    for p in range(3):
        ref_part = oracle.build_partition(row_ptr, col, 3, p, bounds)
        lb, ub, hg = ref_part["lb"], ref_part["ub"], ref_part["halo_gid"]
        part = binding.mgg_build_partition(row_ptr, col, 3, p, bounds, xcd_min_deg=30)
        d_b = [None if b is None else to_dev(b) for b in biases]
        got = {}
        for order in ("agg_first", "update_first"):
            # an output view with padded rows checks that nothing is written beyond the last column
            buf = torch.full((ub - lb, dims[-1] + 3), float("nan"), dtype=torch.float32, device=DEV)
            out = binding.mgg_layer_forward(part, mode, to_dev(x[lb:ub]), to_dev(x[hg]) if hg.size else None,
                                            [to_dev(m) for m in weights], acts, eps=0.25, biases=d_b, out=buf[:, :dims[-1]],
                                            order=order)
            torch.cuda.synchronize()
            assert torch.isnan(buf[:, dims[-1]:]).all()
            got[order] = to_host64(out)
        ref = oracle.layer_forward(row_ptr, col, mode, x[lb:ub], weights, acts, eps=0.25, lb=lb, ub=ub, x_halo=x[hg],
                                   halo_gid=hg, biases=biases)
        xa = np.abs(inputs.bf16_bits_to_f32(x)) if bf16 else np.abs(x)
        s = oracle.aggregate(row_ptr, col, mode, xa[lb:ub], lb=lb, ub=ub, x_halo=xa[hg], halo_gid=hg, eps=0.25)
        for i, m in enumerate(weights):
            s = s @ np.abs(oracle.to_f64(m)) + (0 if biases[i] is None else np.abs(biases[i]))
        bound = BF16_LAYER_ATOL * s if bf16 else 2e-6 * s + 2.0 * max(dims[:-1]) * 2.0 ** -24 * s
        for order in got:
            assert_close(got[order], ref, 2e-2 if bf16 else 1e-4, bound, f"{mode} {dims} part {p} {order}")
        part.destroy()


@pytest.mark.parametrize("seed", range(24))
def test_aggregate_random_graphs_and_schedules(seed):
    """Seeded random cases: small graphs with hubs, duplicates, self-loops and empty rows, random
    widths, dtypes, modes, shares and schedule knobs."""
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.integers(2, 400))
    hubs = rng.integers(0, n, size=3)
    rows = []
    for v in range(n):
        d = int(rng.choice([0, 1, 3, 17, 40, 300 if v in hubs else 5]))
        rows.append(sorted(rng.integers(0, n, size=d).tolist()))
    row_ptr, col = inputs.csr_from_adjacency_lists(rows)
    parts = int(rng.integers(1, 5))
    bounds = np.array([0] + sorted(rng.integers(0, n + 1, size=parts - 1).tolist()) + [n], dtype=np.int64)
    dim = int(rng.choice([1, 5, 16, 47, 64, 100, 130, 256, 602]))
    bf16 = bool(rng.integers(0, 2))
    mode = str(rng.choice(["gcn", "gin"]))
    x = rng.standard_normal((n, dim)).astype(np.float32)
    if bf16:
        x = inputs.to_bf16_bits(x)
    build = dict(ps=int(rng.choice([1, 4, 32, 64])), dist=int(rng.choice([1, 2, 16])), short_max=int(rng.choice([-1, 2, 16])),
                 wpb=int(rng.choice([1, 4, 8])), xcd_min_deg=int(rng.choice([-1, 1, 20, 256])),
                 hot_phases=int(rng.choice([-1, 0, 2])), hot_rows=int(rng.choice([0, 3, 50])), min_piece=int(rng.choice([1, 4, 16])))
    ld_pad = int(rng.choice([0, 0, 3, 8]))
    for p in range(parts):
        if bounds[p + 1] > bounds[p]:
            check_aggregate(row_ptr, col, parts, p, bounds, x, mode, eps=float(rng.choice([0.0, 0.5, -1.0])), build=build,
                            ld_pad=ld_pad, what=f"seed {seed} part {p} dim {dim} {build}")


# ----------------------------------------------------------------------------- HIP graph capture
def test_layer_forward_captured_without_any_eager_call():
    """A layer forward takes everything it needs from its arguments (the partial sums of cut rows pass
    through the workspace): the very first call on a fresh partition can be the one that is captured,
    at a width no earlier call ever used."""
    w = inputs.config(5, shrink=5)
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    assert part.info.n_split_items > 0 and part.info.reserved_dim == 0
    hg = part.export()["halo_gid"]
    rng = np.random.default_rng(11)
    dims = (328, 72)                                     # wider than anything this partition has seen (nothing)
    x = rng.standard_normal((w.row_ptr.size - 1, dims[0])).astype(np.float32)
    wt = (0.1 * rng.standard_normal(dims)).astype(np.float32)
    xl, xh, dw = to_dev(x[w.lb:w.ub]), to_dev(x[hg]), [to_dev(wt)]
    wsp = torch.empty(binding.mgg_layer_workspace_bytes(part, "gcn", dw, ["relu"]), dtype=torch.uint8, device=DEV)
    out = torch.full((int(part.info.n_own), dims[1]), float("nan"), device=DEV)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        binding.mgg_layer_forward(part, "gcn", xl, xh, dw, ["relu"], workspace=wsp, out=out)
    torch.cuda.synchronize()
    for rep in range(3):
        out.fill_(float("nan"))
        wsp.random_(0, 255)                              # whatever the workspace held must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = to_host64(out)
        ref = oracle.layer_forward(w.row_ptr, w.col, "gcn", x[w.lb:w.ub], [wt], ["relu"], lb=w.lb, ub=w.ub, x_halo=x[hg], halo_gid=hg)
        agg = oracle.aggregate(w.row_ptr, w.col, "gcn", x[w.lb:w.ub], lb=w.lb, ub=w.ub, x_halo=x[hg], halo_gid=hg)
        s = np.abs(agg) @ np.abs(wt).astype(np.float64)
        assert_close(got, ref, 1e-4, 2e-6 * s + 2.0 * dims[0] * 2.0 ** -24 * s, f"captured layer, replay {rep}")
    info = binding.PartitionInfo()
    import ctypes
    binding.lib().mgg_partition_info(part.handle, ctypes.byref(info))
    assert info.reserved_dim == 0
    part.destroy()


def test_aggregate_refuses_a_width_that_was_not_reserved():
    """mgg_aggregate allocates nothing: on a partition that cuts rows into several items the width has to
    be reserved first (the Python binding does that on its own; the raw call is made here)."""
    import ctypes
    w = inputs.config(2, shrink=5)
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds, reserve_dim=32)
    assert part.info.n_split_items > 0 and part.info.reserved_dim == 32
    hg = part.export()["halo_gid"]
    xl, xh = to_dev(w.x[w.lb:w.ub]), to_dev(w.x[hg])
    out = torch.full((int(part.info.n_own), w.dim), 3.0, device=DEV)
    lib = binding.lib()
    args = (part.handle, binding.AGG_GCN_SYM, ctypes.c_float(0.0), binding.F32, ctypes.c_void_p(xl.data_ptr()), ctypes.c_void_p(xh.data_ptr()))
    st = lib.mgg_aggregate(*args, w.dim, w.dim, ctypes.c_void_p(out.data_ptr()), w.dim, None)
    assert st == binding.ERR_INVALID_ARG and b"mgg_partition_reserve" in lib.mgg_last_error()
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
    st = lib.mgg_aggregate(*args, 32, w.dim, ctypes.c_void_p(out.data_ptr()), w.dim, None)      # the reserved width works
    assert st == binding.OK
    assert lib.mgg_partition_reserve(part.handle, w.dim) == binding.OK
    st = lib.mgg_aggregate(*args, w.dim, w.dim, ctypes.c_void_p(out.data_ptr()), w.dim, None)
    assert st == binding.OK
    torch.cuda.synchronize()
    want = binding.mgg_aggregate(part, "gcn", xl, xh)
    assert torch.equal(out, want)
    part.destroy()


def test_layer_forward_in_a_hip_graph():
    """A layer forward allocates nothing, synchronises nothing and records no memset, so it can be
    captured in a HIP graph.  Every replay -- with new inputs, and with eager work and
    synchronisations in between -- must reproduce the eager result bit for bit."""
    w = inputs.config(2, shrink=5)
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    hg = part.export()["halo_gid"]
    layer = w.layers[0]
    xl, xh = to_dev(w.x[w.lb:w.ub]), to_dev(w.x[hg])
    ws = [to_dev(m) for m in layer.weights]
    wsp = torch.empty(binding.mgg_layer_workspace_bytes(part, layer.mode, ws, layer.acts), dtype=torch.uint8, device=DEV)
    out = torch.empty((int(part.info.n_own), layer.dims[-1]), device=DEV)
    side = torch.empty(1 << 20, device=DEV)

    def forward():
        binding.mgg_layer_forward(part, layer.mode, xl, xh, ws, layer.acts, workspace=wsp, out=out)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        forward()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        forward()
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    for rep in range(4):
        xl.copy_(to_dev(rng.standard_normal(tuple(xl.shape)).astype(np.float32)))
        xh.copy_(to_dev(rng.standard_normal(tuple(xh.shape)).astype(np.float32)))
        with torch.cuda.stream(stream):
            forward()
        torch.cuda.synchronize()
        want = out.clone()
        out.fill_(float("nan"))
        side.normal_()                              # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep} differs from the eager result"
    part.destroy()


def test_gather_probe_orders_the_memory_levels():
    """The bare gather kernel behind the roofline table: rows from a table inside L2 arrive faster than
    rows from a table in the Infinity Cache, and those faster than rows from HBM."""
    l2 = binding.mgg_probe_gather(2 << 20, 256, n_gathers=1 << 22, iters=3)
    mall = binding.mgg_probe_gather(64 << 20, 256, n_gathers=1 << 22, iters=3)
    hbm = binding.mgg_probe_gather(2 << 30, 1024, n_gathers=1 << 22, iters=3)
    assert l2 > mall > 0 and l2 > hbm > 0
    assert l2 > 8000.0                                   # beyond the HBM peak: a cache figure


# ----------------------------------------------------------------------------- embedding bags
@pytest.mark.parametrize("dim,bf16,lo_hi,knobs", [(64, False, (0, 5000), {}), (16, False, (2000, 2600), dict(ps=8, dist=2)),
                                                   (128, True, (0, 20000), {}), (47, False, (0, 0), dict(xcd_min_deg=16)),
                                                   (100, True, (19000, 20000), dict(hot_phases=2, hot_rows=64)), (256, False, (3, 9), dict(short_max=-1))])
def test_bag_sum(dim, bf16, lo_hi, knobs):
    """Embedding-bag sum through the aggregation path (section 8.3): Zipf-distributed lookups, empty
    and very large bags, the table cut into a local slice and a halo table of the distinct other rows."""
    rng = np.random.default_rng(dim)
    table_rows, n_bags = 20000, 3000
    sizes = rng.integers(0, 60, size=n_bags)
    sizes[:4] = [0, 1, 3000, 17]
    ptr = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    idx = ((rng.zipf(1.1, size=ptr[-1]) - 1) % table_rows).astype(np.int32)
    table = rng.standard_normal((table_rows, dim)).astype(np.float32)
    if bf16:
        table = inputs.to_bf16_bits(table)
    lo, hi = lo_hi
    part = binding.mgg_build_bags(ptr, idx, table_rows, lo, hi, **knobs)
    hg = part.export()["halo_gid"]
    t_local = to_dev(table[lo:hi]) if hi > lo else None
    t_halo = to_dev(table[hg]) if hg.size else None
    buf = torch.full((n_bags, dim + 3), float("nan"), dtype=torch.float32, device=DEV)
    out = binding.mgg_bag_sum(part, t_local, t_halo, out=buf[:, :dim], dim=dim)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:, dim:]).all()
    ref = oracle.bag_sum(ptr, idx, table)
    scale = oracle.bag_sum(ptr, idx, np.abs(inputs.bf16_bits_to_f32(table)) if bf16 else np.abs(table))
    got = to_host64(out)
    assert np.all(np.abs(got - ref) <= 1e-6 * np.maximum(1.0, scale) + 1e-4 * np.abs(ref)), np.abs(got - ref).max()
    assert np.all(got[0] == 0.0)                                    # the empty bag
    with pytest.raises(binding.MggError):
        binding.mgg_aggregate(part, "gin", t_local if t_local is not None else t_halo, t_halo)
    part.destroy()
