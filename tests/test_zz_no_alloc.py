"""mgg_aggregate_static: the entry point that allocates nothing (the partial sums of cut rows go to a
fixed array inside the library's device code) against mgg_aggregate, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2209_06800_amd import binding, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(shrink, dim, mode, seed):
    """One share of the R-MAT workload of config 2, shrunk: (partition, x_local, x_halo, oracle value)."""
    w = inputs.config(2, shrink=shrink)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((w.row_ptr.size - 1, dim)).astype(np.float32)
    ref_part = oracle.build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    hg = ref_part["halo_gid"]
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    assert part.info.n_split_items > 0, "the case must cut rows into several items, or no scratch is used"
    ref = oracle.aggregate(w.row_ptr, w.col, mode, x[w.lb:w.ub], lb=w.lb, ub=w.ub, x_halo=x[hg], halo_gid=hg, eps=0.25)
    return part, torch.from_numpy(x[w.lb:w.ub]).to(DEV), torch.from_numpy(x[hg]).to(DEV), ref


def test_static_scratch_entry_point_matches_mgg_aggregate():
    """Two calls in a row, the second on a smaller partition and a narrower width (the array keeps the
    first call's contents): each equals mgg_aggregate bit for bit (same kernels, same order of the
    partial sums) and meets the fp32 bar against the oracle.  The static call comes first, on a partition
    for which nothing was ever reserved."""
    for shrink, dim, mode, seed in ((3, 100, "gcn", 1), (5, 48, "gin", 2)):
        part, xl, xh, ref = _case(shrink, dim, mode, seed)
        assert part.info.reserved_dim == 0
        out = torch.full((int(part.info.n_own), dim + 4), float("nan"), device=DEV)
        got = binding.mgg_aggregate_static(part, mode, xl, xh, eps=0.25, out=out[:, :dim])
        torch.cuda.synchronize()
        assert torch.isnan(out[:, dim:]).all()
        info = binding.PartitionInfo()
        binding.lib().mgg_partition_info(part.handle, ctypes.byref(info))
        assert info.reserved_dim == 0                      # the static call reserved nothing on the partition
        want = binding.mgg_aggregate(part, mode, xl, xh, eps=0.25)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        g = got.double().cpu().numpy()
        if mode == "gcn":
            assert np.all(np.abs(g - ref) <= 1e-6 + 1e-4 * np.abs(ref))
        else:                                              # unnormalised sums: the absolute term follows sum |x_u|
            args, kwargs = _abs_args(shrink, dim, seed)
            s = oracle.aggregate(*args, **kwargs)
            assert np.all(np.abs(g - ref) <= 1e-6 * np.maximum(1.0, s) + 1e-4 * np.abs(ref))
        part.destroy()


def _abs_args(shrink, dim, seed):
    w = inputs.config(2, shrink=shrink)
    rng = np.random.default_rng(seed)
    x = np.abs(rng.standard_normal((w.row_ptr.size - 1, dim)).astype(np.float32))
    hg = oracle.build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)["halo_gid"]
    return (w.row_ptr, w.col, "gin", x[w.lb:w.ub]), dict(lb=w.lb, ub=w.ub, x_halo=x[hg], halo_gid=hg, eps=0.25)


def test_static_scratch_refuses_what_does_not_fit():
    """A partition whose partial sums at the given width exceed the fixed array is an error, not a launch."""
    w = inputs.config(2, shrink=3)
    part = binding.mgg_build_partition(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)
    dim = 1
    while binding.mgg_aggregate_scratch_bytes(part, dim) <= (64 << 20):
        dim *= 2
    n, h = int(part.info.n_own), int(part.info.num_halo)
    xl, xh = torch.zeros((n, dim), device=DEV), torch.zeros((h, dim), device=DEV)
    out = torch.full((n, dim), 7.0, device=DEV)
    with pytest.raises(binding.MggError) as e:
        binding.mgg_aggregate_static(part, "gcn", xl, xh, out=out)
    assert e.value.status == binding.ERR_UNSUPPORTED and "fixed scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                        # nothing was written
    # half that width fits
    binding.mgg_aggregate_static(part, "gcn", xl[:, : dim // 2], xh[:, : dim // 2], out=out[:, : dim // 2])
    torch.cuda.synchronize()
    part.destroy()
