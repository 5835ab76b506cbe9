"""CPU-only checks of libmgg: the library loads and exports every symbol the header declares,
the host partition builder agrees bit for bit with the oracle's independent builder, work
items form a valid schedule, and bad arguments come back as error codes."""
import ctypes
import json
import os
import re

import numpy as np
import pytest

import oracle
from paper_2209_06800_amd import binding, inputs
from paper_2209_06800_amd.binding import MggError

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mgg.h")).read()
    declared = set(re.findall(r"\b(mgg_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTED_SYMBOLS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in binding.mgg_version()


def _compare_with_oracle(row_ptr, col, parts, p, bounds, **opts):
    want = oracle.build_partition(row_ptr, col, parts, p, bounds)
    part = binding.mgg_build_partition(row_ptr, col, parts, p, bounds, host_only=True, **opts)
    got = part.export()
    info = part.info
    assert (info.lb, info.ub, info.n_own) == (want["lb"], want["ub"], want["n_own"])
    assert info.on_device == 0
    for key in ("local_row_ptr", "local_col", "remote_row_ptr", "remote_col", "halo_gid", "halo_peer_ptr",
                "deg_own", "deg_halo"):
        assert np.array_equal(got[key].astype(np.int64), want[key].astype(np.int64)), key
    for kind in ("local", "remote"):
        row, start, end = oracle.neighbor_groups(want[f"{kind}_row_ptr"], info.ps)
        assert np.array_equal(got[f"grp_{kind}_row"], row)
        assert np.array_equal(got[f"grp_{kind}_start"], start)
        assert np.array_equal(got[f"grp_{kind}_end"], end)
    hp = opts.get("hot_phases", 0)
    if opts.get("xcd_min_deg", 0) < 0:
        assert info.class_mode == 0
    elif hp != 0:
        assert info.class_mode == (2 if hp > 0 else 1)
    else:
        assert info.class_mode in (1, 2)                     # the library chooses
    _check_schedule(got, info, hot_by_popularity=info.class_mode == 2)
    part.destroy()
    return got, info


def _source_class(x):
    return ((x.astype(np.uint64) * np.uint64(0x9E3779B1)) & np.uint64(0xFFFFFFFF)) >> np.uint64(29)


def _check_schedule(got, info, hot_by_popularity=True):
    """Several schedules are valid; check that this one covers every neighbour exactly once,
    keeps items within one row and within ps * dist neighbours per list, uses each scratch slot
    once, walks a per-row permutation of the canonical columns, and -- for rows regrouped by
    source class -- gives every item a single class equal to the XCD its workgroup lands on."""
    n_own = info.n_own
    lrp, rrp = got["local_row_ptr"].astype(np.int64), got["remote_row_ptr"].astype(np.int64)
    deg = np.diff(lrp) + np.diff(rrp)
    seen_rows = np.zeros(n_own, dtype=np.int64)
    np.add.at(seen_rows, got["short_rows"], 1)
    if info.short_max >= 0:
        assert np.all(deg[got["short_rows"]] <= info.short_max)
        assert np.all(np.diff(deg[got["short_rows"]]) <= 0)            # longest first
    run = info.ps * info.dist
    valid = got["item_row"] >= 0                                       # the rest is padding
    pos = np.nonzero(valid)[0]
    rows = got["item_row"][valid].astype(np.int64)
    lbeg, lend = got["item_lbeg"][valid].astype(np.int64), got["item_lend"][valid].astype(np.int64)
    rbeg, rend = got["item_rbeg"][valid].astype(np.int64), got["item_rend"][valid].astype(np.int64)
    slots = got["item_slot"][valid]
    assert np.all(got["item_slot"][~valid] == -1)
    item_rows = np.unique(rows)
    seen_rows[item_rows] += 1
    assert np.all(seen_rows == 1)                                      # every row in exactly one bin
    for beg, end, rp in ((lbeg, lend, lrp), (rbeg, rend, rrp)):
        assert np.all(end - beg <= run) and np.all(end >= beg)
        assert np.all(beg >= rp[rows]) and np.all(end <= rp[rows + 1])  # inside the item's row
        ne = end > beg
        order = np.argsort(beg[ne], kind="stable")
        b, e = beg[ne][order], end[ne][order]
        assert np.all(e[:-1] <= b[1:])                                  # no neighbour twice
        cover = np.zeros(n_own, dtype=np.int64)
        np.add.at(cover, rows, end - beg)
        assert np.array_equal(cover[item_rows], np.diff(rp)[item_rows])   # no neighbour missed
    whole = slots < 0
    counts = np.bincount(rows, minlength=n_own)
    assert np.all(counts[rows[whole]] == 1) and np.all(counts[rows[~whole]] > 1)
    assert np.array_equal(np.sort(slots[~whole]), np.arange(info.n_split_items))
    assert info.n_split_rows == np.unique(rows[~whole]).size
    assert info.n_groups_local == int(np.sum(-(-np.diff(lrp) // info.ps)))
    assert info.n_groups_remote == int(np.sum(-(-np.diff(rrp) // info.ps)))
    # the kernel's column order is the canonical one permuted inside each row
    for canon, sched, rp in ((got["local_col"], got["sched_local_col"], lrp), (got["remote_col"], got["sched_remote_col"], rrp)):
        row_of = np.repeat(np.arange(n_own, dtype=np.int64), np.diff(rp))
        big = np.int64(1) << 32
        assert np.array_equal(np.sort(row_of * big + canon), np.sort(row_of * big + sched))
    if info.xcd_min_deg > 0:
        assert got["item_row"].size % (8 * info.wpb) == 0                # 8 XCDs x wpb items per workgroup
        xcd = (pos // info.wpb) % 8
        cl, ch = got["src_class_local"], got["src_class_halo"]
        n_hot = 8 * info.n_phases
        assert np.all((cl >= -1) & (cl < n_hot)) and np.all((ch >= -1) & (ch < n_hot))
        if hot_by_popularity:
            # classes follow the gather counts: every hot class holds at most hot_rows table rows, no row of
            # phase p + 1 is gathered more often than a row of phase p, cold rows are the least gathered
            cnt = np.concatenate([np.bincount(got["local_col"], minlength=n_own),
                                  np.bincount(got["remote_col"], minlength=info.num_halo)])
            cls = np.concatenate([cl, ch])
            if n_hot:
                assert np.bincount(cls[cls >= 0], minlength=n_hot).max() <= info.hot_rows
                assert cnt[cls >= 0].min() >= info.hot_min_count
                lo = [cnt[(cls >= 0) & (cls // 8 == ph)].min() for ph in range(info.n_phases)]
                hi = [cnt[(cls >= 0) & (cls // 8 == ph)].max() for ph in range(info.n_phases)]
                assert all(lo[i] >= hi[i + 1] for i in range(info.n_phases - 1))
                if (cls < 0).any():
                    assert cnt[cls < 0].max() <= lo[-1]
                # phase 0 is dealt round-robin: the 8 classes of a phase differ by at most one row
                sizes = np.bincount(cls[(cls >= 0) & (cls < 8)], minlength=8)
                assert sizes.max() - sizes.min() <= 1
        # an item of a regrouped row gathers rows of one class only; a hot item runs on the XCD of its class,
        # after every item of an earlier phase in that XCD's queue; hot pieces hold at least min_piece neighbours
        regrouped = np.nonzero(deg[rows] >= info.xcd_min_deg)[0]
        rng = np.random.default_rng(0)
        last_phase = np.full(8, -1)
        piece_size = {}
        for i in (regrouped if regrouped.size <= 6000 else np.sort(rng.choice(regrouped, 6000, replace=False))):
            c = np.concatenate([cl[got["sched_local_col"][lbeg[i]:lend[i]]], ch[got["sched_remote_col"][rbeg[i]:rend[i]]]])
            if c.size == 0:
                continue
            r = rows[i]
            row_cls = np.concatenate([cl[got["local_col"][lrp[r]:lrp[r + 1]]], ch[got["remote_col"][rrp[r]:rrp[r + 1]]]])
            row_count = np.bincount(row_cls[row_cls >= 0], minlength=max(n_hot, 1))   # neighbours of this row per class
            hot = c[c >= 0]
            if hot.size == c.size and np.all(hot == hot[0]) and row_count[hot[0]] >= info.min_piece:
                assert hot[0] % 8 == xcd[i]
                assert hot[0] // 8 >= last_phase[xcd[i]]
                last_phase[xcd[i]] = hot[0] // 8
                piece_size[(r, hot[0])] = piece_size.get((r, hot[0]), 0) + c.size
            else:
                # the row's cold piece: cold rows plus classes too small to stand alone
                assert np.all(row_count[hot] < info.min_piece)
        if regrouped.size <= 6000:
            for (r, h), v in piece_size.items():                         # a hot piece is never cut short
                row_cls = np.concatenate([cl[got["local_col"][lrp[r]:lrp[r + 1]]], ch[got["remote_col"][rrp[r]:rrp[r + 1]]]])
                assert v == np.count_nonzero(row_cls == h)
    else:
        assert np.array_equal(got["sched_local_col"], got["local_col"])
        assert np.array_equal(got["sched_remote_col"], got["remote_col"])
        assert np.all(valid)
        assert np.all(got["src_class_local"] == -1) and np.all(got["src_class_halo"] == -1)


def test_partition_matches_hand_written_fixture():
    fx = json.load(open(os.path.join(GOLDEN, "tiny_partition.json")))
    row_ptr, col = inputs.csr_from_adjacency_lists(fx["adjacency"])
    for p, want in enumerate(fx["parts"]):
        part = binding.mgg_build_partition(row_ptr, col, 2, p, fx["bounds"], ps=2, host_only=True)
        got = part.export()
        for key in ("local_row_ptr", "local_col", "remote_row_ptr", "remote_col", "halo_gid", "halo_peer_ptr",
                    "deg_own", "deg_halo"):
            assert got[key].tolist() == want[key], (p, key)
        for kind in ("local", "remote"):
            g = want[f"groups_ps2_{kind}"]
            assert got[f"grp_{kind}_row"].tolist() == g["row"]
            assert got[f"grp_{kind}_start"].tolist() == g["start"]
            assert got[f"grp_{kind}_end"].tolist() == g["end"]


@pytest.mark.parametrize("xcd_min_deg", [-1, 1, 24, 300])
@pytest.mark.parametrize("parts,ps,dist,short_max", [(1, 0, 0, 0), (4, 32, 16, 16), (4, 2, 1, -1), (3, 7, 3, 5),
                                                     (8, 64, 1, 40), (2, 1, 1, 1)])
def test_partition_bit_exact_against_oracle(parts, ps, dist, short_max, xcd_min_deg):
    wpb = {-1: 0, 1: 1, 24: 16, 300: 3}[xcd_min_deg]
    hot = {-1: {}, 1: dict(hot_rows=16, hot_phases=3, min_piece=1, hot_min_count=1),
           24: dict(hot_rows=40, hot_phases=31, min_piece=3, hot_min_count=2), 300: dict(hot_phases=-1)}[xcd_min_deg]
    rng = np.random.default_rng(parts * 100 + ps)
    row_ptr, col = inputs.rmat_graph(12, 50000, 0.57, 0.19, 0.19, 0.05, rng)
    n = row_ptr.size - 1
    bounds = inputs.equal_node_bounds(n, parts)
    for p in range(parts):
        _compare_with_oracle(row_ptr, col, parts, p, bounds, ps=ps, dist=dist, short_max=short_max,
                             xcd_min_deg=xcd_min_deg, wpb=wpb, **hot)


def test_partition_with_self_loops_duplicates_and_empty_ranges():
    row_ptr, col = inputs.csr_from_adjacency_lists([[0, 1, 1, 3], [0], [], [0, 3, 3]])
    bounds = [0, 2, 2, 4]                     # the middle range is empty
    for p in range(3):
        got, info = _compare_with_oracle(row_ptr, col, 3, p, np.array(bounds), ps=2, dist=1, short_max=-1)
    assert info.n_own == 2
    empty = binding.mgg_build_partition(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), host_only=True)
    assert empty.info.n_own == 0 and empty.info.n_items == 0


def test_default_bounds_are_the_equal_node_split():
    rng = np.random.default_rng(5)
    row_ptr, col = inputs.rmat_graph(10, 5000, 0.45, 0.22, 0.22, 0.11, rng, n_nodes=1000)
    for parts in (1, 3, 7):
        b = inputs.equal_node_bounds(1000, parts)
        for p in range(parts):
            part = binding.mgg_build_partition(row_ptr, col, parts, p, None, host_only=True)
            assert (part.info.lb, part.info.ub) == (b[p], b[p + 1])


def test_scaled_configs_bit_exact():
    for cfg, shrink in ((2, 6), (3, 8), (5, 7)):
        w = inputs.config(cfg, shrink=shrink)
        _compare_with_oracle(w.row_ptr, w.col, w.parts, w.part_id, w.bounds)


def test_edge_balanced_split_matches_oracle():
    rng = np.random.default_rng(9)
    row_ptr, _ = inputs.rmat_graph(13, 100000, 0.57, 0.19, 0.19, 0.05, rng)
    for parts in (1, 2, 4, 8, 16, 31):
        assert np.array_equal(binding.mgg_split_edge_balanced(row_ptr, parts),
                              oracle.split_edge_balanced(row_ptr, parts))


def _status(fn, *a, **k):
    with pytest.raises(MggError) as e:
        fn(*a, **k)
    return e.value.status


def test_bad_arguments_are_error_codes_not_crashes():
    rp = np.array([0, 1, 2], dtype=np.int64)
    col = np.array([1, 0], dtype=np.int32)
    ho = dict(host_only=True)
    assert _status(binding.mgg_build_partition, np.array([0, 2, 1]), col, **ho) == binding.ERR_BAD_GRAPH
    assert _status(binding.mgg_build_partition, np.array([1, 1, 2]), col, **ho) == binding.ERR_BAD_GRAPH
    assert _status(binding.mgg_build_partition, rp, np.array([1, 2], dtype=np.int32), **ho) == binding.ERR_BAD_GRAPH
    assert _status(binding.mgg_build_partition, rp, np.array([-1, 0], dtype=np.int32), **ho) == binding.ERR_BAD_GRAPH
    assert _status(binding.mgg_build_partition, rp, col, 2, 2, **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_partition, rp, col, 2, -1, **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_partition, rp, col, 0, 0, **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_partition, rp, col, 2, 0, [0, 3, 2], **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_partition, rp, col, 2, 0, [0, 1, 3], **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_partition, rp, col, ps=65, **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_partition, rp, col, dist=-3, **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_partition, rp, col, wpb=17, **ho) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_set_option, "no_such_option", 1) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_set_option, "lds_halo", 7) == binding.ERR_INVALID_ARG
    lib = binding.lib()
    assert lib.mgg_build_partition(2, None, None, 1, 0, None, None, None) == binding.ERR_INVALID_ARG
    h = ctypes.c_void_p()
    assert lib.mgg_build_partition(2, None, None, 1, 0, None, None, ctypes.byref(h)) == binding.ERR_INVALID_ARG
    assert h.value is None and b"NULL" in lib.mgg_last_error()
    lib.mgg_partition_destroy(None)


def test_device_calls_refuse_a_host_only_partition():
    part = binding.mgg_build_partition(np.array([0, 1, 2]), np.array([1, 0], dtype=np.int32), host_only=True)
    lib = binding.lib()
    st = lib.mgg_aggregate(part.handle, 0, 0.0, 0, ctypes.c_void_p(256), None, 4, 4, ctypes.c_void_p(512), 4, None)
    assert st == binding.ERR_INVALID_ARG and b"host-only" in lib.mgg_last_error()
    assert lib.mgg_update(4, 0, None, 4, 4, 0, None, None, 4, 0, 0, None, 4, None) == binding.ERR_INVALID_ARG
    assert lib.mgg_update(4, 1, ctypes.c_void_p(256), 4, 4, 0, ctypes.c_void_p(256), None, 4, 0, 0,
                          ctypes.c_void_p(512), 4, None) == binding.ERR_UNSUPPORTED


def test_reserve_and_static_calls_refuse_a_host_only_partition():
    part = binding.mgg_build_partition(np.array([0, 1, 2]), np.array([1, 0], dtype=np.int32), host_only=True)
    lib = binding.lib()
    assert lib.mgg_partition_reserve(part.handle, 64) == binding.ERR_INVALID_ARG and b"host-only" in lib.mgg_last_error()
    assert lib.mgg_partition_reserve(None, 64) == binding.ERR_INVALID_ARG
    st = lib.mgg_aggregate_static(part.handle, 0, 0.0, 0, ctypes.c_void_p(256), None, 4, 4, ctypes.c_void_p(512), 4, None)
    assert st == binding.ERR_INVALID_ARG and b"host-only" in lib.mgg_last_error()
    assert binding.mgg_aggregate_scratch_bytes(part, 0) == 0
    assert part.info.reserved_dim == 0


def test_binding_checks_what_the_c_abi_cannot_see():
    """Both embedding tables travel as bare pointers with one leading dimension: a halo table of
    another dtype, device or row stride, or a buffer with too few rows, is refused before the call."""
    import torch
    rng = np.random.default_rng(8)
    row_ptr, col = inputs.rmat_graph(9, 4000, 0.57, 0.19, 0.19, 0.05, rng)
    part = binding.mgg_build_partition(row_ptr, col, 2, 0, None, host_only=True)
    n, h = int(part.info.n_own), int(part.info.num_halo)
    assert h > 0
    xl, xh = torch.zeros(n, 16), torch.zeros(h, 16)
    out = torch.zeros(n, 16)
    cases = {
        "stride": (xl, torch.zeros(h, 24)[:, :16], out),             # a padded halo table next to a contiguous local one
        "dtype": (xl, xh.to(torch.bfloat16), out),
        "short halo": (xl, xh[: h - 1], out),
        "short local": (xl[: n - 1], xh, out),
        "short out": (xl, xh, out[: n - 1]),
        "narrow out": (xl, xh, torch.zeros(n, 8)),
        "no halo": (xl, None, out),
    }
    for name, (a, b, o) in cases.items():
        with pytest.raises(ValueError):
            binding.mgg_aggregate(part, "gcn", a, b, out=o)
        with pytest.raises(ValueError):
            binding.mgg_aggregate_static(part, "gcn", a, b, out=o)
    with pytest.raises(ValueError):
        binding.mgg_layer_forward(part, "gcn", xl, torch.zeros(h, 24)[:, :16], [torch.zeros(16, 4)], ["none"],
                                  workspace=torch.zeros(8, dtype=torch.uint8))
    with pytest.raises(ValueError):
        binding.mgg_layer_forward(part, "gcn", xl, xh, [torch.zeros(16, 4)], ["none"], workspace=torch.zeros(8, dtype=torch.uint8),
                                  out=torch.zeros(n - 1, 4))
    # consistent tables pass the checks and reach the library, which refuses the host-only partition
    with pytest.raises((MggError, TypeError)):
        binding.mgg_aggregate(part, "gcn", xl, xh, out=out)


def test_aggregation_switches_belong_to_a_partition():
    """mgg_set_option sets the defaults new partitions start from; mgg_partition_set_option changes one
    partition and no other."""
    rp, col = np.array([0, 1, 2]), np.array([1, 0], dtype=np.int32)
    a = binding.mgg_build_partition(rp, col, host_only=True)
    binding.mgg_set_option("col_slab_bytes", 128)
    binding.mgg_set_option("items_per_wave", 3)
    try:
        b = binding.mgg_build_partition(rp, col, host_only=True)
    finally:
        binding.mgg_set_option("col_slab_bytes", 0)
        binding.mgg_set_option("items_per_wave", 0)
    assert (a.get_option("col_slab_bytes"), a.get_option("items_per_wave")) == (0, 0)        # built before: untouched
    assert (b.get_option("col_slab_bytes"), b.get_option("items_per_wave")) == (128, 3)
    a.set_option("lds_halo", 1)
    a.set_option("split_phases", 1)
    assert a.get_option("lds_halo") == 1 and b.get_option("lds_halo") == 0 and binding.mgg_get_option("lds_halo") == 0
    for key, bad in (("col_slab_bytes", 96), ("items_per_wave", 65), ("short_per_wave", -1), ("lds_halo", 2), ("update_stream", 1), ("nope", 0)):
        assert _status(a.set_option, key, bad) == binding.ERR_INVALID_ARG
    with pytest.raises(MggError):
        a.get_option("update_stream")
    lib = binding.lib()
    assert lib.mgg_partition_set_option(None, b"lds_halo", 1) == binding.ERR_INVALID_ARG


def test_gather_probe_checks_its_arguments():
    lib = binding.lib()
    g = ctypes.c_double()
    assert lib.mgg_probe_gather(1 << 20, 100, 1 << 20, 1, 1, ctypes.byref(g)) == binding.ERR_INVALID_ARG        # row size
    assert lib.mgg_probe_gather(64, 256, 1 << 20, 1, 1, ctypes.byref(g)) == binding.ERR_INVALID_ARG             # table smaller than a row
    assert lib.mgg_probe_gather(1 << 20, 256, 100, 1, 1, ctypes.byref(g)) == binding.ERR_INVALID_ARG            # too few gathers
    assert lib.mgg_probe_gather(1 << 20, 256, 1 << 20, 0, 1, ctypes.byref(g)) == binding.ERR_INVALID_ARG
    assert lib.mgg_probe_gather(1 << 20, 256, 1 << 20, 1, 1, None) == binding.ERR_INVALID_ARG


def test_options_round_trip():
    assert binding.mgg_get_option("items_per_wave") == 0
    for v in (1, 8, 64, 0):
        binding.mgg_set_option("items_per_wave", v)
        assert binding.mgg_get_option("items_per_wave") == v
    for bad in (-1, 65):
        assert _status(binding.mgg_set_option, "items_per_wave", bad) == binding.ERR_INVALID_ARG
    for key in ("split_phases", "lds_halo", "update_stream"):
        old = binding.mgg_get_option(key)
        binding.mgg_set_option(key, 1 - old)
        assert binding.mgg_get_option(key) == 1 - old
        binding.mgg_set_option(key, old)
    assert binding.mgg_get_option("col_slab_bytes") == 0
    for v in (1, 64, 128, 4096, 0):
        binding.mgg_set_option("col_slab_bytes", v)
        assert binding.mgg_get_option("col_slab_bytes") == v
    for bad in (-1, 3, 96, 8192):
        assert _status(binding.mgg_set_option, "col_slab_bytes", bad) == binding.ERR_INVALID_ARG


def test_layer_workspace_bytes_follow_the_order():
    """Host-side planning of mgg_layer_forward: the aggregate-first form needs the aggregation
    result (and the hidden activations of a 2-linear MLP); the update-first form needs the two
    transformed tables instead.  No GPU is touched: the weight pointers are never dereferenced."""
    rng = np.random.default_rng(3)
    row_ptr, col = inputs.rmat_graph(10, 8000, 0.57, 0.19, 0.19, 0.05, rng)
    part = binding.mgg_build_partition(row_ptr, col, 2, 0, None, host_only=True)
    n, h = part.info.n_own, part.info.num_halo
    lib = binding.lib()

    def need(dims, order, w_dtype=binding.F32):
        d = binding.LayerDesc()
        d.mode, d.n_linear, d.w_dtype, d.order = binding.AGG_GCN_SYM, len(dims) - 1, w_dtype, order
        for i, v in enumerate(dims):
            d.dims[i] = v
        return int(lib.mgg_layer_workspace_bytes(part.handle, ctypes.byref(d)))

    r256 = lambda v: -(-v // 256) * 256
    # the partial sums of rows cut into several work items pass through the workspace as well
    si = int(part.info.n_split_items)
    assert si > 0
    scr = lambda width: r256(si * width * 4)
    assert binding.mgg_aggregate_scratch_bytes(part, 100) == si * 104 * 4
    assert binding.mgg_aggregate_scratch_bytes(part, 40) == si * 40 * 4
    assert need((100, 40), binding.ORDER_AGG_FIRST) == r256(n * 104 * 4) + scr(104) + 256
    assert need((100, 40), binding.ORDER_UPDATE_FIRST) == r256(n * 40 * 4) + r256(h * 40 * 4) + scr(40) + 256
    assert need((100, 40, 7), binding.ORDER_AGG_FIRST) == r256(n * 104 * 4) + r256(n * 40 * 4) + scr(104) + 256
    assert need((100, 40, 7), binding.ORDER_UPDATE_FIRST) == 2 * r256(n * 40 * 4) + r256(h * 40 * 4) + scr(40) + 256
    # AUTO reorders when the transformed rows are at most 3/4 of the input bytes: 40 * 4 <= 0.75 * 100 * 4
    assert need((100, 40), binding.ORDER_AUTO) == max(need((100, 40), binding.ORDER_AGG_FIRST), need((100, 40), binding.ORDER_UPDATE_FIRST))
    assert need((100, 90), binding.ORDER_AUTO) == need((100, 90), binding.ORDER_AGG_FIRST)
    assert need((100, 40), 7) == 0 and need((100, 0), 0) == 0 and need((100,), 0) == 0


def test_automatic_choice_of_source_classes():
    """hot_phases = 0: popularity phases when the most gathered rows of one phase receive less than
    half of all gathers, hash classes otherwise."""
    rng = np.random.default_rng(8)
    # skewed: R-MAT hubs take most gathers -> by hash
    row_ptr, col = inputs.rmat_graph(12, 60000, 0.57, 0.19, 0.19, 0.05, rng)
    part = binding.mgg_build_partition(row_ptr, col, 2, 0, None, host_only=True, hot_rows=8, xcd_min_deg=8)
    cnt = np.sort(np.bincount(np.concatenate([part.export()["local_col"], part.info.n_own + part.export()["remote_col"]])))[::-1]
    share = cnt[:64].sum() / cnt.sum()
    assert part.info.class_mode == (2 if share < 0.5 else 1)
    # flat: a random regular-ish graph, every row gathered about equally often -> by popularity
    n = 4096
    col2 = rng.integers(0, n, size=n * 16).astype(np.int32)
    row_ptr2 = np.arange(0, n * 16 + 1, 16, dtype=np.int64)
    part2 = binding.mgg_build_partition(row_ptr2, col2, 1, 0, None, host_only=True, hot_rows=8, xcd_min_deg=8)
    assert part2.info.class_mode == 2 and part2.info.n_phases == 4
    # skewed by construction: 64 hub rows take nine tenths of the gathers -> by hash
    hub = rng.integers(0, 64, size=n * 16)
    col3 = np.where(rng.random(n * 16) < 0.9, hub, col2).astype(np.int32)
    part3 = binding.mgg_build_partition(row_ptr2, col3, 1, 0, None, host_only=True, hot_rows=8, xcd_min_deg=8)
    assert part3.info.class_mode == 1


def test_partition_fuzz_against_oracle():
    """Random small graphs (duplicates, self-loops, empty rows, directed), random bounds (empty ranges
    allowed) and random schedule knobs: integer structures bit-exact against the oracle's builder, and a
    valid schedule whatever the knobs."""
    from hypothesis import given, settings, strategies as st, HealthCheck

    @settings(max_examples=80, deadline=None, suppress_health_check=list(HealthCheck), derandomize=True)
    @given(st.data())
    def run(data):
        n = data.draw(st.integers(1, 48))
        rows = [data.draw(st.lists(st.integers(0, n - 1), max_size=data.draw(st.sampled_from([0, 2, 5, 40])))) for _ in range(n)]
        row_ptr, col = inputs.csr_from_adjacency_lists([sorted(r) for r in rows])
        parts = data.draw(st.integers(1, 5))
        cuts = sorted(data.draw(st.lists(st.integers(0, n), min_size=parts - 1, max_size=parts - 1)))
        bounds = np.array([0] + cuts + [n], dtype=np.int64)
        opts = dict(ps=data.draw(st.sampled_from([1, 2, 7, 32, 64])), dist=data.draw(st.sampled_from([1, 2, 16])),
                    short_max=data.draw(st.sampled_from([-1, 1, 3, 16])), wpb=data.draw(st.sampled_from([1, 4, 16])),
                    xcd_min_deg=data.draw(st.sampled_from([-1, 1, 4, 30])),
                    hot_phases=data.draw(st.sampled_from([-1, 0, 1, 3, 31])), hot_rows=data.draw(st.sampled_from([1, 2, 5, 100])),
                    min_piece=data.draw(st.sampled_from([1, 2, 9])), hot_min_count=data.draw(st.sampled_from([1, 2, 4])))
        for p in range(parts):
            _compare_with_oracle(row_ptr, col, parts, p, bounds, **opts)

    run()


def test_bag_partition_structures():
    """mgg_build_bags: lookups inside the local slice become local columns rebased to the slice, the
    others halo slots over the distinct remote rows in ascending order -- rebuilt here with numpy."""
    rng = np.random.default_rng(2)
    table_rows, lo, hi = 3000, 700, 1900
    sizes = rng.integers(0, 40, size=500)
    sizes[:3] = [0, 1, 400]
    ptr = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    idx = (rng.zipf(1.2, size=ptr[-1]) % table_rows).astype(np.int32)
    for knobs in (dict(), dict(ps=4, dist=2, xcd_min_deg=8, short_max=2), dict(hot_phases=3, hot_rows=16, xcd_min_deg=4, min_piece=2)):
        part = binding.mgg_build_bags(ptr, idx, table_rows, lo, hi, host_only=True, **knobs)
        info, got = part.info, part.export()
        assert (info.n_own, info.lb, info.ub, info.n_local_rows, info.is_bags) == (500, lo, hi, hi - lo, 1)
        is_local = (idx >= lo) & (idx < hi)
        halo = np.unique(idx[~is_local])
        assert np.array_equal(got["halo_gid"], halo)
        bag_of = np.repeat(np.arange(500), sizes)
        assert np.array_equal(got["local_row_ptr"], np.concatenate([[0], np.cumsum(np.bincount(bag_of[is_local], minlength=500))]))
        assert np.array_equal(got["remote_row_ptr"], np.concatenate([[0], np.cumsum(np.bincount(bag_of[~is_local], minlength=500))]))
        assert np.array_equal(got["local_col"], idx[is_local] - lo)
        assert np.array_equal(got["remote_col"], np.searchsorted(halo, idx[~is_local]))
        assert np.array_equal(got["deg_own"], sizes)
        _check_schedule(got, info, hot_by_popularity=info.class_mode == 2)
        part.destroy()
    # errors
    assert _status(binding.mgg_build_bags, ptr, idx, table_rows, 10, 5, host_only=True) == binding.ERR_INVALID_ARG
    assert _status(binding.mgg_build_bags, ptr, idx, 100, 0, 50, host_only=True) == binding.ERR_BAD_GRAPH
    assert _status(binding.mgg_build_bags, np.array([0, 3, 2]), idx[:3], table_rows, 0, 5, host_only=True) == binding.ERR_BAD_GRAPH
