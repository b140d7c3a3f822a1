"""GPU tests: the HIP path against the CPU oracle, element by element, through the C ABI.

Kernel maps must be bit-exact (after the canonical sort, and - where the library promises an
order - in that order too); outputs must agree within 1e-5 (fp32) / 2e-2 (fp16, bf16 inputs
with fp32 accumulation) of the largest reference magnitude.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_07710_amd import binding as sc
from paper_2402_07710_amd import synth
from tests import pins

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}
TDT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def to_dev(x_f32: np.ndarray, dtype: str):
    return torch.from_numpy(np.ascontiguousarray(x_f32)).to(DEV).to(TDT[dtype]).contiguous()


def run_layer(coords, feat, weight, K, stride, mode, dtype, out_dtype=None, grid_dims=None):
    """Whole layer on the GPU.  Returns (buffers, counts, out_coords np, feat_out np float64).
    grid_dims: use the dense location table over that box instead of the hash table."""
    n = len(coords)
    C_in, C_out = weight.shape[1], weight.shape[2]
    buf = sc.LayerBuffers(n, K, stride, mode, C_in, C_out, dtype, out_dtype, device=DEV, grid_dims=grid_dims)
    d_coords = torch.from_numpy(np.ascontiguousarray(coords, dtype=np.int32)).to(DEV).reshape(-1, 4)
    d_feat = to_dev(feat.reshape(n, C_in), dtype)
    d_w = to_dev(weight, dtype)
    buf.layer(d_coords, d_feat, d_w)
    h = buf.read_counts()
    n_out = int(h.n_out)
    out_coords = buf.out_coords[:n_out].cpu().numpy()
    out = buf.feat_out[:n_out].to(torch.float64).cpu().numpy()
    return buf, h, out_coords, out


def exported_map(buf, h):
    pin, pout, ost = buf.export(h)
    return dict(pair_in=pin.cpu().numpy(), pair_out=pout.cpu().numpy(), offset_start=ost.cpu().numpy().astype(np.int64))


def assert_maps_equal(gpu_km, out_coords, ref_km, exact_order):
    """Bit-exact comparison of two kernel maps after canonical sorting (and without it where
    the order is part of the contract)."""
    g = dict(gpu_km, out_coords=out_coords)
    assert np.array_equal(g["offset_start"], ref_km["offset_start"]), "per-offset pair counts differ"
    oc_g, per_g = oracle.canonical_pairs(g)
    oc_r, per_r = oracle.canonical_pairs(ref_km)
    assert np.array_equal(oc_g, oc_r), "output coordinate sets differ"
    for k, (a, b) in enumerate(zip(per_g, per_r)):
        assert np.array_equal(a, b), f"pairs of offset {k} differ"
    if exact_order:
        assert np.array_equal(out_coords, ref_km["out_coords"])
        assert np.array_equal(g["pair_in"], ref_km["pair_in"])
        assert np.array_equal(g["pair_out"], ref_km["pair_out"])


def rel_err(got, ref):
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30)) if ref.size else 0.0


def check_layer(coords, K, stride, mode, C_in, C_out, dtype, seed=0, out_dtype=None, threads=8, grid_dims=None):
    n = len(coords)
    feat = synth.features(n, C_in, dtype, seed)
    weight = synth.weights(K ** 3, C_in, C_out, dtype, seed)
    buf, h, out_coords, out = run_layer(coords, feat, weight, K, stride, mode, dtype, out_dtype, grid_dims)
    ref_km = oracle.kmap(coords, K, stride, mode)
    assert h.n_in == n and h.n_out == ref_km["n_out"] and h.n_pairs == ref_km["offset_start"][-1]
    assert list(h.per_offset[:K ** 3]) == list(np.diff(ref_km["offset_start"]))
    assert_maps_equal(exported_map(buf, h), out_coords, ref_km, exact_order=True)
    ref = oracle.conv(feat, weight, ref_km, threads=threads)
    err = rel_err(out, ref)
    assert err <= TOL[dtype], f"max relative error {err:.3e} > {TOL[dtype]}"
    return err


# ---- location table --------------------------------------------------------------------------
@pytest.mark.parametrize("n,grid", [(1, 4), (63, 8), (2000, 64), (50000, 64)])
def test_hash_finds_every_key(n, grid):
    say(f"hash n={n} grid={grid}")
    coords = synth.uniform_cells(n, grid, seed=n)
    coords[:, 0] = np.arange(n) % 3
    d_coords = torch.from_numpy(coords).to(DEV)
    table = torch.empty(sc.sc_hash_bytes(n), dtype=torch.uint8, device=DEV)
    counts = torch.zeros(sc.COUNTS_BYTES + 8, dtype=torch.uint8, device=DEV)
    sc.sc_hash_build(d_coords, table, counts)
    h = sc.sc_counts_read(counts)
    assert h.n_in == n and h.status == 0
    rows = torch.empty(n, dtype=torch.int32, device=DEV)
    sc.sc_hash_lookup(table, n, d_coords, rows)
    assert torch.equal(rows.cpu(), torch.arange(n, dtype=torch.int32))
    # absent keys: same cells in a batch slot that is not used, and shifted cells
    absent = coords.copy()
    absent[:, 0] = 7
    rows2 = torch.empty(n, dtype=torch.int32, device=DEV)
    sc.sc_hash_lookup(table, n, torch.from_numpy(absent).to(DEV), rows2)
    assert bool((rows2 == -1).all())
    present = {tuple(r) for r in coords.tolist()}
    shifted = coords.copy()
    shifted[:, 3] += 1
    want = np.array([-1 if tuple(r) not in present else 0 for r in shifted.tolist()])
    sc.sc_hash_lookup(table, n, torch.from_numpy(shifted).to(DEV), rows2)
    got = rows2.cpu().numpy()
    assert np.array_equal(got == -1, want == -1)
    hit = got >= 0
    assert np.array_equal(coords[got[hit]], shifted[hit])


def test_hash_reports_duplicates_and_range():
    say("hash errors")
    coords = synth.uniform_cells(500, 16, seed=1)
    dup = coords.copy()
    dup[400] = dup[17]
    table = torch.empty(sc.sc_hash_bytes(500), dtype=torch.uint8, device=DEV)
    counts = torch.zeros(sc.COUNTS_BYTES + 8, dtype=torch.uint8, device=DEV)
    sc.sc_hash_build(torch.from_numpy(dup).to(DEV), table, counts)
    assert sc.sc_counts_read(counts, check=False).status == sc.SC_EDUP
    bad = coords.copy()
    bad[3, 2] = 65535
    sc.sc_hash_build(torch.from_numpy(bad).to(DEV), table, counts)
    assert sc.sc_counts_read(counts, check=False).status == sc.SC_ERANGE
    bad[3, 2] = -1
    sc.sc_hash_build(torch.from_numpy(bad).to(DEV), table, counts)
    assert sc.sc_counts_read(counts, check=False).status == sc.SC_ERANGE
    # a clean build clears the latch
    sc.sc_hash_build(torch.from_numpy(coords).to(DEV), table, counts)
    assert sc.sc_counts_read(counts).status == 0



def fresh_table(n):
    table = torch.empty(sc.sc_hash_bytes(n), dtype=torch.uint8, device=DEV)
    counts = torch.zeros(sc.COUNTS_BYTES + 8, dtype=torch.uint8, device=DEV)
    return table, counts


def lookup_np(table, n, query):
    rows = torch.empty(len(query), dtype=torch.int32, device=DEV)
    sc.sc_hash_lookup(table, n, torch.from_numpy(np.ascontiguousarray(query, dtype=np.int32)).to(DEV), rows)
    return rows.cpu().numpy()


def test_hash_rebuild_sees_only_the_last_build():
    """A table that is built again without the filling pass: keys of earlier builds are gone,
    also when the new set overlaps the old one or reuses its slots."""
    say("hash rebuild epochs")
    n = 3000
    sets = [synth.uniform_cells(n, 24, seed=s) for s in (1, 2, 3)]
    sets.append(sets[0][::-1].copy())                      # an old set again, rows renumbered
    sets.append(np.roll(sets[1], 7, axis=0))
    table, counts = fresh_table(n)
    everything = np.unique(np.concatenate(sets), axis=0)
    for epoch, coords in enumerate(sets):
        d = torch.from_numpy(coords).to(DEV)
        if epoch == 0:
            sc.sc_hash_build(d, table, counts)
        else:
            sc.sc_hash_rebuild(d, table, epoch, counts)
        h = sc.sc_counts_read(counts)
        assert h.n_in == n and h.status == 0
        assert np.array_equal(lookup_np(table, n, coords), np.arange(n))
        want = {tuple(c): i for i, c in enumerate(coords.tolist())}
        got = lookup_np(table, n, everything)
        assert np.array_equal(got, np.array([want.get(tuple(c), -1) for c in everything.tolist()]))
    # epochs need not be consecutive, only unused
    coords = synth.uniform_cells(n, 24, seed=9)
    sc.sc_hash_rebuild(torch.from_numpy(coords).to(DEV), table, sc.SC_HASH_EPOCH_MAX, counts)
    assert np.array_equal(lookup_np(table, n, coords), np.arange(n))
    got = lookup_np(table, n, everything)
    want = {tuple(c): i for i, c in enumerate(coords.tolist())}
    assert np.array_equal(got, np.array([want.get(tuple(c), -1) for c in everything.tolist()]))


def test_hash_rebuild_with_fewer_and_more_rows():
    """The capacity is the one the table was filled with, whatever n later builds bring."""
    say("hash rebuild sizes")
    n0 = 2000
    table, counts = fresh_table(n0)
    sc.sc_hash_build(torch.from_numpy(synth.uniform_cells(n0, 20, seed=1)).to(DEV), table, counts)
    for epoch, n in enumerate([1, 130, 1999, 2000, 0, 700], start=1):
        coords = synth.uniform_cells(n, 20, seed=10 + epoch) if n else np.zeros((0, 4), np.int32)
        d = torch.from_numpy(coords).to(DEV).reshape(-1, 4)
        sc.sc_hash_rebuild(d, table, epoch, counts)
        h = sc.sc_counts_read(counts)
        assert h.n_in == n and h.status == 0
        if n:
            assert np.array_equal(lookup_np(table, n0, coords), np.arange(n))
        probe = synth.uniform_cells(500, 20, seed=77)
        want = {tuple(c): i for i, c in enumerate(coords.tolist())}
        assert np.array_equal(lookup_np(table, n0, probe), np.array([want.get(tuple(c), -1) for c in probe.tolist()]))


def test_hash_rebuild_layers_match_oracle_across_the_epoch_wrap():
    """Layer after layer on one set of buffers: more builds than there are epochs, so the table
    is refilled on the way; every layer must give the oracle's map and output."""
    say("hash rebuild layers")
    n, C = 700, 32
    buf = sc.LayerBuffers(n, 3, 1, "subm", C, C, "f16", device=DEV)
    cases = []
    for s in range(3):
        coords = synth.uniform_cells(n, 14, seed=40 + s)
        feat = synth.features(n, C, "f16", s)
        weight = synth.weights(27, C, C, "f16", s)
        km = oracle.kmap(coords, 3, 1, "subm")
        cases.append((torch.from_numpy(coords).to(DEV), to_dev(feat, "f16"), to_dev(weight, "f16"), km,
                      oracle.conv(feat, weight, km)))
    seen_epochs = set()
    for it in range(sc.SC_HASH_EPOCH_MAX + 8):
        d_coords, d_feat, d_w, km, ref = cases[it % 3]
        buf.layer(d_coords, d_feat, d_w)
        seen_epochs.add(buf.epoch)
        if it < 6 or it > sc.SC_HASH_EPOCH_MAX - 3:
            h = buf.read_counts()
            assert h.status == 0 and h.n_pairs == km["offset_start"][-1]
            assert_maps_equal(exported_map(buf, h), buf.out_coords.cpu().numpy(), km, exact_order=True)
        else:
            assert buf.read_counts(with_pairs=False).status == 0
        assert rel_err(buf.feat_out[:n].to(torch.float64).cpu().numpy(), ref) <= TOL["f16"]
    assert seen_epochs == set(range(sc.SC_HASH_EPOCH_MAX + 1))


def test_hash_rebuild_errors_surface_at_the_map_build():
    say("hash rebuild errors")
    n = 500
    coords = synth.uniform_cells(n, 16, seed=1)
    d_good = torch.from_numpy(coords).to(DEV)
    dup = coords.copy()
    dup[400] = dup[17]
    bad = coords.copy()
    bad[3, 0] = sc.SC_BATCH_MAX + 1
    for mode, K, s in (("subm", 3, 1), ("strided", 2, 2), ("strided", 3, 2)):
        buf = sc.LayerBuffers(n, K, s, mode, 32, 32, "f16", device=DEV)
        buf.hash_build(d_good)                                   # fills the table (epoch 0)
        buf.kmap_build(d_good)
        assert buf.read_counts(check=False).status == 0
        for wrong, code in ((dup, sc.SC_EDUP), (bad, sc.SC_ERANGE)):
            d = torch.from_numpy(wrong).to(DEV)
            buf.hash_build(d)                                    # a rebuild: the error waits in the table
            assert buf.epoch >= 1
            buf.kmap_build(d)
            assert buf.read_counts(check=False, with_pairs=False).status == code
            buf.hash_build(d_good)                               # and does not outlive its build
            buf.kmap_build(d_good)
            assert buf.read_counts(check=False).status == 0
    # more rows than the table was filled for: refused by the build, reported like the others
    table = torch.empty(sc.sc_hash_bytes(4 * n), dtype=torch.uint8, device=DEV)
    counts = torch.zeros(sc.COUNTS_BYTES + 8, dtype=torch.uint8, device=DEV)
    sc.sc_hash_build(d_good[:100].contiguous(), table, counts)           # capacity 4096
    big = torch.from_numpy(synth.uniform_cells(1100, 16, seed=5)).to(DEV)
    sc.sc_hash_rebuild(big, table, 1, counts)
    kmap = torch.empty(sc.sc_kmap_bytes(1100, 3, 1, "subm"), dtype=torch.uint8, device=DEV)
    sc.sc_kmap_build(big, table, 3, 1, "subm", None, kmap, None, counts)
    assert sc.sc_counts_read(counts, check=False).status == sc.SC_ECAP


def test_hash_rebuild_error_with_epochs_out_of_order():
    """Epochs may be used in any order between two sc_hash_build calls: an error left under a
    higher epoch must not hide the error of a later build with a lower one."""
    say("hash rebuild errors, epochs 5 then 3")
    n = 500
    coords = synth.uniform_cells(n, 16, seed=1)
    dup = coords.copy()
    dup[400] = dup[17]
    bad = coords.copy()
    bad[7, 3] = -4
    table, counts = fresh_table(n)
    kmap = torch.empty(sc.sc_kmap_bytes(n, 3, 1, "subm"), dtype=torch.uint8, device=DEV)
    sc.sc_hash_build(torch.from_numpy(coords).to(DEV), table, counts)
    for epoch, wrong, code in ((5, dup, sc.SC_EDUP), (3, dup, sc.SC_EDUP), (4, bad, sc.SC_ERANGE), (2, coords, 0),
                               (1, dup, sc.SC_EDUP)):
        d = torch.from_numpy(wrong).to(DEV)
        sc.sc_hash_rebuild(d, table, epoch, counts)
        sc.sc_kmap_build(d, table, 3, 1, "subm", None, kmap, None, counts)
        assert sc.sc_counts_read(counts, check=False).status == code, (epoch, code)


def test_hash_rebuild_of_a_large_table():
    """Above 64 MiB of table a rebuild fills the table after all (and then reports its errors
    like sc_hash_build): same results as for small tables, whichever way the library takes."""
    say("hash rebuild, large table")
    n = 530_000                                             # capacity 2^23 slots = 128 MiB
    assert sc.sc_hash_bytes(n) == (1 << 23) * 16 + 256
    table, counts = fresh_table(n)
    kmap = torch.empty(sc.sc_kmap_bytes(n, 3, 1, "subm"), dtype=torch.uint8, device=DEV)
    prev = None
    for epoch in range(2):
        coords = synth.uniform_cells(n, 110, seed=100 + epoch)
        d = torch.from_numpy(coords).to(DEV)
        if epoch == 0:
            sc.sc_hash_build(d, table, counts)
        else:
            sc.sc_hash_rebuild(d, table, epoch, counts)
        assert sc.sc_counts_read(counts).status == 0
        assert np.array_equal(lookup_np(table, n, coords[::7]), np.arange(n)[::7])
        if prev is not None:                                # the previous build's keys are gone
            gone = prev[:5000]
            want = {tuple(c): i for i, c in enumerate(coords.tolist())}
            assert np.array_equal(lookup_np(table, n, gone), np.array([want.get(tuple(c), -1) for c in gone.tolist()]))
        sc.sc_kmap_build(d, table, 3, 1, "subm", None, kmap, None, counts)
        h = sc.sc_counts_read(counts, kmap, n, 3, 1, "subm")
        ref = oracle.kmap(coords, 3, 1, "subm")
        assert h.status == 0 and h.n_pairs == ref["offset_start"][-1]
        assert list(h.per_offset[:27]) == list(np.diff(ref["offset_start"]))
        prev = coords
    dup = prev.copy()
    dup[1234] = dup[99999]
    sc.sc_hash_rebuild(torch.from_numpy(dup).to(DEV), table, 2, counts)
    assert sc.sc_counts_read(counts, check=False).status == sc.SC_EDUP


def test_hash_batch_index_range():
    say("hash batch range")
    coords = synth.uniform_cells(200, 8, seed=3)
    coords[:, 0] = np.arange(200) % (sc.SC_BATCH_MAX + 1)
    table, counts = fresh_table(200)
    sc.sc_hash_build(torch.from_numpy(coords).to(DEV), table, counts)
    assert sc.sc_counts_read(counts).status == 0
    assert np.array_equal(lookup_np(table, 200, coords), np.arange(200))
    coords[7, 0] = sc.SC_BATCH_MAX + 1
    sc.sc_hash_build(torch.from_numpy(coords).to(DEV), table, counts)
    assert sc.sc_counts_read(counts, check=False).status == sc.SC_ERANGE


# ---- dense location table ---------------------------------------------------------------------
@pytest.mark.parametrize("n,box", [(1, (1, 4, 4, 4)), (63, (3, 8, 8, 8)), (2000, (3, 64, 64, 64)), (50000, (3, 64, 64, 41))])
def test_grid_finds_every_key(n, box):
    say(f"grid n={n} box={box}")
    coords = synth.uniform_cells(n, min(box[1:]), seed=n)
    coords[:, 0] = np.arange(n) % box[0]
    d_coords = torch.from_numpy(coords).to(DEV)
    grid = torch.empty(sc.sc_grid_bytes(*box), dtype=torch.uint8, device=DEV)
    sc.sc_grid_clear(grid, box)
    counts = torch.zeros(sc.COUNTS_BYTES + 8, dtype=torch.uint8, device=DEV)
    sc.sc_grid_build(d_coords, grid, box, 1, counts)
    h = sc.sc_counts_read(counts)
    assert h.n_in == n and h.status == 0
    rows = torch.empty(n, dtype=torch.int32, device=DEV)
    sc.sc_grid_lookup(grid, box, 1, d_coords, rows)
    assert torch.equal(rows.cpu(), torch.arange(n, dtype=torch.int32))
    # another epoch sees nothing; queries outside the box are absent, not errors
    sc.sc_grid_lookup(grid, box, 2, d_coords, rows)
    assert bool((rows == -1).all())
    outside = coords.copy()
    outside[:, 3] += box[3]
    outside[::2, 1] = -1
    sc.sc_grid_lookup(grid, box, 1, torch.from_numpy(outside).to(DEV), rows)
    assert bool((rows == -1).all())
    present = {tuple(r): i for i, r in enumerate(coords.tolist())}
    shifted = coords.copy()
    shifted[:, 3] = (shifted[:, 3] + 1) % box[3]
    want = np.array([present.get(tuple(r), -1) for r in shifted.tolist()], dtype=np.int32)
    sc.sc_grid_lookup(grid, box, 1, torch.from_numpy(shifted).to(DEV), rows)
    assert np.array_equal(rows.cpu().numpy(), want)


def test_grid_reports_duplicates_and_range():
    """The dense build stores blindly; the kernel-map build, which reads every row's own cell,
    reports rows outside the box and rows that share a coordinate."""
    say("grid errors")
    box = (2, 16, 16, 16)
    coords = synth.uniform_cells(500, 16, seed=1)
    grid = torch.empty(sc.sc_grid_bytes(*box), dtype=torch.uint8, device=DEV)
    sc.sc_grid_clear(grid, box)
    counts = torch.zeros(sc.COUNTS_BYTES + 8, dtype=torch.uint8, device=DEV)
    kmap = torch.empty(sc.sc_kmap_bytes(500, 3, 1, "subm"), dtype=torch.uint8, device=DEV)

    def status_of(c, epoch):
        d = torch.from_numpy(c).to(DEV)
        sc.sc_grid_build(d, grid, box, epoch, counts)
        sc.sc_kmap_build_grid(d, grid, box, epoch, 3, kmap, counts)
        return sc.sc_counts_read(counts, check=False).status

    dup = coords.copy()
    dup[400] = dup[17]
    assert status_of(dup, 1) == sc.SC_EDUP
    for epoch, (col, val) in enumerate([(2, 16), (2, -1), (0, 2), (3, 65535)], start=2):
        bad = coords.copy()
        bad[3, col] = val
        assert status_of(bad, epoch) == sc.SC_ERANGE, (col, val)
    # a clean build clears the latch, and the cells of the failed builds are stale
    assert status_of(coords, 9) == 0
    rows = torch.empty(500, dtype=torch.int32, device=DEV)
    sc.sc_grid_lookup(grid, box, 9, torch.from_numpy(coords).to(DEV), rows)
    assert torch.equal(rows.cpu(), torch.arange(500, dtype=torch.int32))


@pytest.mark.parametrize("K", [1, 3, 5, 7])
@pytest.mark.parametrize("n", [1, 65, 1000])
def test_grid_layer_small(K, n):
    say(f"grid layer K={K} n={n}")
    box = (2, 12, 12, 12)
    coords = synth.uniform_cells(n, 12, seed=K + n)
    coords[:, 0] = np.arange(n) % 2
    check_layer(coords, K, 1, "subm", 32, 32, "f16", seed=K, grid_dims=box)


def test_grid_reuse_across_builds_without_clearing():
    """Several different voxel sets through ONE array: every build must only see its own cells."""
    say("grid epochs")
    box = (1, 20, 20, 20)
    n_max = 3000
    buf = sc.LayerBuffers(n_max, 3, 1, "subm", 32, 32, "f16", device=DEV, grid_dims=box)
    for it, n in enumerate([3000, 700, 2500, 64, 1]):
        coords = synth.uniform_cells(n, 20, seed=100 + it)
        b = sc.LayerBuffers(n, 3, 1, "subm", 32, 32, "f16", device=DEV, grid_dims=box)
        b.table, b.epoch = buf.table, buf.epoch            # the same array, the running epoch counter
        d_coords = torch.from_numpy(coords).to(DEV)
        b.hash_build(d_coords)
        b.kmap_build(d_coords)
        buf.epoch = b.epoch
        h = b.read_counts()
        ref_km = oracle.kmap(coords, 3, 1, "subm")
        assert h.n_pairs == ref_km["offset_start"][-1]
        assert_maps_equal(exported_map(b, h), coords, ref_km, exact_order=True)


# ---- whole layers, small: several tiles and a ragged tail --------------------------------------
@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 128, 129, 1000])
@pytest.mark.parametrize("dtype,C", [("f32", 16), ("f16", 32)])
def test_subm_tile_edges(n, dtype, C):
    say(f"subm edges n={n} {dtype}")
    coords = synth.uniform_cells(n, 6 if n < 200 else 12, seed=n)
    check_layer(coords, 3, 1, "subm", C, C, dtype, seed=n)


@pytest.mark.parametrize("K,s", [(2, 2), (3, 3), (4, 4)])
@pytest.mark.parametrize("n", [1, 64, 65, 700])
def test_strided_small(K, s, n):
    say(f"strided K={K} n={n}")
    coords = synth.uniform_cells(n, 10, seed=100 + n)
    coords[:, 0] = np.arange(n) % 2
    check_layer(coords, K, s, "strided", 32, 64, "f16", seed=n)
    check_layer(coords, K, s, "strided", 8, 24, "f32", seed=n)


def test_strided_map_of_a_set_too_large_for_the_in_kernel_scan():
    """More than 4096 blocks of 1024 inputs: the block counts are then scanned by a kernel of
    their own (below that, every workgroup of the pairs kernel scans them itself)."""
    say("strided map, 4.3 M inputs")
    n = 4_300_000
    coords = synth.uniform_cells(n, 180, seed=11)
    buf = sc.LayerBuffers(n, 2, 2, "strided", 32, 32, "f16", device=DEV)
    d = torch.from_numpy(coords).to(DEV)
    buf.kmap_build(d, standalone=True)
    h = buf.read_counts()
    ref_km = oracle.kmap(coords, 2, 2, "strided")
    assert h.status == 0 and h.n_out == ref_km["n_out"] and h.n_pairs == n
    assert_maps_equal(exported_map(buf, h), buf.out_coords[:h.n_out].cpu().numpy(), ref_km, exact_order=True)


@pytest.mark.parametrize("K,s", [(3, 2), (3, 1), (4, 2), (5, 2), (5, 3), (2, 1), (5, 5), (7, 7)])
@pytest.mark.parametrize("n", [1, 65, 900])
def test_strided_general_kernel_and_stride(K, s, n):
    """K != stride (and K == stride beyond 4): every input belongs to up to ceil(K/s)^3 output
    cells; output numbering by first occurrence (input row, then offset) must be the oracle's."""
    say(f"strided general K={K} s={s} n={n}")
    coords = synth.uniform_cells(n, 14, seed=K * 100 + s * 10 + n)
    coords[:, 0] = np.arange(n) % 2
    check_layer(coords, K, s, "strided", 32, 32, "f16", seed=n)


def test_strided_general_on_lidar_scene():
    say("strided K=3 s=2 on the cfg2 voxel set")
    coords = synth.lidar_scene(0)
    check_layer(coords, 3, 2, "strided", 32, 64, "f16", threads=16)


@pytest.mark.parametrize("s", [2, 3])
@pytest.mark.parametrize("dtype,n", [("f16", 700), ("bf16", 20000)])
def test_strided_64_channel_layer(s, dtype, n):
    """K = 3 strided layers of 64 -> 64 channels run the kernel of the 64-channel submanifold
    layer: here its row count comes from the device and is far below the grid's row capacity."""
    say(f"strided K=3 s={s} 64->64 {dtype} n={n}")
    coords = synth.lidar_scene(6)[:n]
    check_layer(coords, 3, s, "strided", 64, 64, dtype, seed=n, threads=16)


@pytest.mark.parametrize("K", [1, 5, 7])
def test_subm_other_kernel_sizes(K):
    say(f"subm K={K}")
    coords = synth.uniform_cells(900, 10, seed=K)
    check_layer(coords, K, 1, "subm", 32, 16, "bf16", seed=K)
    check_layer(coords[:300], K, 1, "subm", 5, 7, "f32", seed=K)


@pytest.mark.parametrize("dtype,C_in,C_out", [("f16", 32, 32), ("f16", 64, 64), ("f16", 128, 128), ("f16", 256, 48),
                                              ("bf16", 64, 64), ("bf16", 32, 256), ("bf16", 128, 16),
                                              ("f32", 16, 16), ("f32", 3, 100), ("f32", 70, 130),
                                              ("f32", 32, 64), ("f32", 64, 32), ("f32", 64, 64), ("f32", 16, 32)])
def test_channel_shapes(dtype, C_in, C_out):
    say(f"channels {dtype} {C_in}->{C_out}")
    coords = synth.uniform_cells(3000, 18, seed=C_in + C_out)     # about half the cells active: ~14 pairs/voxel
    coords[:, 0] = np.arange(len(coords)) % 2
    check_layer(coords, 3, 1, "subm", C_in, C_out, dtype, seed=1)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_fp32_output_of_16bit_layer(dtype):
    say(f"fp32 output {dtype}")
    coords = synth.uniform_cells(2000, 14, seed=9)
    err = check_layer(coords, 3, 1, "subm", 64, 32, dtype, seed=2, out_dtype="f32")
    assert err < 1e-5        # 16-bit inputs are exact in fp32; only the summation order differs


def test_empty_input():
    say("empty")
    coords = np.zeros((0, 4), np.int32)
    for mode, K, s in (("subm", 3, 1), ("strided", 2, 2)):
        buf = sc.LayerBuffers(0, K, s, mode, 32, 32, "f16", device=DEV)
        d_coords = torch.zeros((0, 4), dtype=torch.int32, device=DEV)
        buf.layer(d_coords, torch.zeros((0, 32), dtype=torch.float16, device=DEV),
                  torch.zeros((K ** 3, 32, 32), dtype=torch.float16, device=DEV))
        h = buf.read_counts()
        assert h.n_in == 0 and h.n_out == 0 and h.n_pairs == 0 and h.status == 0


def test_domain_edges_and_batches():
    """Voxels on the faces of the key domain: probes that leave it must miss, not wrap."""
    say("domain edges")
    m = sc.SC_COORD_MAX
    pts = []
    for b in (0, 5, sc.SC_BATCH_MAX):
        for x in (0, 1, m - 1, m):
            for y in (0, m):
                for z in (0, 1, m):
                    pts.append((b, x, y, z))
    coords = np.array(pts, dtype=np.int32)
    check_layer(coords, 3, 1, "subm", 32, 32, "f16", seed=3)
    check_layer(coords, 5, 1, "subm", 4, 4, "f32", seed=3)
    check_layer(coords, 2, 2, "strided", 32, 32, "bf16", seed=3)


def test_strided_reports_duplicates():
    say("strided dup")
    coords = synth.uniform_cells(300, 8, seed=2)
    coords[200] = coords[5]
    buf = sc.LayerBuffers(300, 2, 2, "strided", 32, 32, "f16", device=DEV)
    d = torch.from_numpy(coords).to(DEV)
    buf.hash_build(d)
    buf.kmap_build(d)
    assert buf.read_counts(check=False).status == sc.SC_EDUP


def test_strided_build_without_a_table_is_self_contained():
    """sc_kmap_build(SC_STRIDED, d_table = NULL): same map as after sc_hash_build, and the build
    starts the counts block itself (n_in, a clean status) whatever the block held before."""
    say("strided standalone")
    for K, s_, n in ((2, 2, 700), (3, 2, 300), (2, 2, 0)):
        coords = synth.uniform_cells(n, 14, seed=K + n) if n else np.zeros((0, 4), np.int32)
        buf = sc.LayerBuffers(n, K, s_, "strided", 32, 32, "f16", device=DEV)
        d_coords = torch.from_numpy(coords).to(DEV).reshape(-1, 4)
        buf.counts.fill_(0x7f)                                  # garbage, incl. a latched "error"
        buf.kmap_build(d_coords, standalone=True)
        h = buf.read_counts()
        ref_km = oracle.kmap(coords, K, s_, "strided")
        assert h.status == 0 and h.n_in == n and h.n_out == ref_km["n_out"] and h.n_pairs == ref_km["offset_start"][-1]
        if n:
            assert_maps_equal(exported_map(buf, h), buf.out_coords[:h.n_out].cpu().numpy(), ref_km, exact_order=True)


def test_maps_and_outputs_are_reproducible_bit_for_bit():
    """The same input gives the same kernel-map bytes, the same output coordinates and the same
    output features on every run, 20 runs of every call (no dependence on thread timing)."""
    say("determinism")
    coords = synth.lidar_scene(1)[:30000]
    d = torch.from_numpy(coords).to(DEV)
    n = len(coords)
    for mode, K, s, C_in, C_out in (("subm", 3, 1, 32, 32), ("strided", 2, 2, 32, 64), ("strided", 3, 2, 32, 32),
                                    ("subm", 3, 1, 64, 64)):
        d_feat = to_dev(synth.features(n, C_in, "f16", 3), "f16")
        d_w = to_dev(synth.weights(K ** 3, C_in, C_out, "f16", 3), "f16")
        buf = sc.LayerBuffers(n, K, s, mode, C_in, C_out, "f16", device=DEV)
        ref = None
        for _ in range(20):
            buf.kmap.zero_()
            buf.feat_out.zero_()
            buf.layer(d, d_feat, d_w)
            h = buf.read_counts()
            pin, pout, ost = buf.export(h)
            cur = (pin.clone(), pout.clone(), ost.clone(), buf.out_coords[:h.n_out].clone(), buf.feat_out[:h.n_out].clone())
            if ref is None:
                ref = cur
            else:
                assert all(torch.equal(a, b) for a, b in zip(ref, cur))


def test_delta_weight_passthrough():
    """W[centre] = I reproduces the input rows bit for bit in every dtype."""
    say("delta weights")
    coords = synth.uniform_cells(1500, 12, seed=4)
    for dtype, C in (("f32", 16), ("f16", 32), ("bf16", 64)):
        feat = synth.features(1500, C, dtype, 5)
        W = np.zeros((27, C, C), np.float32)
        W[13] = np.eye(C)
        _, _, _, out = run_layer(coords, feat, W, 3, 1, "subm", dtype)
        assert np.array_equal(out, feat.astype(np.float64))


SHIFT_SHAPES = [("f32", 16, 16, 1500), ("f16", 32, 32, 1500), ("f16", 32, 32, 40000), ("f16", 64, 64, 1500),
                ("bf16", 128, 128, 1500), ("f16", 32, 64, 1500), ("bf16", 64, 128, 1500), ("f16", 256, 32, 600)]


@pytest.mark.parametrize("dtype,C_in,C_out,n", SHIFT_SHAPES)
def test_shifted_delta_weights(dtype, C_in, C_out, n):
    """W[k0] = (I | 0) for one offset k0 other than the centre: output row i must equal, bit for
    bit, the first C_out (or all C_in) channels of the input row of the voxel at p_i + d_k0 - pad,
    or zero where there is none.  Pins the per-offset indexing of every dedicated kernel (the 40,000
    row case takes the four-tiles-per-workgroup form of the 32 -> 32 kernel)."""
    say(f"shifted delta {dtype} {C_in}->{C_out} n={n}")
    grid = 12 if n <= 1500 else 40
    coords = synth.uniform_cells(n, grid, seed=n + C_in)
    feat = synth.features(n, C_in, dtype, 6)
    lookup = {tuple(r): i for i, r in enumerate(coords.tolist())}
    cc = min(C_in, C_out)
    for k0 in (0, 5, 24, 26):
        W = np.zeros((27, C_in, C_out), np.float32)
        W[k0, :cc, :cc] = np.eye(cc)
        _, _, _, out = run_layer(coords, feat, W, 3, 1, "subm", dtype)
        d = (k0 // 9 - 1, (k0 // 3) % 3 - 1, k0 % 3 - 1)
        src = np.array([lookup.get((b, x + d[0], y + d[1], z + d[2]), -1) for b, x, y, z in coords.tolist()])
        want = np.zeros((n, C_out))
        hit = src >= 0
        want[hit, :cc] = feat[src[hit], :cc]
        assert np.array_equal(out, want), k0


def test_resident_kernel_with_four_tiles_per_workgroup_fp32_output():
    """32 -> 32 channels on >= 512 tiles takes the NT = 4 form of the resident kernel: held to
    the oracle with fp32 output (only the order of summation differs: 1e-5)."""
    say("32->32, 512+ tiles, fp32 output")
    coords = synth.lidar_scene(4)[:40000]
    err = check_layer(coords, 3, 1, "subm", 32, 32, "f16", seed=4, out_dtype="f32", threads=16)
    assert err <= 1e-5


# ---- map reuse and the inverse layer ------------------------------------------------------------
def test_one_map_serves_several_layers():
    """Layers over the same coordinates share one table and one map (the offset table is built
    once per index set): two submanifold layers with different weights and channel counts."""
    say("map reuse")
    coords = synth.lidar_scene(3)[:20000]
    n = len(coords)
    d_coords = torch.from_numpy(coords).to(DEV)
    buf = sc.LayerBuffers(n, 3, 1, "subm", 32, 64, "f16", device=DEV)
    buf.hash_build(d_coords)
    buf.kmap_build(d_coords)
    ref_km = oracle.kmap(coords, 3, 1, "subm")
    f1 = synth.features(n, 32, "f16", 1)
    w1 = synth.weights(27, 32, 64, "f16", 1)
    buf.conv_fwd(to_dev(f1, "f16"), to_dev(w1, "f16"))
    out1 = buf.feat_out[:n].clone()
    assert rel_err(out1.double().cpu().numpy(), oracle.conv(f1, w1, ref_km, threads=8)) <= TOL["f16"]
    # second layer: the first layer's output as input, other weights, same map
    f2 = out1.float().cpu().numpy()
    w2 = synth.weights(27, 64, 64, "f16", 2)
    out2 = torch.empty((n, 64), dtype=torch.float16, device=DEV)
    ws = torch.empty(max(sc.sc_conv_workspace_bytes(3, 64, 64, "f16"), 16), dtype=torch.uint8, device=DEV)
    sc.sc_conv_fwd(out1, to_dev(w2, "f16"), out2, buf.kmap, buf.counts, 3, 1, "subm", ws)
    assert rel_err(out2.double().cpu().numpy(), oracle.conv(f2, w2, ref_km, threads=8)) <= TOL["f16"]


@pytest.mark.parametrize("K,dtype,C_c,C_f", [(2, "f16", 64, 32), (2, "bf16", 128, 128), (3, "f16", 32, 32), (2, "f32", 8, 5),
                                             (3, "f16", 64, 64), (3, "bf16", 64, 64)])
def test_inverse_layer(K, dtype, C_c, C_f):
    """Up-sampling: the strided layer's map transposed; every fine row gets parent . W[offset]."""
    say(f"inverse K={K} {dtype}")
    coords = synth.lidar_scene(4)[:30000]
    n = len(coords)
    d_coords = torch.from_numpy(coords).to(DEV)
    buf = sc.LayerBuffers(n, K, K, "strided", 32, 32, "f16", device=DEV)
    buf.hash_build(d_coords)
    buf.kmap_build(d_coords)
    h = buf.read_counts()
    ref_km = oracle.kmap(coords, K, K, "strided")
    ref_inv = oracle.transpose_map(ref_km)
    n_c = int(h.n_out)
    assert n_c == ref_km["n_out"]
    kmap_inv = torch.empty(sc.sc_kmap_bytes(n, K, K, "inverse"), dtype=torch.uint8, device=DEV)
    sc.sc_kmap_transpose(buf.kmap, n, K, K, buf.counts, kmap_inv)
    h_inv = sc.sc_counts_read(buf.counts, kmap_inv, n, K, K, "inverse")
    assert h_inv.n_pairs == n
    pin, pout, ost = sc.sc_kmap_export(kmap_inv, n, K, K, "inverse", h_inv)
    assert np.array_equal(ost.cpu().numpy(), ref_inv["offset_start"])
    assert np.array_equal(pin.cpu().numpy(), ref_inv["pair_in"])
    assert np.array_equal(pout.cpu().numpy(), ref_inv["pair_out"])
    feat_c = synth.features(n_c, C_c, dtype, 7)
    w = synth.weights(K ** 3, C_c, C_f, dtype, 7)
    out = torch.empty((n, C_f), dtype=TDT[dtype], device=DEV)
    ws = torch.empty(max(sc.sc_conv_workspace_bytes(K, C_c, C_f, dtype), 16), dtype=torch.uint8, device=DEV)
    sc.sc_conv_fwd(to_dev(feat_c, dtype), to_dev(w, dtype), out, kmap_inv, buf.counts, K, K, "inverse", ws, n_map=n)
    ref = oracle.conv(feat_c, w, ref_inv, threads=8)
    err = rel_err(out.double().cpu().numpy(), ref)
    assert err <= TOL[dtype], err


@pytest.mark.parametrize("K,dtype,C_c,C_f,out_dtype", [(2, "f16", 64, 32, None), (2, "bf16", 32, 32, None),
                                                       (2, "f16", 64, 64, "f32"), (2, "bf16", 128, 64, None),
                                                       (3, "f16", 32, 32, None)])
def test_upsampling_from_the_strided_map(K, dtype, C_c, C_f, out_dtype):
    """sc_conv_up_fwd: the inverse layer without a transposed map, against the oracle's inverse
    layer and against the library's own transpose + sc_conv_fwd(SC_INVERSE)."""
    say(f"up-sampling K={K} {dtype} {C_c}->{C_f} out={out_dtype}")
    coords = synth.lidar_scene(5)[:20011]
    n = len(coords)
    d_coords = torch.from_numpy(coords).to(DEV)
    buf = sc.LayerBuffers(n, K, K, "strided", 32, 32, "f16", device=DEV)
    buf.kmap_build(d_coords, standalone=True)
    n_c = int(buf.read_counts().n_out)
    ref_km = oracle.kmap(coords, K, K, "strided")
    assert n_c == ref_km["n_out"]
    feat_c = synth.features(n_c, C_c, dtype, 9)
    w = synth.weights(K ** 3, C_c, C_f, dtype, 9)
    odt = TDT[out_dtype or dtype]
    fine = torch.full((n, C_f), float("nan"), dtype=odt, device=DEV)
    sc.sc_conv_up_fwd(to_dev(feat_c, dtype), n, to_dev(w, dtype), fine, buf.kmap, buf.counts, K)
    ref = oracle.conv(feat_c, w, oracle.transpose_map(ref_km), threads=8)
    got = fine.double().cpu().numpy()
    assert np.isfinite(got).all(), "a fine row was not written"
    assert rel_err(got, ref) <= TOL[dtype]
    # the same layer through the transposed map: identical bits (one product per row either way)
    kmap_inv = torch.empty(sc.sc_kmap_bytes(n, K, K, "inverse"), dtype=torch.uint8, device=DEV)
    sc.sc_kmap_transpose(buf.kmap, n, K, K, buf.counts, kmap_inv)
    fine2 = torch.empty((n, C_f), dtype=odt, device=DEV)
    ws = torch.empty(max(sc.sc_conv_workspace_bytes(K, C_c, C_f, dtype), 16), dtype=torch.uint8, device=DEV)
    sc.sc_conv_fwd(to_dev(feat_c, dtype), to_dev(w, dtype), fine2, kmap_inv, buf.counts, K, K, "inverse", ws, n_map=n)
    assert torch.equal(fine, fine2)


def test_upsampling_small_and_ragged():
    say("up-sampling small")
    for n in (1, 17, 64, 65, 700):
        coords = synth.uniform_cells(n, 12, seed=n)
        d_coords = torch.from_numpy(coords).to(DEV)
        buf = sc.LayerBuffers(n, 2, 2, "strided", 32, 32, "f16", device=DEV)
        buf.kmap_build(d_coords, standalone=True)
        n_c = int(buf.read_counts().n_out)
        ref_km = oracle.kmap(coords, 2, 2, "strided")
        feat_c = synth.features(n_c, 64, "f16", n)
        w = synth.weights(8, 64, 32, "f16", n)
        fine = torch.full((n, 32), float("nan"), dtype=torch.float16, device=DEV)
        sc.sc_conv_up_fwd(to_dev(feat_c, "f16"), n, to_dev(w, "f16"), fine, buf.kmap, buf.counts, 2)
        ref = oracle.conv(feat_c, w, oracle.transpose_map(ref_km), threads=2)
        got = fine.double().cpu().numpy()
        assert np.isfinite(got).all()
        assert rel_err(got, ref) <= TOL["f16"]
    with pytest.raises(sc.ScError):
        sc.sc_conv_up_fwd(to_dev(feat_c, "f16")[:, :32].contiguous(), n, to_dev(synth.weights(8, 32, 48, "f16", 1), "f16"),
                          torch.empty((n, 48), dtype=torch.float16, device=DEV), buf.kmap, buf.counts, 2)


def test_random_layers():
    """A seeded sweep over layer kinds, kernel sizes, strides, channel counts, element types, sizes
    and both location tables, each layer checked like the named ones (map bit-exact, output within
    tolerance)."""
    rng = np.random.default_rng(2024)
    for it in range(48):
        kind = rng.choice(["subm", "strided", "strided_general"])
        dtype = str(rng.choice(["f16", "bf16", "f32"]))
        if dtype == "f32":
            C_in, C_out = int(rng.choice([3, 8, 16, 32, 48])), int(rng.choice([5, 16, 32, 64]))
        else:
            C_in, C_out = int(rng.choice([32, 64, 128])), int(rng.choice([16, 32, 48, 64, 128]))
        if kind == "subm":
            mode, K, s = "subm", int(rng.choice([1, 3, 3, 3, 5])), 1
        elif kind == "strided":
            mode, K = "strided", int(rng.choice([2, 2, 3, 4]))
            s = K
        else:
            mode, K = "strided", int(rng.choice([3, 3, 4, 5]))
            s = int(rng.integers(1, K))
        g = int(rng.choice([6, 12, 20, 30]))
        n = max(1, int(min(rng.integers(1, 12000), g ** 3 * 0.6)))
        coords = synth.uniform_cells(n, g, seed=int(rng.integers(1 << 30)))
        coords[:, 0] = rng.integers(0, 3, size=n)
        coords = np.unique(coords, axis=0)
        rng.shuffle(coords)
        coords = np.ascontiguousarray(coords.astype(np.int32))
        if mode == "strided" and K != s:
            coords = coords[:3000]
        grid = (3, g, g, g) if mode == "subm" and rng.random() < 0.3 else None
        say(f"random layer {it}: {mode} K={K} s={s} {dtype} {C_in}->{C_out} n={len(coords)} box={g} grid={grid is not None}")
        check_layer(coords, K, s, mode, C_in, C_out, dtype, seed=it, threads=8, grid_dims=grid)


# ---- the five named configurations at full size ----------------------------------------------
def sampled_rows_reference(feat, weight, ref_km, rows, threads=16):
    """The oracle's outputs on `rows` only: the pairs of other output rows are dropped first."""
    K3 = len(ref_km["offset_start"]) - 1
    keep = np.isin(ref_km["pair_out"], rows)
    ost = np.zeros(K3 + 1, np.int64)
    for k in range(K3):
        sl = slice(ref_km["offset_start"][k], ref_km["offset_start"][k + 1])
        ost[k + 1] = ost[k] + int(keep[sl].sum())
    sub = dict(ref_km, pair_in=ref_km["pair_in"][keep], pair_out=ref_km["pair_out"][keep], offset_start=ost)
    return oracle.conv(feat, weight, sub, threads=threads)


# The 64 -> 64 kernel puts 1..8 tiles into a workgroup depending on how many tiles there are per
# CU (4 beyond 8 per CU), and spreads a workgroup's tiles over the row range: tile = wavefront *
# units + unit.  One size per setting on a 256-CU device, fp32 output held to the fp32 tolerance.
@pytest.mark.parametrize("n_tiles,dtype", [(t, "f16") for t in (255, 300, 600, 1000, 1200, 1500, 1700, 2040, 2300)] +
                         [(t, "bf16") for t in (300, 1700, 2300)])
def test_64_channel_layer_at_every_tiles_per_workgroup(n_tiles, dtype):
    n = n_tiles * 64 - 37                      # ragged last tile
    say(f"64->64 {dtype} tiles={n_tiles} n={n}")
    side = int(np.ceil((n / 0.22) ** (1.0 / 3.0)))      # ~6 neighbours per voxel
    coords = synth.uniform_cells(n, side, seed=n_tiles)
    order = np.lexsort((coords[:, 3], coords[:, 2], coords[:, 1], coords[:, 0]))     # rows in x, y, z order
    coords = np.ascontiguousarray(coords[order])
    feat = synth.features(n, 64, dtype, 3)
    weight = synth.weights(27, 64, 64, dtype, 3)
    buf, h, out_coords, out = run_layer(coords, feat, weight, 3, 1, "subm", dtype, out_dtype="f32")
    ref_km = oracle.kmap(coords, 3, 1, "subm")
    assert h.n_pairs == ref_km["offset_start"][-1]
    assert_maps_equal(exported_map(buf, h), out_coords, ref_km, exact_order=True)
    rng = np.random.default_rng(n_tiles)
    # a random sample, both ends, and whole tiles on either side of the places where one
    # wavefront's share of the row range ends and the next one's begins
    per_cu = -(-n_tiles // 256)
    nwv = 4 if per_cu > 8 else per_cu
    units = -(-n_tiles // nwv)
    edges = [np.arange(max(0, w * units * 64 - 96), min(n, w * units * 64 + 96)) for w in range(1, nwv)]
    rows = np.unique(np.concatenate([rng.choice(n, 4000, replace=False), np.arange(0, 130), np.arange(n - 130, n)] + edges))
    ref = sampled_rows_reference(feat, weight, ref_km, rows)
    err = rel_err(out[rows], ref[rows])
    say(f"  sampled rows {len(rows)} max rel err {err:.3e}")
    assert err <= 1e-5


@pytest.mark.parametrize("dims,C", [((257, 257, 257), 64), ((512, 256, 256), 32)])
def test_layers_of_tens_of_millions_of_voxels(dims, C):
    """Table, map and convolution far beyond the named workloads.  (257, 257, 257), 64 channels:
    34 M voxels, the feature array passes 4 GiB, where the 64 -> 64 layer leaves the kernel with
    32-bit buffer offsets for the streaming kernel.  (512, 256, 256), 32 channels: exactly
    SC_N_MAX = 2^26 voxels, the largest input the library accepts.
    The voxel set has a closed form: cells (3i+1, 3j+1, 3k+1) and (3i+1, 3j+1, 3k+2) for
    (i, j, k) < dims, rows in that order, so row r has exactly one neighbour, row r^1, at dz = +1
    (offset 14) for even r and dz = -1 (offset 12) for odd r, and out[r] = in[r].W[13] +
    in[r^1].W[14 or 12] (the definition of the layer written out, Algorithm 2 with two terms),
    evaluated here in float64 on sampled rows."""
    I, J, Kd = dims
    n = 2 * I * J * Kd
    assert n <= sc.SC_N_MAX
    say(f"{C}->{C} f16, n={n}: feature array {n * C * 2 / 2 ** 30:.2f} GiB")
    r = torch.arange(n, device=DEV, dtype=torch.int64)
    t, cell = r & 1, r >> 1
    k, j, i = cell % Kd, (cell // Kd) % J, cell // (Kd * J)
    d_coords = torch.stack([torch.zeros_like(r), 3 * i + 1, 3 * j + 1, 3 * k + 1 + t], dim=1).to(torch.int32).contiguous()
    del r, t, cell, k, j, i
    gen = torch.Generator(device=DEV)
    gen.manual_seed(34)
    d_feat = torch.randn((n, C), generator=gen, device=DEV, dtype=torch.float32).to(torch.float16)
    weight = synth.weights(27, C, C, "f16", 34)
    d_w = to_dev(weight, "f16")
    buf = sc.LayerBuffers(n, 3, 1, "subm", C, C, "f16", device=DEV)
    buf.layer(d_coords, d_feat, d_w)
    h = buf.read_counts()
    assert h.status == 0 and h.n_out == n and h.n_pairs == 2 * n
    per_offset = [int(h.per_offset[q]) for q in range(27)]
    assert per_offset[13] == n and per_offset[12] == n // 2 and per_offset[14] == n // 2 and sum(per_offset) == 2 * n
    rng = np.random.default_rng(34)
    mid = (1 << 32) // (2 * C)          # the row at byte 2^32 of the feature array
    rows = np.unique(np.concatenate([rng.choice(n, 6000, replace=False), np.arange(0, 256), np.arange(n - 256, n),
                                     np.arange(min(mid, n) - 256, min(mid + 256, n))]))
    assert rows.min() >= 0 and rows.max() < n
    idx = torch.from_numpy(rows).to(DEV)
    f_own = d_feat[idx].double().cpu().numpy()
    f_nb = d_feat[idx ^ 1].double().cpu().numpy()
    w64 = weight.astype(np.float64)
    k_nb = np.where(rows % 2 == 0, 14, 12)
    ref = f_own @ w64[13] + np.einsum("rc,rcd->rd", f_nb, w64[k_nb])
    got = buf.feat_out[idx].double().cpu().numpy()
    err = rel_err(got, ref)
    say(f"  sampled rows {len(rows)} max rel err {err:.3e}")
    assert err <= TOL["f16"]
    # the table itself on the sampled rows, through the library's look-up: the neighbour's row number
    q = d_coords[idx].clone()
    q[:, 3] += torch.from_numpy(np.where(rows % 2 == 0, 1, -1)).to(DEV).to(torch.int32)
    found = torch.empty(len(rows), dtype=torch.int32, device=DEV)
    sc.sc_hash_lookup(buf.table, n, q.contiguous(), found)
    assert np.array_equal(found.cpu().numpy().astype(np.int64), rows ^ 1)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "target64"])
def test_named_config_full(name):
    say(f"config {name}")
    cfg = synth.make_config(name)
    err = check_layer(cfg["coords"], cfg["K"], cfg["stride"], cfg["mode"], cfg["C_in"], cfg["C_out"], cfg["dtype"],
                      threads=16)
    say(f"  {name}: N={len(cfg['coords'])} max rel err {err:.3e}")


@pytest.mark.parametrize("n,C_in,C_out,dtype", [(1, 32, 32, "f16"), (65, 64, 64, "bf16"), (1000, 32, 64, "f16"),
                                                 (1500, 64, 128, "f16"), (700, 128, 128, "bf16")])
def test_fused_dense_layer_small(n, C_in, C_out, dtype):
    """sc_conv_fwd_grid (look-ups inside the convolution, no kernel map) against the oracle, incl.
    voxels on the faces of the box and two batches."""
    say(f"fused dense layer n={n} {C_in}->{C_out} {dtype}")
    box = (2, 12, 12, 12)
    coords = synth.uniform_cells(n, 12, seed=n)
    coords[:, 0] = np.arange(n) % 2
    feat = synth.features(n, C_in, dtype, 1)
    weight = synth.weights(27, C_in, C_out, dtype, 1)
    buf = sc.LayerBuffers(n, 3, 1, "subm", C_in, C_out, dtype, device=DEV, grid_dims=box)
    buf.feat_out.fill_(float("nan"))
    buf.layer_fused(torch.from_numpy(coords).to(DEV), to_dev(feat, dtype), to_dev(weight, dtype))
    ref = oracle.conv(feat, weight, oracle.kmap(coords, 3, 1, "subm"), threads=8)
    err = rel_err(buf.feat_out[:n].double().cpu().numpy(), ref)
    assert err <= TOL[dtype], err


@pytest.mark.parametrize("name", ["cfg2", "cfg4", "target64", "cfg5"])
def test_fused_dense_layer_equals_three_call_layer(name):
    """The fused layer against the hash-table layer (which the tests above and below hold to the
    oracle), with fp32 outputs.  Where both run the same kernel the results are equal bit for bit;
    the 64-channel layer has its own kernel on the three-call path (another order of summation),
    there the two must agree to fp32 summation error."""
    say(f"config {name}, fused dense layer")
    cfg = synth.make_config(name)
    n = len(cfg["coords"])
    d_coords = torch.from_numpy(cfg["coords"]).to(DEV)
    d_feat, d_w = to_dev(cfg["feat"], cfg["dtype"]), to_dev(cfg["weight"], cfg["dtype"])
    a = sc.LayerBuffers(n, 3, 1, "subm", cfg["C_in"], cfg["C_out"], cfg["dtype"], "f32", device=DEV)
    a.layer(d_coords, d_feat, d_w)
    b = sc.LayerBuffers(n, 3, 1, "subm", cfg["C_in"], cfg["C_out"], cfg["dtype"], "f32", device=DEV, grid_dims=cfg["box"])
    b.layer_fused(d_coords, d_feat, d_w)
    torch.cuda.synchronize()
    if (cfg["C_in"], cfg["C_out"]) == (64, 64):
        err = float((a.feat_out[:n] - b.feat_out[:n]).abs().max() / a.feat_out[:n].abs().max())
        say(f"  {name}: fused vs three calls {err:.2e}")
        assert err <= 2e-6
    else:
        assert torch.equal(a.feat_out[:n], b.feat_out[:n])


PACKED_SHAPES = [(3, 1, "subm", "f16", 32, 32), (3, 1, "subm", "bf16", 64, 64), (3, 1, "subm", "f16", 128, 128),
                 (3, 1, "subm", "f16", 32, 64), (3, 1, "subm", "bf16", 64, 128), (2, 2, "strided", "f16", 32, 64),
                 (2, 2, "strided", "f16", 64, 64), (2, 2, "strided", "bf16", 128, 128), (3, 1, "subm", "f16", 256, 48),
                 (5, 1, "subm", "f16", 32, 32), (3, 1, "subm", "f32", 16, 16), (3, 2, "strided", "f16", 64, 64)]


@pytest.mark.parametrize("K,stride,mode,dtype,C_in,C_out", PACKED_SHAPES)
def test_packed_weights_give_the_same_layer(K, stride, mode, dtype, C_in, C_out):
    """sc_conv_weight_pack + sc_conv_fwd_packed: the same bits as sc_conv_fwd on raw weights, for
    every dedicated kernel and the generic one; the layer itself is held to the oracle."""
    say(f"packed weights K={K} s={stride} {mode} {dtype} {C_in}->{C_out}")
    coords = synth.lidar_scene(5)[:3000]
    n = len(coords)
    feat = synth.features(n, C_in, dtype, 3)
    weight = synth.weights(K ** 3, C_in, C_out, dtype, 3)
    for out_dtype in (None, "f32"):
        buf, h, out_coords, out = run_layer(coords, feat, weight, K, stride, mode, dtype, out_dtype)
        raw = buf.feat_out[:int(h.n_out)].clone()
        d_w = to_dev(weight, dtype)
        packed = sc.sc_conv_weight_pack(d_w, K)
        buf.feat_out.fill_(float("nan"))
        buf.conv_fwd_packed(to_dev(feat, dtype), packed)
        torch.cuda.synchronize()
        assert torch.equal(buf.feat_out[:int(h.n_out)], raw)
        ref = oracle.conv(feat, weight, oracle.kmap(coords, K, stride, mode))
        err = rel_err(out, ref)
        tol = 1e-5 if out_dtype == "f32" or dtype == "f32" else TOL[dtype]
        assert err <= tol, f"{err:.3e}"


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4", "target64", "cfg5"])
def test_named_config_dense_table(name):
    """The submanifold configurations again with the dense location table over the config's box:
    the kernel map must be the oracle's, bit for bit (cfg5: the map only, its outputs are checked
    with the hash-table build below - the convolution does not know which table made the map)."""
    say(f"config {name}, dense table")
    cfg = synth.make_config(name)
    if name != "cfg5":
        err = check_layer(cfg["coords"], cfg["K"], cfg["stride"], cfg["mode"], cfg["C_in"], cfg["C_out"], cfg["dtype"],
                          threads=16, grid_dims=cfg["box"])
        say(f"  {name}: max rel err {err:.3e}")
        return
    coords = cfg["coords"]
    n = len(coords)
    buf = sc.LayerBuffers(n, 3, 1, "subm", 128, 128, "f16", device=DEV, grid_dims=cfg["box"])
    d_coords = torch.from_numpy(coords).to(DEV)
    buf.hash_build(d_coords)
    buf.kmap_build(d_coords)
    h = buf.read_counts()
    ref_km = oracle.kmap(coords, 3, 1, "subm")
    assert h.n_pairs == ref_km["offset_start"][-1]
    assert_maps_equal(exported_map(buf, h), coords, ref_km, exact_order=True)


def test_cfg5_full_map_and_sampled_outputs():
    """~1M voxels, C=128: the whole kernel map is compared; outputs are compared on a sample of
    rows the oracle computes one by one (its triple loop over the full set takes minutes)."""
    say("config cfg5")
    cfg = synth.make_config("cfg5")
    coords, feat, weight = cfg["coords"], cfg["feat"], cfg["weight"]
    n = len(coords)
    buf, h, out_coords, out = run_layer(coords, feat, weight, 3, 1, "subm", "f16")
    ref_km = oracle.kmap(coords, 3, 1, "subm")
    say(f"  cfg5: N={n} P={ref_km['offset_start'][-1]}")
    assert h.n_pairs == ref_km["offset_start"][-1]
    assert_maps_equal(exported_map(buf, h), out_coords, ref_km, exact_order=True)
    rng = np.random.default_rng(0)
    # a random sample, both ends, and whole 64-row tiles on either side of every place where the
    # convolution's tile numbering changes hands: a workgroup of 8 wavefronts takes tiles
    # w * units + unit (w = wavefront), and the units go to the 8 XCDs in eighths
    units = (n + 511) // 512
    chunk = (units + 7) // 8
    edges = [np.arange(max(0, (w * units + c * chunk) * 64 - 128), min(n, (w * units + c * chunk) * 64 + 128))
             for w in range(8) for c in range(8)]
    rows = np.unique(np.concatenate([rng.choice(n, 20000, replace=False), np.arange(0, 200), np.arange(n - 200, n)] + edges))
    keep = np.isin(ref_km["pair_out"], rows)
    ost = np.zeros(28, np.int64)
    for k in range(27):
        sl = slice(ref_km["offset_start"][k], ref_km["offset_start"][k + 1])
        ost[k + 1] = ost[k] + int(keep[sl].sum())
    sub = dict(ref_km, pair_in=ref_km["pair_in"][keep], pair_out=ref_km["pair_out"][keep], offset_start=ost)
    ref = oracle.conv(feat, weight, sub, threads=16)
    err = rel_err(out[rows], ref[rows])
    say(f"  cfg5 sampled rows {len(rows)} max rel err {err:.3e}")
    assert err <= TOL["f16"]
    # every row, through a property that holds at any size: the sum of each 64-row tile of the
    # output equals sum_k (sum of the rows the tile gathers at k) . W[k] (tests/pins.py, checked
    # against the oracle's row-by-row result in the CPU suite).  The outputs are fp16: a tile sum
    # carries up to 64 roundings of 2^-11 relative each, ~2.5e-4 of the largest tile sum in
    # practice, while one wrong or missing row moves its tile's sum by a few per cent of it.
    tiles = -(-n // 64)
    padded = np.zeros((tiles * 64, out.shape[1]))
    padded[:n] = out
    got = padded.reshape(tiles, 64, -1).sum(axis=1)
    want = pins.group_sums_by_linearity(feat, weight, ref_km, 64)
    err_t = rel_err(got, want)
    say(f"  cfg5 sums of all {tiles} tiles: max rel err {err_t:.3e}")
    assert err_t <= 2e-3
