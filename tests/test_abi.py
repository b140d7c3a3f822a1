"""CPU tests: the C-ABI library builds, loads and exports every symbol include/sc.h declares;
host-side argument checks and size queries (no kernel is launched)."""
import ctypes
import os
import re

import pytest

from paper_2402_07710_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in sc.h but not exported by libsc.so"
    assert sorted(binding.SYMBOLS) == names


def test_counts_struct_layout():
    assert ctypes.sizeof(binding.ScCounts) == 24 + 343 * 4 + 4
    assert binding.ScCounts.per_offset.offset == 24
    assert binding.ScCounts.status.offset == 24 + 343 * 4


def test_size_queries(lib):
    # 16-byte slots; capacity = power of two >= 32n while that is at most 2^22 slots, never below 8n
    # or 1024; plus the 256-byte header
    assert lib.sc_hash_bytes(0) == 1024 * 16 + 256
    assert lib.sc_hash_bytes(32) == 1024 * 16 + 256
    assert lib.sc_hash_bytes(33) == 2048 * 16 + 256
    assert lib.sc_hash_bytes(1000) == 32768 * 16 + 256
    assert lib.sc_hash_bytes(1025) == 65536 * 16 + 256
    assert lib.sc_hash_bytes(131072) == (1 << 22) * 16 + 256
    assert lib.sc_hash_bytes(200000) == (1 << 22) * 16 + 256          # 16n < 2^22 <= 32n: capped
    assert lib.sc_hash_bytes(524288) == (1 << 22) * 16 + 256          # exactly 8n
    assert lib.sc_hash_bytes(524289) == (1 << 23) * 16 + 256          # 8n rules from here on
    assert lib.sc_hash_bytes(-1) == 0
    assert lib.sc_out_bound(500, 3, 1, binding.SC_SUBM) == 500
    assert lib.sc_out_bound(500, 2, 2, binding.SC_STRIDED) == 500
    # K != stride: an input can sit in ceil(K/s)^3 output cells
    assert lib.sc_out_bound(500, 3, 2, binding.SC_STRIDED) == 500 * 8
    assert lib.sc_out_bound(500, 3, 1, binding.SC_STRIDED) == 500 * 27
    assert lib.sc_out_bound(500, 5, 5, binding.SC_STRIDED) == 500
    assert lib.sc_out_bound(500, 2, 3, binding.SC_STRIDED) == -1     # stride > K leaves inputs unused
    assert lib.sc_out_bound(1 << 24, 3, 2, binding.SC_STRIDED) == -1  # more candidates than rows a map can hold
    assert lib.sc_out_bound(500, 3, 2, binding.SC_INVERSE) == -1
    assert lib.sc_out_bound(500, 2, 1, binding.SC_SUBM) == -1      # even K has no centre
    assert lib.sc_out_bound(500, 3, 2, binding.SC_SUBM) == -1      # submanifold stride is 1
    assert lib.sc_kmap_bytes(500, 9, 1, binding.SC_SUBM) == 0
    # tile-major offset table: header + 4 mask words per tile + one int32 per (row, offset)
    b = lib.sc_kmap_bytes(6400, 3, 1, binding.SC_SUBM)
    assert b >= 100 * 64 * 27 * 4 + 100 * 16 and b < 100 * 64 * 27 * 4 + 100 * 16 + 1024
    assert lib.sc_kmap_scratch_bytes(6400, 2, 2, binding.SC_STRIDED) > 32768 * 16 + 6400 * 4
    assert lib.sc_conv_workspace_bytes(3, 64, 64, binding.SC_F16) == 27 * 64 * 64 * 2
    assert lib.sc_conv_workspace_bytes(3, 16, 16, binding.SC_F32) == 0
    # dense location table: one 8-byte cell per site
    assert lib.sc_grid_bytes(1, 1408, 1600, 41) == 1408 * 1600 * 41 * 8
    assert lib.sc_grid_bytes(2, 3, 5, 7) == 1792                       # 210 cells, rounded up to 256 bytes
    assert lib.sc_grid_bytes(0, 4, 4, 4) == 0 and lib.sc_grid_bytes(1, 4, -4, 4) == 0
    assert lib.sc_grid_bytes(1, 65536, 4, 4) == 0                      # a side beyond the coordinate range
    assert lib.sc_grid_bytes(1, 65535, 65535, 3) == 0                  # more than 2^33 sites


def test_host_side_argument_errors(lib):
    # null pointers and bad shapes are rejected before anything is enqueued (no GPU needed)
    assert lib.sc_hash_build(None, 10, None, 0, None, None) == binding.SC_EINVAL
    assert lib.sc_hash_build(None, -1, 16, 0, 16, None) == binding.SC_EINVAL
    assert lib.sc_hash_build(16, 10, 32, 8, 48, None) == binding.SC_ECAP
    assert lib.sc_hash_build(17, 10, 32, 1 << 20, 48, None) == binding.SC_EINVAL      # misaligned
    for epoch in (0, -1, binding.SC_HASH_EPOCH_MAX + 1):
        assert lib.sc_hash_rebuild(16, 10, 32, 1 << 20, epoch, 48, None) == binding.SC_EINVAL
    assert lib.sc_hash_rebuild(16, 10, 32, 8, 1, 48, None) == binding.SC_ECAP
    assert lib.sc_hash_rebuild(None, 10, 32, 1 << 20, 1, 48, None) == binding.SC_EINVAL
    assert lib.sc_kmap_build(16, 10, 32, 2, 1, binding.SC_SUBM, None, 64, 1 << 20, None, 0, 80, None) == binding.SC_EINVAL
    assert lib.sc_kmap_build(16, 10, 32, 3, 1, binding.SC_SUBM, None, 64, 8, None, 0, 80, None) == binding.SC_ECAP
    assert lib.sc_kmap_build(16, 10, None, 3, 1, binding.SC_SUBM, None, 64, 1 << 20, None, 0, 80, None) == binding.SC_EINVAL
    assert lib.sc_conv_fwd(16, 10, 32, 48, 10, 64, 1 << 20, 80, 3, 1, binding.SC_SUBM, 24, 32, binding.SC_F16,
                           binding.SC_F16, 96, 1 << 20, None) == binding.SC_EINVAL   # C_in not 32/64/128/256
    assert lib.sc_conv_fwd(16, 10, 32, 48, 10, 64, 1 << 20, 80, 3, 1, binding.SC_SUBM, 32, 32, binding.SC_F16,
                           binding.SC_BF16, 96, 1 << 20, None) == binding.SC_EINVAL  # output type mismatch
    assert lib.sc_conv_fwd(16, 10, 32, 48, 10, 64, 1 << 20, 80, 3, 1, binding.SC_SUBM, 32, 32, binding.SC_F16,
                           binding.SC_F16, 96, 16, None) == binding.SC_ECAP          # workspace too small
    gb = lib.sc_grid_bytes(1, 8, 8, 8)
    assert lib.sc_grid_build(16, 10, 32, gb, 1, 8, 8, 8, 0, 48, None) == binding.SC_EINVAL       # epoch 0 is "never"
    assert lib.sc_grid_build(16, 10, 32, gb - 1, 1, 8, 8, 8, 1, 48, None) == binding.SC_ECAP
    assert lib.sc_grid_build(16, 10, 32, gb, 1, 8, 0, 8, 1, 48, None) == binding.SC_EINVAL
    assert lib.sc_grid_clear(None, gb, 1, 8, 8, 8, None) == binding.SC_EINVAL
    assert lib.sc_grid_lookup(32, 1, 8, 8, 8, 0, 16, 4, 48, None) == binding.SC_EINVAL
    assert lib.sc_kmap_build_grid(16, 10, 32, gb, 1, 8, 8, 8, 1, 2, 64, 1 << 20, 80, None) == binding.SC_EINVAL  # even K
    assert lib.sc_kmap_build_grid(16, 10, 32, gb, 1, 8, 8, 8, 1, 3, 64, 8, 80, None) == binding.SC_ECAP
    assert lib.sc_conv_fwd_grid(16, 32, 10, 48, gb, 1, 8, 8, 8, 1, 64, 80, 5, 32, 32, binding.SC_F16, binding.SC_F16,
                                96, 1 << 20, None) == binding.SC_EINVAL                 # 3x3x3 only
    assert lib.sc_conv_fwd_grid(16, 32, 10, 48, gb, 1, 8, 8, 8, 1, 64, 80, 3, 32, 32, binding.SC_F32, binding.SC_F32,
                                96, 1 << 20, None) == binding.SC_EINVAL                 # 16-bit layers only
    assert lib.sc_conv_fwd_grid(16, 32, 10, 48, gb, 1, 8, 8, 8, 1, 64, 80, 3, 32, 32, binding.SC_F16, binding.SC_F16,
                                96, 16, None) == binding.SC_ECAP                        # workspace too small
    # sc_conv_up_fwd(feat_coarse, n_map, weight, feat_fine, kmap, kmap_bytes, counts, K, C_in, C_out, dt_in, dt_out, stream)
    F16, F32 = binding.SC_F16, binding.SC_F32
    assert lib.sc_conv_up_fwd(16, 10, 32, 48, 64, 1 << 20, 80, 5, 32, 32, F16, F16, None) == binding.SC_EINVAL   # K
    assert lib.sc_conv_up_fwd(16, 10, 32, 48, 64, 1 << 20, 80, 2, 32, 32, F32, F32, None) == binding.SC_EINVAL   # dtype
    assert lib.sc_conv_up_fwd(16, 10, 32, 48, 64, 1 << 20, 80, 2, 32, 32, F16, binding.SC_BF16, None) == binding.SC_EINVAL
    assert lib.sc_conv_up_fwd(16, 10, 32, 48, 64, 8, 80, 2, 32, 32, F16, F16, None) == binding.SC_ECAP           # map blob
    assert lib.sc_conv_up_fwd(16, 10, 32, 48, 64, 1 << 20, 80, 2, 32, 48, F16, F16, None) == binding.SC_EINVAL   # shape
    assert lib.sc_conv_up_fwd(16, 10, None, 48, 64, 1 << 20, 80, 2, 32, 32, F16, F16, None) == binding.SC_EINVAL
    assert lib.sc_conv_up_fwd(17, 10, 32, 48, 64, 1 << 20, 80, 2, 32, 32, F16, F16, None) == binding.SC_EINVAL   # misaligned
    assert binding.strerror(binding.SC_EDUP) == "duplicate input coordinate"
    assert binding.strerror(12345) == "unknown status"


def _insert_probe_lengths(lib, coords, n):
    """Simulate the table build on the host with the library's own probe sequence: number of
    attempts every key needs until it finds a free slot."""
    taken = set()
    lengths = []
    for b, x, y, z in coords:
        t = 0
        while True:
            slot = lib.sc_hash_probe_slot(int(b), int(x), int(y), int(z), t, n)
            assert slot >= 0
            if slot not in taken:
                taken.add(slot)
                break
            t += 1
        lengths.append(t + 1)
    return lengths


def test_probe_sequence_on_lattice_aligned_keys(lib):
    """Voxel sets whose coordinates are all multiples of 2 or 4 (down-sampled sets kept at the
    original scale) must not pile up on a few places of every 64-slot region."""
    import numpy as np
    rng = np.random.default_rng(5)
    n = 20000
    cells = rng.choice(48 ** 3, size=n, replace=False)
    for lattice in (1, 2, 4):
        coords = [(0, (c // 2304) * lattice, ((c // 48) % 48) * lattice, (c % 48) * lattice) for c in cells.tolist()]
        lengths = _insert_probe_lengths(lib, coords, n)
        assert sum(lengths) / n < 1.1, (lattice, sum(lengths) / n)
        assert max(lengths) <= 6, (lattice, max(lengths))
    assert lib.sc_hash_probe_slot(0, -1, 0, 0, 0, n) == -1
