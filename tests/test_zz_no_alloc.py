"""GPU test of sc_kmap_build_noalloc: the kernel-map build whose scratch lives in a fixed device
array of the library.  Called through the C ABI (raw ctypes), its results must equal those of
sc_kmap_build bit for bit: maps, output coordinates, counts; two calls in a row on the same GPU,
the second with a smaller input (the shared array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2402_07710_amd import binding as sc
from paper_2402_07710_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def build_both(lib, coords, K, stride, mode):
    """(reference results, no-alloc results) of one build; each a dict of host arrays."""
    n = len(coords)
    d_coords = torch.from_numpy(np.ascontiguousarray(coords, dtype=np.int32)).to(DEV).reshape(-1, 4)
    stream = torch.cuda.current_stream().cuda_stream
    bound = sc.sc_out_bound(n, K, stride, mode)
    results = []
    for variant in ("scratch argument", "library array"):
        table = torch.empty(max(sc.sc_hash_bytes(n), 16), dtype=torch.uint8, device=DEV)
        counts = torch.zeros(sc.COUNTS_BYTES + 8, dtype=torch.uint8, device=DEV)
        kmap = torch.zeros(max(sc.sc_kmap_bytes(n, K, stride, mode), 16), dtype=torch.uint8, device=DEV)
        out_coords = torch.full((max(bound, 1), 4), -7, dtype=torch.int32, device=DEV)
        rc = lib.sc_hash_build(d_coords.data_ptr(), n, table.data_ptr(), table.numel(), counts.data_ptr(), stream)
        assert rc == sc.SC_OK
        if variant == "scratch argument":
            scratch = torch.empty(max(sc.sc_kmap_scratch_bytes(n, K, stride, mode), 16), dtype=torch.uint8, device=DEV)
            rc = lib.sc_kmap_build(d_coords.data_ptr(), n, table.data_ptr(), K, stride, sc.MODES[mode],
                                   out_coords.data_ptr(), kmap.data_ptr(), kmap.numel(), scratch.data_ptr(),
                                   scratch.numel(), counts.data_ptr(), stream)
        else:
            rc = lib.sc_kmap_build_noalloc(d_coords.data_ptr(), n, table.data_ptr(), K, stride, sc.MODES[mode],
                                           out_coords.data_ptr(), kmap.data_ptr(), kmap.numel(), counts.data_ptr(),
                                           stream)
        assert rc == sc.SC_OK, (variant, rc)
        h = sc.ScCounts()
        rc = lib.sc_counts_read(counts.data_ptr(), ctypes.byref(h), kmap.data_ptr(), n, K, stride, sc.MODES[mode], stream)
        assert rc == sc.SC_OK, (variant, rc)
        pin, pout, ost = sc.sc_kmap_export(kmap, n, K, stride, mode, h)
        results.append(dict(n_out=int(h.n_out), n_pairs=int(h.n_pairs), per_offset=list(h.per_offset[:K ** 3]),
                            out_coords=out_coords[:int(h.n_out)].cpu().numpy(), pin=pin.cpu().numpy(),
                            pout=pout.cpu().numpy(), ost=ost.cpu().numpy()))
    return results


def assert_same(a, b):
    assert a["n_out"] == b["n_out"] and a["n_pairs"] == b["n_pairs"] and a["per_offset"] == b["per_offset"]
    for key in ("out_coords", "pin", "pout", "ost"):
        assert np.array_equal(a[key], b[key]), key


@pytest.mark.parametrize("K,stride,mode,n_first,n_second", [(2, 2, "strided", 40000, 9000), (3, 2, "strided", 6000, 700),
                                                             (3, 1, "subm", 5000, 300)])
def test_noalloc_build_equals_the_build_with_a_scratch_argument(K, stride, mode, n_first, n_second):
    lib = sc.load(build_if_missing=False)
    scene = synth.lidar_scene(3)
    for n in (n_first, n_second):            # two calls in a row, the second with fewer rows
        print(f"noalloc K={K} s={stride} {mode} n={n}", flush=True)
        ref, got = build_both(lib, scene[:n], K, stride, mode)
        assert ref["n_pairs"] > 0
        assert_same(ref, got)


def test_noalloc_build_refuses_what_does_not_fit():
    lib = sc.load(build_if_missing=False)
    n = 200_000                               # K == stride needs 8 slots of 16 bytes per row: far above 16 MiB
    assert sc.sc_kmap_scratch_bytes(n, 2, 2, "strided") > (16 << 20)
    dummy = torch.zeros(64, dtype=torch.uint8, device=DEV)
    rc = lib.sc_kmap_build_noalloc(dummy.data_ptr(), n, None, 2, 2, sc.SC_STRIDED, dummy.data_ptr(), dummy.data_ptr(),
                                   sc.sc_kmap_bytes(n, 2, 2, "strided"), dummy.data_ptr(), None)
    assert rc == sc.SC_ECAP
