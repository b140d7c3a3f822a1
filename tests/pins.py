"""Checks that pin the CPU oracle to facts fixed by the paper and by mathematics.

Every function takes an oracle object (`oracle.Oracle`) and raises AssertionError when the
oracle disagrees with the pinned fact.  They are written against the oracle's *interface* only
so the same checks can be run on deliberately broken builds of the oracle source (the mutant
test), which shows that the pins can tell a wrong oracle from a right one.
"""
from __future__ import annotations

import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ---------------------------------------------------------------------------------------------
# an independent dense evaluation (numpy arrays over the whole grid, no coordinate lookups)
# ---------------------------------------------------------------------------------------------
def dense_conv3d(coords, feat, weight, K, stride, mode, grid, n_batch):
    """Dense 3-D correlation over a full grid: zero-padded "same" for submanifold layers,
    stride-s "valid" from the origin for strided layers (Section II-B's dense convolution).
    Returns (dense output [B,X',Y',Z',C_out], active-output mask [B,X',Y',Z'])."""
    C_in, C_out = weight.shape[1], weight.shape[2]
    pad = (K - 1) // 2 if mode == "subm" else 0
    # dense input with a margin of K cells on every side so all windows are in range
    m = K
    dense = np.zeros((n_batch, grid + 2 * m, grid + 2 * m, grid + 2 * m, C_in))
    occ = np.zeros(dense.shape[:4], dtype=bool)
    for row, f in zip(coords, feat):
        b, x, y, z = (int(v) for v in row)
        dense[b, x + m, y + m, z + m] = f
        occ[b, x + m, y + m, z + m] = True
    if mode == "subm":
        n_o = grid
    else:
        n_o = (grid - 1) // stride + 1          # every q with q*s <= grid-1 can be reached
    out = np.zeros((n_batch, n_o, n_o, n_o, C_out))
    hit = np.zeros((n_batch, n_o, n_o, n_o), dtype=bool)
    for dx in range(K):
        for dy in range(K):
            for dz in range(K):
                k = (dx * K + dy) * K + dz
                sl = tuple(slice(m + d - pad, m + d - pad + (n_o - 1) * stride + 1, stride)
                           for d in (dx, dy, dz))
                win = dense[(slice(None),) + sl]              # [B, n_o, n_o, n_o, C_in]
                out += win @ weight[k]
                hit |= occ[(slice(None),) + sl]
    if mode == "subm":
        active = occ[:, m:m + grid, m:m + grid, m:m + grid]
    else:
        active = hit
    return out, active


def check_dense(orc, rng, grid, n, K, stride, mode, C_in, C_out, n_batch=1):
    """Oracle output equals the dense evaluation at every active output site, and the oracle's
    output sites are exactly the dense evaluation's active sites."""
    cells = rng.choice(n_batch * grid ** 3, size=n, replace=False)
    b, rem = np.divmod(cells, grid ** 3)
    x, rem = np.divmod(rem, grid * grid)
    y, z = np.divmod(rem, grid)
    coords = np.stack([b, x, y, z], axis=1).astype(np.int32)
    feat = rng.standard_normal((n, C_in))
    weight = rng.standard_normal((K ** 3, C_in, C_out))
    out_coords, out, km = orc.sparse_conv(coords, feat, weight, K, stride, mode)
    ref, active = dense_conv3d(coords, feat, weight, K, stride, mode, grid, n_batch)
    assert len(out_coords) == int(active.sum()), (len(out_coords), int(active.sum()))
    seen = np.zeros_like(active)
    for row, f in zip(out_coords, out):
        bb, xx, yy, zz = (int(v) for v in row)
        assert active[bb, xx, yy, zz], f"oracle output site {row} is not an active dense site"
        assert not seen[bb, xx, yy, zz], f"oracle output site {row} listed twice"
        seen[bb, xx, yy, zz] = True
        np.testing.assert_allclose(f, ref[bb, xx, yy, zz], rtol=1e-12, atol=1e-12)
    if mode == "subm":
        assert np.array_equal(out_coords, coords)


# ---------------------------------------------------------------------------------------------
# the paper's worked figures and equations
# ---------------------------------------------------------------------------------------------
def _read_blocks(path):
    blocks, cur = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0].isalpha() and len(tok) == 1:
            cur = tok[0]
            blocks[cur] = []
        elif tok[0] == "ERRATUM":
            blocks.setdefault("ERRATUM", []).append([int(t) for t in tok[1:]])
        else:
            blocks[cur].append([int(t) for t in tok])
    return blocks


def check_fig_subm_2d(orc):
    """Section II-B figure: 7x7 input, 3x3 kernel, printed 5x5 interior result."""
    blk = _read_blocks(os.path.join(GOLDEN, "fig_subm_2d.txt"))
    I = np.array(blk["INPUT"])
    Kk = np.array(blk["KERNEL"], dtype=np.float64)
    R = np.array(blk["RESULT"], dtype=np.float64)
    for r, c, printed, defined in blk["ERRATUM"]:
        assert R[r, c] == printed
        R[r, c] = defined
    rows, cols = np.nonzero(I)
    coords = np.stack([np.zeros_like(rows), rows, cols, np.zeros_like(rows)], axis=1).astype(np.int32)
    feat = I[rows, cols].astype(np.float64)[:, None]
    W = np.zeros((27, 1, 1))
    for dx in range(3):
        for dy in range(3):
            W[(dx * 3 + dy) * 3 + 1, 0, 0] = Kk[dx, dy]        # the dz = centre plane
    out_coords, out, _ = orc.sparse_conv(coords, feat, W, 3, 1, "subm")
    got = np.zeros((7, 7))
    got[out_coords[:, 1], out_coords[:, 2]] = out[:, 0]
    # inactive centres produce no output row (the figure's red cells) ...
    assert len(out_coords) == int(I.sum())
    # ... and the interior agrees with the printed matrix
    np.testing.assert_array_equal(got[1:6, 1:6], R)


def check_fig_oft_2d(orc):
    """Section III-C figure: OFT rows of three diagonal points, columns 0, 4 and 8."""
    pts, rows = {}, {}
    order = []
    for line in open(os.path.join(GOLDEN, "fig_oft_2d.txt")):
        tok = line.split()
        if not tok or tok[0].startswith("#"):
            continue
        if tok[0] == "POINT":
            pts[tok[1]] = (int(tok[2]), int(tok[3]))
            order.append(tok[1])
        elif tok[0] == "ROW":
            rows[tok[1]] = tok[2:5]
    # give the three points non-trivial row indices by surrounding them with far-away filler
    names = ["f0", order[2], "f1", order[0], order[1]]
    xy = {"f0": (5, 50), "f1": (50, 5), **pts}
    coords = np.array([[0, xy[nm][0], xy[nm][1], 0] for nm in names], dtype=np.int32)
    km = orc.kmap(coords, 3, 1, "subm")
    oft = np.full((len(coords), 27), -1, dtype=np.int64)
    ost = km["offset_start"]
    for k in range(27):
        for e in range(ost[k], ost[k + 1]):
            assert oft[km["pair_out"][e], k] == -1
            oft[km["pair_out"][e], k] = km["pair_in"][e]
    index = {nm: i for i, nm in enumerate(names)}
    for nm, (c0, c4, c8) in rows.items():
        for col2d, want in zip((0, 4, 8), (c0, c4, c8)):
            dx, dy = divmod(col2d, 3)
            k = (dx * 3 + dy) * 3 + 1
            expect = -1 if want == "-1" else index[want]
            assert oft[index[nm], k] == expect, (nm, col2d, oft[index[nm], k], expect)


def check_eq_cell_mapping(orc):
    """Section III-B eq. 1-5 on single points (K = s)."""
    for line in open(os.path.join(GOLDEN, "eq_cell_mapping.txt")):
        tok = line.split()
        if not tok or tok[0].startswith("#"):
            continue
        x, y, z, s, k, ox, oy, oz, ko = (int(t) for t in tok)
        km = orc.kmap(np.array([[3, x, y, z]], dtype=np.int32), k, s, "strided")
        assert km["n_out"] == 1
        assert tuple(km["out_coords"][0]) == (3, ox, oy, oz)
        ost = km["offset_start"]
        assert ost[-1] == 1 and ost[ko] == 0 and ost[ko + 1] == 1, (ko, ost)


# ---------------------------------------------------------------------------------------------
# structural facts of kernel maps
# ---------------------------------------------------------------------------------------------
def check_symmetry_and_centre(orc, coords, K):
    """Submanifold maps: (i,j) at k <=> (j,i) at K³-1-k; the centre offset is the identity."""
    km = orc.kmap(coords, K, 1, "subm")
    ost = km["offset_start"]
    K3 = K ** 3
    sets = [set(zip(km["pair_in"][ost[k]:ost[k + 1]].tolist(), km["pair_out"][ost[k]:ost[k + 1]].tolist()))
            for k in range(K3)]
    for k in range(K3):
        assert len(sets[k]) == ost[k + 1] - ost[k]
        assert sets[K3 - 1 - k] == {(o, i) for (i, o) in sets[k]}
    n = len(coords)
    assert sets[(K3 - 1) // 2] == {(i, i) for i in range(n)}


def check_delta_weights(orc, coords, feat, K):
    """W[centre] = I, else 0 reproduces the input bit for bit; W[k0] = I for another k0 is a
    pure shift: row i receives the row of the voxel at p_i + d_k0 - pad, or zero."""
    C = feat.shape[1]
    K3 = K ** 3
    pad = (K - 1) // 2
    W = np.zeros((K3, C, C))
    W[(K3 - 1) // 2] = np.eye(C)
    _, out, _ = orc.sparse_conv(coords, feat, W, K, 1, "subm")
    assert np.array_equal(out, feat.astype(np.float64))
    lookup = {tuple(int(v) for v in row): i for i, row in enumerate(coords)}
    for k0 in (0, 5, K3 - 1, K3 - 3):
        W = np.zeros((K3, C, C))
        W[k0] = np.eye(C)
        d = (k0 // (K * K), (k0 // K) % K, k0 % K)
        _, out, _ = orc.sparse_conv(coords, feat, W, K, 1, "subm")
        for i, row in enumerate(coords):
            nb = (int(row[0]), int(row[1]) + d[0] - pad, int(row[2]) + d[1] - pad, int(row[3]) + d[2] - pad)
            j = lookup.get(nb)
            want = feat[j] if j is not None else np.zeros(C)
            assert np.array_equal(out[i], want), (k0, i)


def check_full_grid_counts(orc, n):
    """All n³ cells active: the K=3 submanifold map has (3n-2)³ pairs; for even n the K=s=2
    strided map has (n/2)³ outputs and exactly that many pairs at every offset."""
    g = np.arange(n)
    x, y, z = np.meshgrid(g, g, g, indexing="ij")
    coords = np.stack([np.zeros(n ** 3, dtype=np.int64), x.ravel(), y.ravel(), z.ravel()], axis=1).astype(np.int32)
    km = orc.kmap(coords, 3, 1, "subm")
    assert km["offset_start"][-1] == (3 * n - 2) ** 3
    # per offset: (n-|dx|)(n-|dy|)(n-|dz|)
    for k in range(27):
        d = (k // 9 - 1, (k // 3) % 3 - 1, k % 3 - 1)
        want = np.prod([n - abs(v) for v in d])
        assert km["offset_start"][k + 1] - km["offset_start"][k] == want
    if n % 2 == 0:
        km = orc.kmap(coords, 2, 2, "strided")
        assert km["n_out"] == (n // 2) ** 3
        assert np.all(np.diff(km["offset_start"]) == (n // 2) ** 3)


def check_isolated_is_matmul(orc, rng):
    """Voxels at pairwise Chebyshev distance >= K: every voxel only sees itself, so the layer
    is one plain matrix product with the centre weight."""
    K, C_in, C_out = 3, 5, 7
    g = np.arange(0, 30, 3)
    x, y, z = np.meshgrid(g, g, g, indexing="ij")
    coords = np.stack([np.ones(x.size, dtype=np.int64), x.ravel(), y.ravel(), z.ravel()], axis=1).astype(np.int32)
    coords = coords[rng.permutation(len(coords))[:200]]
    feat = rng.standard_normal((len(coords), C_in))
    W = rng.standard_normal((27, C_in, C_out))
    _, out, km = orc.sparse_conv(coords, feat, W, K, 1, "subm")
    assert km["offset_start"][-1] == len(coords)
    np.testing.assert_allclose(out, feat @ W[13], rtol=1e-13, atol=1e-13)


def check_strided_partition(orc, coords, s):
    """K = s strided map: every input appears in exactly one pair, the outputs are the distinct
    cells floor(p/s) numbered by first occurrence, and each pair's offset is p - floor(p/s)*s."""
    km = orc.kmap(coords, s, s, "strided")
    n = len(coords)
    assert km["offset_start"][-1] == n
    assert np.array_equal(np.sort(km["pair_in"]), np.arange(n))
    q = coords.copy()
    q[:, 1:] //= s
    _, first = np.unique(q, axis=0, return_index=True)
    want = q[np.sort(first)]
    assert np.array_equal(km["out_coords"], want)
    ost = km["offset_start"]
    for k in range(s ** 3):
        for e in range(ost[k], ost[k + 1]):
            i, o = km["pair_in"][e], km["pair_out"][e]
            d = coords[i, 1:] - km["out_coords"][o, 1:] * s
            assert coords[i, 0] == km["out_coords"][o, 0]
            assert (d[0] * s + d[1]) * s + d[2] == k


def check_invariances(orc, rng, coords, K, stride, mode, C_in=3, C_out=4):
    n = len(coords)
    # keep every window clear of the q >= 0 boundary, where a translated set gains outputs
    coords = coords + np.array([0, K * stride, K * stride, K * stride], dtype=np.int32)
    f1, f2 = rng.standard_normal((n, C_in)), rng.standard_normal((n, C_in))
    W1, W2 = rng.standard_normal((K ** 3, C_in, C_out)), rng.standard_normal((K ** 3, C_in, C_out))
    oc, o11, km = orc.sparse_conv(coords, f1, W1, K, stride, mode)
    # linearity in the features and in the weights
    np.testing.assert_allclose(orc.conv(2.5 * f1 - f2, W1, km), 2.5 * o11 - orc.conv(f2, W1, km), atol=1e-11)
    np.testing.assert_allclose(orc.conv(f1, W1 + 3 * W2, km), o11 + 3 * orc.conv(f1, W2, km), atol=1e-11)
    # translation by a multiple of the stride: same map, outputs shifted by t/stride
    t = np.array([0, 4 * stride, 2 * stride, 6 * stride], dtype=np.int32)
    oc_t, o_t, km_t = orc.sparse_conv(coords + t, f1, W1, K, stride, mode)
    assert np.array_equal(oc_t, oc + t // np.array([1, stride, stride, stride]))
    assert np.array_equal(km_t["pair_in"], km["pair_in"]) and np.array_equal(km_t["pair_out"], km["pair_out"])
    assert np.array_equal(o_t, o11)
    # permuting the input rows permutes submanifold outputs identically
    if mode == "subm":
        perm = rng.permutation(n)
        _, o_p, _ = orc.sparse_conv(coords[perm], f1[perm], W1, K, stride, mode)
        np.testing.assert_allclose(o_p, o11[perm], atol=1e-12)
    # batches never interact: two copies in different batch slots = two separate results
    c2 = coords.copy()
    c2[:, 0] += int(coords[:, 0].max()) + 1
    both = np.concatenate([coords, c2])
    oc_b, o_b, _ = orc.sparse_conv(both, np.concatenate([f1, f2]), W1, K, stride, mode)
    _, o22, _ = orc.sparse_conv(c2, f2, W1, K, stride, mode)
    m = len(oc)
    assert np.array_equal(oc_b[:m], oc) and np.array_equal(oc_b[m:, 1:], oc[:, 1:])
    np.testing.assert_allclose(o_b[:m], o11, atol=1e-12)
    np.testing.assert_allclose(o_b[m:], o22, atol=1e-12)


def alg2_out_major(feat_in, oft, w_paper):
    """Algorithm 2 evaluated in its own loop order (output row, output channel, offset, input
    channel) on an offset table, with the weight laid out [C_out][K³][C_in] as the algorithm
    indexes it."""
    n_out, K3 = oft.shape
    C_out, _, C_in = w_paper.shape
    out = np.zeros((n_out, C_out))
    for i in range(n_out):
        for o in range(C_out):
            s = 0.0
            for k in range(K3):
                j = oft[i, k]
                if j != -1:
                    for c in range(C_in):
                        s += feat_in[j, c] * w_paper[o, k, c]
            out[i, o] = s
    return out


def check_alg2_formulation(orc, rng, coords, K, stride, mode, C_in=3, C_out=2):
    """The per-offset pair-list evaluation equals Algorithm 2's out-major evaluation."""
    n = len(coords)
    feat = rng.standard_normal((n, C_in))
    W = rng.standard_normal((K ** 3, C_in, C_out))
    _, out, km = orc.sparse_conv(coords, feat, W, K, stride, mode)
    oft = np.full((km["n_out"], K ** 3), -1, dtype=np.int64)
    ost = km["offset_start"]
    for k in range(K ** 3):
        sl = slice(ost[k], ost[k + 1])
        assert np.all(oft[km["pair_out"][sl], k] == -1)
        oft[km["pair_out"][sl], k] = km["pair_in"][sl]
    ref = alg2_out_major(feat, oft, np.ascontiguousarray(W.transpose(2, 0, 1)))
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)


def group_sums_by_linearity(feat, weight, km, rows_per_group):
    """Sums of the layer output over groups of consecutive output rows, without evaluating the
    layer row by row: the sum over a group of sum_k in[i].W[k] is sum_k (sum of the input rows
    the group gathers at k).W[k] - one sparse row-sum and one matrix product per offset.
    Needs only a kernel map and library matrix products, so it reaches sizes at which the triple
    loop takes minutes.  Returns [ceil(n_out / rows_per_group)][C_out] in float64."""
    import scipy.sparse as sp
    K3, C_in, C_out = weight.shape
    n_in, n_out = feat.shape[0], int(km["n_out"])
    n_groups = -(-n_out // rows_per_group)
    f64, w64 = np.asarray(feat, dtype=np.float64), np.asarray(weight, dtype=np.float64)
    ost = km["offset_start"]
    total = np.zeros((n_groups, C_out))
    for k in range(K3):
        sl = slice(int(ost[k]), int(ost[k + 1]))
        pi, po = np.asarray(km["pair_in"][sl], dtype=np.int64), np.asarray(km["pair_out"][sl], dtype=np.int64)
        if pi.size == 0:
            continue
        gather = sp.csr_matrix((np.ones(pi.size), (po // rows_per_group, pi)), shape=(n_groups, n_in))
        total += (gather @ f64) @ w64[k]
    return total


def check_group_sums(orc, rng, coords, K, stride, mode, rows_per_group, C_in=5, C_out=3):
    """group_sums_by_linearity agrees with the oracle's output summed over the same groups."""
    n = len(coords)
    feat = rng.standard_normal((n, C_in))
    W = rng.standard_normal((K ** 3, C_in, C_out))
    _, out, km = orc.sparse_conv(coords, feat, W, K, stride, mode)
    n_out = km["n_out"]
    n_groups = -(-n_out // rows_per_group)
    padded = np.zeros((n_groups * rows_per_group, C_out))
    padded[:n_out] = out
    ref = padded.reshape(n_groups, rows_per_group, C_out).sum(axis=1)
    np.testing.assert_allclose(group_sums_by_linearity(feat, W, km, rows_per_group), ref, rtol=1e-11, atol=1e-11)


def check_expected_pairs_uniform(orc):
    """Uniform-random occupancy (2,000 of 64³ cells): P = N + (ordered neighbour pairs), whose
    expectation is N(N-1)/(V-1) times the mean number of in-grid neighbours."""
    from paper_2402_07710_amd import synth
    coords = synth.uniform_cells(2000, 64, seed=0)
    km = orc.kmap(coords, 3, 1, "subm")
    N, V, g = 2000, 64 ** 3, 64
    mean_nb = ((3 * g - 2) ** 3 - g ** 3) / g ** 3           # in-grid neighbours per cell
    expect = N + N * (N - 1) / (V - 1) * mean_nb
    P = int(km["offset_start"][-1])
    assert abs(P - expect) < 5 * np.sqrt(expect - N), (P, expect)


def check_inverse_is_adjoint(orc, rng, coords, s, C_f=3, C_c=4):
    """The inverse layer built from a strided map is the adjoint of the strided layer when every
    W[k] is transposed: <y, down(x; W)> = <up(y; W^T), x> for all x, y (Section III-E: the same
    parent / offset relation, read in the other direction)."""
    import oracle
    n = len(coords)
    km = orc.kmap(coords, s, s, "strided")
    W = rng.standard_normal((s ** 3, C_f, C_c))
    x = rng.standard_normal((n, C_f))
    y = rng.standard_normal((km["n_out"], C_c))
    down = orc.conv(x, W, km)
    up = orc.conv(y, np.ascontiguousarray(W.transpose(0, 2, 1)), oracle.transpose_map(km))
    assert up.shape == (n, C_f)
    np.testing.assert_allclose(np.sum(y * down), np.sum(up * x), rtol=1e-10)
    # and row by row: a fine row only hears from the cell that contains it
    inv = oracle.transpose_map(km)
    assert inv["offset_start"][-1] == n and np.array_equal(np.sort(inv["pair_out"]), np.arange(n))
    cell = coords.copy()
    cell[:, 1:] //= s
    assert np.array_equal(km["out_coords"][inv["pair_in"]], cell[inv["pair_out"]])


def run_all(orc, seed=0):
    """Every pin in one call (used on the real oracle and on each mutant)."""
    rng = np.random.default_rng(seed)
    check_fig_subm_2d(orc)
    check_fig_oft_2d(orc)
    check_eq_cell_mapping(orc)
    for (grid, n, K, s, mode, ci, co, nb) in [
        (6, 40, 3, 1, "subm", 3, 2, 1), (5, 60, 3, 1, "subm", 2, 3, 2), (7, 30, 5, 1, "subm", 2, 2, 1),
        (6, 50, 2, 2, "strided", 3, 2, 1), (7, 40, 3, 3, "strided", 2, 2, 2), (6, 30, 3, 2, "strided", 2, 3, 1),
        (5, 125, 3, 1, "subm", 1, 1, 1), (4, 1, 3, 1, "subm", 2, 2, 1), (6, 216, 2, 2, "strided", 1, 2, 1),
    ]:
        check_dense(orc, rng, grid, n, K, s, mode, ci, co, nb)
    from paper_2402_07710_amd import synth
    c = synth.uniform_cells(300, 8, seed=3)
    c[:, 0] = rng.integers(0, 2, len(c))
    check_symmetry_and_centre(orc, c, 3)
    check_symmetry_and_centre(orc, c[:100], 5)
    check_delta_weights(orc, c, rng.standard_normal((len(c), 4)).astype(np.float32), 3)
    check_full_grid_counts(orc, 4)
    check_full_grid_counts(orc, 5)
    check_isolated_is_matmul(orc, rng)
    check_strided_partition(orc, c, 2)
    check_strided_partition(orc, c, 3)
    check_invariances(orc, rng, c, 3, 1, "subm")
    check_invariances(orc, rng, c, 2, 2, "strided")
    check_invariances(orc, rng, c[:80], 3, 2, "strided")
    check_alg2_formulation(orc, rng, c[:120], 3, 1, "subm")
    check_alg2_formulation(orc, rng, c[:120], 2, 2, "strided")
    check_expected_pairs_uniform(orc)
    check_inverse_is_adjoint(orc, rng, c, 2)
