"""CPU test: the pins can tell a wrong oracle from a right one.

Each case plants one plausible mistake in a copy of the oracle's source (a flipped offset
direction, a transposed weight, a swapped axis in the offset numbering, ...), builds it into a
temporary library and runs the same pin checks on it; every such build must fail a pin, and the
unmodified source must pass them all.  Nothing here touches the GPU.
"""
import os

import pytest

import oracle
from oracle import build as obuild
from tests import pins

MUTANTS = {
    "offset_direction_flipped": ("outs[o][1] * stride + d[0] - pad", "outs[o][1] * stride - d[0] + pad"),
    "offset_numbering_xz_swapped": ("d[0] = k / (K * K);\n    d[1] = (k / K) % K;\n    d[2] = k % K;",
                                    "d[2] = k / (K * K);\n    d[1] = (k / K) % K;\n    d[0] = k % K;"),
    "weight_transposed": ("Wk[(size_t)ci * C_out + co]", "Wk[(size_t)co * C_in + ci]"),
    "batch_ignored_in_lookup": ("Coord p{outs[o][0],", "Coord p{0,"),
    "no_padding": ("(mode == 0) ? (K - 1) / 2 : 0", "(mode == 0) ? 0 : 0"),
    "last_offset_dropped": ("for (int k = 0; k < K3; ++k) {\n            const double* Wk",
                            "for (int k = 0; k < K3 - 1; ++k) {\n            const double* Wk"),
    "stride_divisibility_ignored": ("t < 0 || t % stride != 0", "t < 0"),
    "stride_not_divided": ("q[1 + a] = t / stride;", "q[1 + a] = t;"),
    "overwrite_instead_of_accumulate": ("fo[co] += fi[ci]", "fo[co] = fi[ci]"),
    "y_offset_uses_x": ("outs[o][2] * stride + d[1] - pad", "outs[o][2] * stride + d[0] - pad"),
    "input_channel_off_by_one": ("for (int ci = 0; ci < C_in; ++ci)", "for (int ci = 1; ci < C_in; ++ci)"),
    "z_offset_uses_y": ("outs[o][3] * stride + d[2] - pad", "outs[o][3] * stride + d[1] - pad"),
    "output_cell_offset_sign": ("int32_t t = coords[4 * i + 1 + a] - d[a];", "int32_t t = coords[4 * i + 1 + a] + d[a];"),
    "offsets_reversed_in_the_sum": ("const double* Wk = weight + (size_t)k * C_in * C_out;",
                                    "const double* Wk = weight + (size_t)(K3 - 1 - k) * C_in * C_out;"),
    "strided_layers_padded": ("(mode == 0) ? (K - 1) / 2 : 0", "(K - 1) / 2"),
    "output_row_of_a_pair_shifted": ("pair_out[total] = (int32_t)o;", "pair_out[total] = (int32_t)((o + 1) % outs.size());"),
}


def test_unmodified_oracle_passes_every_pin(orc):
    pins.run_all(orc)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(obuild.SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    msrc = tmp_path / "mutant.cpp"
    msrc.write_text(src.replace(old, new))
    lib = obuild.build(force=True, src=str(msrc), lib=str(tmp_path / f"lib_{name}.so"))
    mutant = oracle.Oracle(lib)
    with pytest.raises((AssertionError, oracle.OracleError, ValueError)):
        pins.run_all(mutant)
