"""Sparse 3-D convolution over voxelised point clouds for MI355X (gfx950).

`binding` holds the calls of include/sc.h (hash build, kernel-map build, convolution);
`synth` holds the seeded synthetic input generators; `build` compiles csrc/ into libsc.so.
"""
