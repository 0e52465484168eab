"""CPU fp64 oracle of the spatially partitioned 3D convolution path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  Nothing here is used by, or shares code with,
the GPU library; the GPU library never falls back to it.
"""
