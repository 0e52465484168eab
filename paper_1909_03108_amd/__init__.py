"""sp3d: spatially partitioned 3x3x3 convolution (forward, data-grad, weight-grad) with
halo pack/unpack for one MI355X, behind a C-ABI library.

`paper_1909_03108_amd.sp3d` is the thin ctypes binding (argument marshalling only); it
loads the HIP library lazily and raises if the library has not been built.
`paper_1909_03108_amd.synth` draws the seeded synthetic workloads.
"""
__all__ = ["sp3d", "synth"]
