"""MI355X-native eigensolver for the normalized Laplacian of sparse similarity graphs.

The compute path lives in ``csrc/`` (HIP kernels for gfx950 behind a C ABI, see ``include/sceig.h``);
``binding`` marshals arguments to it and ``workloads`` builds seeded synthetic inputs.  Nothing is
imported eagerly so that the input generators can be used without the built library.
"""
__all__ = ["binding", "workloads", "build"]
