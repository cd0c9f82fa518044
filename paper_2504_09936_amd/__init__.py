"""KeepKV hot path for MI355X (gfx950): HIP kernels behind a C-ABI library.

`paper_2504_09936_amd.workloads`  seeded synthetic inputs (numpy only).
`paper_2504_09936_amd.binding`    ctypes binding of libkeepkv.so (loads the HIP library;
                                   raises if it has not been built).
`paper_2504_09936_amd.build`      compiles csrc/*.hip for gfx950 into libkeepkv.so.
"""
__all__ = ["workloads", "binding", "build"]
