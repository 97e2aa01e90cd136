"""TernGrad hot path for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

Submodules are imported on demand so that `workloads` (input generators) can be
used without loading the HIP library:
    paper_1705_07878_amd.binding    -- ctypes binding of libterngrad.so
    paper_1705_07878_amd.workloads  -- seeded synthetic gradients
    paper_1705_07878_amd.build      -- hipcc build of the library
"""
__all__ = ["binding", "workloads", "build"]
