"""MI355X (gfx950) kernels for the local work of Beaver-triple multiplication
and truncation over Z_2^64, behind the C ABI declared in include/spin.h.

`paper_2402_02320_amd.spin` is the ctypes binding; `workloads` draws the seeded
synthetic inputs.  Importing the package loads nothing native."""
