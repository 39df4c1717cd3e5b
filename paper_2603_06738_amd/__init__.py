"""RIB window attention for AMD MI355X (gfx950): hand-written HIP kernels behind
a C-ABI library, plus a thin ctypes binding.  Importing the package loads
nothing; the library is opened on the first call into `binding`."""
