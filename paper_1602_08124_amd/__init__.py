"""MI355X-native vDNN: HIP kernels + memory manager behind a C ABI (libvdnn.so), with a thin
Python binding.  Build the library with `python -m paper_1602_08124_amd.build` (or
`__graft_entry__.build()`); importing the binding fails loudly when the library is missing."""
