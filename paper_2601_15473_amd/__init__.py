"""SKLinear forward/backward for AMD MI355X (gfx950): a C-ABI library of HIP
kernels (``libsk``) and a thin ctypes binding with the same entry-point names.

The binding is loaded lazily (``from paper_2601_15473_amd import libsk``) so
that the input generators in ``workloads`` can be imported on their own."""
