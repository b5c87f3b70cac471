"""Hidden Transfer tree-verify decoding on MI355X: thin ctypes binding over libht.so.

Every step of the decode path runs in the HIP kernels of libht.so; this package only marshals
arguments (torch supplies device memory and the stream).  There is no CPU fallback: importing
`paper_2404_12022_amd.binding` raises if the library has not been built.
"""
