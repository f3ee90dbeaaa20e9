"""MI355X (gfx950) implementation of the TriAttention KV-cache compression step.

The work is done by hand-written HIP kernels behind a C ABI (include/tri.h, libtri.so);
`binding` marshals torch tensors into that ABI and nothing more.  There is no CPU fallback:
importing `binding` without a built libtri.so raises.
"""
