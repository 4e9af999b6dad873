"""fp64 CPU oracle for the chunked causal attention path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  The product path (the HIP library and its Python binding) never does.

`definition`  : ctypes front end of fpdt_oracle.c -- the plain unchunked definition.
`chunked`     : the chunk-by-chunk method of the paper in numpy, used to
                cross-check the definition (and the other way round).
"""
from . import definition, chunked  # noqa: F401
