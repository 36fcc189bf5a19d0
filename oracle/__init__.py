"""CPU oracle for the Visual Perception Engine hot path -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  The product (the HIP library and its Python binding) never does, and this
package never imports the product.

`ops`   -- ctypes wrappers over the fp64 C operators in vpe_oracle.c
`model` -- the encoder and the three heads written out with those operators
"""
from . import ops, model  # noqa: F401
from .ops import build  # noqa: F401
