"""Float64 CPU oracle of the LiSA attention path -- test infrastructure only.

Two independent statements of the same definitions live here:
  * ``oracle.cref``  -- ctypes binding of ``lisa_oracle.c`` (row-addressable, plain loops,
    optional OpenMP over rows), used for parity tests and the CPU baseline timing;
  * ``oracle.npref`` -- whole-tensor numpy version (einsum / matmul as library steps),
    used on small inputs to cross-check the C code.
Nothing in the product package imports this directory.
"""
