"""TEST INFRASTRUCTURE ONLY: slow, plain CPU oracles for the micro-batched
convolution method (arXiv 1804.04806).

* ``oracle.conv``    -- fp64 direct convolution (Forward, BackwardData,
  BackwardFilter), a ctypes front for ``conv_oracle.c``.
* ``oracle.planner`` -- exhaustive enumeration of micro-batch divisions (WR) and
  of per-kernel configuration products under one budget (WD).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It imports nothing from the HIP package and the HIP package imports
nothing from here.
"""
