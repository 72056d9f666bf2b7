"""CPU oracles for the build's hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It imports nothing from the HIP product package and the product
package imports nothing from here.

* :mod:`oracle.conv`  -- ctypes front end of ``conv_oracle.c`` (seven-loop fp64 convolution).
* :mod:`oracle.ga`    -- step-by-step genetic search (Section 2.3 "Genetic search", eqs. 1-2).
"""
