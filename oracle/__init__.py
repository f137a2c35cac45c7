"""HiKonv oracle package -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Three independent CPU artefacts, none of which shares code with the HIP library:

* ``direct``   -- the plain int64 definitions (C, loops only) of 1-D convolution,
                  the DNN convolution layer, ReLU+requantise, 2x2 max-pool and the
                  bit-dense container layout.  This is what GPU results are compared to.
* ``plan_model``   -- the paper's slice / guard-bit rules and its exhaustive
                  throughput search (Algorithm 1), in Python.
* ``packed_model`` -- the packed algorithm itself (pack, one wide multiply, overlap-add,
                  split, sign correction) in exact Python big-integer arithmetic; used to
                  test the paper's identities on the CPU.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.
"""
from . import direct, plan_model, packed_model  # noqa: F401
