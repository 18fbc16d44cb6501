"""CPU oracle for the radial-attention hot path.  TEST INFRASTRUCTURE ONLY.

Everything in this package is a plain, slow, definition-level implementation of what
the GPU library computes, written from the paper (Radial Attention, arXiv 2506.19852):

* ``oracle.mask``       -- the 4-D token mask of Sec. 4.2 ("Formal definition"), its
                           flattening, the attention sink (App. A.1), and the reduction
                           to 128x128 blocks (Sec. 4.2 "Hardware-friendly block sparsity").
* ``oracle.attention``  -- Eq. 1 / Eq. 2 (softmax attention with an additive {-inf, 0}
                           mask) and its analytic gradient, in float64 numpy.
* ``oracle/mask_scan.c``-- the same token-level definition as ``oracle.mask``, as a plain
                           C double loop over all token pairs so that the block mask of the
                           large workloads can be produced by brute force.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It imports nothing from the product package and shares no
code, table or constant with the HIP path.
"""
