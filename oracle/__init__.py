"""A2CiD2 CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Serial, event-by-event, fp64.  Only tests/, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library never does and the
two share no code.

  oracle.core   -- ctypes view of a2cid_oracle.c: mixing, gradient and gossip
                   jumps, the serial event loop, observables, the Poisson-clock
                   event source.
  oracle.graph  -- topologies, Laplacian, chi_1, chi_2 and the hyper-parameter
                   rule of Proposition 3.2 (numpy).
  oracle.levels -- the plain definition of the vertex-disjoint level packing.
"""
