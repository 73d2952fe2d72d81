"""TEST INFRASTRUCTURE ONLY: slow, plain CPU oracles written from the paper.

``direct``     -- Eq. (1) of Section 3 (the layer definition) in C, fp64 accumulation.
``winograd``   -- the transform matrices of Eq. (7) and Eq. (15) as exact rationals, and
                  Algorithm 1 taken stage by stage in numpy float64 / rationals.
``complexity`` -- the multiplication counts and the arithmetic-complexity model of
                  Sections 4 and 5, and the flop/throughput accounting of Section 7.

Nothing under this package is imported by the GPU library or its Python binding; only
the tests, the smoke check and the benchmark's CPU-baseline leg may use it.
"""
