"""CPU oracle for the all-gather -> GEMM hot path. TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may import
this package. It imports nothing from the HIP package and the HIP package imports nothing from it.

* :mod:`oracle.gemm`     - the result of the pair, by its definition (paper Sec. II-B, Fig. 3(a)-(b)),
                           in plain C with fp64 accumulation (``ficco_oracle.c``).
* :mod:`oracle.schedule` - the decomposition/ordering rules (Sec. III, Sec. V-A/B), the static
                           descriptors OTB and MT (Sec. IV-B, IV-C), the ideal-overlap model and
                           the DIL/CIL ratios (Sec. IV-A), and the schedule heuristic's decision
                           rule (Sec. V-C), in plain Python.
* :mod:`oracle.grouped`  - expert-parallel dispatch -> grouped expert GEMM: piece layout for unequal
                           per-peer token counts and the per-expert products.
* :mod:`oracle.reduce`   - the adding half of a reduce-scatter (fp32 in ascending GPU order, one
                           rounding), in numpy.
"""
