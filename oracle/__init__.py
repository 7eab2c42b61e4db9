"""CPU oracle for the merged-gradient hot path of MG-WFBP.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this: it exists so that the
tests, the smoke check and the benchmark's `cpu_baseline` leg have a slow, plain statement of what
the HIP path must compute.  It shares no code, tables or helpers with the HIP path.

  oracle.plan      cost model (Eq. 10), timeline (Eq. 6-8), merge properties (Eq. 12-14),
                   Algorithm 1, exhaustive search, grouping (Algorithm 2) and buffer layout (Sec. 5.3)
  oracle.pipeline  pack / reduce / unpack + SGD-momentum update as plain numpy loops (Sec. 5.3, Eq. 2)
"""
