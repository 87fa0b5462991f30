"""CPU oracle for the WaveTune hot path -- TEST INFRASTRUCTURE, not product code.

Plain, slow, obviously-correct implementations written from the paper:

  gemm.py        fp64-accumulating GEMM on storage-rounded operands (Sec. 3.2, tiled-GEMM
                 paragraph: C = A.B with A in R^{MxK}, B in R^{KxN}); bf16 / e4m3 decoders.
  gemm_ref.c     the same triple loop in C (row-parallel) for shapes Python cannot finish.
  geometry.py    Phi: (M,N,K) -> (G,L) (Table 2, Dense-GEMM row), wave count (Sec. 3.2/3.3),
                 resident-block capacity, greedy-dispatch simulation (Sec. 3.2, Fig. 4).
  sampler.py     wave-aligned regions, sub-intervals, representative grid sizes, workload
                 instantiation (Sec. 4.2).
  fit.py         shared micro choice, per-bucket bilinear least squares, extrapolation
                 coefficients, dual table (Sec. 4.3, 4.5).
  select.py      two-stage runtime selection on a dual table (Sec. 4.4, 4.5) and a reader
                 for the binary table file the product library writes.
  exhaustive.py  brute-force search over a latency table (Sec. 5.1, brute-force baseline).
  attention.py   scaled dot-product attention in fp64 and the attention row of the abstraction
                 (Table 2, FlashAttention row; Sec. 4.2 head-aligned grid sizes; Eq. 6).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It imports nothing from the product package and shares no code or tables with it.  Three feasibility
limits of the product (split-K workspace floats, split-K tile count, anchor slots per table bucket) are
not results of the method; the oracle takes them as arguments (geometry.split_fits, fit.thin_anchors,
select.read_table), None meaning "no limit", and the tests pass in the values the product's header states.

Pins (tests/test_oracle_*.py) tie each function to facts fixed by the paper or by mathematics;
a function whose behaviour could not be pinned says "parity unpinned" in its docstring.
"""
