"""CPU oracle for the tile-wise (TW) / tile-vector-wise (TVW) sparse GEMM.

TEST INFRASTRUCTURE ONLY.  Nothing here is on the product path: only the
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It shares no code with the HIP library and imports nothing from it.

What it holds, each piece written out plainly in NumPy fp64 / Python ints:

  gemm.py   C = A . (B (.) mask): the definition the sparse kernels must reach
            (Section III-A problem statement; Section V "skips computing
            partial sums for pruned elements"), plus a brute-force per-element
            version that pins it.
  prune.py  one-shot TW / VW(2:4) / TVW mask construction following the steps
            of Algorithms 2 and 3 with magnitude scores.
  pack.py   the canonical *logical* packed form: kept-column list, per-tile
            kept-row lists, compressed tile offsets (Section V, "Tile Fusion
            and Compressed Tile Offset"), condensed values and 2:4 positions.

Pins (tests/test_oracle_*.py): brute force with math.fsum, the 0 %-sparsity =
dense case, exact zeros for pruned rows/columns, linearity over disjoint
masks, the worked index/offset example of Section V, the column-regrouping
example of Section III-A, the closed forms of Algorithm 3, the G=1 and
single-tile limits named in the introduction, and pack/unpack round trips.
Nothing that involves trained weights or accuracy is covered: parity unpinned
and out of scope for those.
"""
