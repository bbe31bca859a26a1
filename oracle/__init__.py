"""CPU oracle for the virtual-tensor hot path.  TEST INFRASTRUCTURE ONLY.

What it computes: the plain definition of what the method must reach.  A chain of
data-movement operators is executed one operator at a time, each into a fresh dense
row-major array (Def. 2 of the paper: O_i[x] = I_j[y] with (j, y) = F(i, x)), and the
consumer (add + row-sum, LayerNorm + linear, GEMM, decode attention) then runs on the
dense result.  The paper states that eliminating the data movement leaves the numbers
unchanged (Sec. 6, numeric equivalence), so this is exactly the value the virtual-tensor
kernels must produce.

Rules this package follows:
  * slow, plain numpy / pure Python; floating point in float64 except where a reading
    fixes the precision (the fp32 row-sum order, the fp16 rounding between LayerNorm
    and the linear layer);
  * it shares no code with the HIP path and imports nothing from the product package;
  * only tests, the smoke check and the benchmark's cpu_baseline leg may import it.

Pins (tests marked "not gpu"): brute-force index enumeration with the per-operator maps
in ``index_maps``, invariants (permute∘inverse, concat∘split, reshape keeps row-major
order), the paper's stride example (Sec. 2.1), the Expand closed form (Eq. 2), the Fig. 3
column boundaries, hand-derived closed forms of the composed maps of the benchmark
chains, and textbook special cases of each consumer.  Full-size end-to-end outputs have
no independent pin (the paper prints none): parity there rests on the same code being
pinned at small sizes.
"""
