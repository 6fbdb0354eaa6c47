"""CPU oracle for the block-attention hot path: TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy implementations of what the path computes, written from the
paper's definitions (Sec. 2.1 masked self-attention; Listing 1 block-parallel attention;
Sec. 4.1 block generation).  Only tests, the smoke check and the benchmark's cpu_baseline
leg may import this package; the product (paper_2510_10620_amd) never does, and this
package never imports the product's kernels or bindings.
"""
