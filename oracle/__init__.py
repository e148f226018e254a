"""CPU oracle for the chunk-plan executor.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the executor must compute: the unchunked
forward of each workload (AutoChunk, arXiv 2401.10652, section 2.2: a chunked
module must give the output of the unchunked module; section 3.3, output
alignment rule).  It shares no code with the GPU path and does not import it.
Only the tests, the smoke check and the benchmark's CPU-baseline leg may use
anything in this package; the product never routes through it.

Parity pins (tests marked "not gpu"):
  transformer.*   brute-force scalar loops on tiny shapes, torch fp64 library
                  routines (layer_norm, scaled_dot_product_attention, linear,
                  gelu), closed forms and invariants of softmax / GELU / causal
                  masking, chunked == unchunked for every legal dim and length.
  pairstack.*     brute-force scalar loops on tiny shapes, einsum witnesses,
                  transpose symmetries between outgoing/incoming and
                  starting/ending forms, reduction of the transition to the
                  feed-forward of the transformer block.
  memory_model.*  hand-computed byte counts of the paper's two activation
                  equations for the five workloads.
No function here is "parity unpinned".
"""
