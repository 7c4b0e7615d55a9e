"""CPU oracle for the RNG-overlap hot path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously correct
CPU implementation of what the HIP path computes: the Philox4x32 block
function, the attention-dropout keep-mask, attention with dropout applied
after softmax, GEMM, bf16 / fp8-e4m3 rounding, and a Llama-style transformer
block.  Only the tests, the smoke check and the `cpu_baseline` leg of the
benchmark may import it.  It shares no code with `paper_2410_07531_amd` and
never imports it.

Floating-point work is done in float64 on inputs that were already rounded to
the dtype under test.  Each function cites the passage of the paper it follows
(section / equation / table), or says that the paper is silent and states the
reading taken.
"""
