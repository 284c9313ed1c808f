"""CPU oracle for the BlockDialect / DialectFP4 hot path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 NumPy
implementation of what the paper defines (Section 3.1 formatbook, Section 3.2
two-stage dialect selection, Section 3.3 quantization / dequantization / block
MAC, Appendix I bit accounting) plus the MXFP4 comparison format (Section 4.1
baseline).  It exists so that the HIP kernels can be compared against something
written directly from the paper.  It shares no code, tables or helpers with the
HIP path, and nothing in the product package imports it.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import it.

Parity status of each function against something other than itself:

  formatbook rows 4 and 5 ......... pinned by the worked example of Section 3.3
                                    and the beneficial-range example of Section 3.2
  formatbook rows 0-3, 6-15 ....... reconstructed from the three formatbook
                                    criteria of Section 3.1; the figure that
                                    prints them is not available as text:
                                    PARITY UNPINNED against the published table
                                    (structural invariants are pinned)
  shared_exponent ................. pinned (closed form, Section 3.1 formula)
  stage-1 / stage-2 selection ..... pinned on the Section 3.2 example and by a
                                    brute-force Voronoi count; tie rule and the
                                    rounded-max-of-8.0 clamp are readings the
                                    paper does not fix (unpinned as readings)
  element rounding ................ pinned (Section 3.3 interval [4.0, 5.75) -> 5.0,
                                    exhaustive brute force with exact rationals)
  dequantize / gemm ............... pinned (closed form, integer formulation in
                                    exact rationals, hand-worked block)
  dfp4_quantize_mse ............... pinned (exhaustive exact-rational search over the 16
                                    dialects; never worse than the two-stage choice;
                                    lossless on a dialect's own grid); the tie rule
                                    (lowest id) is a reading the paper does not fix
  dfp4_quantize_block64 ........... pinned (the exhaustive per-block search run on
                                    64-element blocks)
  dfp4_quantize_block16,
  dfp4_dequantize_block,
  dfp4_gemm_blocks ................ pinned (the exhaustive per-block search run on
                                    16-element blocks; exact-rational product of the
                                    brute force's own dequantization)
  round_to_bf16, dfp4_gemm_requant  pinned (library bf16 conversion; a hand-worked block
                                    whose products sit on and just below a bf16 midpoint,
                                    so that dropping the bf16 step or rounding in one
                                    step changes a code)
  mxfp4_* ......................... rounding mode is a reading (round to nearest,
                                    ties to even code, saturating): pinned against an
                                    exact-rational brute force of that reading only
"""
