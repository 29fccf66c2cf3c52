"""CPU oracle of the Sali-Cache pre-attention filter.  TEST INFRASTRUCTURE ONLY.

A plain, slow, step-by-step NumPy implementation of what the HIP library
computes, written from the paper (Methodology: Temporal Filtering via Optical
Flow, Eq. 5-6; Spatial Filtering via Saliency-Guided Quantization, Eq. 7-8;
Just-In-Time Dequantization; Algorithm 1; Implementation Details).  It shares
no code, tables or constants modules with the HIP path and imports nothing
from the `paper_2602_14236_amd` package.  Only the tests, the smoke check and
the benchmark's `cpu_baseline` leg may import it; the product never does.

Precision: the flow field is computed in float64 (the paper fixes none); the
saliency stages are integer arithmetic; quantisation follows the fp32
operation sequence stated in `oracle.quant` because there floating point
decides integer codes.

Pins (tests/test_oracle_*.py, CPU only):
  flow      zero flow on identical frames; exact recovery of the expansion of a quadratic
            image and of its translate; integer translation of a textured image; the
            lambda = 0 single-iteration case against an independently written weighted
            least-squares solve; rational gate boundary; and the whole coarse-to-fine
            estimate on a tiny sub-pixel-shifted texture against a second, pixel-by-pixel
            implementation of the definition (per-pixel lstsq expansion, direct 2-D window
            sums of 2x2 matrix products, np.linalg.solve), to 1e-9.
  saliency  brute-force loops on 8x8 images, CIE L*a*b* closed form within one level,
            step edges, hysteresis chains, uniform-variance image.
  quant     round-trip error <= scale/2, power-of-two scaling invariance, negation,
            extreme codes, closed-form byte counts, brute-force ranks on tiny inputs.
  attention (single-query attention over the cache, float64) a library scaled-dot-product
            attention on an all-FP16 cache, uniform-logits and dominant-key closed forms,
            brute-force loops with a pointer frame and pruned tokens, log-sum-exp merge.
"""
