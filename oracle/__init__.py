"""CPU oracle of the Stream Batch denoising step (StreamDiffusion, arXiv 2312.12491).

TEST INFRASTRUCTURE ONLY.  Plain, slow PyTorch-CPU / numpy code in float64, written
from the paper's equations; it shares no code with the HIP library and must never be
imported by the product package.  Only the tests, the smoke check and the bench's
CPU-baseline leg may call it.

Pin status (what each part is checked against, in tests/test_oracle_*.py):
  unet.py   : every op against brute-force loops from the textbook definition on tiny
              shapes; wiring against the publicly known parameter counts of the SD-1.5 /
              SD-2.1 shaped nets; ResBlock, transformer block and the whole net at a micro shape
              against the definition written as scalar Python loops, with planted wiring mistakes
              (tests/test_oracle_blocks.py).  Whole-net numerics at SD shape: PARITY UNPINNED beyond
              that (random weights, the paper prints no worked example).
  stream.py : Stream Batch == sequential denoising (Sec. 3.1); R-CFG -> CFG collapse
              (Eq. 2 vs Eq. 6); slot-0 identities of Eq. 5 / Eq. 7; Eq. 4 inverting Eq. 1;
              U-Net evaluation counts n / n+1 / 2n (Sec. 3.3); public schedule values.
  image.py  : the tiny autoencoder around the U-Net (appendix: the paper only names it; the layers are this
              build's definition): encoder, decoder and Block against scalar Python loops at a small width,
              closed-form parameter count, saturation and dead-block cases, planted wiring mistakes.
              Numerics at width 64 / 512x512: PARITY UNPINNED beyond that (random weights).
  ssf.py    : Eq. 8-9 special cases (identical, orthogonal, eta = 1), python-int brute
              force of the integer sums, empirical skip frequency.
"""
