"""CPU oracle for parallel speculative decoding (PEARL).

TEST INFRASTRUCTURE ONLY.  Plain, slow NumPy code written from the paper; it shares
no code with the HIP library and must never be imported by the product path.  Only
the test-suite, the smoke check and the benchmark's CPU-baseline leg may use it.

Modules
-------
transformer : decoder forward with a KV cache (the "M_p(.)" / "M_q(.)" of Section 2)
sampling    : softmax, inverse-CDF draw, the acceptance rule of Eq. (1), residual resampling
loops       : autoregressive decoding, vanilla speculative decoding (Section 2) and the
              pre-verify / post-verify loop (Section 3, Algorithms 1 and 2)

Pins (tests/test_oracle_*.py): multi-token forward == sequential forwards, RoPE invariants,
brute-force attention on tiny sizes, chi-square exactness of speculative sampling and of the whole
loop on toy models, closed-form tokens/step, the Figure 3 trace, greedy equivalences.

Parity unpinned: anything that depends on real-text acceptance rates (mean accepted tokens,
speed-up ratios of the paper's tables) - these need the paper's checkpoints and datasets.
"""
