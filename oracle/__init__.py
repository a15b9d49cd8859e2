"""CPU oracle for the asynchronous-denoising hot path (AsyncDiff, arXiv 2406.06911).

This package is TEST INFRASTRUCTURE, not product code: it is a plain, slow, fp64 NumPy
restatement of what the GPU library computes, written from the paper (Section 3.1 for the
sampler, Section 3.2 and Appendix A for the schedule) and from the textbook definitions of
the UNet building blocks.  Only the tests, the smoke check and the benchmark's CPU-baseline
leg may import it.  It shares no code with the HIP path and never imports it.

Parity status: every function here is pinned by tests/test_oracle_*.py except end-to-end
image quality against the paper's tables (needs trained weights and captions): parity unpinned.
"""
