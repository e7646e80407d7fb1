"""CPU fp64 oracle for the V-TiMePReSt / I-TiMePReSt stage hot path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
numpy (fp64) restatement of what one pipeline stage computes under the
paper's weight rules.  It exists to check the HIP library and is imported
only by the tests, by the smoke check and by the benchmark's CPU-baseline leg.
It shares no code with the HIP path and must never be used as a fallback for
it.

What follows the paper and where:
  significance.py  f(delta) and the intermediate-weight coefficients
                   (Section "I-TiMePReSt", Eq. 1-2; Appendix A.1, A.2)
  schedule.py      nF1B order of forward/backward/update events and the
                   weight version each one sees (Section "Methodology",
                   Sections "V-TiMePReSt" and "I-TiMePReSt", worked examples),
                   at mini-batch and at micro-batch granularity (the latter
                   with or without updates in the middle of a pass)
  layers.py        textbook layer mathematics (dense, convolution, pooling,
                   normalisations, attention, ReLU, GELU, softmax
                   cross-entropy); the paper gives no formulas for these
  stage.py         one stage: forward per micro-batch on the latest weights,
                   one backward per mini-batch on the prescribed weights, the
                   stash of stale versions and its retention rule (Section
                   "Memory Overhead"), SGD-momentum update per mini-batch
  pipeline.py      K stages driven through the event order on one host; on
                   the micro-batch clock also the parent method TiMePReSt,
                   whose passes read the versions of their start (Section
                   "V-TiMePReSt", Challenge 1)

Parity status: every function here is pinned by tests that run without a GPU
(closed forms, the paper's worked version examples, finite differences,
reduction to sequential mini-batch SGD, brute force on tiny inputs).  The
absolute accuracy/loss curves of the paper's figures are "parity unpinned":
the figures are not available and the datasets are not used.
"""
