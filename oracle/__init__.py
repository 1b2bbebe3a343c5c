"""CPU oracle for one zero-bubble pipeline stage (arXiv 2401.10241).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, obviously-correct
definition of what the stage computes, written from the paper.  It is imported
by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg and by
nothing else; the product (the HIP library and its Python binding) never
imports it and it never imports the product.

Contents
  layers.py     F / B / W of a pre-LN GPT decoder layer in fp64 (Sec. 1: the
                split of backward into input-gradient and parameter-gradient
                passes; Sec. 2.3 + Table 1: transformer shape and FLOP model)
  schedule.py   per-stage pass order of 1F1B, ZB-H1, ZB-H2 (Sec. 2, 2.1, 2.2),
                stash-occupancy model (Appendix G memory deltas) and a p-stage
                timing simulator for the bubble-rate metric (Sec. 5.3)
  optimizer.py  AdamW Step / Rollback (Appendix C, Algorithm 1) and the
                post-validation protocol (Sec. 4)
  stage.py      a whole stage: parameters, stashes, gradient accumulation,
                dependency checks, optimizer

Every function is pinned by tests/test_oracle_*.py to something other than
itself (finite differences, closed forms, the paper's printed tables, brute
force); no function here is "parity unpinned".
"""
