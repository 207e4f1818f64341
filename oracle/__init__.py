"""CPU oracle for the 1F1B weight-stashed stage step (PipeDream, Sections 3.3-3.5 and 4).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy statement of
what the hot path computes.  Only the test-suite, the smoke check and the
benchmark's ``cpu_baseline`` leg may import it; the product package never does,
and nothing here imports the product package or its kernels.

Modules
  schedule  -- NOAM, per-stage in-flight depth, the static 1F1B op list, the
               event-driven multi-stage simulator (integers only)
  layers    -- textbook layer maths (Linear, ReLU, softmax cross-entropy, ...)
               and the bf16 rounding points of the mixed-precision mode
  pipeline  -- stage state (version ring, stash, momentum), F / B / U, the
               pipeline run, and the flat-loop form of the staleness equation
  partition -- the layer partitioner of Section 3.2: stage time, boundary cost,
               the dynamic program over (layers, machines), NOAM
  replicated-- a stage replicated over several machines (Sections 3.3 and 4): round-robin
               routing, the parameter server's summed update, a pipeline with such stages
  checkpoint-- the per-stage checkpoint file (Section 4): layout and checksum
               written out in plain Python; pinned by hand-computed checksums

Pins (tests/test_oracle_*.py): the paper's 4-stage worked example (Section 3.4),
the closed-form version rule read off the staleness equation of Section 3.4,
reduction to sequential minibatch SGD for one stage / one active minibatch
(checked against torch autograd + torch.optim.SGD), finite differences for every
layer's backward, the no-idle steady state under unit costs (Section 3.3), and a
no-stashing negative control; for the partitioner, exhaustive enumeration of
every pipeline on small problems, closed-form special cases and a hand-worked
example; for replicated stages, synchronous data-parallel SGD in torch (Section 4's
special case), a hand-worked example and a torch flat loop of the staleness rule.
Start-up slot positions of the timeline figure
(Figure "example pipeline") are parity unpinned: the figure is not available.
"""
