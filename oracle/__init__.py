"""CPU oracle for the kFkB stage engine.  TEST INFRASTRUCTURE ONLY.

Plain, slow, float64 numpy statements of what one pipeline stage computes and
of the order a kFkB plan runs it in.  Nothing here is tuned, blocked or fused,
and nothing here is used by the product path: only the tests, the smoke check
and the benchmark's CPU-baseline leg import this package.  It shares no code
with the HIP kernels or their Python binding.

Modules
  stage_math  transformer-block forward / backward (the stage computation)
  schedule    kFkB micro-batch order, live-activation count, memory model,
              one whole iteration with gradient accumulation
  transfer_sim  discrete-event model of the delayed inter-stage transfers
                (timing only: "parity unpinned" beyond its closed-form checks)
  tuner       cost model and online choice of k (moving averages of measured
              transfer times, estimated iteration length per candidate plan)
  pipeline    S stages, each under its own kFkB plan: the order one executor
              issues their ops in, one iteration, a timing model (the timing
              is "parity unpinned" beyond its closed forms)
"""
