"""CPU oracle for the Bamboo stage hot path (arXiv 2204.12013).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only the tests, the smoke check and the benchmark's cpu_baseline leg
do.  It shares no code with the HIP path: plain numpy float64, one function per
mathematical step, no blocking or fusion.

Modules
  layer     transformer layer forward/backward (the computation that FNC/BNC
            and FRC/BRC of Section 5.1 both denote)
  schedule  1F1B program, slot timeline, FRC insertion, failover merge
            (Sections 2, 5.2)
  stage     a stage executing an instruction list with simulated neighbours
            (Sections 5.1, 5.2: eager FRC, lazy BRC, recovery)
  ends      the two ends of the model that the wrap-around stage works on (Section 5.1: the
            last node fetches the input samples to run the first node's layers): token and
            position embedding at the front, LM head and mean cross-entropy at the back
  optim     Adam update (Section 7 names the optimizer) and replica weight
            synchronisation (Section 5.1 requires equal parameters)

Pins (see tests/test_oracle_*.py): finite differences, an independent autograd
implementation, closed forms for the timeline, the paper's worked values, brute
force over tiny pipelines.  Input distributions for biases/LayerNorm parameters
and the upstream-gradient scale are not fixed by the paper: parity unpinned for
those choices (they are inputs, not arithmetic).
"""
