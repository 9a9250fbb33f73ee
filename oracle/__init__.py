"""CPU oracle for the BanditSpec speculative-decoding round (arXiv 2505.15141).

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 numpy code that states what the
hot path computes, written from the paper's definitions (Sec. 2, Alg. 2-5,
App. A "Vanilla Speculative Decoding", full versions of UCBSpec / EXP3Spec).
Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import it.  It shares no code with the HIP library and never imports it.

Modules
  philox      counter-based Philox4x32-10 and the uniform conventions
  sampling    softmax at temperature, inverse-CDF categorical draw,
              accept/reject + residual/bonus sampling (vanilla SD, App. A)
  bandit      UCBSpec (Alg. 4 / full version) and EXP3Spec (Alg. 5 / full version)
  forward     decoder-only transformer forward, full recompute, no KV cache
  spec_round  draft proposal, one speculative round, the BanditSpec loop (Alg. 3)

Pins (tests/test_oracle_*.py): brute-force enumeration of the output law on
tiny vocabularies (Prop. 3.1), truncated-geometric closed forms (Prop. 4.5),
hand-evaluated UCB radii and EXP3 probabilities, the FTRL characterisation of
the EXP3 weights (App. C), Random123 known-answer vectors for Philox, and
library-routine reductions of the forward pass.
Parity unpinned: the transformer architecture details the paper never states
(norm epsilon, RoPE pairing) - they are fixed by convention, not by the paper.
"""
