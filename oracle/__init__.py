"""CPU oracle for one DiffuSpec speculative round.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, readable CPU statement of
what the round computes, written from the paper.  It exists so that the HIP path can
be checked against something independent.  It shares no code with the HIP path and
must never be imported by it: only the tests, the smoke check and the benchmark's
`cpu_baseline` leg may use it.

Precision: the decoder forward works in float64 on the given (fp32 / bf16-exact)
weights and rounds logits once to float32.  Lattice, path search and acceptance take
float32 logits / log-scores as data and follow the float32 operation order stated in
each function, because those steps end in integer decisions.

Pins (tests marked "not gpu"): KV-cached forward == full-sequence recompute; a third
implementation in primitive PyTorch CPU ops; RoPE shift invariance; GQA == MHA with
replicated heads; mask-row symmetry; causality; softmax mass == 1 and top-M == stable
full sort; hand-made mass-pruning rows; brute-force enumeration of all lattice paths and
a Viterbi DP for the path search; both forms of the accepted-length formula; hand traces
of the draft-length controller; refinement with one step == the single-pass draft, update-set sizes
and order checked against an independent sort; stochastic verification against the exact output
distribution it must reproduce (enumerated over a uniform grid on a tiny vocabulary) and numpy's
searchsorted for the inverse CDF; the path search with a tiny causal LM as its proxy against an exhaustive
enumeration whose proxy scores come from one uncached causal pass, and against the proxy-free search at
lambda = 1.  Beams narrower than exhaustive: a hand-worked three-position lattice on which beams 4, 2 and 1
return three different paths (the prefix of the optimum is pruned), with hand-computed scores and margins; beyond
such examples the narrow-beam path is fixed by the step-by-step reading of the search procedure (depth-synchronous
pruning, the stated keep order), which no closed form pins.
"""
from . import model, lattice, cps, accept, adl, round, refine, sample  # noqa: F401
