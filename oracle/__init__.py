"""CPU oracle for the BranchGRPO tree rollout (arXiv 2509.06040).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy
implementation of what the GPU library computes, written from the paper.  It
shares no code with the HIP path and must never be imported by the product
package; only the test-suite, the smoke check and the benchmark's CPU-baseline
leg use it.

Modules (each function cites the passage of the paper it follows):

  philox   counter-based noise: Philox4x32-10 words -> uniforms -> normals
  tree     level-ordered rollout-tree topology (Sec. 3.2 "Preliminaries")
  sde      Euler-Maruyama step of the reverse SDE (Eq. 1, App. B.1) and the
           Gaussian transition log-density (ratio of Eq. 5)
  dit      the synthetic DiT velocity network the workloads define
  rollout  tree rollout (Alg. 1, tree-building loop; Eq. 2) and the flat
           sequential rollout it is compared with
  rewards  synthetic leaf rewards standing in for the paper's reward models
  fusion   reward fusion (Eq. 3) and depth-wise normalisation (Eq. 4)
  prune    width / depth pruning (Sec. 3.4) and the kept-edge set
  objective  clipped GRPO objective value over edges (Eq. 5)

Pins: see tests/test_oracle_*.py.  Unpinned items are listed in each module's
header.
"""
