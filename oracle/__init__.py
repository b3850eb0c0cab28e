"""TEST INFRASTRUCTURE ONLY -- CPU oracle for DeFT tree-attention decode.

Nothing in the product path may import this package: it exists so that tests,
the smoke check and the benchmark's cpu_baseline leg have an independent,
slow, obviously-correct statement of what the HIP path must compute.

  tree_attention       fp64 attention over each query's root-to-node path
                       (plain C, tree_attention_oracle.c; Section 3.1 definition);
                       tree_attention_paged is the same over a paged pool (Section 4.2)
  plan.flatten_plan    the DeFT-Flatten QKV-preparation plan (Algorithm 3,
                       Remark 3.1) in plain Python
  deft_flatten         the two-stage algorithm itself (Algorithm 4, eq. 1) in
                       fp64 numpy, used to check that plan + merge reproduce
                       the plain definition
"""

from .attention import build, tree_attention, tree_attention_paged, library_path  # noqa: F401
