"""CPU oracle package -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke run and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP path and never imports it.

  oracle.attn   exact causal softmax attention + gradients in fp64 (C, OpenMP),
                the plain definition of paper Eq. 1 with the causal mask of Sec. 4.3
  oracle.plan   independent integer re-implementation of the zigzag shard plan,
                and fp64 per-step partials + log-sum-exp merge used to check that
                sharded-and-merged equals unsharded
"""
