"""MI355X-native policy-gradient head: fused LM-head log-prob, TRLOO advantages and
clipped-surrogate forward/backward, as hand-written HIP kernels behind a C ABI.

`binding` wraps the shared library (it is loaded on first use and fails loudly
when the library has not been built); `synth` draws seeded synthetic workloads.
"""
