"""CPU oracle for the WLB-LLM hot path (test infrastructure, not the product).

Plain, slow, fp64 / exact-integer implementations written from the paper:
document-masked causal attention forward and backward, the context-parallel
sharding maps, and the greedy variable-length packer.  Only the tests, the
smoke check and the benchmark's cpu_baseline leg may import this package; the
HIP path never does, and this package imports nothing from the HIP path.
"""
