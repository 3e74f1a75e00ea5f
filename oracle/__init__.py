"""CPU oracle for the Actor rollout.  TEST INFRASTRUCTURE ONLY.

A plain, slow definition of what `Response <- Actor.generate(Query)` (Alg. 1 and
Alg. 2 of the paper) computes for a Llama-style decoder (Sec. V-A): per-token
logits of a decoder-only transformer, a seeded temperature / top-p sampler and
the per-token log-probabilities.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the HIP library never does, and the two share no
code.  Everything is float64 on torch CPU tensors unless a caller asks for
float32; `torch.matmul` is the only library primitive used as a step.
"""
