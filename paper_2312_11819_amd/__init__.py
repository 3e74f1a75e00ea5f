"""MI355X-native Actor rollout (prefill + KV-cached decode) behind a C-ABI library.

`binding` loads the HIP shared library and mirrors its entry points; `synth`
holds the seeded input generators.  Nothing here computes on the CPU.
"""
