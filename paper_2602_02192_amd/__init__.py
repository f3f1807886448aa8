"""MI355X-native GRPO rollout generation (batched autoregressive decoding with
per-token sampler log-probabilities and policy-version swaps).

Sub-modules:
  synth  -- seeded synthetic model/prompt generators (no arithmetic of the method)
  echo   -- ctypes binding of the C-ABI library (loads the HIP shared object)

Importing this package does not load the HIP library; `paper_2602_02192_amd.echo`
does, and raises if it has not been built.
"""
