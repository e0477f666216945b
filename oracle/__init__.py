"""CPU fp64 oracle for the dLLM rollout denoising step -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It shares no code with the HIP library and never calls it.

Layers:
  dlm_oracle.c   attention rows and LM-head rows, plain definitions in double
  ref.py         numpy-facing wrappers (concatenate KV segments, call the C code)
  denoise.py     selection/commit rule and the block rollout loop, plain Python
  sampling.py    counter-based noise and Gumbel-max token sampling, numpy
  backward.py    gradient of block attention (dQ, dK, dV), dense numpy

Parity pins live in tests/test_oracle_*.py (pure-Python brute force on tiny
inputs, closed forms, metamorphic identities, textbook special cases).
"""
from .ref import (KV, attention, attention_varlen, block_diffusion_train_attention, lmhead,  # noqa: F401
                  num_threads, build)  # noqa: F401
from .denoise import select_commit, OracleRollout, full_pass, seq_logprob  # noqa: F401
from . import sampling, backward  # noqa: F401,E402
