"""MI355X-native hot path of dLLM rollout denoising (block attention, LM-head
confidence, unmask/commit) behind a C-ABI HIP library.

Submodules:
  synth     seeded synthetic inputs (no method arithmetic; shared with the test oracle's callers)
  binding   ctypes binding to libdlm.so (argument marshalling only)
  rollout   block rollout driver built on the binding

Nothing here falls back to a CPU implementation: using `binding` without the
built HIP library raises.
"""
__all__ = ["synth", "binding", "rollout"]
