"""MI355X-native server-side step of split federated LoRA fine-tuning (SplitLoRA).

Sub-modules:
  synth    seeded synthetic inputs (no method arithmetic; importable without a GPU)
  binding  ctypes binding of libslora.so, the C-ABI library of HIP kernels
Nothing is imported eagerly so that `synth` can be used on machines without the
built library.
"""
__all__ = ["synth", "binding"]
