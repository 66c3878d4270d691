"""MI355X-native per-layer training compute (conv2d fwd / dgrad / wgrad, dense fwd+bwd)
at the small per-GPU batches that strong scaling forces, behind a C-ABI library.

`binding` loads the HIP library and mirrors its entry points; `synth` and
`workloads` hold seeded inputs and layer shapes only.  Submodules are imported
on demand so that the input generators can be used without the GPU library.
"""
__all__ = ["binding", "synth", "workloads"]
