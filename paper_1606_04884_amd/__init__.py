"""fp32 NCHW conv2d training kernels for MI355X (gfx950) behind a C ABI.

`binding` mirrors include/mi355conv.h; `synth` holds seeded inputs and the layer
tables of the benchmark configurations; `build` compiles csrc/ with hipcc.
"""
__all__ = ["binding", "synth", "build"]
