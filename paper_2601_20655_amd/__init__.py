"""MI355X-native DiT attention hot path (self-attention with 3-axis RoPE, cross-attention
with a key-padding mask) behind a C-ABI library of hand-written gfx950 kernels.

`binding` marshals arguments to the C ABI; `workloads` makes seeded synthetic inputs.
Nothing here computes attention on the CPU: without the built HIP library every call fails.
"""
__version__ = "0.1.0"
