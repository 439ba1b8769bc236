"""MI355X-native block-denoising step of a MoE diffusion LLM (hand-written gfx950 HIP kernels behind a C-ABI).

`binding` loads libdinfer.so and raises if it is not built: there is no CPU or PyTorch fallback.
"""
