"""Seeded synthetic workloads shaped like the self-attention layers LinFusion replaces.

Holds no arithmetic of the method: only shapes, seeds and the Gaussian draw.  Q, K, V are
i.i.d. N(0, 1) drawn in fp32 from one torch generator per tensor, then rounded (to nearest
even) to the storage dtype; the rounded values are what both the library and the oracle see.
They stand in for the activations of the SD-v1.5 / v2.1 / XL attention layers on the paper's
image workloads, which need weights and datasets that are not available here.
"""
from __future__ import annotations

import numpy as np
import torch

BASE_SEED = 240902097

# name -> (cfg index, B, H, N, d, dtype, k_scale)
CONFIGS = {
    "sd15_256_f32": dict(idx=1, B=1, H=8, N=32 * 32, d=40, dtype="f32", k_scale=1.0),
    "sd15_512_f16": dict(idx=2, B=2, H=8, N=64 * 64, d=40, dtype="f16", k_scale=1.0),
    "sd21_768_f16": dict(idx=3, B=2, H=5, N=96 * 96, d=64, dtype="f16", k_scale=1.0),
    "sd21_768_f16_peaky": dict(idx=3, B=2, H=5, N=96 * 96, d=64, dtype="f16", k_scale=4.0),
    "sdxl_2048_A_bf16": dict(idx=4, B=2, H=10, N=128 * 128, d=64, dtype="bf16", k_scale=1.0),
    "sdxl_2048_B_bf16": dict(idx=5, B=2, H=20, N=64 * 64, d=64, dtype="bf16", k_scale=1.0),
    "sd15_16k_f16": dict(idx=6, B=1, H=8, N=2048 * 1024, d=40, dtype="f16", k_scale=1.0),
    # the deeper levels of the SD-v1.5 UNet (640 and 1280 channels over 8 heads): at 512 px, and at the
    # 16K-image resolution of the headline workload (tokens / 4 and / 16)
    "sd15_512_d80_f16": dict(idx=7, B=2, H=8, N=32 * 32, d=80, dtype="f16", k_scale=1.0),
    "sd15_512_d160_f16": dict(idx=8, B=2, H=8, N=16 * 16, d=160, dtype="f16", k_scale=1.0),
    "sd15_16k_d80_f16": dict(idx=9, B=1, H=8, N=1024 * 512, d=80, dtype="f16", k_scale=1.0),
    "sd15_16k_d160_f16": dict(idx=10, B=1, H=8, N=512 * 256, d=160, dtype="f16", k_scale=1.0),
    "sd15_16k_d160_bf16": dict(idx=10, B=1, H=8, N=512 * 256, d=160, dtype="bf16", k_scale=1.0),
}
EPS = 1e-6


def config(name: str) -> dict:
    """A named workload, or an ad-hoc one written as "B=2,H=8,N=16384,d=40,dtype=f16"."""
    if name in CONFIGS:
        return CONFIGS[name]
    c = dict(idx=99, k_scale=1.0)
    for item in name.split(","):
        key, val = item.split("=")
        c[key] = val if key == "dtype" else int(val)
    if not {"B", "H", "N", "d", "dtype"} <= set(c):
        raise KeyError(f"unknown workload {name!r}")
    return c

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}
ITEMSIZE = {"f32": 4, "f16": 2, "bf16": 2}


def draw(shape, seed: int, dtype: str, device="cpu", scale: float = 1.0) -> torch.Tensor:
    """N(0,1) * scale drawn in fp32 on `device` with its own generator, rounded to `dtype`."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if scale != 1.0:
        x = x * scale
    return x.to(TORCH_DTYPE[dtype]).contiguous()


def make_qkv(B, H, N, d, dtype, idx=0, k_scale=1.0, device="cpu", seed_offset=0):
    base = BASE_SEED + 1000 * idx + 10 * seed_offset
    q = draw((B, H, N, d), base + 0, dtype, device)
    k = draw((B, H, N, d), base + 1, dtype, device, scale=k_scale)
    v = draw((B, H, N, d), base + 2, dtype, device)
    return q, k, v


def make_qkv_widths(B, H, N, d_qk, d_v, dtype, idx=0, device="cpu"):
    """q, k ~ N(0, 1) of width d_qk and v ~ N(0, 1) of width d_v (feature width other than the value width)."""
    base = BASE_SEED + 1000 * idx + 700
    return (draw((B, H, N, d_qk), base + 0, dtype, device), draw((B, H, N, d_qk), base + 1, dtype, device),
            draw((B, H, N, d_v), base + 2, dtype, device))


def make_mlp_inputs(B, H, N, d, dtype, idx=0, device="cpu", zero_start=False):
    """Stand-ins for what the two-branch MLPs in front of the mixer hand over, token-major [B, N, H*d]:
    a_q, a_k (linear-branch results) and v ~ N(0, 1); t_q, t_k (results of the second branch's Linear)
    ~ N(0.5, 1.5^2) so that the LayerNorm has a mean and a scale to remove; per-channel affine
    gamma ~ N(1, 0.25^2), beta ~ N(0, 0.5^2) in fp32 (both zero with `zero_start`: the state the paper
    initialises the second branch to).  Returns (a_q, t_q, a_k, t_k, v, gamma_q, beta_q, gamma_k, beta_k)."""
    base = BASE_SEED + 1000 * idx + 500
    C = H * d
    a_q = draw((B, N, C), base + 0, dtype, device)
    a_k = draw((B, N, C), base + 1, dtype, device)
    v = draw((B, N, C), base + 2, dtype, device)
    t_q = (draw((B, N, C), base + 3, "f32", device, scale=1.5) + 0.5).to(TORCH_DTYPE[dtype])
    t_k = (draw((B, N, C), base + 4, "f32", device, scale=1.5) + 0.5).to(TORCH_DTYPE[dtype])
    if zero_start:
        vecs = [torch.zeros(C, dtype=torch.float32, device=device) for _ in range(4)]
    else:
        vecs = [draw((C,), base + 5, "f32", device, scale=0.25) + 1.0, draw((C,), base + 6, "f32", device, scale=0.5),
                draw((C,), base + 7, "f32", device, scale=0.25) + 1.0, draw((C,), base + 8, "f32", device, scale=0.5)]
    return (a_q, t_q, a_k, t_k, v, *vecs)


def make_config(name: str, device="cpu"):
    c = config(name)
    return make_qkv(c["B"], c["H"], c["N"], c["d"], c["dtype"], c["idx"], c["k_scale"], device)


def stored_numpy(t: torch.Tensor) -> np.ndarray:
    """Storage of a tensor as the oracle takes it: float32 array, or uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    return t.view(torch.int16).numpy().view(np.uint16)


def algorithmic_bytes(B, H, N, d, dtype) -> int:
    """q, k, v read once and out written once."""
    return 4 * B * H * N * d * ITEMSIZE[dtype]
