"""Seeded synthetic workloads shaped like the paper's (App. B.1-B.3).

This module only draws numbers and rounds them to the kernels' input type; it contains none
of the method's arithmetic and is the one module that both the tests' oracle side and the
GPU side take their inputs from.

Every generator returns host numpy arrays holding the values *after* rounding to the input
dtype (round-to-nearest-even), as float32: the oracle widens exactly these values to fp64,
and `to_device` ships exactly these values to the GPU in the input dtype, so both sides
start from identical numbers.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np
import torch

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
DTYPE_CODE = {"f32": 0, "bf16": 1, "f16": 2}


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array -> same values rounded (RNE) to `dtype`, still stored as float32."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(_TORCH_DTYPE[dtype]).to(torch.float32).numpy()


def to_device(x: np.ndarray, dtype: str, device: str = "cuda:0") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(_TORCH_DTYPE[dtype]).to(device)


def matmul_inputs(M: int, N: int, K: int, dtype: str, seed: int, dist: str = "normal") -> Tuple[np.ndarray, np.ndarray]:
    """A[M,K], B[K,N].  dist "normal": N(0,1)/sqrt(K); "uniform": U[-1,1]."""
    rng = np.random.default_rng(seed)
    if dist == "uniform":
        A = rng.uniform(-1.0, 1.0, size=(M, K))
        B = rng.uniform(-1.0, 1.0, size=(K, N))
    else:
        A = rng.standard_normal((M, K), dtype=np.float32) / np.sqrt(K)
        B = rng.standard_normal((K, N), dtype=np.float32) / np.sqrt(K)
    return round_to(A, dtype), round_to(B, dtype)


def bmm_inputs(batch: int, M: int, N: int, K: int, dtype: str, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """A[b,M,K], B[b,K,N] ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((batch, M, K), dtype=np.float32)
    B = rng.standard_normal((batch, K, N), dtype=np.float32)
    return round_to(A, dtype), round_to(B, dtype)


def bmm_ta_inputs(batch: int, M: int, N: int, K: int, dtype: str, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """First operand stored transposed: At[b,K,M], B[b,K,N] ~ N(0,1); C[b] = At[b]^T B[b]."""
    rng = np.random.default_rng(seed)
    At = rng.standard_normal((batch, K, M), dtype=np.float32)
    B = rng.standard_normal((batch, K, N), dtype=np.float32)
    return round_to(At, dtype), round_to(B, dtype)


def conv_inputs(B: int, Cin: int, H: int, W: int, Cout: int, Hk: int, Wk: int, dtype: str, seed: int
                ) -> Tuple[np.ndarray, np.ndarray]:
    """image[B,Cin,H,W] ~ U[0,1), kernel[Cout,Cin,Hk,Wk] ~ N(0, 0.05^2)."""
    rng = np.random.default_rng(seed)
    img = rng.random((B, Cin, H, W), dtype=np.float32)
    ker = 0.05 * rng.standard_normal((Cout, Cin, Hk, Wk), dtype=np.float32)
    return round_to(img, dtype), round_to(ker, dtype)


# The graded workloads: name -> (operator kind, dims as opevo_op_create takes them, dtype, seed)
WORKLOADS: Dict[str, dict] = {
    "mm64_f32": dict(kind="matmul", dims=(64, 64, 64), dtype="f32", seed=1234, dist="uniform"),
    "mm1_bf16": dict(kind="matmul", dims=(512, 1024, 1024), dtype="bf16", seed=1235, dist="normal"),
    "bmm_attn_bf16": dict(kind="bmm", dims=(128, 128, 128, 64), dtype="bf16", seed=1236),
    "conv56_bf16": dict(kind="conv2d", dims=(1, 64, 56, 56, 64, 3, 3, 1, 1), dtype="bf16", seed=1237),
    "mm8192_bf16": dict(kind="matmul", dims=(8192, 8192, 8192), dtype="bf16", seed=1238, dist="normal"),
    "conv14_bf16": dict(kind="conv2d", dims=(32, 256, 14, 14, 256, 3, 3, 1, 1), dtype="bf16", seed=1239),
    # the paper's own operator shapes (App. B.1-B.3) with untransposed operands
    "mm2_bf16": dict(kind="matmul", dims=(512, 4096, 1024), dtype="bf16", seed=1240, dist="normal"),
    "mm3_bf16": dict(kind="matmul", dims=(512, 1024, 4096), dtype="bf16", seed=1241, dist="normal"),
    "bmm1_bf16": dict(kind="bmm", dims=(960, 128, 64, 128), dtype="bf16", seed=1242),
    "bmm2_bf16": dict(kind="bmm_ta", dims=(960, 128, 64, 128), dtype="bf16", seed=1245),   # (128x128)^T . (128x64)
    "bmm3_bf16": dict(kind="bmm_ta", dims=(960, 64, 64, 128), dtype="bf16", seed=1246),    # (128x64)^T . (128x64)
    "c1_bf16": dict(kind="conv2d", dims=(512, 3, 227, 227, 64, 11, 11, 4, 0), dtype="bf16", seed=1243),
    "c2_bf16": dict(kind="conv2d", dims=(512, 64, 27, 27, 192, 5, 5, 1, 2), dtype="bf16", seed=1244),
    # the MatMul / BMM shapes at the paper's own precision (fp32 inputs, fp32 MFMA atoms)
    "mm1_f32": dict(kind="matmul", dims=(512, 1024, 1024), dtype="f32", seed=1235, dist="normal"),
    "mm2_f32": dict(kind="matmul", dims=(512, 4096, 1024), dtype="f32", seed=1240, dist="normal"),
    "mm3_f32": dict(kind="matmul", dims=(512, 1024, 4096), dtype="f32", seed=1241, dist="normal"),
    "bmm1_f32": dict(kind="bmm", dims=(960, 128, 64, 128), dtype="f32", seed=1242),
    "bmm2_f32": dict(kind="bmm_ta", dims=(960, 128, 64, 128), dtype="f32", seed=1245),
    "bmm3_f32": dict(kind="bmm_ta", dims=(960, 64, 64, 128), dtype="f32", seed=1246),
    "c1_f32": dict(kind="conv2d", dims=(512, 3, 227, 227, 64, 11, 11, 4, 0), dtype="f32", seed=1243),
    "c2_f32": dict(kind="conv2d", dims=(512, 64, 27, 27, 192, 5, 5, 1, 2), dtype="f32", seed=1244),
    "mm8192_f16": dict(kind="matmul", dims=(8192, 8192, 8192), dtype="f16", seed=1238, dist="normal"),
    "mm8192_f32": dict(kind="matmul", dims=(8192, 8192, 8192), dtype="f32", seed=1238, dist="normal"),
}


def workload_inputs(name: str) -> Tuple[np.ndarray, np.ndarray]:
    """(first operand, second operand) in the order the kernels take them: MatMul/BMM (A, B);
    BMM with a transposed first operand (At, B); Conv2d (kernel tensor, image)."""
    w = WORKLOADS[name]
    if w["kind"] == "matmul":
        M, N, K = w["dims"]
        return matmul_inputs(M, N, K, w["dtype"], w["seed"], w.get("dist", "normal"))
    if w["kind"] == "bmm":
        b, M, N, K = w["dims"]
        return bmm_inputs(b, M, N, K, w["dtype"], w["seed"])
    if w["kind"] == "bmm_ta":
        b, M, N, K = w["dims"]
        return bmm_ta_inputs(b, M, N, K, w["dtype"], w["seed"])
    B, Cin, H, W, Cout, Hk, Wk, _, _ = w["dims"]
    img, ker = conv_inputs(B, Cin, H, W, Cout, Hk, Wk, w["dtype"], w["seed"])
    return ker, img
