"""Seeded synthetic logits, bit-reproducible on host and device (input tooling only).

Stand-in for ComputeLogits(L) of Algorithm 2: the language model itself is outside the
constrained-decoding path.  Values are approximately N(0, sigma) and are produced with
integer arithmetic only, so a host (numpy) and a device (HIP) implementation of this one
definition agree bit for bit:

  element index   e = (step * batch + b) * n_tokens + t                    (64-bit)
  three words     z_k = splitmix64_output(seed, 3 e + k),  k = 0, 1, 2
                  where output n of the stream is mix(seed + (n + 1) * 0x9E3779B97F4A7C15)
                  and mix is the splitmix64 finaliser (xor-shift 30, multiply
                  0xBF58476D1CE4E5B9, xor-shift 27, multiply 0x94D049BB133111EB, xor-shift 31)
  Irwin-Hall sum  S = sum of the twelve 16-bit fields of z_0, z_1, z_2     (0 .. 786420)
  value           x = (S - 393210) * (sigma / 65536)                       exact in fp32
  bf16            round-to-nearest-even of the fp32 bit pattern to its top 16 bits

sigma must be a power of two so that the scaling is exact.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
M1 = np.uint64(0xBF58476D1CE4E5B9)
M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * M1
    z = (z ^ (z >> np.uint64(27))) * M2
    return z ^ (z >> np.uint64(31))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even of finite fp32 values to bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def gen_logits(seed: int, step: int, batch: int, n_tokens: int, sigma: float, dtype: str,
               b_lo: int = 0, b_hi: int | None = None) -> np.ndarray:
    """Rows [b_lo, b_hi) of the step's [batch, n_tokens] logits: float32 ("f32") or
    uint16 bf16 bit patterns ("bf16")."""
    b_hi = batch if b_hi is None else b_hi
    scale = np.float32(sigma / 65536.0)
    assert float(scale) * 65536.0 == sigma and np.log2(sigma) == int(np.log2(sigma))
    out = np.empty((b_hi - b_lo, n_tokens), dtype=np.float32)
    t = np.arange(n_tokens, dtype=np.uint64)
    with np.errstate(over="ignore"):
        for b in range(b_lo, b_hi):
            e = (np.uint64(step) * np.uint64(batch) + np.uint64(b)) * np.uint64(n_tokens) + t
            s = np.zeros(n_tokens, dtype=np.int64)
            for k in range(3):
                z = _mix(np.uint64(seed) + (np.uint64(3) * e + np.uint64(k + 1)) * GOLDEN)
                for sh in (0, 16, 32, 48):
                    s += ((z >> np.uint64(sh)) & np.uint64(0xFFFF)).astype(np.int64)
            out[b - b_lo] = (s - 393210).astype(np.float32) * scale
    if dtype == "f32":
        return out
    if dtype == "bf16":
        return f32_to_bf16_bits(out)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- device twin
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "gen_logits.hip")
_LIB = os.path.join(_HERE, "libtdfa_workloads.so")
_lib = None

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(force: bool = True) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["hipcc", *HIPCC_FLAGS, "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def gen_logits_device(out_ptr: int, seed: int, step: int, batch: int, n_tokens: int,
                      row_stride: int, sigma: float, dtype: str, stream: int = 0) -> None:
    """Fill device memory at out_ptr ([batch, row_stride] elements) on `stream` (a hipStream_t)."""
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (loads the HIP runtime the process uses)
        build(force=False)
        _lib = C.CDLL(_LIB)
    rc = _lib.tdfa_workload_gen_logits(C.c_void_p(out_ptr), C.c_uint64(seed), C.c_uint64(step),
                                       C.c_int32(batch), C.c_int32(n_tokens), C.c_int64(row_stride),
                                       C.c_float(sigma), C.c_int(0 if dtype == "f32" else 1),
                                       C.c_void_p(stream))
    if rc != 0:
        raise RuntimeError(f"gen_logits_device failed: hip error {rc}")
