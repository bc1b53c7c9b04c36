"""Seeded synthetic inputs for segment attention.

This module holds NONE of the method's arithmetic: it only draws numbers,
rounds them to the storage type and describes the benchmark workloads.  It is
the one module that both the HIP path's tests and the CPU oracle's tests use,
so that both sides see bit-identical inputs.

Generator: a counter-based stream -- element ``i`` of stream ``seed`` is a
function of ``(seed, i)`` alone (splitmix64 finaliser on a 64-bit counter, two
uniforms, Box-Muller), so values do not depend on numpy's or torch's RNG
versions, on chunking, or on the order of generation.

Workloads: character-level language-model shapes of the paper's runs
(Section 5.1: 8 heads of width 64, batch 4; Section 5.4: 16 heads of width
128; sequence lengths up to 50,112, Table 3).  The paper trains on enwik8;
attention cost does not depend on the values, so i.i.d. Gaussian activations
of those shapes stand in for that dataset.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    x = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
    z = x
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
    return z ^ (z >> np.uint64(31))


def _normal_chunk(base, lo, hi, std, out):
    with np.errstate(over="ignore"):
        ctr = np.arange(lo, hi, dtype=np.uint64)
        a = _splitmix64(base ^ (ctr * np.uint64(2)))
        b = _splitmix64(base ^ (ctr * np.uint64(2) + np.uint64(1)))
        # 53-bit uniforms; u1 in (0, 1], u2 in [0, 1)
        u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
        u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[lo:hi] = (z * std).astype(np.float32)


def normal_f32(seed: int, n: int, std: float = 1.0, chunk: int = 1 << 20, workers: int = 8) -> np.ndarray:
    """``n`` samples of N(0, std^2) as float32; element i depends on (seed, i) only.

    Chunks are drawn by a small thread pool (numpy releases the GIL); the values do
    not depend on the chunking.
    """
    out = np.empty(n, dtype=np.float32)
    with np.errstate(over="ignore"):
        base = _splitmix64(np.array([seed], dtype=np.uint64))[0]
    spans = [(lo, min(n, lo + chunk)) for lo in range(0, n, chunk)]
    if len(spans) <= 1 or workers <= 1:
        for lo, hi in spans:
            _normal_chunk(base, lo, hi, std, out)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda sp: _normal_chunk(base, sp[0], sp[1], std, out), spans))
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration: a sequence of l_x tokens split into N segments."""
    name: str
    B: int
    l_x: int
    N: int
    H: int
    d: int
    causal: bool
    qkv_std: float      # std of Q, K, V entries
    seed: int           # base seed; streams seed+0..3 are Q, K, V, dO

    @property
    def l_s(self) -> int:
        return self.l_x // self.N

    def offsets(self):
        return [i * self.l_s for i in range(self.N)]

    def pairs(self) -> int:
        """Unmasked (query, key) pairs of the whole sequence, times B*H."""
        per = self.l_x * (self.l_x + 1) // 2 if self.causal else self.l_x * self.l_x
        return per * self.B * self.H

    def segment_pairs(self, i: int) -> int:
        s0, l_s = i * self.l_s, self.l_s
        per = l_s * s0 + l_s * (l_s + 1) // 2 if self.causal else l_s * self.l_x
        return per * self.B * self.H


# The five configurations this build is measured and checked on.
WORKLOADS = {
    "tiny": Workload("tiny", B=1, l_x=1024, N=4, H=4, d=64, causal=True, qkv_std=1.0, seed=0),
    "lx8k": Workload("lx8k", B=2, l_x=8192, N=8, H=8, d=64, causal=True, qkv_std=1.0, seed=2000),
    "lx24k": Workload("lx24k", B=4, l_x=24576, N=6, H=16, d=64, causal=True, qkv_std=0.125, seed=3000),
    "lx32k_d128": Workload("lx32k_d128", B=1, l_x=32768, N=16, H=16, d=128, causal=False, qkv_std=1.0, seed=4000),
    "lx50k": Workload("lx50k", B=1, l_x=50112, N=48, H=8, d=64, causal=True, qkv_std=1.0, seed=5000),
    # segments as short as the paper's largest runs give one GPU: 58 rows of a 50,112-token sequence
    "lx50k_skinny": Workload("lx50k_skinny", B=4, l_x=50112, N=864, H=8, d=64, causal=True, qkv_std=1.0, seed=6000),
}


def make_inputs(B, l_x, H, d, seed, qkv_std=1.0):
    """Full-sequence Q, K, V, dO as float32 arrays [B, l_x, H, d] from streams seed+0..3."""
    n = B * l_x * H * d
    shape = (B, l_x, H, d)
    q = normal_f32(seed + 0, n, qkv_std).reshape(shape)
    k = normal_f32(seed + 1, n, qkv_std).reshape(shape)
    v = normal_f32(seed + 2, n, qkv_std).reshape(shape)
    d_out = normal_f32(seed + 3, n, 1.0).reshape(shape)
    return q, k, v, d_out


def workload_inputs(w: Workload):
    return make_inputs(w.B, w.l_x, w.H, w.d, w.seed, w.qkv_std)


def make_projection_inputs(B, l_x, H, d, seed, qkv_std=1.0):
    """Inputs of the linear maps around the attention: x [B, l_x, E], W_q [E, E], W_kv [E, 2E]
    (E = H d) as float32, from streams seed+4..6.  x ~ N(0, 1); weight entries ~ N(0, qkv_std^2 / E),
    so that projected rows have the standard deviation qkv_std the attention workloads use."""
    E = H * d
    x = normal_f32(seed + 4, B * l_x * E, 1.0).reshape(B, l_x, E)
    w_std = qkv_std / float(np.sqrt(E))
    w_q = normal_f32(seed + 5, E * E, w_std).reshape(E, E)
    w_kv = normal_f32(seed + 6, E * 2 * E, w_std).reshape(E, 2 * E)
    return x, w_q, w_kv
