"""Counter-based synthetic tensor generator (numpy reference implementation).

This module only makes *inputs*: activations, weights, router biases and
per-layer k vectors.  It holds none of the MoE arithmetic and is the one piece
of code that both the CPU oracle's tests and the HIP path's tests may import.

Definition (identical in ``csrc/synth_host.c`` and ``csrc/synth_device.hip``):

* ``mix64`` is the output function of SplitMix64 (Steele, Lea, Flood 2014):
  ``z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27;
  z *= 0x94D049BB133111EB; z ^= z >> 31``.
* ``key = mix64(seed ^ mix64(tensor_id + GOLDEN))``.
* Element ``i`` draws the three stream outputs
  ``h_m = mix64(key + (3*i + m + 1) * GOLDEN)``, ``m = 0, 1, 2``
  (a SplitMix64 stream whose state starts at ``key``).
* The twelve 16-bit fields of ``h_0, h_1, h_2`` are summed to ``S`` (exact
  integer); ``z = (2*S - 12*65535) / 131072`` is an Irwin-Hall(12) variate:
  mean 0, variance 1 - 2**-32, ``|z| < 6``, exactly representable in fp64.
* value ``= fp32_rne(fp64(sigma) * z)``; for bf16 tensors that fp32 value is
  then rounded to nearest-even bf16.

Every step is integer arithmetic or a single IEEE operation, so the numpy, C
and HIP implementations produce identical bits, and any element can be
regenerated on its own from ``(seed, tensor_id, i)``.
"""
from __future__ import annotations

import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

BASE_SEED = 0x4C455849  # ASCII "LEXI"

# tensor kinds; tensor_id = layer * 16 + kind
KIND_X = 0
KIND_W_ROUTER = 1
KIND_W_GATE = 2
KIND_W_UP = 3
KIND_W_DOWN = 4
KIND_WS_GATE = 5
KIND_WS_UP = 6
KIND_WS_DOWN = 7
KIND_W_SHARED_GATE = 8
KIND_BIAS_PERM = 9
KIND_KVEC = 10


def tensor_id(layer: int, kind: int) -> int:
    return int(layer) * 16 + int(kind)


def mix64(z):
    """SplitMix64 output function on uint64 scalars or arrays (wraps mod 2**64)."""
    with np.errstate(over="ignore"):
        z = np.asarray(z, dtype=np.uint64)
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def tensor_key(seed: int, tid: int) -> np.uint64:
    with np.errstate(over="ignore"):
        inner = mix64(np.uint64(tid) + GOLDEN)
        return mix64(np.uint64(seed) ^ inner)


def _field_sum(key: np.uint64, idx: np.ndarray) -> np.ndarray:
    """Sum of the twelve 16-bit fields drawn for each element index."""
    with np.errstate(over="ignore"):
        idx = idx.astype(np.uint64)
        total = np.zeros(idx.shape, dtype=np.int64)
        for m in range(3):
            h = mix64(key + (np.uint64(3) * idx + np.uint64(m + 1)) * GOLDEN)
            for sh in (0, 16, 32, 48):
                total += ((h >> np.uint64(sh)) & np.uint64(0xFFFF)).astype(np.int64)
        return total


def normal_f64(seed: int, tid: int, start: int, count: int) -> np.ndarray:
    """Unit-variance variates z for elements start .. start+count-1 (fp64, exact)."""
    key = tensor_key(seed, tid)
    idx = np.arange(start, start + count, dtype=np.uint64)
    s = _field_sum(key, idx)
    return (2 * s - 12 * 65535).astype(np.float64) / 131072.0


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit pattern (uint16). Finite inputs."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def fill(seed: int, tid: int, count: int, sigma: float, dtype: str, start: int = 0) -> np.ndarray:
    """Generate `count` elements: dtype 'f32' -> float32 array, 'bf16' -> uint16 bit patterns."""
    out_f32 = np.empty(count, dtype=np.float32)
    chunk = 1 << 22
    for c0 in range(0, count, chunk):
        n = min(chunk, count - c0)
        z = normal_f64(seed, tid, start + c0, n)
        out_f32[c0:c0 + n] = (np.float64(sigma) * z).astype(np.float32)
    if dtype == "f32":
        return out_f32
    if dtype == "bf16":
        return f32_to_bf16_bits(out_f32)
    raise ValueError(f"unknown dtype {dtype!r}")


def uniform_u64(seed: int, tid: int, count: int) -> np.ndarray:
    """Plain SplitMix64 stream outputs, used by the integer generators below."""
    key = tensor_key(seed, tid)
    with np.errstate(over="ignore"):
        idx = np.arange(1, count + 1, dtype=np.uint64)
        return mix64(key + idx * GOLDEN)


def seeded_permutation(seed: int, tid: int, n: int) -> np.ndarray:
    """Permutation of 0..n-1: argsort of n stream outputs (ties broken by index)."""
    h = uniform_u64(seed, tid, n)
    return np.argsort(h, kind="stable").astype(np.int64)


def zipf_router_bias(seed: int, layer: int, E: int, s: float = 1.1) -> np.ndarray:
    """Per-expert additive logit bias -s*ln(rank_e), rank a seeded permutation of 1..E.

    Makes the selection probability fall off roughly like rank**-s, i.e. the
    load imbalance across experts that batched MoE inference meets in practice.
    """
    perm = seeded_permutation(seed, tensor_id(layer, KIND_BIAS_PERM), E)
    rank = np.empty(E, dtype=np.int64)
    rank[perm] = np.arange(1, E + 1)
    return (-np.float64(s) * np.log(rank.astype(np.float64))).astype(np.float32)


def k_vector(seed: int, L: int, budget: int, k_min: int, k_max: int, moves_per_layer: int = 4) -> np.ndarray:
    """Per-layer k vector with sum == budget and k_min <= k_l <= k_max.

    Starts from the flattest vector and applies L*moves_per_layer balanced
    +1/-1 moves (one layer up, another down, rejected when out of bounds), the
    sum-preserving mutation an evolutionary search over allocations uses.
    """
    if not (L * k_min <= budget <= L * k_max):
        raise ValueError("budget outside [L*k_min, L*k_max]")
    base, extra = divmod(budget, L)
    k = np.full(L, base, dtype=np.int64)
    k[:extra] += 1
    n_moves = L * moves_per_layer
    h = uniform_u64(seed, tensor_id(0, KIND_KVEC), 2 * n_moves)
    for m in range(n_moves):
        i = int(h[2 * m] % np.uint64(L))
        j = int(h[2 * m + 1] % np.uint64(L))
        if i == j:
            continue
        if k[i] + 1 <= k_max and k[j] - 1 >= k_min:
            k[i] += 1
            k[j] -= 1
    assert int(k.sum()) == budget and k.min() >= k_min and k.max() <= k_max
    return k.astype(np.int32)
