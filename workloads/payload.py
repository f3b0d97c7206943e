"""Seeded payload bytes of the synthetic tensors.

A copy path is value-agnostic, so every tensor but config 1's 16-bit
parameters is filled with a counter pattern: 32-bit word i of tensor t is a
bijective integer hash of (seed, t, i).  The pattern makes any misplaced,
truncated or shifted copy visible, and can be regenerated one tensor at a time
for workloads of hundreds of GiB.  Config 1 states its parameters as
N(0, 0.02) with seed 0; those are drawn here as fp16.

The GPU library fills large workloads on the device with its own
implementation of the same counter function (stated in words in the header);
this numpy version is the one expected values are built from.
"""

from __future__ import annotations

import numpy as np

PAYLOAD_SEED = 0

_M32 = np.uint64(0xFFFFFFFF)


def _hash32(x: np.ndarray) -> np.ndarray:
    """Bijective 32-bit finaliser (xor-shift / odd-multiply rounds) on uint64
    lanes holding 32-bit values."""
    x = x & _M32
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & _M32
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & _M32
    x ^= x >> np.uint64(16)
    return x


def payload_words(tensor: int, n_words: int, seed: int = PAYLOAD_SEED, first_word: int = 0) -> np.ndarray:
    """32-bit words first_word .. first_word+n_words-1 of tensor `tensor`.

    word(i) = hash32( i*0x9E3779B1 + tensor*0x85EBCA77 + seed*0xC2B2AE3D  mod 2^32 )
    """
    i = np.arange(first_word, first_word + n_words, dtype=np.uint64)
    base = (int(tensor) * 0x85EBCA77 + int(seed) * 0xC2B2AE3D) & 0xFFFFFFFF
    x = (i * np.uint64(0x9E3779B1) + np.uint64(base)) & _M32
    return _hash32(x).astype(np.uint32)


def payload_bytes(tensor: int, n_bytes: int, seed: int = PAYLOAD_SEED) -> np.ndarray:
    """The first n_bytes bytes (little-endian words) of tensor `tensor`'s pattern."""
    n_words = (int(n_bytes) + 3) // 4
    return payload_words(tensor, n_words, seed).view(np.uint8)[: int(n_bytes)].copy()


def gaussian_fp16_bytes(tensor: int, n_bytes: int, seed: int = PAYLOAD_SEED, std: float = 0.02) -> np.ndarray:
    """fp16(N(0, std)) bytes for a 16-bit parameter tensor; one generator per
    tensor, keyed by (seed, tensor), so tensors can be drawn independently."""
    rng = np.random.default_rng([int(seed), int(tensor)])
    n = (int(n_bytes) + 1) // 2
    x = (rng.standard_normal(n, dtype=np.float32) * np.float32(std)).astype(np.float16)
    return x.view(np.uint8)[: int(n_bytes)].copy()


def workload_payload(wl, tensor: int, seed: int = PAYLOAD_SEED) -> np.ndarray:
    """Initial bytes of one tensor of a workload."""
    n = int(wl.tensor_bytes[tensor])
    if wl.gaussian_p16 and int(wl.tensor_kind[tensor]) == 0:
        return gaussian_fp16_bytes(tensor, n, seed)
    return payload_bytes(tensor, n, seed)
