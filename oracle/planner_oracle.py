"""CPU ORACLE of the partitioner / planner -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Plain Python written from the paper's §3 (arXiv 2407.14417): given the available GPU memory and a task's
preference, decide how many experts are 4-bit, which experts those are (assigned at random), and which
experts stay in GPU memory (4-bit experts first).  Only tests may import this file; it shares no code with
the library's planner.

Steps, in the paper's order and notation:
  throughput preference: Num_E,16 from Eq. 1,
        floor((Mem_GPU - Size_N.E. - Num_E * Size_E,4) / (3 * Size_E,4))   if Mem_GPU > Size_N.E. + Num_E * Size_E,4
        0                                                                    otherwise
      (clamped to Num_E: the paper omits the clamp, more memory than the 16-bit model needs changes nothing);
      Num_E,4 = Num_E - Num_E,16.
  quality preference: Num_E,4 is given by the task.
  quantized attribute: a seeded random choice of Num_E,4 experts (§3: assigned to experts randomly).
  location attribute: experts are given GPU memory in the order "4-bit first, then 16-bit", each class in
      expert order, while the budget Mem_GPU - Size_N.E. - swap space lasts (§3: 4-bit experts are assigned to
      the GPU first; a swap space is set aside for expert misses).
Readings where the paper is silent: the clamp above; within a class experts are taken in index order; an
expert that does not fit ends its class (no skipping ahead); the budget is never negative.

Pins: tests/test_planner.py -- Eq. 1 against a brute-force search for the largest feasible count when a 16-bit
expert is exactly four 4-bit experts; the boundary Mem_GPU = Size_N.E. + Num_E * Size_E,4 gives 0; the paper's
own sizes (336 MB experts, 3.16 GB non-expert part, 256 experts) give all-16-bit at the 16-bit model size;
monotonicity in memory; residency never exceeds the budget; 4-bit experts resident before any 16-bit one.
"""
from __future__ import annotations

from typing import List, Tuple

THROUGHPUT, QUALITY = 0, 1

_M = (1 << 64) - 1


def _mix64(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M
    return z ^ (z >> 31)


def num_e16_eq1(mem_gpu: int, size_ne: int, num_e: int, size_e4: int) -> int:
    """Eq. 1, with the clamp to Num_E."""
    if mem_gpu > size_ne + num_e * size_e4:
        return min(num_e, (mem_gpu - size_ne - num_e * size_e4) // (3 * size_e4))
    return 0


def random_mask(num_e: int, num_e4: int, seed: int) -> List[int]:
    """1 = 4-bit.  Fisher-Yates shuffle of 0..num_e-1 driven by a splitmix64 stream; the first num_e4 entries of
    the shuffled order are quantized (same recipe as the seeded input generator's mask)."""
    key = _mix64((_mix64(seed) + 0x5EED0A5C) & _M)
    order = list(range(num_e))
    for i in range(num_e - 1, 0, -1):
        j = _mix64((key + i) & _M) % (i + 1)
        order[i], order[j] = order[j], order[i]
    mask = [0] * num_e
    for e in order[:num_e4]:
        mask[e] = 1
    return mask


def plan(mem_gpu: int, size_ne: int, size_e16: int, size_e4: int, num_e: int, preference: int, num_e4: int,
         seed: int, swap: int = 0) -> Tuple[List[int], List[int]]:
    """Returns (quantized[num_e], resident[num_e])."""
    if preference == THROUGHPUT:
        num_e4 = num_e - num_e16_eq1(mem_gpu, size_ne, num_e, size_e4)
    quantized = random_mask(num_e, num_e4, seed)
    budget = max(0, mem_gpu - size_ne - swap)
    resident = [0] * num_e
    for cls, size in ((1, size_e4), (0, size_e16)):
        for e in range(num_e):
            if quantized[e] != cls:
                continue
            if budget < size:
                break
            budget -= size
            resident[e] = 1
    return quantized, resident
