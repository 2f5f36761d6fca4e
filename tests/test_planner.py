"""Partitioner / planner (paper §3, Eq. 1): pins of the Python oracle, then the library's host-only moe_plan
against the oracle, field by field.  Runs without a GPU."""
import random

import numpy as np
import pytest

from oracle import planner_oracle as po
from paper_2407_14417_amd import binding as mm
from paper_2407_14417_amd import synth

MB, GB = 10 ** 6, 10 ** 9
# sizes the paper prints (§4.1): 336 MB per 16-bit expert, 3.16 GB of non-expert layers, 32 x 8 experts
S16, SNE, NE = 336 * MB, 3160 * MB, 256
S4 = S16 // 4


# ---------------------------------------------------------------- oracle pins

def _brute_force_num_e16(mem, ne, n, s4):
    """Largest count of 16-bit experts (each exactly four 4-bit sizes) such that everything fits."""
    best = 0
    for c in range(n + 1):
        if ne + (n - c) * s4 + c * 4 * s4 <= mem:
            best = c
    return best


@pytest.mark.parametrize("seed", range(5))
def test_eq1_equals_brute_force_search(seed):
    rng = random.Random(seed)
    for _ in range(200):
        n = rng.randint(1, 40)
        s4 = rng.randint(1, 1000)
        ne = rng.randint(0, 5000)
        mem = rng.randint(0, ne + 5 * n * s4)
        got = po.num_e16_eq1(mem, ne, n, s4)
        if mem > ne + n * s4:
            assert got == _brute_force_num_e16(mem, ne, n, s4)
        else:
            assert got == 0


def test_eq1_boundary_and_paper_sizes():
    assert po.num_e16_eq1(SNE + NE * S4, SNE, NE, S4) == 0                 # exactly the all-4-bit model: strict ">"
    assert po.num_e16_eq1(SNE + NE * S4 + 3 * S4 - 1, SNE, NE, S4) == 0
    assert po.num_e16_eq1(SNE + NE * S4 + 3 * S4, SNE, NE, S4) == 1        # one promotion costs 3 x Size_E,4
    assert po.num_e16_eq1(SNE + NE * S16, SNE, NE, S4) == NE               # the 16-bit model fits: all 16-bit
    assert po.num_e16_eq1(10 ** 15, SNE, NE, S4) == NE                     # clamp
    # the paper's A100: 80 GB hold the all-4-bit model (3.16 + 256 x 0.084 = 24.7 GB) and 219 promotions
    assert po.num_e16_eq1(80 * GB, SNE, NE, S4) == (80 * GB - SNE - NE * S4) // (3 * S4) == 219


def test_random_mask_is_the_generators_mask():
    for n, n4, seed in ((256, 128, 0), (256, 128, 1), (8, 3, 7), (1, 1, 0), (5, 0, 2)):
        assert po.random_mask(n, n4, seed) == synth.precision_mask(n, n4, seed).tolist()


def test_plan_invariants():
    rng = random.Random(0)
    for _ in range(300):
        n = rng.randint(1, 64)
        s4 = rng.randint(1, 100)
        s16 = rng.randint(s4, 5 * s4)
        ne = rng.randint(0, 300)
        mem = rng.randint(0, ne + n * s16 + 50)
        swap = rng.choice([0, s16])
        pref = rng.choice([po.THROUGHPUT, po.QUALITY])
        n4 = rng.randint(0, n)
        q, r = po.plan(mem, ne, s16, s4, n, pref, n4, seed=rng.randint(0, 9), swap=swap)
        if pref == po.QUALITY:
            assert sum(q) == n4
        else:
            assert sum(q) == n - po.num_e16_eq1(mem, ne, n, s4)
        used = sum(s4 if q[e] else s16 for e in range(n) if r[e])
        assert used <= max(0, mem - ne - swap)
        # 4-bit first: a 16-bit expert is resident only if every 4-bit one is
        if any(r[e] and not q[e] for e in range(n)):
            assert all(r[e] for e in range(n) if q[e])
        # within a class, residents form a prefix in expert order
        for cls in (0, 1):
            flags = [r[e] for e in range(n) if q[e] == cls]
            assert flags == sorted(flags, reverse=True)


def test_more_memory_never_evicts():
    prev = -1
    for mem in range(0, SNE + NE * S16 + S16, 7 * S4):
        q, r = po.plan(mem, SNE, S16, S4, NE, po.QUALITY, 128, seed=3)
        assert sum(r) >= prev
        prev = sum(r)
    assert prev == NE


# ---------------------------------------------------------------- library against the oracle

@pytest.fixture(scope="module")
def L():
    return mm.lib()


def test_library_plan_equals_oracle(L):
    rng = random.Random(1)
    for _ in range(300):
        n = rng.randint(1, 300)
        s4 = rng.randint(1, 10 ** 8)
        s16 = rng.randint(s4, 5 * s4)
        ne = rng.randint(0, 10 ** 9)
        mem = rng.randint(0, ne + n * s16 + 1000)
        swap = rng.choice([0, s16])
        pref = rng.choice([mm.PREFER_THROUGHPUT, mm.PREFER_QUALITY])
        n4 = rng.randint(0, n)
        seed = rng.randint(0, 2 ** 40)
        res, q, r = mm.moe_plan(mem, ne, s16, s4, n, pref, n4, seed, swap)
        oq, orr = po.plan(mem, ne, s16, s4, n, pref, n4, seed, swap)
        assert q == oq and r == orr
        assert res.num_e4 == sum(oq) and res.num_e16 == n - sum(oq)
        assert res.resident_e4 == sum(1 for e in range(n) if oq[e] and orr[e])
        assert res.resident_e16 == sum(1 for e in range(n) if not oq[e] and orr[e])
        assert res.bytes_resident == ne + sum(s4 if oq[e] else s16 for e in range(n) if orr[e])


def test_library_plan_mixtral_with_this_librarys_format(L):
    """Sizes of this library's 4-bit format (4.5 bits per weight): the all-4-bit model of 256 experts needs
    3.16 GB + 256 x 99.09 MB = 28.5 GB; an 80 GB device then promotes floor(51.47 GB / 297.3 MB) = 173 experts."""
    s16, s4 = 352_321_536, 99_090_432
    res, q, r = mm.moe_plan(80 * GB, SNE, s16, s4, NE, mm.PREFER_THROUGHPUT)
    assert res.num_e16 == (80 * GB - SNE - NE * s4) // (3 * s4) == 173
    assert res.resident_e4 == res.num_e4 == NE - 173 and res.resident_e16 == 173    # Eq. 1 is conservative here
    res, q, r = mm.moe_plan(20 * GB, SNE, s16, s4, NE, mm.PREFER_THROUGHPUT)
    assert res.num_e16 == 0 and res.resident_e4 == (20 * GB - SNE) // s4 and res.resident_e16 == 0


def test_library_plan_rejects_bad_requests(L):
    for kwargs in (dict(num_experts=0), dict(size_e4=0), dict(num_e4=9, preference=mm.PREFER_QUALITY),
                   dict(num_e4=-1, preference=mm.PREFER_QUALITY), dict(preference=5)):
        a = dict(mem_gpu=100, size_non_expert=1, size_e16=4, size_e4=1, num_experts=8, preference=0, num_e4=0)
        a.update(kwargs)
        with pytest.raises(mm.MoeError):
            mm.moe_plan(**a)
