"""Pins of the grid sampler with 3 x 3 and 4 x 4 cells (keep ratios k/9, k/16).  The paper names grid-wise
sampling and fixes no generator, so what can be pinned is structure (exact counts, k per full cell, the edge rule,
canonical order), uniformity (every slot and every k-subset of a cell equally often), an independently written
decoder of the same specification, and stored vectors.  Generator constants: parity unpinned by the paper."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from oracle import sbp_oracle as so

HERE = os.path.dirname(os.path.abspath(__file__))


def _second_implementation(B, P, H, W, k, cell, seed, stream, shared=False, per_sample=True):
    """Same specification, written differently: factorial-base digits taken from the least significant end,
    slots picked by list deletion on an explicit free list kept as a boolean array, positions through a mask image."""
    n = cell * cell
    fact = math.factorial(n)
    N = P + H * W
    base = so._absorb(so._absorb(0, seed), stream)
    out = []
    for b in range(B):
        hb = so._absorb(base, b if per_sample else 0)
        img = np.zeros((H, W), dtype=bool)
        cw = (W + cell - 1) // cell
        for cy in range((H + cell - 1) // cell):
            for cx in range(cw):
                h = so._absorb(hb, 0 if shared else cy * cw + cx)
                p = (h * fact) // (1 << 64)
                digits = []
                for radix in range(1, n + 1):          # least significant digit first: p = sum d_i * i!
                    digits.append(p % radix)
                    p //= radix
                digits.reverse()                        # most significant first: digit t in [0, n - 1 - t]
                free = np.ones(n, dtype=bool)
                order = []
                for d in digits:
                    s = int(np.flatnonzero(free)[d])
                    free[s] = False
                    order.append(s)
                inside = [s for s in order if cell * cy + s // cell < H and cell * cx + s % cell < W]
                kc = k if len(inside) == n else max(1, int(math.floor(k * len(inside) / n + 0.5)))
                for s in inside[:kc]:
                    img[cell * cy + s // cell, cell * cx + s % cell] = True
        rows = []
        for cy in range((H + cell - 1) // cell):       # canonical order: cells row-major, slots ascending
            for cx in range(cw):
                for s in range(n):
                    y, x = cell * cy + s // cell, cell * cx + s % cell
                    if y < H and x < W and img[y, x]:
                        rows.append(b * N + P + y * W + x)
        out.extend(list(range(b * N, b * N + P)) + rows)
    return np.asarray(out, dtype=np.int32)


@pytest.mark.parametrize("geom", [(2, 1, 9, 12, 4, 3), (1, 0, 7, 10, 5, 3), (2, 0, 8, 8, 4, 4), (1, 1, 14, 14, 8, 4),
                                  (3, 0, 5, 6, 1, 4), (1, 0, 3, 3, 9, 3), (2, 2, 13, 5, 16, 4), (1, 0, 1, 1, 2, 3)])
def test_counts_structure_and_second_implementation(geom):
    B, P, H, W, k, cell = geom
    n = cell * cell
    for seed, stream in ((0, 0), (5, 77), (2**64 - 1, 2**63)):
        idx = oracle.sample_indices_cells(B, P, H, W, k, cell, seed, stream)
        assert idx.dtype == np.int32
        assert len(idx) == oracle.keep_count_cells(B, P, H, W, k, cell) == len(set(idx.tolist()))
        assert np.array_equal(idx, _second_implementation(B, P, H, W, k, cell, seed, stream))
        N = P + H * W
        for b in range(B):
            mine = idx[(idx >= b * N) & (idx < (b + 1) * N)] - b * N
            assert list(mine[:P]) == list(range(P))
            img = np.zeros(H * W, dtype=int); img[mine[P:] - P] = 1; img = img.reshape(H, W)
            for cy in range(-(-H // cell)):
                for cx in range(-(-W // cell)):
                    blk = img[cell * cy:cell * cy + cell, cell * cx:cell * cx + cell]
                    want = k if blk.size == n else max(1, int(math.floor(k * blk.size / n + 0.5)))
                    assert blk.sum() == want, (cy, cx)


def test_every_slot_and_every_subset_equally_often():
    # one full 3 x 3 cell, k = 4: 126 subsets; 12600 draws -> 100 each on average
    cell, k, draws = 3, 4, 12600
    counts = {}
    slot = np.zeros(9)
    for st in range(draws):
        idx = tuple(oracle.sample_indices_cells(1, 0, 3, 3, k, cell, 11, st).tolist())
        counts[idx] = counts.get(idx, 0) + 1
        slot[list(idx)] += 1
    assert len(counts) == math.comb(9, 4)
    exp = draws / math.comb(9, 4)
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    assert chi2 < 125 + 5 * math.sqrt(2 * 125)            # chi-square with 125 degrees of freedom, +5 sigma
    assert np.all(np.abs(slot / draws - k / 9) < 0.02)
    # 4 x 4, k = 8: every slot half of the time
    slot = np.zeros(16)
    for st in range(4000):
        slot[oracle.sample_indices_cells(1, 0, 4, 4, 8, 4, 3, st)] += 1
    assert np.all(np.abs(slot / 4000 - 0.5) < 0.04)


def test_permutation_index_covers_its_range_and_first_digit_is_uniform():
    n = 16
    fact = math.factorial(n)
    first = np.zeros(n)
    for i in range(8000):
        h = so._absorb(so._absorb(123, i), 0)
        p = (h * fact) >> 64
        assert 0 <= p < fact
        rank = so._slot_ranks_cells(h, n)
        assert sorted(rank) == list(range(n))
        first[rank.index(0)] += 1
    assert np.all(np.abs(first / 8000 - 1 / n) < 0.015)
    assert so._slot_ranks_cells(0, 9) == list(range(9))                     # p = 0: identity
    assert so._slot_ranks_cells(2**64 - 1, 9) == list(range(8, -1, -1))     # p = 9! - 1: reversal


def test_shared_pattern_and_shared_batch():
    B, P, H, W, k, cell = 2, 0, 9, 9, 3, 3
    idx = oracle.sample_indices_cells(B, P, H, W, k, cell, 5, 6, mode=oracle.GRID_SHARED)
    img = np.zeros(B * H * W, dtype=int); img[idx] = 1; img = img.reshape(B, H, W)
    for b in range(B):
        ref = img[b, :3, :3]
        for cy in range(3):
            for cx in range(3):
                assert np.array_equal(img[b, 3 * cy:3 * cy + 3, 3 * cx:3 * cx + 3], ref)
    assert not np.array_equal(img[0], img[1])
    idx = oracle.sample_indices_cells(B, P, H, W, k, cell, 5, 6, per_sample=False)
    img = np.zeros(B * H * W, dtype=int); img[idx] = 1; img = img.reshape(B, H, W)
    assert np.array_equal(img[0], img[1])


def test_golden_vectors():
    n = 0
    for line in open(os.path.join(HERE, "golden", "sampler_cells_golden.txt")):
        if line.startswith("#"):
            continue
        head, vals = line.split(":")
        B, P, H, W, k, cell, mode, ps, seed, stream = (int(v) for v in head.split())
        want = np.array([int(v) for v in vals.split()], dtype=np.int32)
        got = oracle.sample_indices_cells(B, P, H, W, k, cell, seed, stream, mode=mode, per_sample=bool(ps))
        assert np.array_equal(got, want)
        n += 1
    assert n == 6


def test_rejects_bad_arguments():
    for cell, k in ((2, 1), (5, 1), (3, 0), (3, 10), (4, 17)):
        with pytest.raises(ValueError):
            oracle.sample_indices_cells(1, 0, 6, 6, k, cell, 0, 0)
