"""Pins of the oracle's other keep-mask samplers: the random mask and temporal (whole-frame) subsets.
The paper fixes their statistics (exact keep ratio, every position visited with equal probability, no grid
structure for the random mask, frames kept whole), not a generator: the generator itself is parity unpinned."""
import itertools

import numpy as np
import pytest

import oracle


def _second_random(B, P, H, W, k, seed, stream_id):
    """Independent construction: rank every position by counting smaller (key, p) pairs."""
    from oracle.sbp_oracle import _absorb
    N, n = P + H * W, H * W
    n_keep = max(1, int(np.floor(k * n / 4 + 0.5)))
    base = _absorb(_absorb(0, seed), stream_id)
    out = []
    for b in range(B):
        hb = _absorb(base, b)
        keys = np.array([_absorb(hb, p) for p in range(n)], dtype=np.uint64)
        rank = np.array([np.sum((keys < keys[p]) | ((keys == keys[p]) & (np.arange(n) < p))) for p in range(n)])
        out += [b * N + p for p in range(P)] + [b * N + P + p for p in range(n) if rank[p] < n_keep]
    return np.asarray(out, dtype=np.int32)


@pytest.mark.parametrize("geom", [(2, 1, 14, 14), (3, 0, 5, 7), (1, 2, 1, 1), (2, 0, 9, 4)])
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_random_mask_counts_order_and_second_implementation(geom, k):
    B, P, H, W = geom
    idx = oracle.sample_indices_random(B, P, H, W, k, 5, 6)
    N = P + H * W
    per = P + oracle.random_keep_count(H, W, k)
    assert idx.size == B * per and len(set(idx.tolist())) == idx.size
    assert np.array_equal(idx, np.sort(idx))                       # canonical order is ascending row id
    for b in range(B):
        part = idx[b * per:(b + 1) * per]
        assert np.array_equal(part[:P], b * N + np.arange(P))      # prefix rows always kept
        assert np.all((part >= b * N) & (part < (b + 1) * N))
    assert np.array_equal(idx, _second_random(B, P, H, W, k, 5, 6))
    if k == 4:
        assert idx.size == B * N
    # the keep ratio is exact: |K_grid / (H W) - k / 4| <= 1 / (2 H W)
    assert abs(oracle.random_keep_count(H, W, k) / (H * W) - k / 4) <= 0.5 / (H * W) + 1e-12 or H * W < 4


def test_random_mask_is_uniform_over_subsets_and_positions():
    # 2 x 2 grid, keep 2: the 6 subsets are equally likely; larger grid: every position has frequency r
    counts = {}
    n = 3000
    for s in range(n):
        key = tuple(oracle.sample_indices_random(1, 0, 2, 2, 2, s, 1).tolist())
        counts[key] = counts.get(key, 0) + 1
    assert len(counts) == 6
    exp = n / 6
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    assert chi2 < 25.7                                              # chi-square, 5 dof, p = 1e-4
    freq = np.zeros(6 * 6)
    for s in range(800):
        freq[oracle.sample_indices_random(1, 0, 6, 6, 2, 77, s)] += 1
    sigma = np.sqrt(800 * 0.25)
    assert np.all(np.abs(freq - 400) < 4.5 * sigma)


def test_random_mask_has_no_grid_structure_and_fresh_masks_per_stream():
    # the grid-wise mask keeps exactly 2 positions of every 2 x 2 cell; a random mask of the same ratio does not
    idx = oracle.sample_indices_random(1, 0, 14, 14, 2, 1, 2)
    m = np.zeros(196, dtype=int); m[idx] = 1
    cells = m.reshape(7, 2, 7, 2).sum(axis=(1, 3))
    assert set(cells.ravel().tolist()) - {2} != set()              # some cell keeps 0, 1, 3 or 4
    other = oracle.sample_indices_random(1, 0, 14, 14, 2, 1, 3)
    assert not np.array_equal(idx, other)
    same = oracle.sample_indices_random(2, 0, 14, 14, 2, 1, 2, per_sample=False)
    assert np.array_equal(same[:98] + 196, same[98:])


@pytest.mark.parametrize("c,k", [(2, 1), (2, 2), (3, 1), (3, 2), (4, 1), (4, 3)])
@pytest.mark.parametrize("T", [8, 9, 10, 3, 1])
def test_temporal_subsets_keep_whole_frames(T, c, k):
    B, P, HW = 2, 1, 5
    idx = oracle.sample_indices_temporal(B, P, T, HW, c, k, 3, 4)
    N = P + T * HW
    nf = oracle.temporal_keep_frames(T, c, k)
    assert idx.size == B * (P + nf * HW) and np.array_equal(idx, np.sort(idx))
    for b in range(B):
        rows = idx[(idx >= b * N) & (idx < (b + 1) * N)] - b * N
        assert np.array_equal(rows[:P], np.arange(P))
        grid = np.zeros(T * HW, dtype=int); grid[rows[P:] - P] = 1
        per_frame = grid.reshape(T, HW).sum(axis=1)
        assert set(per_frame.tolist()) <= {0, HW}                  # frames are kept whole or not at all
        kept = per_frame // HW
        for cell in range(T // c):
            assert kept[cell * c:(cell + 1) * c].sum() == k        # every full cell keeps exactly k frames
        if T % c:
            assert kept[(T // c) * c:].sum() == max(1, (2 * k * (T % c) + c) // (2 * c))


def test_temporal_subsets_visit_every_frame_equally():
    T, c, k = 8, 4, 1
    freq = np.zeros(T)
    for s in range(1200):
        idx = oracle.sample_indices_temporal(1, 0, T, 1, c, k, 9, s)
        freq[idx] += 1
    sigma = np.sqrt(1200 * 0.25 * 0.75)
    assert np.all(np.abs(freq - 300) < 4.5 * sigma)
    # all C(4, 2) frame pairs of a cell occur
    seen = {tuple(oracle.sample_indices_temporal(1, 0, 4, 1, 4, 2, 1, s).tolist()) for s in range(200)}
    assert seen == set(itertools.combinations(range(4), 2))
