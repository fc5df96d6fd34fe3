"""Pins for the oracle's grid-wise keep-set sampler.

The paper fixes the structure (a fixed share of every local neighbourhood is
kept, a fresh draw every step visits all positions equally often, the keep ratio
is kept rows over all rows); the generator itself is this repository's
specification, pinned here to the published SplitMix64 sequence, to a second
implementation written differently, and to stored vectors.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sampler_golden.txt")
MASK = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def test_mixer_reproduces_published_splitmix64_sequence():
    # SplitMix64 (Steele, Lea, Flood, OOPSLA 2014): outputs for state seeds 1234567 and 0.
    s, out = 1234567, []
    for _ in range(5):
        s = (s + GAMMA) & MASK
        out.append(oracle.mix64(s))
    assert out == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                   4593380528125082431, 16408922859458223821]
    assert oracle.mix64(GAMMA) == 0xE220A8397B1DCDAF


# ---- a second implementation, written differently (vectorised, table of permutations) ----
_PERMS = np.array(list(itertools.permutations(range(4))), dtype=np.int64)  # lexicographic order


def _mix_np(z):
    z = z.astype(np.uint64)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def _absorb_np(h, v):
    with np.errstate(over="ignore"):
        return _mix_np(np.asarray(h, dtype=np.uint64) + np.asarray(v, dtype=np.uint64) + np.uint64(GAMMA))


def _second_sampler(B, P, H, W, k, seed, stream, shared=False, per_sample=True):
    N = P + H * W
    ch, cw = (H + 1) // 2, (W + 1) // 2
    base = _absorb_np(_absorb_np(np.uint64(0), np.uint64(seed)), np.uint64(stream))
    keep = np.zeros((B, N), dtype=bool)
    keep[:, :P] = True
    cells = np.arange(ch * cw, dtype=np.uint64)
    for b in range(B):
        hb = _absorb_np(base, np.uint64(b if per_sample else 0))
        h = _absorb_np(hb, np.zeros_like(cells) if shared else cells)
        p = ((h >> np.uint64(32)) * np.uint64(24)) >> np.uint64(32)
        perm = _PERMS[p.astype(np.int64)]            # perm[c, t] = slot of rank t (p-th lexicographic permutation)
        for c in range(ch * cw):
            cy, cx = divmod(c, cw)
            order = [s for s in perm[c] if 2 * cy + (s >> 1) < H and 2 * cx + (s & 1) < W]
            nv = len(order)
            kc = k if nv == 4 else max(1, (2 * k * nv + 4) // 8)
            for s in order[:kc]:
                keep[b, P + (2 * cy + (s >> 1)) * W + 2 * cx + (s & 1)] = True
    return keep


def _canonical_from_mask(keep, P, H, W):
    """Canonical order: sample, prefix, cell row-major, slot ascending."""
    B, N = keep.shape
    out = []
    for b in range(B):
        out += [b * N + p for p in range(P)]
        for cy in range((H + 1) // 2):
            for cx in range((W + 1) // 2):
                for s in range(4):
                    y, x = 2 * cy + (s >> 1), 2 * cx + (s & 1)
                    if y < H and x < W and keep[b, P + y * W + x]:
                        out.append(b * N + P + y * W + x)
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("geom", [(2, 0, 4, 4), (3, 1, 14, 14), (2, 0, 5, 7), (1, 2, 3, 3), (2, 1, 1, 6)])
@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("mode", [oracle.GRID_PER_CELL, oracle.GRID_SHARED])
def test_matches_second_implementation(geom, k, mode):
    B, P, H, W = geom
    for per_sample in (True, False):
        a = oracle.sample_indices(B, P, H, W, k, seed=77, stream_id=5, mode=mode, per_sample=per_sample)
        keep = _second_sampler(B, P, H, W, k, 77, 5, shared=(mode == oracle.GRID_SHARED), per_sample=per_sample)
        np.testing.assert_array_equal(a, _canonical_from_mask(keep, P, H, W))
        assert a.size == oracle.keep_count(B, P, H, W, k)


@pytest.mark.parametrize("r,k", [(0.25, 1), (0.5, 2), (0.75, 3), (1.0, 4), (0.3, 1), (0.4, 2), (0.125, 1), (0.9, 4)])
def test_k_from_ratio(r, k):
    assert oracle.k_from_ratio(r) == k


def test_keep_ratio_is_exact_on_even_grids():
    for (B, P, H, W) in [(2, 0, 14, 14), (64, 1, 14, 14), (2, 0, 200, 336), (2, 0, 50, 84)]:
        for k in (1, 2, 3, 4):
            K = oracle.keep_count(B, P, H, W, k)
            assert K == B * (P + k * H * W // 4)
    # the sizes quoted for the workloads
    assert oracle.keep_count(2, 0, 14, 14, 2) == 196
    assert oracle.keep_count(64, 1, 14, 14, 2) == 6336
    assert [oracle.keep_count(64, 1, 14, 14, k) for k in (1, 2, 3, 4)] == [3200, 6336, 9472, 12608]
    assert oracle.keep_count(2, 0, 200, 336, 2) == 67200
    assert oracle.keep_count(2, 0, 100, 168, 2) == 16800
    assert [oracle.keep_count(2, 0, 50, 84, k) for k in (1, 2, 4)] == [2100, 4200, 8400]


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_structure_every_cell_keeps_exactly_k(k):
    B, P, H, W = 3, 1, 8, 10
    N = P + H * W
    idx = oracle.sample_indices(B, P, H, W, k, seed=3, stream_id=8)
    assert idx.dtype == np.int32
    assert np.unique(idx).size == idx.size
    assert idx.min() >= 0 and idx.max() < B * N
    keep = np.zeros(B * N, dtype=bool)
    keep[idx] = True
    keep = keep.reshape(B, N)
    assert keep[:, :P].all()
    grid = keep[:, P:].reshape(B, H // 2, 2, W // 2, 2)
    assert np.all(grid.sum(axis=(2, 4)) == k)
    if k == 4:
        np.testing.assert_array_equal(np.sort(idx), np.arange(B * N))


def test_4x4_grid_k1_layout():
    # 4x4 grid, one kept slot per cell: 4 indices, one in each quadrant cell, in cell order.
    idx = oracle.sample_indices(1, 0, 4, 4, 1, seed=0, stream_id=0)
    assert idx.size == 4
    cells = [((i // 4) // 2) * 2 + (i % 4) // 2 for i in idx]
    assert cells == [0, 1, 2, 3]


def test_fresh_stream_gives_fresh_mask_and_same_inputs_give_same_mask():
    a = oracle.sample_indices(2, 0, 14, 14, 2, seed=0, stream_id=1)
    b = oracle.sample_indices(2, 0, 14, 14, 2, seed=0, stream_id=2)
    c = oracle.sample_indices(2, 0, 14, 14, 2, seed=0, stream_id=1)
    d = oracle.sample_indices(2, 0, 14, 14, 2, seed=1, stream_id=1)
    np.testing.assert_array_equal(a, c)
    assert not np.array_equal(a, b)
    assert not np.array_equal(a, d)


def test_per_sample_flag():
    H = W = 6
    shared = oracle.sample_indices(3, 0, H, W, 2, seed=4, stream_id=0, per_sample=False)
    per = oracle.sample_indices(3, 0, H, W, 2, seed=4, stream_id=0, per_sample=True)
    s = shared.reshape(3, -1) - (np.arange(3) * H * W)[:, None]
    assert np.array_equal(s[0], s[1]) and np.array_equal(s[0], s[2])
    p = per.reshape(3, -1) - (np.arange(3) * H * W)[:, None]
    assert not np.array_equal(p[0], p[1])


def test_shared_mode_is_a_lattice_and_two_complementary_draws_cover_everything():
    # one slot pattern for all cells of a sample: k=2 keeps a regular lattice, and the pattern
    # together with its complement visits every position (the paper's two-iteration remark).
    H, W = 6, 8
    idx = oracle.sample_indices(1, 0, H, W, 2, seed=2, stream_id=0, mode=oracle.GRID_SHARED)
    keep = np.zeros(H * W, dtype=bool)
    keep[idx] = True
    g = keep.reshape(H // 2, 2, W // 2, 2).transpose(0, 2, 1, 3).reshape(-1, 4)
    assert np.all(g == g[0])
    assert g[0].sum() == 2
    assert np.all(keep | ~keep) and (~keep).sum() == H * W // 2


def test_every_position_is_visited_with_frequency_r():
    # "statistically visit every spatial location with equal importance"
    H, W, draws = 4, 6, 4000
    for k in (1, 2, 3):
        cnt = np.zeros(H * W)
        for t in range(draws):
            cnt[oracle.sample_indices(1, 0, H, W, k, seed=123, stream_id=t)] += 1
        r = k / 4.0
        sigma = np.sqrt(draws * r * (1 - r))
        assert np.all(np.abs(cnt - draws * r) < 4.5 * sigma)


def test_all_subsets_of_a_cell_are_equally_likely_and_cells_are_independent():
    draws = 6000
    seen = {}
    joint = np.zeros((2, 2))
    for t in range(draws):
        idx = oracle.sample_indices(1, 0, 2, 4, 2, seed=9, stream_id=t)
        keep = np.zeros(8, dtype=bool)
        keep[idx] = True
        g = keep.reshape(2, 2, 2)   # y, cell, xslot
        c0 = tuple(int(v) for v in (g[0, 0, 0], g[0, 0, 1], g[1, 0, 0], g[1, 0, 1]))
        seen[c0] = seen.get(c0, 0) + 1
        joint[int(keep[0]), int(keep[2])] += 1       # slot 0 of cell 0 vs slot 0 of cell 1
    assert len(seen) == 6                               # C(4,2) subsets
    exp = draws / 6.0
    assert all(abs(v - exp) < 5 * np.sqrt(exp) for v in seen.values())
    assert np.all(np.abs(joint - draws / 4.0) < 5 * np.sqrt(draws * 0.25 * 0.75))


def _read_golden():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, vals = line.split(":")
            cases.append((tuple(int(v) for v in head.split()), np.array([int(v) for v in vals.split()], dtype=np.int32)))
    return cases


def test_golden_vectors():
    cases = _read_golden()
    assert len(cases) >= 6
    for (B, P, H, W, k, mode, per_sample, seed, stream), want in cases:
        got = oracle.sample_indices(B, P, H, W, k, seed, stream, mode=mode, per_sample=bool(per_sample))
        np.testing.assert_array_equal(got, want)
        keep = _second_sampler(B, P, H, W, k, seed, stream, shared=(mode == oracle.GRID_SHARED),
                               per_sample=bool(per_sample))
        np.testing.assert_array_equal(_canonical_from_mask(keep, P, H, W), want)
