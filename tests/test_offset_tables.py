"""Host logic of the tap-offset form of the convolution Hessian (Section 3, Eq. 2 with X the unfolded input of a
stride-1 k x k convolution), checked on the CPU against the definition.

With M the zero-padded maps and W_a the window of padded positions that tap a = (a_y, a_x) visits,
    H[(a, c), (b, c')] = sum over images and q in W_a of M[q, c] * M[q + (b - a), c'].
The library forms the blocks of the taps (0, 0) and (0, k - 1) directly and every other block as the base block with the
same tap offset plus a signed sum of correlations over single rows / columns ("strips").  fobq_debug_offset_tables
returns that list; here every block rebuilt from it is compared with the brute-force sum, on integer-valued maps so
that every sum is exact in fp64 and the comparison is for equality."""
import itertools

import numpy as np
import pytest

import paper_2509_05576_amd as fobq


def _padded(rng, n_img, h, w, c, pad):
    maps = rng.integers(-3, 4, size=(n_img, h, w, c)).astype(np.float64)
    mp = np.zeros((n_img, h + 2 * pad, w + 2 * pad, c))
    mp[:, pad:pad + h, pad:pad + w, :] = maps
    return mp


def _corr(mp, ys, xs, dy, dx):
    """sum over images and the positions ys x xs of M[q, c] * M[q + (dy, dx), c'] -> (c, c')"""
    a = mp[:, ys[0]:ys[1], xs[0]:xs[1], :]
    b = mp[:, ys[0] + dy:ys[1] + dy, xs[0] + dx:xs[1] + dx, :]
    return np.einsum("nyxc,nyxd->cd", a, b)


GEOMETRIES = [(3, 1, 5, 6), (3, 0, 6, 5), (3, 2, 4, 7), (2, 1, 5, 5), (2, 0, 4, 6), (3, 1, 3, 3), (3, 1, 1, 2), (3, 3, 2, 2)]


@pytest.mark.parametrize("k,pad,h,w", GEOMETRIES)
def test_every_block_is_its_base_block_plus_the_listed_strips(k, pad, h, w):
    fobq.load_library()
    tables = fobq.fobq_debug_offset_tables(k, pad, h, w)
    assert tables is not None
    jobs, pairs, terms = tables
    rng = np.random.default_rng(1000 * k + 100 * pad + 10 * h + w)
    mp = _padded(rng, 2, h, w, 3, pad)
    hp, wp = h + 2 * pad, w + 2 * pad
    ho, wo = hp - k + 1, wp - k + 1

    def block(a, b):
        return _corr(mp, (a[0], a[0] + ho), (a[1], a[1] + wo), b[0] - a[0], b[1] - a[1])

    def strip(job):
        kind, coord, start, length, dy, dx = job
        if kind == 0:
            return _corr(mp, (coord, coord + 1), (start, start + length), dy, dx)
        return _corr(mp, (start, start + length), (coord, coord + 1), dy, dx)

    seen = set()
    for ta, tb, t0, t1 in pairs:
        a, b = (ta // k, ta % k), (tb // k, tb % k)
        dy, dx = b[0] - a[0], b[1] - a[1]
        assert dy > 0 or (dy == 0 and dx >= 0)                 # canonical orientation only
        a0 = (0, 0 if dx >= 0 else k - 1)
        assert a != a0                                         # base blocks need no correction
        b0 = (a0[0] + dy, a0[1] + dx)
        assert 0 <= b0[0] < k and 0 <= b0[1] < k               # the base block exists
        rebuilt = block(a0, b0)
        for job, sign in terms[t0:t1]:
            assert sign in (-1, 1)
            rebuilt = rebuilt + sign * strip(jobs[job])
        assert np.array_equal(rebuilt, block(a, b)), f"taps {a} {b}"
        seen.add((ta, tb))
    # every pair in canonical orientation is either a base block or listed exactly once
    want = set()
    for ta, tb in itertools.product(range(k * k), repeat=2):
        a, b = (ta // k, ta % k), (tb // k, tb % k)
        dy, dx = b[0] - a[0], b[1] - a[1]
        if (dy > 0 or (dy == 0 and dx >= 0)) and a != (0, 0 if dx >= 0 else k - 1):
            want.add((ta, tb))
    assert seen == want and len(pairs) == len(want)
    # no strip reads outside the padded maps
    for kind, coord, start, length, dy, dx in jobs:
        ys = (coord, coord + 1) if kind == 0 else (start, start + length)
        xs = (start, start + length) if kind == 0 else (coord, coord + 1)
        assert 0 <= ys[0] and ys[1] <= hp and 0 <= xs[0] and xs[1] <= wp
        assert 0 <= ys[0] + dy and ys[1] + dy <= hp and 0 <= xs[0] + dx and xs[1] + dx <= wp


def test_blocks_are_the_unfolded_hessian():
    # the block formula itself against X X^T of the unfolded input (rows tap-major: (ky, kx, c))
    k, pad, h, w, c = 3, 1, 4, 5, 2
    rng = np.random.default_rng(5)
    mp = _padded(rng, 2, h, w, c, pad)
    hp, wp = h + 2 * pad, w + 2 * pad
    ho, wo = hp - k + 1, wp - k + 1
    rows = []
    for ky in range(k):
        for kx in range(k):
            for ch in range(c):
                rows.append(mp[:, ky:ky + ho, kx:kx + wo, ch].reshape(-1))
    X = np.stack(rows)
    G = X @ X.T
    for ta, tb in itertools.product(range(k * k), repeat=2):
        a, b = (ta // k, ta % k), (tb // k, tb % k)
        blk = _corr(mp, (a[0], a[0] + ho), (a[1], a[1] + wo), b[0] - a[0], b[1] - a[1])
        assert np.array_equal(blk, G[ta * c:(ta + 1) * c, tb * c:(tb + 1) * c])


def test_geometries_outside_the_tables_and_bad_arguments():
    fobq.load_library()
    assert fobq.fobq_debug_offset_tables(4, 1, 8, 8) is None          # 16 taps: more than the tables hold
    assert fobq.fobq_debug_offset_tables(1, 0, 8, 8) is None          # 1 x 1: nothing to do by offsets
    assert fobq.fobq_debug_offset_tables(3, 0, 2, 8) is None          # maps smaller than the kernel
    with pytest.raises(fobq.FobqError):
        fobq.fobq_debug_offset_tables(3, -1, 8, 8)
