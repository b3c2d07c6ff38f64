"""Pins for the CPU oracle's inverse density importance sub-sampling (Sec. 3.2), CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from helpers import grid2d


def test_phi_bruteforce_and_grid_closed_form():
    rng = np.random.default_rng(0)
    B, N, K = 2, 29, 5
    pos = rng.random((B, 3, N)).astype(np.float32)
    nbr = rng.integers(0, N, size=(B, K, N)).astype(np.int32)
    phi = oracle.idiss_phi(pos, nbr)
    p = pos.astype(np.float64)
    for b in range(B):
        for l in range(N):
            ref = sum(np.linalg.norm(p[b, :, nbr[b, k, l]] - p[b, :, l]) for k in range(K))
            assert abs(phi[b, l] - ref) <= 1e-13 * max(1.0, ref)
    # regular grid, the 3x3 offsets: four neighbours at h, four at h*sqrt(2), the point itself at 0
    H, W, h = 7, 9, 0.5
    gpos, gnbr, _ = grid2d(H, W, h)
    gphi = oracle.idiss_phi(gpos, gnbr).reshape(H, W)
    np.testing.assert_allclose(gphi[1:-1, 1:-1], 4 * h + 4 * h * np.sqrt(2.0), rtol=1e-12)


def _reference_sample(phi, u):
    """The same procedure with exact rationals / Python integers, written independently."""
    N, Ns = len(phi), len(u)
    lg = (N - 1).bit_length()
    bits = min(28, 51 - lg)
    mx = np.float32(phi.max())
    if mx > 0:
        scale = np.float32(np.float32(2.0 ** bits) / mx)
        q = [int(np.float32(np.float32(x) * scale)) for x in phi]
    else:
        q = [1] * N
    C = np.cumsum(np.array(q, dtype=object))
    Q = int(C[-1])
    out = []
    for j in range(Ns):
        # strata of whole units, lengths differing by at most one: the first Q mod Ns get the extra unit
        width, rem = divmod(Q, Ns)
        lens = [width + (1 if i < rem else 0) for i in range(Ns)]
        assert sum(lens) == Q
        start, ln = sum(lens[:j]), lens[j]
        t = start + int(Fraction(int(u[j]), 2 ** 32) * ln)
        out.append(next(i for i in range(N) if C[i] > t))
    return out


def test_sample_matches_exact_integer_reference():
    rng = np.random.default_rng(1)
    for N, Ns in ((50, 12), (64, 64), (33, 1), (200, 50)):
        phi = rng.random((2, N)).astype(np.float32)
        phi[0, ::7] = 0.0                                   # never drawn
        phi[1, 3] = 40.0                                    # far heavier than a stratum: drawn several times
        u = rng.integers(0, 2 ** 32, size=(2, Ns), dtype=np.uint64).astype(np.uint32)
        sel = oracle.idiss_sample(phi, u)
        for b in range(2):
            assert list(sel[b]) == _reference_sample(phi[b], u[b])
        assert (np.diff(sel, axis=1) >= 0).all()
        assert not np.isin(sel[0], np.arange(0, N, 7)).any()
    # few units (all-zero phi gives one unit per point): the strata's uneven lengths decide the draw
    for N, Ns in ((10, 4), (7, 3), (23, 5)):
        phi = np.zeros((1, N), np.float32)
        for seed in range(20):
            u = np.random.default_rng(seed).integers(0, 2 ** 32, size=(1, Ns), dtype=np.uint64).astype(np.uint32)
            assert list(oracle.idiss_sample(phi, u)[0]) == _reference_sample(phi[0], u[0])


def _reference_sample_integers(k, kmax, u, bits):
    """The draw for weights phi_l = k_l / 2^27 in integer arithmetic alone: q_l = floor(k_l 2^bits / kmax).  Nothing of
    the procedure's float32 steps is retyped; on such weights, with kmax a power of two, those steps are exact, so the
    oracle must return exactly this."""
    q = [(int(v) << bits) // int(kmax) for v in k]
    C = np.cumsum(np.array(q, dtype=object)) if len(q) < 4096 else np.cumsum(np.array(q, dtype=np.int64))
    Q, Ns = int(C[-1]), len(u)
    assert Q < 2 ** 62
    width, rem = divmod(Q, Ns)
    out = []
    for j in range(Ns):
        start = j * width + min(j, rem)
        ln = width + (1 if j < rem else 0)
        t = start + ((int(u[j]) * ln) >> 32)
        out.append(int(np.searchsorted(C, t, side="right")))
    return out


@pytest.mark.parametrize("N,Ns,log2_top", [(40, 10, 27), (97, 31, 26), (64, 16, 28), (300, 75, 27), (2 ** 23 + 1, 64, 27)])
def test_quantisation_against_integer_arithmetic_on_dyadic_weights(N, Ns, log2_top):
    # weights k / 2^27 with 24-bit k and a power of two as the largest: the procedure's float32 quotient 2^bits / max and
    # its products are exact, so its integer weights must be floor(k 2^bits / kmax) computed in integers.  Largest
    # weight 2 (log2_top = 28) leaves half-integers for the floor to act on; N above 2^23 lowers the resolution to
    # 2^27, below it the resolution is 2^28.
    rng = np.random.default_rng(N)
    bits = min(28, 51 - (N - 1).bit_length())
    assert bits == (27 if N > 2 ** 23 else 28)
    k = rng.integers(1, 2 ** 24, size=N, dtype=np.int64) | 1
    k[::9] = 0
    k[int(rng.integers(0, N))] = 2 ** log2_top
    phi = (k.astype(np.float64) * 2.0 ** -27).astype(np.float32)
    assert np.array_equal(phi.astype(np.float64) * 2.0 ** 27, k.astype(np.float64))
    u = rng.integers(0, 2 ** 32, size=(1, Ns), dtype=np.uint64).astype(np.uint32)
    # half of the draws are aimed at the last unit of one point's share and the first unit of the next one's, where an
    # integer weight that is off by one anywhere before them changes the point drawn
    q = [(int(v) << bits) // 2 ** log2_top for v in k]
    C = np.cumsum(np.array(q, dtype=np.int64))
    width, rem = divmod(int(C[-1]), Ns)
    aimed = 0
    for j in range(0, Ns, 2):
        start, ln = j * width + min(j, rem), width + (1 if j < rem else 0)
        inside = np.flatnonzero((C > start) & (C < start + ln))
        if len(inside) == 0 or ln >= 2 ** 32:
            continue
        x = int(C[inside[len(inside) // 2]]) - start - (j // 2) % 2
        u[0, j] = -((-x << 32) // ln)                        # the least u with floor(u ln / 2^32) = x
        assert (int(u[0, j]) * ln) >> 32 == x
        aimed += 1
    assert aimed >= min(Ns, 8) // 2 - 1 or width >= 2 ** 32   # (a stratum wider than 2^32 cannot be hit to the unit)
    got = [int(v) for v in oracle.idiss_sample(phi[None], u)[0]]
    assert got == _reference_sample_integers(k, 2 ** log2_top, u[0], bits)


def test_sample_uniform_density_is_one_point_per_block():
    # equal phi: the strata are equal blocks of points, one point drawn from each
    N, Ns = 4096, 1024
    phi = np.full((1, N), 0.37, np.float32)
    rng = np.random.default_rng(2)
    u = rng.integers(0, 2 ** 32, size=(1, Ns), dtype=np.uint64).astype(np.uint32)
    sel = oracle.idiss_sample(phi, u)[0]
    assert np.array_equal(sel // 4, np.arange(Ns))
    assert len(np.unique(sel % 4)) == 4                     # the random words move the draw inside a block
    # all-zero phi (coincident points) falls back to the same uniform draw
    assert np.array_equal(oracle.idiss_sample(np.zeros((1, N), np.float32), u)[0], sel)


def test_sample_frequencies_are_proportional_to_phi():
    rng = np.random.default_rng(3)
    N, Ns, trials = 60, 15, 4000
    phi = (0.2 + rng.random(N)).astype(np.float32)
    counts = np.zeros(N)
    for _ in range(trials):
        u = rng.integers(0, 2 ** 32, size=(1, Ns), dtype=np.uint64).astype(np.uint32)
        np.add.at(counts, oracle.idiss_sample(phi[None], u)[0], 1)
    expect = trials * Ns * phi.astype(np.float64) / phi.astype(np.float64).sum()
    assert np.abs(counts - expect).max() <= 5.0 * np.sqrt(expect.max())      # five sigma of a Poisson count
    assert abs(counts.sum() - trials * Ns) == 0


def test_make_distinct_bruteforce_and_properties():
    rng = np.random.default_rng(9)
    for N, Ns in ((30, 12), (10, 10), (50, 1), (40, 35), (1000, 400)):
        for trial in range(20):
            sel = np.sort(rng.integers(0, N, size=(2, Ns)), axis=1).astype(np.int32)
            if trial % 3 == 0:
                sel[0, Ns // 2:] = N - 1                      # a pile of repeats at the very end
            out = oracle.selection_make_distinct(sel, N)
            for b in range(2):
                s = [int(v) for v in sel[b]]
                for j in range(1, Ns):                         # the rule, in plain Python
                    if s[j] <= s[j - 1]:
                        s[j] = s[j - 1] + 1
                for j in range(Ns - 1, -1, -1):
                    s[j] = min(s[j], N - Ns + j)
                assert list(out[b]) == s
            assert (np.diff(out, axis=1) > 0).all() and out.min() >= 0 and out.max() < N
            keep = np.ones_like(sel, bool)
            keep[:, 1:] = sel[:, 1:] != sel[:, :-1]
            # away from a packed tail, the first occurrence of every drawn point stays where it was unless an
            # earlier run of repeats had spilled over it
            untouched = (out == sel)
            assert untouched[:, 0].all() or (sel[:, 0] > N - Ns).any()
    distinct = np.array([[1, 4, 9, 20]], np.int32)
    assert np.array_equal(oracle.selection_make_distinct(distinct, 25), distinct)   # nothing to do: unchanged
