"""Pins of the oracle's data-derived codebook (oracle/dd.py): the histogram arithmetic against a
one-weight-at-a-time version, numpy's histogram and conservation laws, the fit against scikit-learn's weighted
k-means and the plain Lloyd iteration on the raw samples, exact-recovery and fixed-point cases, and
the library's host fit (sop_dd_fit) against the oracle's."""
import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA, dd as DD
import sop_inputs as si


def _layer(M=48, K=512, seed=11, bf16=True):
    W = si.student_t_weights(M, K, 4.0, seed, row_sigma=0.5, outlier_frac=0.002)
    if bf16:
        W = si.bf16_round(W)
    c = si.channel_norms(K, 1.0, seed + 1)
    return W, c


@pytest.mark.parametrize("g", [8, 16, 32, 64])
def test_vectorised_histogram_equals_the_loop_version(g):
    W, c = _layer(M=6, K=256, seed=3 + g)
    W[1, :g] = 0.0                                                   # an all-zero block is skipped
    W[2, g:2 * g] = -np.abs(W[2, g:2 * g])                            # one-signed block
    for cc in (c, None):
        assert np.array_equal(DD.histogram(W, cc, g, 256), DD.histogram_loops(W, cc, g, 256))


def test_histogram_conserves_weight_and_places_samples():
    W, c = _layer()
    H = 1024
    h = DD.histogram(W, c, 16, H)
    x, wt = DD.samples(W, c, 16)
    cs = 2.0 ** 20 / float(c.max())
    # every sample adds rint(c*cs): the total is within half a unit per sample of sum(c)*cs
    assert abs(h.sum() - wt.sum() * cs) <= 0.5 * x.size + 1e-6 * wt.sum() * cs
    # the weighted mean of the bin centres is the samples' weighted mean to within half a bin
    centres = -1.0 + (2.0 * np.arange(H) + 1.0) / H
    assert abs((h * centres).sum() / h.sum() - (wt * x).sum() / wt.sum()) < 1.0 / H
    # per bin: the weight it holds is that of the samples inside its edges
    edges = -1.0 + np.arange(H + 1) * (2.0 / H)
    ref = np.histogram(np.minimum(x, np.nextafter(1.0, 0.0)), bins=edges, weights=np.rint(wt * cs))[0]
    assert np.abs(ref - h).max() <= 2.0 ** 21 and abs(ref.sum() - h.sum()) < 1.0   # at most a sample on an edge moves
    # every block contributes its largest-magnitude element at |x| = 1: the end bins hold them
    assert h[0] > 0 and h[H - 1] > 0


def test_power_of_two_rescaling_of_c_and_w_changes_nothing():
    W, c = _layer(seed=21)
    h = DD.histogram(W, c, 16, 512)
    assert np.array_equal(h, DD.histogram(W, c * np.float32(8.0), 16, 512))
    assert np.array_equal(h, DD.histogram(W * np.float32(2.0 ** -7), c, 16, 512))
    # negating the layer mirrors the histogram, up to samples that sit exactly on a bin edge
    hn = DD.histogram(-W, c, 16, 512)
    assert hn.sum() == h.sum() and np.abs(hn[::-1] - h).sum() < 0.05 * h.sum()


@pytest.mark.parametrize("weighted", [False, True])
def test_fit_matches_sample_based_clustering(weighted):
    from sklearn.cluster import KMeans
    W, c = _layer(M=96, K=1024, seed=31)
    cc = c if weighted else None
    H, iters = 4096, 12
    init = OA.nf(4)
    cent = DD.fit(DD.histogram(W, cc, 16, H), 16, iters, init)
    x, wt = DD.samples(W, cc, 16)
    # (a) the oracle's plain weighted Lloyd iteration on the raw samples
    ref = OA.lloyd_1d(x, wt if weighted else None, init, iters)
    assert np.max(np.abs(cent - ref)) < 2.5 * (2.0 / H)
    # (b) scikit-learn's Lloyd k-means, same start, same number of rounds
    km = KMeans(n_clusters=16, init=init.reshape(-1, 1), n_init=1, max_iter=iters, tol=0.0, algorithm="lloyd")
    km.fit(x.reshape(-1, 1), sample_weight=wt if weighted else None)
    sk = np.sort(km.cluster_centers_.ravel())
    assert np.max(np.abs(cent - sk)) < 2.5 * (2.0 / H)
    # the channel-norm weighting matters: the two fits differ by far more than the tolerance
    if weighted:
        plain = DD.fit(DD.histogram(W, None, 16, H), 16, iters, init)
        assert np.max(np.abs(cent - plain)) > 5 * (2.0 / H)


def test_fit_recovers_levels_that_are_exactly_there():
    rng = np.random.default_rng(5)
    levels = np.array([-1.0, -0.75, -0.5, -0.375, -0.25, -0.125, -0.0625, 0.0, 0.0625, 0.1875, 0.25,
                       0.4375, 0.5, 0.625, 0.875, 1.0])
    M, K, g = 32, 256, 16
    idx = rng.integers(0, 16, size=(M, K // g, g))
    idx[:, :, 0] = 15                                                 # every block holds +1 (its largest magnitude)
    scale = 2.0 ** rng.integers(-4, 4, size=(M, K // g, 1))
    W = (levels[idx] * scale).reshape(M, K).astype(np.float32)
    c = si.channel_norms(K, 1.0, 6)
    h = DD.histogram(W, c, g, 2048)
    assert np.count_nonzero(h) == 16
    start = levels + rng.uniform(-0.02, 0.02, size=16)
    cent = DD.fit(h, 16, 3, np.sort(start))
    assert np.max(np.abs(cent - levels)) <= 1.0 / 2048                # a level is known to within its bin


def test_fit_reaches_a_fixed_point_and_lowers_the_distortion():
    W, c = _layer(M=64, K=1024, seed=41)
    h = DD.histogram(W, c, 16, 2048)
    H = 2048
    centres = -1.0 + (np.arange(H) + 0.5) * (2.0 / H)

    def distortion(cent):
        d = np.abs(centres[:, None] - cent[None, :]).min(axis=1)
        return float((h * d * d).sum())

    prev = OA.nf(4)
    values = [distortion(prev)]
    for _ in range(6):
        prev = DD.fit(h, 16, 1, prev)
        values.append(distortion(prev))
    assert all(b <= a * (1 + 1e-9) for a, b in zip(values, values[1:])) and values[-1] < 0.95 * values[0]
    far = DD.fit(h, 16, 400, OA.nf(4))
    assert np.array_equal(far, DD.fit(h, 16, 1, far))                # one more round changes nothing
    assert far[0] < 0 < far[-1] and np.all(np.diff(far) > 0)


def test_library_host_fit_equals_the_oracle_fit():
    W, c = _layer(M=64, K=1024, seed=51)
    for H, n_bits, iters in ((1024, 4, 20), (4096, 5, 7), (256, 3, 50)):
        h = DD.histogram(W, c, 16, H)
        init = OA.to_f32(OA.nf(n_bits))
        mine = sop.sop_dd_fit(h, 2 ** n_bits, iters, init)
        ref = DD.fit(h, 2 ** n_bits, iters, init.astype(np.float64))
        assert np.array_equal(mine, ref.astype(np.float32))
    # histograms with empty stretches, clusters and few samples (cells that stay empty, midpoints that fall on
    # bin centres), random start grids and round counts: same grid, or both reject
    rng = np.random.default_rng(52)
    for trial in range(120):
        H = int(rng.choice([64, 256, 1024, 4096]))
        if trial % 3 == 0:
            x = rng.standard_t(3, size=4000)
            x = x / np.abs(x).max()
        elif trial % 3 == 1:
            x = rng.uniform(-1, 1, size=int(rng.integers(40, 400)))
        else:
            x = np.concatenate([rng.normal(-0.5, 0.05, 500), rng.normal(0.6, 0.02, 500), [-1.0, 1.0]]).clip(-1, 1)
        h = np.histogram(x, bins=H, range=(-1, 1))[0].astype(np.int64) * int(rng.integers(1, 1 << 20))
        n = int(rng.choice([4, 16, 32]))
        init = np.sort(rng.uniform(-1, 1, n)).astype(np.float32)
        if np.unique(init).size < n:
            continue
        iters = int(rng.integers(0, 25))
        try:
            ref = DD.fit(h, n, iters, init.astype(np.float64)).astype(np.float32)
        except Exception:
            ref = None
        if ref is not None and not (np.all(np.diff(ref) > 0) and ref[0] < 0 < ref[-1]):
            ref = None                                                # the library rejects what cannot be an atom
        try:
            mine = sop.sop_dd_fit(h, n, iters, init)
        except sop.SopError:
            mine = None
        assert (mine is None) == (ref is None), trial
        if mine is not None:
            assert np.array_equal(mine, ref), trial
    with pytest.raises(sop.SopError) as e:                            # a one-sided result cannot be an atom
        hh = np.zeros(256, dtype=np.int64)
        hh[200:] = 5
        sop.sop_dd_fit(hh, 4, 5, np.array([0.55, 0.6, 0.7, 0.9], dtype=np.float32))
    assert e.value.status == 3


def test_block_mask_equals_zeroing_the_other_blocks():
    W, c = _layer(M=40, K=512, seed=61)
    g = 16
    rng = np.random.default_rng(62)
    mask = (rng.random(40 * 512 // g) < 0.3).astype(np.uint8)
    Wz = (W.reshape(-1, g) * mask[:, None]).reshape(W.shape).astype(np.float32)
    h = DD.histogram(W, c, g, 512, block_mask=mask)
    assert np.array_equal(h, DD.histogram(Wz, c, g, 512))
    assert 0 < h.sum() < DD.histogram(W, c, g, 512).sum()
    assert np.array_equal(DD.histogram(W, c, g, 512, block_mask=np.ones_like(mask)), DD.histogram(W, c, g, 512))
    assert DD.histogram(W, c, g, 512, block_mask=np.zeros_like(mask)).sum() == 0


def test_steps_one_to_four_refit_on_the_worst_blocks_helps():
    """Step 2 ranks by block cosine under L_a, step 3 fits L_b on the rest, step 4 picks per block."""
    from oracle import partition as PT, pairsearch as ps
    W, c = _layer(M=64, K=1024, seed=71)
    g = 16
    fmt = ps.make_fmt(0, 4, 4)
    La = OA.to_f32(OA.nf(4))
    r1 = ps.pair_search(W, c, [La], g, fmt)
    n_top = PT.top_count(60.0, r1.blk_cos.shape[1])
    tau, pool_b, n_a = PT.partition(r1.blk_cos[0], n_top, True)
    assert n_a >= n_top and pool_b.sum() == pool_b.size - n_a
    # the fitting pool holds the blocks L_a serves worst
    assert r1.blk_cos[0][pool_b == 1].max() < tau <= r1.blk_cos[0][pool_b == 0].min()
    Lb = OA.to_f32(DD.fit(DD.histogram(W, c, g, 1024, block_mask=pool_b), 16, 12, OA.nf(4)))
    r2 = ps.pair_search(W, c, [La, Lb], g, fmt)
    assert r2.acos_pair[0] > r2.acos_atom[0] and r2.acos_pair[0] > r2.acos_atom[1]
    # fitted on its own pool, L_b beats a fit on all blocks there (in the scale-free block cosine:
    # the fit works on block-normalised weights, so every block counts alike)
    Lall = OA.to_f32(DD.fit(DD.histogram(W, c, g, 1024), 16, 12, OA.nf(4)))
    r3 = ps.pair_search(W, c, [Lb, Lall], g, fmt)
    pool = pool_b == 1
    assert r3.blk_cos[0][pool].mean(dtype=np.float64) > r3.blk_cos[1][pool].mean(dtype=np.float64)
