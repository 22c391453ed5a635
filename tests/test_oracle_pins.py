"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests needs a GPU.  Each pins a part of oracle/kf_oracle.c to
something other than itself: closed forms (Eq. 12), limits the paper states for
the temperature (Sec. 3.3.1), the constants it prints for the Gumbel pdf
(Sec. 4.4.3), textbook properties of Eq. 7 (CDF, Gumbel-max), an independent
numpy/scipy evaluation of Eq. 1 / Eq. 4 / Eq. 11 / Alg. 1, and brute force.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import kf_oracle as ko

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def paper_constants():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def bf16_round(a):
    """float32 -> nearest-even bf16, returned as uint16 bits (input prep only)."""
    b = a.astype(np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return b.astype(np.uint16)


def as_f64(a):
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def make_cache(rng, L, B, H, d, cap, n, dtype=ko.F32, pos=None):
    c = ko.OracleCache(L, B, H, d, cap, dtype)
    K = rng.standard_normal((L, B, H, n, d)).astype(np.float32)
    V = rng.standard_normal((L, B, H, n, d)).astype(np.float32)
    if dtype == ko.BF16:
        K, V = bf16_round(K), bf16_round(V)
    c.K[..., :n, :] = K
    c.V[..., :n, :] = V
    c.pos[..., :n] = np.arange(n) if pos is None else pos
    c.len[...] = n
    return c


def rand_vec(rng, shape, dtype):
    a = rng.standard_normal(shape).astype(np.float32)
    return bf16_round(a) if dtype == ko.BF16 else a


def zeta_matrix(noise, seed, layer, head, q_positions, k_positions):
    return np.array([[ko.zeta(noise, seed, layer, head, int(qp), int(kp)) for kp in k_positions]
                     for qp in q_positions])


# ----------------------------------------------------------------------------
# P11  tau schedule, Eq. 12
# ----------------------------------------------------------------------------
def test_tau_closed_form():
    pc = paper_constants()
    for T in (1, 7, 32, 512, 2048):
        taus = [ko.tau(t, T, pc["tau_init"], pc["tau_end"]) for t in range(T + 1)]
        assert taus[0] == pc["tau_init"]                      # prompt iteration
        assert abs(taus[T] - pc["tau_end"]) < 1e-6            # last decode step
        assert all(b > a for a, b in zip(taus, taus[1:]))     # increments by dtau > 0
        for t in (1, T // 2, T):
            exact = pc["tau_init"] + t * (pc["tau_end"] - pc["tau_init"]) / T
            assert abs(taus[t] - exact) < 1e-6
    assert ko.tau(5, 10, 1.5, 1.5) == 1.5                     # fixed temperature


# ----------------------------------------------------------------------------
# P8  noise distribution: Eq. 7 and the constants printed in Sec. 4.4.3
# ----------------------------------------------------------------------------
def _noise_sample(n_q=600, n_k=600, seed=20240309, layer=3, head=5):
    return np.array([[ko.noise_bits(seed, layer, head, qp, kp) for kp in range(n_k)]
                     for qp in range(1000, 1000 + n_q)], dtype=np.uint64)


def test_noise_uniform_bits_and_gumbel_moments():
    pc = paper_constants()
    bits = _noise_sample()
    N = bits.size
    # every output bit is fair
    for b in range(32):
        frac = ((bits >> np.uint64(b)) & np.uint64(1)).mean()
        assert abs(frac - 0.5) < 4.5 * 0.5 / math.sqrt(N), (b, frac)
    z = np.array([ko.gumbel(int(v)) for v in bits.ravel()[:200000]])
    n = z.size
    # mean and std printed in the paper; 4 sigma of the sampling error
    assert abs(z.mean() - pc["gumbel_mean"]) < 4 * pc["gumbel_std"] / math.sqrt(n) + 5e-5
    assert abs(z.std() - pc["gumbel_std"]) < 4 * 1.1 * pc["gumbel_std"] / math.sqrt(n) + 5e-5
    # Kolmogorov-Smirnov against the CDF of Eq. 7's pdf, exp(-exp(-z))
    ks = scipy.stats.kstest(z, lambda t: np.exp(-np.exp(-t)))
    assert ks.pvalue > 1e-3, ks
    assert np.isfinite(z).all() and z.min() > -2.9 and z.max() < 16.7


def test_noise_gumbel_is_inverse_cdf_of_eq7():
    # u = (2*(bits>>9)+1)/2^24, CDF(zeta) must give u back: pins sign and form
    for bits in (0, 1 << 9, 0x7FFFFFFF, 0x80000000, 0xFFFFFFFF, 123456789):
        u = (2 * (bits >> 9) + 1) / 2.0 ** 24
        z = ko.gumbel(bits)
        assert abs(math.exp(-math.exp(-z)) - u) < 1e-12


def test_noise_independence_across_positions_heads_seeds():
    bits = _noise_sample(300, 300)
    u = (bits >> np.uint64(9)).astype(np.float64) / 2 ** 23
    N = u.size
    lim = 4.5 / math.sqrt(N)
    c = lambda a, b: np.corrcoef(a.ravel(), b.ravel())[0, 1]
    assert abs(c(u[:, :-1], u[:, 1:])) < lim          # adjacent key positions
    assert abs(c(u[:-1, :], u[1:, :])) < lim          # adjacent query positions (steps)
    assert abs(c(u[:-1, :-1], u[1:, 1:])) < lim       # diagonal
    assert abs(c(u, u.T)) < lim                       # (q,k) vs (k,q)
    other = np.array([[ko.noise_bits(20240309, 3, 6, qp, kp) for kp in range(300)]
                      for qp in range(1000, 1300)], dtype=np.uint64)
    assert abs(c(u, (other >> np.uint64(9)).astype(np.float64))) < lim   # neighbouring head
    other = np.array([[ko.noise_bits(20240308, 3, 5, qp, kp) for kp in range(300)]
                      for qp in range(1000, 1300)], dtype=np.uint64)
    assert abs(c(u, (other >> np.uint64(9)).astype(np.float64))) < lim   # neighbouring seed
    # the layer enters the key: neighbouring layers (and layers far apart) draw unrelated streams at the
    # same seed, head and positions -- per-layer scores (Sec. 4.4.1) rest on per-layer noise
    for other_layer in (4, 2, 27):
        other = np.array([[ko.noise_bits(20240309, other_layer, 5, qp, kp) for kp in range(300)]
                          for qp in range(1000, 1300)], dtype=np.uint64)
        assert abs(c(u, (other >> np.uint64(9)).astype(np.float64))) < lim, other_layer
        assert (other != bits).mean() > 0.999, other_layer
    # layer and head are separate coordinates: (layer 3, head 5) is not (layer 5, head 3)
    other = np.array([[ko.noise_bits(20240309, 5, 3, qp, kp) for kp in range(300)]
                      for qp in range(1000, 1300)], dtype=np.uint64)
    assert abs(c(u, (other >> np.uint64(9)).astype(np.float64))) < lim
    # no duplicated streams: all 32-bit words of one row distinct from the next row's
    assert (bits[0] != bits[1]).mean() > 0.999


def test_gaussian_adjustment_draws_two_unrelated_uniforms():
    """Eq. 5 needs a normal variate, i.e. (Box-Muller) two independent uniforms per logit.  The second one
    is the generator's word at the key position with its top bit flipped: it must be unrelated to the
    first, and the variate must be the Box-Muller combination of exactly these two words."""
    pc = paper_constants()
    seed, layer, head = 424242, 2, 7
    qps, kps = range(500, 700), range(0, 300)
    b1 = np.array([[ko.noise_bits(seed, layer, head, qp, kp) for kp in kps] for qp in qps], dtype=np.uint64)
    b2 = np.array([[ko.noise_bits(seed, layer, head, qp, kp ^ 0x80000000) for kp in kps] for qp in qps],
                  dtype=np.uint64)
    u1 = (2.0 * (b1 >> np.uint64(9)).astype(np.float64) + 1.0) / 2.0 ** 24
    u2 = (2.0 * (b2 >> np.uint64(9)).astype(np.float64) + 1.0) / 2.0 ** 24
    N = u1.size
    lim = 4.5 / math.sqrt(N)
    corr = lambda a, b: np.corrcoef(a.ravel(), b.ravel())[0, 1]
    assert (b1 != b2).mean() > 0.999
    assert abs(corr(u1, u2)) < lim                                  # linear
    assert abs(corr(np.log(u1), np.cos(2 * np.pi * u2))) < lim      # radius against angle
    assert abs(corr((u1 - 0.5) ** 2, (u2 - 0.5) ** 2)) < lim        # second order
    # joint uniformity on an 8x8 grid (chi-square, 63 degrees of freedom)
    cells = np.histogram2d(u1.ravel(), u2.ravel(), bins=8, range=[[0, 1], [0, 1]])[0]
    chi2 = ((cells - N / 64.0) ** 2 / (N / 64.0)).sum()
    assert chi2 < scipy.stats.chi2.ppf(0.9995, 63), chi2
    # the variate itself, from these two words (textbook Box-Muller, mean and std as printed in Sec. 4.4.3)
    g = np.array([[ko.zeta(ko.NOISE_GAUSSIAN, seed, layer, head, qp, kp) for kp in kps] for qp in qps])
    want = pc["gumbel_mean"] + pc["gumbel_std"] * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    np.testing.assert_allclose(g, want, rtol=0, atol=1e-9)
    # and its radial and angular parts are independent: the squared distance from the mean is exponential
    # whatever the sign of the variate
    r2 = ((g - pc["gumbel_mean"]) / pc["gumbel_std"]) ** 2
    assert abs(corr(r2, np.sign(g - pc["gumbel_mean"]))) < lim


def test_noise_golden_file_matches_oracle():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "noise_bits.txt")) if not l.startswith("#")]
    assert len(rows) > 100
    for r in rows:
        assert ko.noise_bits(*map(int, r[:5])) == int(r[5])


def test_gaussian_and_constant_adjustments():
    pc = paper_constants()
    assert ko.zeta(ko.NOISE_CONSTANT, 1, 2, 3, 4, 5) == pc["constant_adjustment"]
    assert ko.zeta(ko.NOISE_NONE, 1, 2, 3, 4, 5) == 0.0
    g = np.array([ko.zeta(ko.NOISE_GAUSSIAN, 7, 1, 2, qp, kp) for qp in range(300) for kp in range(300)])
    n = g.size
    assert abs(g.mean() - pc["gumbel_mean"]) < 4 * pc["gumbel_std"] / math.sqrt(n)
    assert abs(g.std() - pc["gumbel_std"]) < 4 * pc["gumbel_std"] / math.sqrt(2 * n)
    ks = scipy.stats.kstest(g, "norm", args=(pc["gumbel_mean"], pc["gumbel_std"]))
    assert ks.pvalue > 1e-3
    assert abs(scipy.stats.skew(g)) < 0.03     # symmetric, unlike the Gumbel (skew 1.14)


# ----------------------------------------------------------------------------
# P7  Gumbel-max: argmax_j (x_j + zeta_j) is distributed as softmax(x)
# ----------------------------------------------------------------------------
def test_gumbel_max_frequencies_follow_softmax():
    x = np.array([0.3, -1.0, 1.2, 0.0, 2.0, -0.5])
    p = scipy.special.softmax(x)
    trials = 40000
    counts = np.zeros(len(x))
    for t in range(trials):
        z = np.array([ko.zeta(ko.NOISE_GUMBEL, 99, 0, 1, t, j) for j in range(len(x))])
        counts[np.argmax(x + z)] += 1
    chi2 = ((counts - trials * p) ** 2 / (trials * p)).sum()
    assert chi2 < scipy.stats.chi2.ppf(0.9995, len(x) - 1), (chi2, counts / trials, p)


# ----------------------------------------------------------------------------
# Independent numpy/scipy evaluation of one decode step (Eq. 1, Eq. 4, Eq. 11)
# ----------------------------------------------------------------------------
def numpy_decode(c, u_idx, q, q_pos, tau, scale, noise, seed, slope):
    l, b, h = u_idx
    m = int(c.len[l, b, h])
    K = as_f64(c.K[l, b, h, :m])
    V = as_f64(c.V[l, b, h, :m])
    pos = c.pos[l, b, h, :m].astype(np.int64)
    x = np.float64(np.float32(scale)) * (K @ as_f64(q)) - slope * (q_pos - pos)
    p = scipy.special.softmax(x)
    z = np.array([ko.zeta(noise, seed, l, h, q_pos, int(kp)) for kp in pos])
    df = scipy.special.softmax((x + z) / np.float64(np.float32(tau)))
    return p @ V, p, df


@pytest.mark.parametrize("dtype", [ko.F32, ko.BF16])
@pytest.mark.parametrize("noise", [ko.NOISE_GUMBEL, ko.NOISE_NONE, ko.NOISE_GAUSSIAN, ko.NOISE_CONSTANT])
def test_decode_step_matches_numpy(dtype, noise):
    rng = np.random.default_rng(5)
    L, B, H, d, cap, n = 2, 2, 3, 16, 40, 29
    # non-trivial, strictly ascending original positions
    pos = np.sort(rng.choice(200, size=(L, B, H, n), replace=True), axis=-1)
    pos = pos + np.arange(n)  # make strictly ascending
    c = make_cache(rng, L, B, H, d, cap, n, dtype, pos=pos)
    c.score[..., :n] = rng.random((L, B, H, n)).astype(np.float32)
    before = c.copy()
    q, kn, vn = (rand_vec(rng, (L, B, H, d), dtype) for _ in range(3))
    seeds = np.array([11, 2 ** 63 + 5], np.uint64)
    slopes = np.array([0.5, 0.0, 0.02], np.float32)
    q_pos, tau, scale = 777, 1.37, 0.25
    out, dp, df = c.decode_step(q, kn, vn, q_pos, tau, scale, noise, seeds, slopes, debug=True)
    assert (c.len == n + 1).all()
    # append semantics: new row at slot n, pos = q_pos, old rows untouched
    assert (c.K[..., n, :] == kn).all() and (c.V[..., n, :] == vn).all()
    assert (c.pos[..., n] == q_pos).all()
    assert (c.K[..., :n, :] == before.K[..., :n, :]).all()
    for l, b, h in itertools.product(range(L), range(B), range(H)):
        o_ref, p_ref, df_ref = numpy_decode(c, (l, b, h), q[l, b, h], q_pos, tau, scale, noise,
                                            int(seeds[b]), float(slopes[h]))
        m = n + 1
        np.testing.assert_allclose(dp[l, b, h, :m], p_ref, rtol=1e-11, atol=1e-300)
        np.testing.assert_allclose(df[l, b, h, :m], df_ref, rtol=1e-11, atol=1e-300)
        np.testing.assert_allclose(out[l, b, h], o_ref.astype(np.float32), rtol=2e-7, atol=1e-30)
        f_ref = (np.append(before.score[l, b, h, :n], 0.0).astype(np.float64) + df_ref).astype(np.float32)
        np.testing.assert_array_equal(c.score[l, b, h, :m], f_ref)
        # P1: both softmaxes are probability vectors
        assert abs(dp[l, b, h, :m].sum() - 1) < 1e-12 and abs(df[l, b, h, :m].sum() - 1) < 1e-12
        # P2: a convex combination of the value rows
        Vm = as_f64(c.V[l, b, h, :m])
        assert (out[l, b, h] <= Vm.max(0) + 1e-6).all() and (out[l, b, h] >= Vm.min(0) - 1e-6).all()
    if noise in (ko.NOISE_NONE, ko.NOISE_CONSTANT):
        pass


def test_no_noise_tau_one_is_plain_attention_and_constant_shift_is_invisible():
    # P4: without adjustment and at tau = 1 the score increment IS the attention
    # probability (accumulated-attention / H2O-style score); a constant added to
    # every logit cancels in the softmax.
    rng = np.random.default_rng(6)
    c = make_cache(rng, 1, 1, 2, 32, 50, 37)
    c2 = c.copy()
    q, kn, vn = (rand_vec(rng, (1, 1, 2, 32), ko.F32) for _ in range(3))
    _, dp, df = c.decode_step(q, kn, vn, 37, 1.0, 0.3, ko.NOISE_NONE, debug=True)
    assert (dp == df).all()
    _, dp2, df2 = c2.decode_step(q, kn, vn, 37, 1.0, 0.3, ko.NOISE_CONSTANT, debug=True)
    np.testing.assert_allclose(df2[..., :38], dp[..., :38], rtol=1e-12)


def test_temperature_limits():
    # Sec. 3.3.1: tau -> infinity gives uniform scores, tau -> 0 a sharp distribution
    rng = np.random.default_rng(7)
    n = 23
    c = make_cache(rng, 1, 1, 2, 16, 30, n)
    q, kn, vn = (rand_vec(rng, (1, 1, 2, 16), ko.F32) for _ in range(3))
    seeds = np.array([5], np.uint64)
    hot = c.copy()
    _, _, df = c.decode_step(q, kn, vn, 100, 1e9, 0.25, ko.NOISE_GUMBEL, seeds, debug=True)
    np.testing.assert_allclose(df[..., :n + 1], 1.0 / (n + 1), rtol=1e-6)
    _, _, df = hot.decode_step(q, kn, vn, 100, 1e-3, 0.25, ko.NOISE_GUMBEL, seeds, debug=True)
    for h in range(2):
        K = as_f64(hot.K[0, 0, h, :n + 1])
        x = 0.25 * (K @ as_f64(q[0, 0, h]))
        z = np.array([ko.zeta(ko.NOISE_GUMBEL, 5, 0, h, 100, int(p)) for p in hot.pos[0, 0, h, :n + 1]])
        j = int(np.argmax(x + z))
        assert df[0, 0, h, j] > 1 - 1e-9 and abs(df[0, 0, h, :n + 1].sum() - 1) < 1e-12


def test_single_token_and_equal_keys():
    # P2 special case: one cached token -> out = its value, increment = 1
    c = ko.OracleCache(1, 1, 1, 8, 4)
    rng = np.random.default_rng(8)
    q, kn, vn = (rand_vec(rng, (1, 1, 1, 8), ko.F32) for _ in range(3))
    out, dp, df = c.decode_step(q, kn, vn, 0, 1.7, 0.35, ko.NOISE_GUMBEL, np.array([3], np.uint64), debug=True)
    np.testing.assert_array_equal(out, vn)
    assert dp[0, 0, 0, 0] == 1.0 and df[0, 0, 0, 0] == 1.0 and c.score[0, 0, 0, 0] == 1.0
    # P12: all keys equal and no noise -> uniform attention, out = mean of values
    n = 12
    c = make_cache(rng, 1, 1, 1, 8, 20, n)
    c.K[...] = 0
    c.K[..., :n, :] = kn[0, 0, 0]
    out, dp, df = c.decode_step(q, kn, vn, n, 1.3, 0.35, ko.NOISE_NONE, debug=True)
    np.testing.assert_allclose(dp[0, 0, 0, :n + 1], 1 / (n + 1), rtol=1e-12)
    np.testing.assert_allclose(df[0, 0, 0, :n + 1], 1 / (n + 1), rtol=1e-12)
    np.testing.assert_allclose(out[0, 0, 0], as_f64(c.V[0, 0, 0, :n + 1]).mean(0), rtol=1e-6, atol=1e-7)


def test_alibi_bias_favours_recent_tokens():
    # MPT's ALiBi: the bias shrinks with distance, so with equal keys the
    # attention decays geometrically with (q_pos - pos): p_j ~ exp(-slope*dist)
    rng = np.random.default_rng(9)
    n = 10
    c = make_cache(rng, 1, 1, 1, 8, 16, n, pos=np.arange(n) * 3)
    c.K[...] = 0
    q = rand_vec(rng, (1, 1, 1, 8), ko.F32)
    zero = np.zeros((1, 1, 1, 8), np.float32)
    slope = 0.125
    q_pos = 40
    _, dp, _ = c.decode_step(q, zero, zero, q_pos, 1.0, 0.3, ko.NOISE_NONE, None,
                             np.array([slope], np.float32), debug=True)
    pos = np.append(np.arange(n) * 3, q_pos)
    ref = np.exp(-slope * (q_pos - pos))
    np.testing.assert_allclose(dp[0, 0, 0, :n + 1], ref / ref.sum(), rtol=1e-12)
    assert (np.diff(dp[0, 0, 0, :n + 1]) > 0).all()


def test_new_pos_mode_uses_slot_distances():
    # Sec. 4.4.2 "New Pos": the position bias sees positions within the reduced cache.  With
    # consecutive original positions ending at q_pos it coincides with "Org Pos"; with gaps
    # (evicted tokens) it is the geometric decay in slot distance.
    rng = np.random.default_rng(19)
    n, slope = 9, 0.25
    zero = np.zeros((1, 1, 1, 8), np.float32)
    q = rand_vec(rng, (1, 1, 1, 8), ko.F32)
    sl = np.array([slope], np.float32)
    c = make_cache(rng, 1, 1, 1, 8, 16, n, pos=np.arange(n))
    c2 = c.copy()
    _, p_org, _ = c.decode_step(q, zero, zero, n, 1.0, 0.3, ko.NOISE_NONE, None, sl, debug=True)
    _, p_new, _ = c2.decode_step(q, zero, zero, n, 1.0, 0.3, ko.NOISE_NONE, None, sl, debug=True, new_pos=True)
    np.testing.assert_allclose(p_org, p_new, rtol=1e-13)
    g = make_cache(rng, 1, 1, 1, 8, 16, n, pos=np.arange(n) * 5)
    g.K[...] = 0
    _, p_gap, _ = g.decode_step(q, zero, zero, 100, 1.0, 0.3, ko.NOISE_NONE, None, sl, debug=True, new_pos=True)
    ref = np.exp(-slope * (n - np.arange(n + 1)))        # slot distances n, n-1, ..., 0
    np.testing.assert_allclose(p_gap[0, 0, 0, :n + 1], ref / ref.sum(), rtol=1e-12)


def test_decode_is_invariant_under_slot_permutation():
    # P12: the cache is a set of (pos, K, V, f) entries; permuting the slots
    # (with their positions) changes neither out nor the increments per position
    rng = np.random.default_rng(10)
    n, d = 17, 16
    c = make_cache(rng, 1, 1, 1, d, 24, n, pos=np.arange(n) * 2 + 1)
    perm = rng.permutation(n)
    c2 = c.copy()
    c2.K[0, 0, 0, :n] = c.K[0, 0, 0, perm]
    c2.V[0, 0, 0, :n] = c.V[0, 0, 0, perm]
    c2.pos[0, 0, 0, :n] = c.pos[0, 0, 0, perm]
    q, kn, vn = (rand_vec(rng, (1, 1, 1, d), ko.F32) for _ in range(3))
    sd = np.array([77], np.uint64)
    o1, _, df1 = c.decode_step(q, kn, vn, 99, 1.5, 0.25, ko.NOISE_GUMBEL, sd, debug=True)
    o2, _, df2 = c2.decode_step(q, kn, vn, 99, 1.5, 0.25, ko.NOISE_GUMBEL, sd, debug=True)
    np.testing.assert_allclose(o1, o2, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(df1[0, 0, 0, perm], df2[0, 0, 0, :n], rtol=1e-12)
    np.testing.assert_allclose(df1[0, 0, 0, n], df2[0, 0, 0, n], rtol=1e-12)


# ----------------------------------------------------------------------------
# Prompt-phase scoring (Sec. 3.4, Alg. 1 prompt branch)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [ko.F32, ko.BF16])
@pytest.mark.parametrize("noise", [ko.NOISE_GUMBEL, ko.NOISE_NONE])
def test_prefill_matches_numpy(dtype, noise):
    rng = np.random.default_rng(11)
    L, B, H, d, n, cap = 1, 2, 2, 16, 33, 40
    c = make_cache(rng, L, B, H, d, cap, n, dtype)
    c.pos[...] = -7
    c.len[...] = 0
    Q = rand_vec(rng, (L, B, H, n, d), dtype)
    seeds = np.array([1234, 99], np.uint64)
    slopes = np.array([0.0, 0.0625], np.float32)
    tau, scale = 1.25, 0.25
    c.prefill_score(Q, n, tau, scale, noise, seeds, slopes)
    assert (c.len == n).all() and (c.pos[..., :n] == np.arange(n)).all()
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    for b, h in itertools.product(range(B), range(H)):
        x = np.float64(np.float32(scale)) * (as_f64(Q[0, b, h]) @ as_f64(c.K[0, b, h, :n]).T)
        x = x - float(slopes[h]) * (i - j)
        z = zeta_matrix(noise, int(seeds[b]), 0, h, range(n), range(n))
        y = (x + z) / np.float64(np.float32(tau))
        y = np.where(j <= i, y, -np.inf)                  # causal: token i sees keys 0..i
        zmat = scipy.special.softmax(y, axis=1)
        f_ref = zmat.sum(axis=0)                          # column sums
        np.testing.assert_allclose(c.score[0, b, h, :n], f_ref, rtol=3e-7)
        assert abs(c.score[0, b, h, :n].astype(np.float64).sum() - n) < 1e-4   # P1: n rows, each sums to 1
        assert c.score[0, b, h, n - 1] <= 1.0            # the last key is seen by one row only


def test_prefill_first_row_and_uniform_case():
    # one prompt token: f = [1].  Equal keys, no noise: row i spreads 1/(i+1)
    # over its i+1 keys, so f[j] = sum_{i>=j} 1/(i+1) = H_n - H_j (harmonic numbers)
    rng = np.random.default_rng(12)
    c = make_cache(rng, 1, 1, 1, 8, 4, 1)
    Q = rand_vec(rng, (1, 1, 1, 1, 8), ko.F32)
    c.prefill_score(Q, 1, 1.0, 0.3, ko.NOISE_GUMBEL, np.array([1], np.uint64))
    assert c.score[0, 0, 0, 0] == 1.0
    n = 20
    c = make_cache(rng, 1, 1, 1, 8, n, n)
    c.K[0, 0, 0, :, :] = c.K[0, 0, 0, 0, :]
    Q = rand_vec(rng, (1, 1, 1, n, 8), ko.F32)
    c.prefill_score(Q, n, 1.0, 0.3, ko.NOISE_NONE)
    harm = np.cumsum(1.0 / np.arange(1, n + 1))
    ref = harm[-1] - np.concatenate([[0.0], harm[:-1]])
    np.testing.assert_allclose(c.score[0, 0, 0], ref, rtol=3e-7)


def test_prefill_of_a_padded_batch_scores_every_prompt_by_itself():
    # a batch of prompts of different lengths, padded at the end to n rows (the paper's performance runs
    # make all prompts equally long; a serving batch is not): every sequence's f is the numpy column sum
    # over ITS rows only -- the padding rows are neither queries nor keys -- whatever the padding holds;
    # equal lengths reproduce the plain call
    rng = np.random.default_rng(13)
    L, B, H, d, n, cap = 2, 3, 2, 16, 29, 32
    n_seq = np.array([29, 1, 12])
    c = make_cache(rng, L, B, H, d, cap, n, ko.BF16)
    Q = rand_vec(rng, (L, B, H, n, d), ko.BF16)
    seeds = np.array([5, 6, 7], np.uint64)
    slopes = np.array([0.0, 0.25], np.float32)
    tau, scale = 1.0, 0.25
    plain = c.copy()
    plain.prefill_score(Q, n, tau, scale, ko.NOISE_GUMBEL, seeds, slopes)
    same = c.copy()
    same.prefill_score(Q, n, tau, scale, ko.NOISE_GUMBEL, seeds, slopes, n_seq=[n] * B)
    np.testing.assert_array_equal(same.score, plain.score)
    c.score[...] = -3.0
    c.pos[...] = -7
    r1 = c.copy()
    r1.prefill_score(Q, n, tau, scale, ko.NOISE_GUMBEL, seeds, slopes, n_seq=n_seq)
    c2, Q2 = c.copy(), Q.copy()
    for b in range(B):     # other padding
        c2.K[:, b, :, n_seq[b]:] = rand_vec(rng, c2.K[:, b, :, n_seq[b]:].shape, ko.BF16)
        Q2[:, b, :, n_seq[b]:] = rand_vec(rng, Q2[:, b, :, n_seq[b]:].shape, ko.BF16)
    r2 = c2.copy()
    r2.prefill_score(Q2, n, tau, scale, ko.NOISE_GUMBEL, seeds, slopes, n_seq=n_seq)
    np.testing.assert_array_equal(r1.score, r2.score)
    for l, b, h in itertools.product(range(L), range(B), range(H)):
        nb = int(n_seq[b])
        assert r1.len[l, b, h] == nb
        assert (r1.pos[l, b, h, :nb] == np.arange(nb)).all() and (r1.pos[l, b, h, nb:] == -7).all()
        assert (r1.score[l, b, h, nb:] == -3.0).all()                     # beyond the prompt: untouched
        i, j = np.meshgrid(np.arange(nb), np.arange(nb), indexing="ij")
        x = np.float64(np.float32(scale)) * (as_f64(Q[l, b, h, :nb]) @ as_f64(c.K[l, b, h, :nb]).T)
        x = x - float(slopes[h]) * (i - j)
        y = (x + zeta_matrix(ko.NOISE_GUMBEL, int(seeds[b]), l, h, range(nb), range(nb))) / tau
        f_ref = scipy.special.softmax(np.where(j <= i, y, -np.inf), axis=1).sum(axis=0)
        np.testing.assert_allclose(r1.score[l, b, h, :nb], f_ref, rtol=3e-7)
        assert abs(r1.score[l, b, h, :nb].astype(np.float64).sum() - nb) < 1e-4


# ----------------------------------------------------------------------------
# "Shared" score function (Sec. 4.4.1): one f for all layers, accumulated over
# layers and decoding steps
# ----------------------------------------------------------------------------
def test_shared_score_is_the_sum_over_layers():
    rng = np.random.default_rng(21)
    L, B, H, d, n, cap = 3, 2, 2, 16, 21, 30
    c = make_cache(rng, L, B, H, d, cap, n, ko.BF16)
    Q = rand_vec(rng, (L, B, H, n, d), ko.BF16)
    seeds = np.array([7, 8], np.uint64)
    slopes = np.array([0.0, 0.125], np.float32)
    tau, scale = 1.5, 0.25
    c.prefill_score(Q, n, tau, scale, ko.NOISE_GUMBEL, seeds, slopes, shared=True)
    # independent evaluation: each layer's causal column sums with numpy/scipy, added up
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    f_ref = np.zeros((B, H, n))
    for l, b, h in itertools.product(range(L), range(B), range(H)):
        x = np.float64(np.float32(scale)) * (as_f64(Q[l, b, h]) @ as_f64(c.K[l, b, h, :n]).T)
        x = x - float(slopes[h]) * (i - j)
        z = zeta_matrix(ko.NOISE_GUMBEL, int(seeds[b]), l, h, range(n), range(n))
        y = np.where(j <= i, (x + z) / np.float64(np.float32(tau)), -np.inf)
        f_ref[b, h] += scipy.special.softmax(y, axis=1).sum(axis=0)
    for l in range(L):
        np.testing.assert_allclose(c.score[l, ..., :n], f_ref, rtol=3e-7)
        np.testing.assert_array_equal(c.score[l], c.score[0])          # one function: all copies equal
    assert abs(c.score[0, ..., :n].astype(np.float64).sum() - L * B * H * n) < 1e-3

    # a decode step adds every layer's increment to the one score
    before = c.copy()
    q, kn, vn = (rand_vec(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    q_pos, tau = n, 1.75
    out, dp, df = c.decode_step(q, kn, vn, q_pos, tau, scale, ko.NOISE_GUMBEL, seeds, slopes, debug=True, shared=True)
    m = n + 1
    inc = np.zeros((B, H, m))
    for l, b, h in itertools.product(range(L), range(B), range(H)):
        o_ref, p_ref, df_ref = numpy_decode(c, (l, b, h), q[l, b, h], q_pos, tau, scale, ko.NOISE_GUMBEL,
                                            int(seeds[b]), float(slopes[h]))
        inc[b, h] += df_ref
        np.testing.assert_allclose(out[l, b, h], o_ref.astype(np.float32), rtol=2e-7, atol=1e-30)  # attention unaffected
    old = np.concatenate([before.score[0, ..., :n].astype(np.float64), np.zeros((B, H, 1))], axis=-1)
    for l in range(L):
        np.testing.assert_allclose(c.score[l, ..., :m], (old + inc), rtol=2e-7)
        np.testing.assert_array_equal(c.score[l], c.score[0])
    assert abs(c.score[0, ..., :m].astype(np.float64).sum() - before.score[0, ..., :n].astype(np.float64).sum()
               - L * B * H) < 1e-4                                       # every layer added a probability vector
    # the same scores everywhere => the same evictions everywhere
    kept = c.select_evict(12, 4)
    for l in range(L):
        np.testing.assert_array_equal(kept[l], kept[0])
        np.testing.assert_array_equal(c.pos[l], c.pos[0])


def test_shared_score_special_cases():
    rng = np.random.default_rng(22)
    B, H, d, n, cap = 1, 2, 8, 12, 16
    seeds = np.array([3], np.uint64)
    # one layer: shared and per-layer are the same thing, bit for bit
    a = make_cache(rng, 1, B, H, d, cap, n)
    b_ = a.copy()
    Q = rand_vec(rng, (1, B, H, n, d), ko.F32)
    a.prefill_score(Q, n, 1.0, 0.3, ko.NOISE_GUMBEL, seeds)
    b_.prefill_score(Q, n, 1.0, 0.3, ko.NOISE_GUMBEL, seeds, shared=True)
    np.testing.assert_array_equal(a.score, b_.score)
    q, kn, vn = (rand_vec(rng, (1, B, H, d), ko.F32) for _ in range(3))
    a.decode_step(q, kn, vn, n, 1.2, 0.3, ko.NOISE_GUMBEL, seeds)
    b_.decode_step(q, kn, vn, n, 1.2, 0.3, ko.NOISE_GUMBEL, seeds, shared=True)
    np.testing.assert_array_equal(a.score, b_.score)
    # L identical layers without noise: the shared score is L times the single layer's
    L = 4
    one = make_cache(rng, 1, B, H, d, cap, n)
    many = ko.OracleCache(L, B, H, d, cap, ko.F32)
    for l in range(L):
        many.K[l], many.V[l] = one.K[0], one.V[0]
    Q1 = rand_vec(rng, (1, B, H, n, d), ko.F32)
    one.prefill_score(Q1, n, 1.0, 0.3, ko.NOISE_NONE)
    many.prefill_score(np.repeat(Q1, L, axis=0), n, 1.0, 0.3, ko.NOISE_NONE, shared=True)
    np.testing.assert_allclose(many.score[2, ..., :n], L * one.score[0, ..., :n].astype(np.float64), rtol=2e-7)
    np.testing.assert_array_equal(many.select_evict(8, 3)[1], one.select_evict(8, 3)[0])
    # layers that do not hold the same tokens cannot share a score
    many.pos[1, 0, 0, 2] += 1
    with pytest.raises(ValueError):
        many.decode_step(*(np.repeat(x, L, axis=0) for x in (q, kn, vn)), n, 1.0, 0.3, ko.NOISE_NONE, shared=True)


# ----------------------------------------------------------------------------
# Grouped-query attention (Sec. 6): G query heads per cached head
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("G", [2, 4])
def test_grouped_queries_equal_replicated_kv_heads(G):
    """A cache whose head serves G query heads computes what a one-query-per-head cache with that head's
    K/V replicated G times computes (attention outputs, per-head increments); its score is the sum of the
    replicas' scores.  The replicated run is the already pinned path, so head numbering, slopes and noise
    streams of the grouped run are pinned through it."""
    rng = np.random.default_rng(31 + G)
    L, B, H, d, n, cap = 2, 2, 2, 16, 19, 26
    grp = make_cache(rng, L, B, H, d, cap, n, ko.BF16)
    rep = ko.OracleCache(L, B, H * G, d, cap, ko.BF16)
    for h in range(H * G):
        rep.K[:, :, h], rep.V[:, :, h] = grp.K[:, :, h // G], grp.V[:, :, h // G]
    Q = rand_vec(rng, (L, B, H * G, n, d), ko.BF16)
    seeds = np.array([41, 42], np.uint64)
    slopes = (0.5 ** np.arange(1, H * G + 1)).astype(np.float32)
    grp.prefill_score(Q, n, 1.25, 0.25, ko.NOISE_GUMBEL, seeds, slopes, q_per_kv=G)
    rep.prefill_score(Q, n, 1.25, 0.25, ko.NOISE_GUMBEL, seeds, slopes)
    f_sum = rep.score.astype(np.float64).reshape(L, B, H, G, cap).sum(axis=3)
    np.testing.assert_allclose(grp.score[..., :n], f_sum[..., :n], rtol=3e-7)
    assert abs(grp.score[..., :n].astype(np.float64).sum() - L * B * H * G * n) < 1e-3
    assert (grp.len == n).all() and (grp.pos[..., :n] == np.arange(n)).all()

    rep.score[...] = np.repeat(grp.score, G, axis=2) / G          # any common starting point will do
    start = grp.score.copy()
    q = rand_vec(rng, (L, B, H * G, d), ko.BF16)
    kn, vn = (rand_vec(rng, (L, B, H, d), ko.BF16) for _ in range(2))
    out_g, p_g, df_g = grp.decode_step(q, kn, vn, n, 1.5, 0.25, ko.NOISE_GUMBEL, seeds, slopes, debug=True, q_per_kv=G)
    out_r, p_r, df_r = rep.decode_step(q, np.repeat(kn, G, axis=2), np.repeat(vn, G, axis=2), n, 1.5, 0.25,
                                       ko.NOISE_GUMBEL, seeds, slopes, debug=True)
    np.testing.assert_array_equal(out_g, out_r)
    np.testing.assert_array_equal(p_g, p_r)
    np.testing.assert_array_equal(df_g, df_r)
    m = n + 1
    inc = df_r.reshape(L, B, H, G, cap).sum(axis=3)
    want = np.concatenate([start[..., :n].astype(np.float64), np.zeros((L, B, H, 1))], axis=-1) + inc[..., :m]
    np.testing.assert_allclose(grp.score[..., :m], want, rtol=2e-7)
    assert (grp.len == m).all() and (grp.pos[..., n] == n).all()
    assert (grp.K[..., n, :] == kn).all() and (grp.V[..., n, :] == vn).all()


def test_grouped_queries_special_cases():
    rng = np.random.default_rng(33)
    B, H, d, n, cap, G = 1, 2, 8, 10, 12, 4
    # identical query heads, no adjustment: every head attends alike, the score gains G times one head's increment
    one = make_cache(rng, 1, B, H, d, cap, n)
    many = one.copy()
    q1 = rand_vec(rng, (1, B, H, d), ko.F32)
    kn, vn = (rand_vec(rng, (1, B, H, d), ko.F32) for _ in range(2))
    o1, _, df1 = one.decode_step(q1, kn, vn, n, 1.0, 0.3, ko.NOISE_NONE, debug=True)
    oG, _, dfG = many.decode_step(np.repeat(q1, G, axis=2), kn, vn, n, 1.0, 0.3, ko.NOISE_NONE, debug=True, q_per_kv=G)
    np.testing.assert_array_equal(oG, np.repeat(o1, G, axis=2))
    np.testing.assert_allclose(many.score[..., :n + 1], G * one.score[..., :n + 1].astype(np.float64), rtol=2e-7)
    # each head draws its own noise: with the adjustment on, identical queries no longer score alike
    noisy = make_cache(rng, 1, B, H, d, cap, n)
    _, _, dfn = noisy.decode_step(np.repeat(q1, G, axis=2), kn, vn, n, 1.0, 0.3, ko.NOISE_GUMBEL,
                                  np.array([9], np.uint64), debug=True, q_per_kv=G)
    assert np.abs(dfn[0, 0, 0, :n + 1] - dfn[0, 0, 1, :n + 1]).max() > 1e-3
    assert abs(dfn[0, 0, :, :n + 1].sum() - H * G) < 1e-9          # a probability vector per query head


# ----------------------------------------------------------------------------
# A batch whose sequences are at different steps: per-sequence position and temperature
# ----------------------------------------------------------------------------
def test_per_sequence_position_and_temperature_equal_separate_runs():
    rng = np.random.default_rng(41)
    L, B, H, d, cap = 2, 3, 2, 16, 24
    lens = rng.integers(8, 20, (1, B, 1)).repeat(L, 0).repeat(H, 2).astype(np.int32)
    c = make_cache(rng, L, B, H, d, cap, 20, ko.BF16)
    c.len[...] = lens
    c.score[...] = rng.random(c.score.shape).astype(np.float32)
    q, kn, vn = (rand_vec(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    seeds = np.array([5, 6, 7], np.uint64)
    slopes = np.array([0.25, 0.03], np.float32)
    q_pos = np.array([40, 25, 33], np.int32)
    taus = np.array([1.25, 1.0, 1.9], np.float32)
    whole = c.copy()
    out = whole.decode_step(q, kn, vn, 0, 1.0, 0.25, ko.NOISE_GUMBEL, seeds, slopes, q_pos_seq=q_pos, tau_seq=taus)
    for b in range(B):                                   # each sequence alone, through the scalar arguments
        one = ko.OracleCache(L, 1, H, d, cap, ko.BF16)
        for nm in ("K", "V", "score", "pos", "len"):
            getattr(one, nm)[...] = getattr(c, nm)[:, b:b + 1]
        o = one.decode_step(q[:, b:b + 1], kn[:, b:b + 1], vn[:, b:b + 1], int(q_pos[b]), float(taus[b]), 0.25,
                            ko.NOISE_GUMBEL, seeds[b:b + 1], slopes)
        np.testing.assert_array_equal(out[:, b:b + 1], o)
        for nm in ("K", "V", "score", "pos", "len"):
            np.testing.assert_array_equal(getattr(whole, nm)[:, b:b + 1], getattr(one, nm))
    assert (whole.pos[0, np.arange(B), 0, lens[0, :, 0]] == q_pos).all()   # each appended token carries its own position
    with pytest.raises(ValueError):
        c.copy().decode_step(q, kn, vn, 0, 1.0, 0.25, ko.NOISE_GUMBEL, seeds, slopes, tau_seq=np.array([1.0, 0.0, 1.0]))


# ----------------------------------------------------------------------------
# Selection + compaction (Alg. 1: S_w, S_key = argmax_(k-w) f[:-w], S_k)
# ----------------------------------------------------------------------------
def brute_force_keep(f, n, k, w):
    """All subsets of the candidates: maximal score sum, then lexicographically
    smallest index tuple (= prefers lower slots among equal scores)."""
    ncand, nkey = n - w, k - w
    best, best_sum = None, None
    for comb in itertools.combinations(range(ncand), nkey):
        s = math.fsum(float(f[i]) for i in comb)
        if best is None or s > best_sum or (s == best_sum and comb < best):
            best, best_sum = comb, s
    return list(best) + list(range(n - w, n))


def test_select_matches_brute_force_with_ties():
    rng = np.random.default_rng(13)
    for trial in range(60):
        n = int(rng.integers(5, 15))
        k = int(rng.integers(1, n))
        w = int(rng.integers(0, k + 1))
        if n - w > 12:
            continue
        c = make_cache(rng, 1, 1, 1, 4, n, n)
        # few distinct dyadic values -> many exact ties, exactly summable
        c.score[0, 0, 0, :n] = rng.integers(0, 4, n).astype(np.float32) * 0.25
        before = c.copy()
        kept = c.select_evict(k, w)
        ref = brute_force_keep(before.score[0, 0, 0], n, k, w)
        assert kept[0, 0, 0].tolist() == ref, (n, k, w, before.score[0, 0, 0].tolist())
        # P3: survivors are bit-identical copies, in order
        assert c.len[0, 0, 0] == k
        np.testing.assert_array_equal(c.K[0, 0, 0, :k], before.K[0, 0, 0, ref])
        np.testing.assert_array_equal(c.V[0, 0, 0, :k], before.V[0, 0, 0, ref])
        np.testing.assert_array_equal(c.score[0, 0, 0, :k], before.score[0, 0, 0, ref])
        np.testing.assert_array_equal(c.pos[0, 0, 0, :k], before.pos[0, 0, 0, ref])


def test_select_equals_stable_sort_topk_and_invariants():
    rng = np.random.default_rng(14)
    L, B, H, d, n, k, w = 2, 2, 2, 8, 300, 120, 24
    c = make_cache(rng, L, B, H, d, n, n, ko.BF16)
    c.score[...] = rng.random((L, B, H, n)).astype(np.float32)
    c.score[..., 50:90] = 0.5                    # a block of ties straddling the threshold region
    c.len[0, 0, 0] = 100                         # a unit below the budget is left alone
    before = c.copy()
    kept = c.select_evict(k, w)
    for l, b, h in itertools.product(range(L), range(B), range(H)):
        n_u = int(before.len[l, b, h])
        if n_u <= k:
            assert c.len[l, b, h] == n_u
            assert kept[l, b, h, :n_u].tolist() == list(range(n_u)) and (kept[l, b, h, n_u:] == -1).all()
            np.testing.assert_array_equal(c.K[l, b, h], before.K[l, b, h])
            continue
        f = before.score[l, b, h, :n_u - w]
        order = np.argsort(-f.astype(np.float64), kind="stable")       # stable: lower slot first
        ref = sorted(order[:k - w].tolist()) + list(range(n_u - w, n_u))
        assert kept[l, b, h].tolist() == ref
        assert c.len[l, b, h] == k
        pos = c.pos[l, b, h, :k]
        assert (np.diff(pos) > 0).all()                                 # order preserved
        assert set(range(n_u - w, n_u)) <= set(pos.tolist())            # recent window kept
        # nothing evicted outscores anything kept among the candidates
        evicted = sorted(set(range(n_u - w)) - set(ref))
        assert before.score[l, b, h, evicted].max() <= before.score[l, b, h, ref[:k - w]].min()


def test_decode_shape_drops_the_single_minimum():
    # P10: with len = k+1 exactly one token leaves: the candidate with the
    # smallest score, the highest slot among equal minima
    rng = np.random.default_rng(15)
    k, w = 40, 8
    n = k + 1
    c = make_cache(rng, 1, 1, 4, 4, n, n)
    c.score[...] = rng.random((1, 1, 4, n)).astype(np.float32) + 1
    c.score[0, 0, 0, [3, 17, 30]] = 0.5         # three equal minima -> slot 30 goes
    c.score[0, 0, 1, 36] = 0.0                  # minimum inside the window is protected
    c.score[0, 0, 2, 0] = 0.25                  # oldest token
    c.score[0, 0, 3, n - w - 1] = 0.25          # last candidate
    before = c.copy()
    kept = c.select_evict(k, w)
    drop = [30, int(np.argmin(before.score[0, 0, 1, :n - w])), 0, n - w - 1]
    for h in range(4):
        assert kept[0, 0, h].tolist() == [i for i in range(n) if i != drop[h]]


def test_layer_and_head_offsets_reproduce_the_units_of_the_full_cache():
    """A cache that holds one layer / one head of a model (layer0, head0) computes exactly what the full
    cache computes for that unit: the offsets enter the noise key and the slope index, nothing else."""
    rng = np.random.default_rng(61)
    L, B, H, d, n, cap = 3, 2, 4, 16, 21, 24
    full = make_cache(rng, L, B, H, d, cap, n, ko.BF16)
    Q = rand_vec(rng, (L, B, H, n, d), ko.BF16)
    q, kn, vn = (rand_vec(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    seeds = np.array([5, 6], np.uint64)
    slopes = np.array([0.5, 0.25, 0.125, 0.0625], np.float32)
    ref = full.copy()
    ref.prefill_score(Q, n, 1.0, 0.25, ko.NOISE_GUMBEL, seeds, slopes)
    ref_pre = ref.score.copy()
    out_ref = ref.decode_step(q, kn, vn, n, 1.25, 0.25, ko.NOISE_GUMBEL, seeds, slopes)
    for l, b, h in [(0, 0, 0), (1, 1, 2), (2, 0, 3)]:
        one = ko.OracleCache(1, 1, 1, d, cap, ko.BF16, layer0=l, head0=h)
        one.K[0, 0, 0], one.V[0, 0, 0] = full.K[l, b, h], full.V[l, b, h]
        one.prefill_score(np.ascontiguousarray(Q[l:l + 1, b:b + 1, h:h + 1]), n, 1.0, 0.25, ko.NOISE_GUMBEL,
                          seeds[b:b + 1], slopes)
        np.testing.assert_array_equal(one.score[0, 0, 0], ref_pre[l, b, h])
        o = one.decode_step(q[l:l + 1, b:b + 1, h:h + 1], kn[l:l + 1, b:b + 1, h:h + 1], vn[l:l + 1, b:b + 1, h:h + 1],
                            n, 1.25, 0.25, ko.NOISE_GUMBEL, seeds[b:b + 1], slopes)
        np.testing.assert_array_equal(o[0, 0, 0], out_ref[l, b, h])
        np.testing.assert_array_equal(one.score[0, 0, 0], ref.score[l, b, h])
    # the offsets matter: the same data under another head index draws other noise
    other = ko.OracleCache(1, 1, 1, d, cap, ko.BF16, layer0=1, head0=1)
    other.K[0, 0, 0], other.V[0, 0, 0] = full.K[1, 1, 2], full.V[1, 1, 2]
    other.prefill_score(np.ascontiguousarray(Q[1:2, 1:2, 2:3]), n, 1.0, 0.25, ko.NOISE_GUMBEL, seeds[1:2], None)
    assert (other.score[0, 0, 0, :n] != ref_pre[1, 1, 2, :n]).mean() > 0.9


def test_hand_worked_window_plus_key_tokens_scenario():
    """Fig. 2(d): a recent window of 2 plus 2 key tokens over three consecutive iterations.  The expected
    retained positions and scores were worked out by hand (tests/golden/fig2d_scenario.txt): the two key
    tokens persist while the window slides."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "fig2d_scenario.txt")) if l.strip() and not l.startswith("#")]
    k, w, d = 4, 2, 4
    c = ko.OracleCache(1, 1, 1, d, k + 1, ko.F32)
    assert rows[0][0] == "start"
    c.pos[0, 0, 0, :k] = [int(v) for v in rows[0][1:1 + k]]
    c.score[0, 0, 0, :k] = [int(v) / 10.0 for v in rows[0][1 + k:1 + 2 * k]]
    c.len[...] = k
    zero = np.zeros((1, 1, 1, d), np.float32)
    q = np.ones((1, 1, 1, d), np.float32)
    for step, row in enumerate(rows[1:]):
        new_pos = k + step
        out = c.decode_step(q, zero, np.full((1, 1, 1, d), float(new_pos), np.float32), new_pos, 1.0 + 0.5 * step, 0.5,
                            ko.NOISE_NONE)
        assert int(c.len[0, 0, 0]) == k + 1
        c.select_evict(k, w)
        assert int(c.len[0, 0, 0]) == k
        assert c.pos[0, 0, 0, :k].tolist() == [int(v) for v in row[1:1 + k]], row[0]
        np.testing.assert_allclose(c.score[0, 0, 0, :k], [int(v) / 10.0 for v in row[1 + k:1 + 2 * k]], rtol=3e-7)
        # equal logits: the attention output is the plain mean of the 5 cached value rows
        np.testing.assert_allclose(out[0, 0, 0], np.full(d, int(row[1 + 2 * k]) / 10.0), rtol=3e-7)


def test_gumbel_adjustment_spreads_the_expected_score():
    """Eq. 9-10: the expectation (over the logit adjustment) of the normalised, Gumbel-adjusted logits is more
    uniform than the plain softmax: H(E[z_Gumbel]) > H(E[z]).  Averaged here over 600 query positions, i.e.
    600 independent draws of the adjustment on the same logits; the new token's key equals an old one, so
    the logits do not depend on the query position."""
    rng = np.random.default_rng(77)
    H_, d, n = 2, 16, 24
    base = make_cache(rng, 1, 1, H_, d, n + 1, n)
    base.K[..., :n, :] *= 2.0                      # a peaked softmax
    q = rng.standard_normal((1, 1, H_, d)).astype(np.float32)
    kn, vn = base.K[..., 0, :].copy(), base.V[..., 0, :].copy()
    seeds = np.array([31337], np.uint64)

    def increments(noise, q_pos):
        c = base.copy()
        c.score[...] = 0.0
        c.decode_step(q, kn, vn, q_pos, 1.0, 0.25, noise, seeds)
        return c.score[0, 0, :, : n + 1].astype(np.float64)

    entropy = lambda p: float(-(p * np.log(p)).sum())
    plain = increments(ko.NOISE_NONE, 100)
    mean_g = np.mean([increments(ko.NOISE_GUMBEL, 100 + t) for t in range(600)], axis=0)
    for h in range(H_):
        assert abs(mean_g[h].sum() - 1.0) < 1e-5
        assert entropy(mean_g[h]) > entropy(plain[h]) + 0.05, (h, entropy(mean_g[h]), entropy(plain[h]))
        # ... while the ranking by expected score still follows the logits (the adjustment regularises,
        # it does not reorder): the top token stays on top
        assert int(np.argmax(mean_g[h])) == int(np.argmax(plain[h]))


def test_select_boundaries():
    rng = np.random.default_rng(16)
    n, k = 20, 8
    for w in (0, k):                             # pure top-k ; pure recent window
        c = make_cache(rng, 1, 1, 1, 4, n, n)
        c.score[...] = rng.random((1, 1, 1, n)).astype(np.float32)
        f = c.score[0, 0, 0].copy()
        kept = c.select_evict(k, w)[0, 0, 0].tolist()
        if w == 0:
            assert kept == sorted(np.argsort(-f, kind="stable")[:k].tolist())
        else:
            assert kept == list(range(n - k, n))
    c = make_cache(rng, 1, 1, 1, 4, n, n)
    with pytest.raises(ValueError):
        c.select_evict(8, 9)                     # w > k
    with pytest.raises(ValueError):
        c.select_evict(0, 0)                     # k < 1


# ----------------------------------------------------------------------------
# Whole algorithm on the tiny configuration: invariants of every step
# ----------------------------------------------------------------------------
def test_tiny_config_end_to_end_invariants():
    import kf_workloads as kw
    wl = kw.CONFIGS["tiny"]
    Q, K, V = kw.prompt_layer(wl, 0)
    c = ko.OracleCache(wl.L, wl.B, wl.H, wl.d, wl.n, ko.F32)
    c.K[0, :, :, :wl.n] = kw.to_oracle(K)
    c.V[0, :, :, :wl.n] = kw.to_oracle(V)
    seeds = kw.noise_seeds(wl)
    c.prefill_score(kw.to_oracle(Q)[None], wl.n, ko.tau(0, wl.T), wl.scale, ko.NOISE_GUMBEL, seeds)
    assert abs(c.score.astype(np.float64).sum() - wl.units * wl.n) < 1e-3
    c.select_evict(wl.k, wl.w)
    assert (c.len == wl.k).all()
    assert (c.pos[..., wl.k - wl.w:wl.k] == np.arange(wl.n - wl.w, wl.n)).all()
    total = c.score[..., :wl.k].astype(np.float64).sum()
    for t in range(1, wl.T + 1):
        q, kn, vn = (kw.to_oracle(a) for a in kw.decode_inputs(wl, t))
        q_pos = wl.n + t - 1
        out = c.decode_step(q, kn, vn, q_pos, ko.tau(t, wl.T), wl.scale, ko.NOISE_GUMBEL, seeds)
        assert (c.len == wl.k + 1).all() and np.isfinite(out).all()
        now = c.score[..., :wl.k + 1].astype(np.float64).sum()
        assert abs(now - total - wl.units) < 1e-4                  # each unit gained exactly 1
        c.select_evict(wl.k, wl.w)
        assert (c.len == wl.k).all()                               # cache never exceeds k after eviction
        pos = c.pos[..., :wl.k]
        assert (np.diff(pos, axis=-1) > 0).all()
        assert (pos[..., wl.k - wl.w:] == np.arange(q_pos - wl.w + 1, q_pos + 1)).all()   # w most recent
        total = c.score[..., :wl.k].astype(np.float64).sum()


# ----------------------------------------------------------------------------
# Property test: the selection against numpy's stable sort on random shapes with ties
# ----------------------------------------------------------------------------
def test_select_random_shapes_against_stable_sort():
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=150, deadline=None)
    @given(st.integers(1, 40), st.integers(0, 40), st.integers(0, 40), st.integers(0, 2 ** 31 - 1), st.integers(1, 6))
    def check(n, k_raw, w_raw, seed, levels):
        k = max(1, min(k_raw, n + 3))
        w = min(w_raw, k)
        rng = np.random.default_rng(seed)
        c = make_cache(rng, 1, 1, 1, 4, n + 4, n)
        f = rng.integers(0, levels, n).astype(np.float32) * 0.5 - 1.0     # few distinct values: many ties, negatives
        c.score[0, 0, 0, :n] = f
        c.pos[0, 0, 0, :n] = np.cumsum(rng.integers(1, 4, n))
        before = c.copy()
        kept = c.select_evict(k, w)[0, 0, 0]
        if n <= k:
            assert c.len[0, 0, 0] == n and (kept[:n] == np.arange(n)).all() and (kept[n:] == -1).all()
            return
        wn = min(w, n)
        cand = n - wn
        # (k-w) largest of the candidates; among equal scores the lower slot: a stable sort of -f does exactly that
        order = np.argsort(-f[:cand], kind="stable")[: k - wn]
        want = np.sort(np.concatenate([order, np.arange(cand, n)])).astype(np.int32)
        np.testing.assert_array_equal(kept, want)
        assert c.len[0, 0, 0] == k
        np.testing.assert_array_equal(c.pos[0, 0, 0, :k], before.pos[0, 0, 0, want])
        np.testing.assert_array_equal(c.score[0, 0, 0, :k], before.score[0, 0, 0, want])
        np.testing.assert_array_equal(c.K[0, 0, 0, :k], before.K[0, 0, 0, want])

    check()


# ----------------------------------------------------------------------------
# Beam search: one cache per beam (Sec. 4 uses 4 beams everywhere)
# ----------------------------------------------------------------------------
def test_beam_fork_copies_the_parent_state():
    rng = np.random.default_rng(31)
    L, B, H, d, cap = 2, 4, 2, 16, 12
    c = make_cache(rng, L, B, H, d, cap, cap, ko.BF16)
    c.score[...] = rng.random(c.score.shape).astype(np.float32)
    c.pos[...] = rng.integers(0, 1000, c.pos.shape)
    c.len[...] = rng.integers(1, cap - 1, c.len.shape)
    before = c.copy()
    same = c.copy()
    same.beam_fork([0, 1, 2, 3])                       # every beam continues itself: nothing moves
    for nm in ("K", "V", "score", "pos", "len"):
        np.testing.assert_array_equal(getattr(same, nm), getattr(before, nm))
    c.beam_fork([0, 0, 2, 0])                          # beams 1 and 3 died; beam 0 has three continuations
    for l, h in itertools.product(range(L), range(H)):
        m = int(before.len[l, 0, h])
        for b in (1, 3):
            assert c.len[l, b, h] == m
            for nm in ("K", "V", "score", "pos"):
                np.testing.assert_array_equal(getattr(c, nm)[l, b, h, :m], getattr(before, nm)[l, 0, h, :m])
                # beyond the parent's length the row keeps what it had
                np.testing.assert_array_equal(getattr(c, nm)[l, b, h, m:], getattr(before, nm)[l, b, h, m:])
        for b in (0, 2):
            for nm in ("K", "V", "score", "pos"):
                np.testing.assert_array_equal(getattr(c, nm)[l, b, h], getattr(before, nm)[l, b, h])
    # a forked beam that is fed what its parent is fed (and draws its noise) answers like its parent
    q = rand_vec(rng, (L, 1, H, d), ko.BF16).repeat(B, axis=1)
    kn = rand_vec(rng, (L, 1, H, d), ko.BF16).repeat(B, axis=1)
    vn = rand_vec(rng, (L, 1, H, d), ko.BF16).repeat(B, axis=1)
    seeds = np.array([5, 5, 5, 5], np.uint64)
    out = c.decode_step(q, kn, vn, 40, 1.5, 0.25, ko.NOISE_GUMBEL, seeds)
    np.testing.assert_array_equal(out[:, 1], out[:, 0])
    np.testing.assert_array_equal(out[:, 3], out[:, 0])
    assert not np.array_equal(out[:, 2], out[:, 0])
    with pytest.raises(ValueError):
        c.beam_fork([1, 0, 2, 3])                      # 0 and 1 swap: neither continues itself
    with pytest.raises(ValueError):
        c.beam_fork([0, 4, 2, 3])


# ----------------------------------------------------------------------------
# Element types: the oracle reads fp32, bf16 and IEEE half; all arithmetic is in double
# ----------------------------------------------------------------------------
def test_sixteen_bit_inputs_are_read_exactly():
    # every bf16 / half value is an fp32 value: a cache holding the same numbers as fp32 must give the
    # same bits at every output (prompt scores, attention output, score increments, survivors)
    rng = np.random.default_rng(41)
    L, B, H, d, n, cap = 1, 2, 2, 16, 19, 24
    for dt in (ko.BF16, ko.F16):
        vals = rng.standard_normal((L, B, H, cap, d)).astype(np.float32)
        vals[0, 0, 0, 0, :4] = [0.0, -0.0, 6.1e-5, 65504.0 if dt == ko.F16 else 3.0e38]   # zero, smallest normal half, largest
        vals[0, 0, 0, 1, :2] = [5.96e-8, -3.0e-6]                                         # half subnormals
        if dt == ko.F16:
            k16 = vals.astype(np.float16)
            back = k16.astype(np.float32)
        else:
            k16 = bf16_round(vals)
            back = (k16.astype(np.uint32) << 16).view(np.float32)
        lo, hi = ko.OracleCache(L, B, H, d, cap, dt), ko.OracleCache(L, B, H, d, cap, ko.F32)
        lo.K[...], hi.K[...] = k16, back
        v = rng.standard_normal((L, B, H, cap, d)).astype(np.float32)
        if dt == ko.F16:
            lo.V[...], hi.V[...] = v.astype(np.float16), v.astype(np.float16).astype(np.float32)
        else:
            lo.V[...], hi.V[...] = bf16_round(v), (bf16_round(v).astype(np.uint32) << 16).view(np.float32)
        q = rng.standard_normal((L, B, H, n, d)).astype(np.float32) * 0.25
        q16 = q.astype(np.float16) if dt == ko.F16 else bf16_round(q)
        q32 = q16.astype(np.float32) if dt == ko.F16 else (q16.astype(np.uint32) << 16).view(np.float32)
        seeds = np.array([3, 4], np.uint64)
        lo.prefill_score(q16, n, 1.0, 0.01, ko.NOISE_GUMBEL, seeds)
        hi.prefill_score(q32, n, 1.0, 0.01, ko.NOISE_GUMBEL, seeds)
        np.testing.assert_array_equal(lo.score, hi.score)
        o16 = lo.decode_step(q16[:, :, :, 0], k16[:, :, :, cap - 1], lo.V[:, :, :, cap - 1].copy(), n, 1.5, 0.01, ko.NOISE_GUMBEL, seeds)
        o32 = hi.decode_step(q32[:, :, :, 0], back[:, :, :, cap - 1], hi.V[:, :, :, cap - 1].copy(), n, 1.5, 0.01, ko.NOISE_GUMBEL, seeds)
        np.testing.assert_array_equal(o16, o32)
        np.testing.assert_array_equal(lo.score, hi.score)
        np.testing.assert_array_equal(lo.select_evict(10, 3), hi.select_evict(10, 3))
        np.testing.assert_array_equal(lo.pos, hi.pos)
        got = lo.K.astype(np.float32) if dt == ko.F16 else (lo.K.astype(np.uint32) << 16).view(np.float32)
        np.testing.assert_array_equal(got[..., :10, :], hi.K[..., :10, :])                # rows moved as 16-bit words

