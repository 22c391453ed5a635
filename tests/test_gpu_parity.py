"""GPU-vs-oracle parity of the three hot calls, element by element, through the
C ABI (python binding -> libkeyformer.so).  Needs a real MI355X: -m gpu."""
import itertools
import os

import numpy as np
import pytest
import torch

import kf_workloads as kw
import paper_2403_09054_amd as kf
from oracle import kf_oracle as ko
from parity_harness import (SCORE_RTOL_PREFILL, LockStep, assert_close_out, assert_close_score, assert_set_equal,
                            assert_state_equal, compare_kept, dev, error_word, host, upload, upload_into)

pytestmark = pytest.mark.gpu


def _extra_seeds():
    """More seeds for the seeded shape sweeps, from the environment (KF_TEST_SEEDS="1,2,3"): the committed
    seeds are what every run covers; anybody hunting a rare case can widen the sweeps without editing them."""
    return [int(x) for x in os.environ.get("KF_TEST_SEEDS", "").replace(",", " ").split()]


SWEEP_SEEDS = [None] + _extra_seeds()   # None: the committed seed

DTYPES = [(ko.BF16, 64), (ko.BF16, 128), (ko.BF16, 256), (ko.F32, 64), (ko.F32, 128), (ko.F16, 64), (ko.F16, 128),
          (ko.F16, 256)]


def bf16_round(a):
    b = a.astype(np.float32).view(np.uint32).astype(np.uint64)
    return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)


def rnd(rng, shape, dtype):
    a = rng.standard_normal(shape).astype(np.float32)
    if dtype == ko.F16:
        return a.astype(np.float16)
    return bf16_round(a) if dtype == ko.BF16 else a


def random_cache(rng, L, B, H, d, cap, dtype, lens):
    oc = ko.OracleCache(L, B, H, d, cap, dtype)
    oc.K[...] = rnd(rng, oc.K.shape, dtype)
    oc.V[...] = rnd(rng, oc.V.shape, dtype)
    oc.score[...] = (rng.random(oc.score.shape) * 3).astype(np.float32)
    # strictly ascending original positions with gaps
    oc.pos[...] = np.cumsum(rng.integers(1, 4, oc.pos.shape), axis=-1).astype(np.int32)
    oc.len[...] = lens
    return oc


# ------------------------------------------------------------------ decode
@pytest.mark.parametrize("dtype,d", DTYPES)
@pytest.mark.parametrize("noise", [ko.NOISE_GUMBEL, ko.NOISE_NONE, ko.NOISE_GAUSSIAN, ko.NOISE_CONSTANT])
@pytest.mark.parametrize("cap", [97, 700, 2100])   # one split; several splits; ragged last split
def test_decode_step_matches_oracle(dtype, d, noise, cap):
    rng = np.random.default_rng(1000 + d + cap + noise)
    L, B, H = 2, 2, 3
    lens = rng.integers(0, cap, (L, B, H)).astype(np.int32)
    lens[0, 0, 0] = 0            # empty cache: the new token attends to itself only
    lens[0, 0, 1] = cap - 1      # fills the cache exactly
    lens[1, 1, 2] = cap          # no room: unit must be skipped and reported
    oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    q, kn, vn = (rnd(rng, (L, B, H, d), dtype) for _ in range(3))
    seeds = np.array([20240309, 2 ** 64 - 3], np.uint64)
    slopes = np.array([0.25, 0.0, 0.0039], np.float32)
    q_pos = int(oc.pos.max()) + 5
    tau, scale = 1.4375, float(1.0 / np.sqrt(np.float32(d)))
    out = torch.full((L, B, H, d), 7.0, dtype=torch.float32, device="cuda")
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, 0, tau, scale, noise, dev(seeds), dev(slopes),
                      out, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 1
    # the oracle refuses a full unit; run it with that unit emptied, then compare the rest
    full = oc.copy()
    oc.len[1, 1, 2] = 0
    out_ref = oc.decode_step(q, kn, vn, q_pos, tau, scale, noise, seeds, slopes)
    got_out, got_len = host(out), host(gc.len)
    assert (got_out[1, 1, 2] == 0).all() and got_len[1, 1, 2] == cap
    ok = np.ones((L, B, H), bool)
    ok[1, 1, 2] = False
    assert (got_len[ok] == oc.len[ok]).all()
    assert_close_out(got_out[ok], out_ref[ok])
    lens_cmp = np.where(ok, oc.len, 0)
    assert_close_score(host(gc.score), oc.score, lens_cmp)
    # K, V, pos: the appended row landed, nothing else moved (bit-exact)
    gK, gV, gpos = host(gc.K), host(gc.V), host(gc.pos)
    for l, b, h in itertools.product(range(L), range(B), range(H)):
        ref = oc if ok[l, b, h] else full
        m = int(ref.len[l, b, h])
        np.testing.assert_array_equal(gK[l, b, h, :m], ref.K[l, b, h, :m])
        np.testing.assert_array_equal(gV[l, b, h, :m], ref.V[l, b, h, :m])
        np.testing.assert_array_equal(gpos[l, b, h, :m], ref.pos[l, b, h, :m])
    # the workspace is reusable: a second step on the same workspace still matches
    q2 = rnd(rng, (L, B, H, d), dtype)
    oc.len[1, 1, 2] = cap
    full_units = oc.len >= cap
    gc2 = upload(oc)
    oc.len[full_units] = 0
    out_ref2 = oc.decode_step(q2, kn, vn, q_pos + 1, tau, scale, noise, seeds, slopes)
    kf.kf_decode_step(gc2, dev(q2), dev(kn), dev(vn), q_pos + 1, 0, tau, scale, noise, dev(seeds),
                      dev(slopes), out, ws)
    torch.cuda.synchronize()
    assert_close_out(host(out)[~full_units], out_ref2[~full_units])


def test_decode_m_hint_shapes_the_launch_only():
    rng = np.random.default_rng(5)
    L, B, H, d, cap = 1, 2, 2, 128, 1500
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, 400)
    q, kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    seeds = np.array([1, 2], np.uint64)
    outs = []
    for hint in (0, 401, 900):
        gc = upload(oc)
        ws = kf.new_workspace(gc)
        out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
        kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), 5000, hint, 1.5, 0.09, ko.NOISE_GUMBEL, dev(seeds),
                          None, out, ws)
        torch.cuda.synchronize()
        assert error_word(ws) == 0
        outs.append((host(out), host(gc.score)))
    ref = oc.copy()
    out_ref = ref.decode_step(q, kn, vn, 5000, 1.5, 0.09, ko.NOISE_GUMBEL, seeds)
    for o, s in outs:
        assert_close_out(o, out_ref)
        assert_close_score(s, ref.score, ref.len)
    # a hint below the true length is reported, not silently truncated
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), 5000, 200, 1.5, 0.09, ko.NOISE_GUMBEL, dev(seeds), None,
                      out, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == L * B * H
    assert (host(gc.len) == 400).all()


# ------------------------------------------------------------------ select + compact
@pytest.mark.parametrize("dtype,d", DTYPES)
@pytest.mark.parametrize("n,k,w", [(65, 64, 16), (1025, 1024, 205), (128, 64, 16), (2048, 1024, 205),
                                   (300, 120, 0), (300, 120, 120), (3000, 1200, 240), (50, 1, 0), (50, 1, 1)])
def test_select_evict_matches_oracle(dtype, d, n, k, w):
    rng = np.random.default_rng(n * 7 + k + w + d)
    L, B, H = 2, 1, 3
    lens = np.full((L, B, H), n, np.int32)
    lens[0, 0, 1] = max(1, k - 3)     # under budget: untouched
    lens[1, 0, 0] = k                 # exactly at budget: untouched
    lens[1, 0, 2] = min(n, k + 1)     # one over
    oc = random_cache(rng, L, B, H, d, n, dtype, lens)
    # exact ties: few distinct score values in one unit, a tie block around the threshold in another
    oc.score[0, 0, 0] = rng.integers(0, 5, n).astype(np.float32) * 0.5
    oc.score[0, 0, 2, n // 4: n // 2] = 1.5
    oc.score[1, 0, 1, :] = 2.0        # everything equal: lowest slots win
    before = oc.copy()
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    kept = torch.full((L, B, H, k), -5, dtype=torch.int32, device="cuda")
    kept_ref = oc.select_evict(k, w)
    kf.kf_select_evict(gc, k, w, kept, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(kept), kept_ref)       # ties included: bit-exact
    assert_state_equal(gc, oc)
    # without kept_idx the result is the same
    gc2 = upload(before)
    kf.kf_select_evict(gc2, k, w, None, ws)
    torch.cuda.synchronize()
    assert_state_equal(gc2, oc)


@pytest.mark.parametrize("seed", list(range(6)) + [1000 + x for x in _extra_seeds()])
def test_select_random_ragged_units(seed):
    """Units of every length in one call (empty, under budget, one over, far over, full), random budget and
    window, scores with many exact ties: survivor lists and compacted state bit-exact against the oracle."""
    rng = np.random.default_rng(400 + seed)
    d, dtype = [(64, ko.BF16), (128, ko.F32), (256, ko.BF16), (128, ko.BF16), (64, ko.F32), (256, ko.BF16)][seed % 6]
    cap = int(rng.integers(40, 700))
    k = int(rng.integers(1, cap + 1))
    w = int(rng.integers(0, k + 1))
    L, B, H = 2, 3, 4
    lens = rng.integers(0, cap + 1, (L, B, H)).astype(np.int32)
    lens.flat[:5] = [0, min(cap, k + 1), cap, k, max(0, k - 1)]
    oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
    oc.score[...] = rng.integers(0, 7, oc.score.shape).astype(np.float32) * 0.25 - 0.5
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    kept = torch.full((L, B, H, k), -5, dtype=torch.int32, device="cuda")
    kept_ref = oc.select_evict(k, w)
    kf.kf_select_evict(gc, k, w, kept, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    np.testing.assert_array_equal(host(kept), kept_ref)
    assert_state_equal(gc, oc)


def test_select_adversarial_eviction_slots():
    # decode shape, evicted slot at the very front, at the last candidate, and mid-way
    rng = np.random.default_rng(3)
    k, w, d = 256, 51, 128
    n = k + 1
    oc = random_cache(rng, 1, 1, 4, d, n, ko.BF16, n)
    oc.score[...] += 1.0
    oc.score[0, 0, 0, 0] = 0.0
    oc.score[0, 0, 1, n - w - 1] = 0.0
    oc.score[0, 0, 2, 100] = 0.0
    oc.score[0, 0, 3, [7, 90, 150]] = 0.5      # equal minima: the highest slot leaves
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    kept = torch.zeros((1, 1, 4, k), dtype=torch.int32, device="cuda")
    kept_ref = oc.select_evict(k, w)
    kf.kf_select_evict(gc, k, w, kept, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(kept), kept_ref)
    assert_state_equal(gc, oc)
    assert [sorted(set(range(n)) - set(kept_ref[0, 0, h].tolist()))[0] for h in range(4)] == [0, n - w - 1, 100, 150]


@pytest.mark.parametrize("d,dtype,k,w", [(128, ko.BF16, 256, 0), (128, ko.BF16, 300, 40), (128, ko.BF16, 100, 10),
                                        (256, ko.BF16, 128, 0), (64, ko.F32, 257, 1), (64, ko.BF16, 512, 100)])
def test_select_two_launch_eviction_at_chunk_boundaries(d, dtype, k, w):
    """Few units: the ordered eviction runs as two launches, the second moving the rows chunk by chunk (R rows
    per workgroup, R = 32 KB / row bytes).  Evicted slots on, next to and far from chunk boundaries, budgets that
    are a multiple of R, smaller than R, and without a window."""
    row_bytes = d * (4 if dtype == ko.F32 else 2)
    R = 2048 // (row_bytes // 16)
    n = k + 1
    ncand = n - w
    slots = sorted({s for s in (0, 1, R - 1, R, R + 1, 2 * R - 1, 2 * R, ncand - 1, ncand - 2, ncand // 2) if 0 <= s < ncand})
    rng = np.random.default_rng(k + d)
    oc = random_cache(rng, 1, 1, len(slots), d, n + 3, dtype, n)
    oc.score[...] += 1.0
    for h, s_ in enumerate(slots):
        oc.score[0, 0, h, s_] = 0.5
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    kept = torch.zeros((1, 1, len(slots), k), dtype=torch.int32, device="cuda")
    kept_ref = oc.select_evict(k, w)
    kf.kf_select_evict(gc, k, w, kept, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    np.testing.assert_array_equal(host(kept), kept_ref)
    assert_state_equal(gc, oc)
    for h, s_ in enumerate(slots):
        assert s_ not in set(kept_ref[0, 0, h].tolist())


# ------------------------------------------------------------------ prefill
@pytest.mark.parametrize("dtype,d", DTYPES)
@pytest.mark.parametrize("n", [1, 31, 33, 128, 129, 300])
def test_prefill_score_matches_oracle(dtype, d, n):
    rng = np.random.default_rng(n + d)
    L, B, H, cap = 1, 2, 2, n + 3
    for noise in (ko.NOISE_GUMBEL, ko.NOISE_NONE) if n not in (33, 300) else (
            ko.NOISE_GUMBEL, ko.NOISE_NONE, ko.NOISE_GAUSSIAN, ko.NOISE_CONSTANT):
        oc = random_cache(rng, L, B, H, d, cap, dtype, 0)
        Q = rnd(rng, (L, B, H, n, d), dtype)
        seeds = np.array([77, 2 ** 40 + 1], np.uint64)
        slopes = np.array([0.0, 0.0625], np.float32)
        tau, scale = 1.0 if noise == ko.NOISE_GUMBEL else 1.3, float(1.0 / np.sqrt(np.float32(d)))
        gc = upload(oc)
        ws = kf.new_workspace(gc, n)
        oc.prefill_score(Q, n, tau, scale, noise, seeds, slopes)
        kf.kf_prefill_score(gc, dev(Q), n, tau, scale, noise, dev(seeds), dev(slopes), ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(gc.len), oc.len)
        np.testing.assert_array_equal(host(gc.pos)[..., :n], oc.pos[..., :n])
        assert_close_score(host(gc.score), oc.score, oc.len, "prefill noise=%d" % noise, rtol=SCORE_RTOL_PREFILL)


@pytest.mark.parametrize("sweep_seed", SWEEP_SEEDS)
def test_prefill_on_random_shapes_matches_oracle(sweep_seed):
    """Seeded sweep over the prompt-scoring call: element types, head sizes, prompt lengths around the tile
    edges and in between, query heads per cached head, every logit adjustment at temperatures on both sides
    of 1, logit scales from flat to peaked, with and without a position bias (each has kernels of its own)."""
    rng = np.random.default_rng(20240311 if sweep_seed is None else 999000 + sweep_seed)
    for case in range(12):
        dtype, d = DTYPES[int(rng.integers(0, len(DTYPES)))]
        n = int(rng.choice([1, 2, 31, 32, 33, 127, 128, 129, int(rng.integers(130, 900))]))
        L, B, H = 1, int(rng.integers(1, 3)), int(rng.integers(1, 4))
        G = int(rng.choice([1, 1, 2, 4]))
        noise = int(rng.choice([ko.NOISE_GUMBEL, ko.NOISE_GUMBEL, ko.NOISE_NONE, ko.NOISE_GAUSSIAN, ko.NOISE_CONSTANT]))
        tau = float(rng.choice([1.0, 1.0, 1.3, 0.6, 2.0]))
        scale = float(rng.choice([1.0, 1.0, 3.0, 0.2])) / float(np.sqrt(np.float32(d)))
        slopes = (rng.random(H * G) * 0.5).astype(np.float32) if rng.integers(0, 2) else None
        oc = random_cache(rng, L, B, H, d, n + int(rng.integers(0, 5)), dtype, 0)
        Q = rnd(rng, (L, B, H * G, n, d), dtype)
        seeds = rng.integers(0, 2 ** 63, B).astype(np.uint64)
        what = "case %d: dtype=%d d=%d n=%d B,H=%d,%d G=%d noise=%d tau=%g scale*sqrt(d)=%g slopes=%s" % (
            case, dtype, d, n, B, H, G, noise, tau, scale * np.sqrt(d), slopes is not None)
        print(what, flush=True)
        gc = upload(oc, G)
        ws = kf.new_workspace(gc, n)
        oc.prefill_score(Q, n, tau, scale, noise, seeds, slopes, q_per_kv=G)
        kf.kf_prefill_score(gc, dev(Q), n, tau, scale, noise, dev(seeds), None if slopes is None else dev(slopes), ws)
        torch.cuda.synchronize()
        assert error_word(ws) == 0, what
        np.testing.assert_array_equal(host(gc.len), oc.len)
        np.testing.assert_array_equal(host(gc.pos)[..., :n], oc.pos[..., :n])
        assert_close_score(host(gc.score), oc.score, oc.len, what, rtol=SCORE_RTOL_PREFILL)
        del gc, ws


@pytest.mark.parametrize("dtype,d,scale", [(ko.BF16, 128, 6.0), (ko.F32, 64, 9.0), (ko.BF16, 256, 0.0)])
def test_prefill_with_logits_far_from_the_rows_reference(dtype, d, scale):
    """Logits spread over hundreds of powers of two (a logit scale far above 1/sqrt(d)): the row sums are
    formed against a reference exponent that starts at the diagonal term, so terms 2^120 and more above it
    must send the reference up (the tile is summed again) instead of overflowing, and rows whose other terms
    all vanish against it keep their diagonal term.  Scale 0: every logit is pure adjustment."""
    rng = np.random.default_rng(int(scale * 10) + d)
    L, B, H, n = 1, 2, 2, 200
    oc = random_cache(rng, L, B, H, d, n, dtype, 0)
    Q = rnd(rng, (L, B, H, n, d), dtype)
    seeds = np.array([3, 4], np.uint64)
    slopes = np.array([0.0, 0.7], np.float32)
    gc = upload(oc)
    ws = kf.new_workspace(gc, n)
    oc.prefill_score(Q, n, 1.0, scale, ko.NOISE_GUMBEL, seeds, slopes)
    kf.kf_prefill_score(gc, dev(Q), n, 1.0, scale, ko.NOISE_GUMBEL, dev(seeds), dev(slopes), ws)
    torch.cuda.synchronize()
    got, ref = host(gc.score).astype(np.float64), oc.score.astype(np.float64)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got.sum(axis=-1), n, rtol=1e-5)          # every row of the softmax sums to one
    big = ref > 1e-12                                                    # below that the sums are lost in fp32
    assert big.sum() > n                                                 # (near one-hot rows: few columns carry the mass)
    assert (np.abs(got - ref)[big] <= SCORE_RTOL_PREFILL * ref[big] + 1e-12).all()
    assert (got[~big] <= 1e-11).all()


def test_prefill_with_a_nan_query_row_stays_confined_to_it():
    """A query row of NaNs makes that row's terms NaN (its sum can never be brought into range: the retry of
    the row sum is bounded), which reaches the columns it contributes to (keys up to its own position) of its
    own unit and nothing else."""
    rng = np.random.default_rng(404)
    L, B, H, d, n, bad = 1, 1, 2, 64, 150, 70
    oc = random_cache(rng, L, B, H, d, n, ko.F32, 0)
    Q = rnd(rng, (L, B, H, n, d), ko.F32)
    Q[0, 0, 0, bad] = np.nan
    seeds = np.array([8], np.uint64)
    gc = upload(oc)
    ws = kf.new_workspace(gc, n)
    scale = float(1.0 / np.sqrt(np.float32(d)))
    kf.kf_prefill_score(gc, dev(Q), n, 1.0, scale, kf.NOISE_GUMBEL, dev(seeds), None, ws)
    torch.cuda.synchronize()
    clean = Q.copy()
    clean[0, 0, 0, bad] = 0.0
    oc.prefill_score(clean, n, 1.0, scale, ko.NOISE_GUMBEL, seeds, None)
    got = host(gc.score)
    assert np.isnan(got[0, 0, 0, : bad + 1]).all()                   # the columns row `bad` contributes to
    sel = np.zeros((L, B, H), np.int32)
    sel[0, 0, 1] = n                                                   # the other unit: untouched by it
    assert_close_score(got, oc.score, sel, rtol=SCORE_RTOL_PREFILL)
    # columns behind the bad row receive nothing from it: the same sums as with that row replaced (rows after it
    # are unchanged, and a zero query row only matters to the columns up to its own position)
    np.testing.assert_allclose(got[0, 0, 0, bad + 1:n], oc.score[0, 0, 0, bad + 1:n], rtol=SCORE_RTOL_PREFILL)


@pytest.mark.parametrize("dtype,d,G,shared", [(ko.BF16, 128, 1, False), (ko.BF16, 256, 1, False), (ko.F32, 64, 1, False),
                                              (ko.BF16, 64, 4, False), (ko.BF16, 128, 1, True)])
def test_prefill_of_a_padded_batch_matches_oracle(dtype, d, G, shared):
    """Prompts of different lengths padded to n rows (cfg.seq_n): every sequence is scored over its own rows."""
    rng = np.random.default_rng(500 + d + G)
    L, H, n = 2, 2, 300
    n_seq = np.array([300, 1, 129, 37, 128, 256], np.int32)
    B = len(n_seq)
    oc = random_cache(rng, L, B, H, d, n + 5, dtype, 3)
    oc.score[...] = -3.0
    oc.pos[...] = -7
    Q = rnd(rng, (L, B, H * G, n, d), dtype)
    seeds = (np.arange(B) * 1000 + 3).astype(np.uint64)
    slopes = (0.5 ** np.arange(1, H * G + 1)).astype(np.float32)
    scale = float(1.0 / np.sqrt(np.float32(d)))
    gc = upload(oc, G)
    ws = kf.new_workspace(gc, n)
    kf.kf_prefill_score(gc, dev(Q), n, 1.0, scale, kf.NOISE_GUMBEL, dev(seeds), dev(slopes), ws,
                        score_mode=kf.SCORE_SHARED if shared else kf.SCORE_PER_LAYER, seq_n=dev(n_seq))
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    oc.prefill_score(Q, n, 1.0, scale, ko.NOISE_GUMBEL, seeds, slopes, shared=shared, q_per_kv=G, n_seq=n_seq)
    assert (oc.len == n_seq[None, :, None]).all()
    np.testing.assert_array_equal(host(gc.len), oc.len)
    np.testing.assert_array_equal(host(gc.pos), oc.pos)                     # -7 kept beyond every prompt's end
    assert_close_score(host(gc.score), oc.score, oc.len, "padded batch", rtol=SCORE_RTOL_PREFILL)
    for b in range(B):
        assert (host(gc.score)[:, b, :, n_seq[b]:] == -3.0).all()


def test_prefill_of_a_padded_batch_reports_lengths_out_of_range():
    rng = np.random.default_rng(501)
    L, B, H, d, n = 2, 3, 2, 64, 70
    oc = random_cache(rng, L, B, H, d, n + 2, ko.BF16, 9)
    Q = rnd(rng, (L, B, H, n, d), ko.BF16)
    n_seq = np.array([0, 71, 33], np.int32)
    seeds = np.array([1, 2, 3], np.uint64)
    gc = upload(oc)
    ws = kf.new_workspace(gc, n)
    kf.kf_prefill_score(gc, dev(Q), n, 1.0, 0.125, kf.NOISE_GUMBEL, dev(seeds), None, ws, seq_n=dev(n_seq))
    torch.cuda.synchronize()
    assert error_word(ws) == 2 * L * H                                      # every unit of the two sequences
    ref = oc.copy()
    one = ko.OracleCache(L, 1, H, d, n + 2, ko.BF16)
    for nm in ("K", "V", "score", "pos", "len"):
        getattr(one, nm)[...] = getattr(oc, nm)[:, 2:3]
    one.prefill_score(np.ascontiguousarray(Q[:, 2:3, :, :33]), 33, 1.0, 0.125, ko.NOISE_GUMBEL, seeds[2:3])
    for nm in ("score", "pos", "len"):
        getattr(ref, nm)[:, 2:3] = getattr(one, nm)
    np.testing.assert_array_equal(host(gc.len), ref.len)                    # skipped units keep their state
    np.testing.assert_array_equal(host(gc.pos), ref.pos)
    np.testing.assert_array_equal(host(gc.score)[:, :2], ref.score[:, :2])
    assert_close_score(host(gc.score), ref.score, ref.len, rtol=SCORE_RTOL_PREFILL)


@pytest.mark.parametrize("layout", [kf.LAYOUT_ORDERED, kf.LAYOUT_SLOT])
def test_padded_batch_from_prompt_through_generation(layout):
    """Sequences with prompts of 40..700 tokens in one batch: prompt scoring with seq_n, the first eviction
    (only the prompts over budget lose tokens), then steps in which every sequence is at its own position."""
    rng = np.random.default_rng(502)
    L, H, d, n, k, w, T = 1, 4, 128, 700, 200, 40, 16
    n_seq = np.array([700, 40, 201, 333], np.int32)
    B = len(n_seq)
    cap = n
    oc = ko.OracleCache(L, B, H, d, cap, ko.BF16)
    oc.K[...] = rnd(rng, oc.K.shape, ko.BF16)
    oc.V[...] = rnd(rng, oc.V.shape, ko.BF16)
    Q = rnd(rng, (L, B, H, n, d), ko.BF16)
    seeds = np.array([11, 12, 13, 14], np.uint64)
    slopes = (0.5 ** np.arange(1, H + 1)).astype(np.float32)
    scale = float(1.0 / np.sqrt(np.float32(d)))
    gc = upload(oc)
    ws = kf.new_workspace(gc, n)
    kf.kf_prefill_score(gc, dev(Q), n, kf.kf_tau(0, T), scale, kf.NOISE_GUMBEL, dev(seeds), dev(slopes), ws, seq_n=dev(n_seq))
    oc.prefill_score(Q, n, ko.tau(0, T), scale, ko.NOISE_GUMBEL, seeds, slopes, n_seq=n_seq)
    kept = torch.zeros((L, B, H, k), dtype=torch.int32, device="cuda")
    before_score, before_len = oc.score.copy(), oc.len.copy()
    kf.kf_select_evict(gc, k, w, kept, ws)                                  # ordered: also what the slot layout starts from
    kept_ref = oc.select_evict(k, w)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    assert compare_kept(host(kept), kept_ref, before_score, before_len, k, w) == 0
    assert (oc.len == np.minimum(n_seq, k)[None, :, None]).all()
    assert_state_equal(gc, oc, kv=True, score_exact=False)
    out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    for t in range(1, T + 1):
        q, kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(3))
        q_pos = (n_seq + t - 1).astype(np.int32)
        taus = np.full(B, kf.kf_tau(t, T), np.float32)
        kf.kf_decode_select_step(gc, dev(q), dev(kn), dev(vn), 0, 0, 1.0, scale, kf.NOISE_GUMBEL, dev(seeds), dev(slopes),
                                 out, k=k, w=w, layout=layout, kept_idx=kept, workspace=ws, seq_q_pos=dev(q_pos),
                                 seq_tau=dev(taus))
        torch.cuda.synchronize()
        assert error_word(ws) == 0
        out_ref = oc.decode_step(q, kn, vn, 0, 1.0, scale, ko.NOISE_GUMBEL, seeds, slopes, q_pos_seq=q_pos, tau_seq=taus)
        assert_close_out(host(out), out_ref, "out step %d" % t)
        before_score, before_len = oc.score.copy(), oc.len.copy()
        kept_ref = oc.select_evict(k, w)
        if layout == kf.LAYOUT_ORDERED:
            assert compare_kept(host(kept), kept_ref, before_score, before_len, k, w) == 0
            assert_state_equal(gc, oc, kv=True, score_exact=False)
            assert_close_score(host(gc.score), oc.score, oc.len, "score step %d" % t, rtol=SCORE_RTOL_PREFILL)   # the GPU's own prompt scores, never resynchronised
        else:
            assert_set_equal(gc, oc, kv=True, score_exact=False)
    assert (oc.len == np.minimum(n_seq + T, k)[None, :, None]).all()      # the short prompt is still growing


# ------------------------------------------------------------------ the five configurations
def test_tiny_config_full_lockstep_and_free_running():
    wl = kw.CONFIGS["tiny"]
    ls = LockStep(wl)
    ls.prefill()
    for t in range(1, wl.T + 1):
        ls.step(t, check_kv=True)
    assert ls.stats["steps"] == wl.T
    print("tiny lockstep", ls.stats)
    # free-running: no resynchronisation at all; report where (if ever) the sets part
    fr = LockStep(wl)
    fr.oc.prefill_score(fr.Q, wl.n, ko.tau(0, wl.T), wl.scale, fr.noise, fr.seeds, fr.slopes)
    kf.kf_prefill_score(fr.gc, dev(fr.Q), wl.n, kf.kf_tau(0, wl.T), wl.scale, fr.noise, fr.d_seeds, None, fr.ws)
    fr.oc.select_evict(wl.k, wl.w)
    kf.kf_select_evict(fr.gc, wl.k, wl.w, None, fr.ws)
    first_div = None
    for t in range(1, wl.T + 1):
        q, kn, vn = kw.decode_inputs(wl, t)
        fr.oc.decode_step(kw.to_oracle(q), kw.to_oracle(kn), kw.to_oracle(vn), wl.n + t - 1, ko.tau(t, wl.T),
                          wl.scale, fr.noise, fr.seeds)
        kf.kf_decode_step(fr.gc, q.cuda(), kn.cuda(), vn.cuda(), wl.n + t - 1, wl.k + 1, kf.kf_tau(t, wl.T),
                          wl.scale, fr.noise, fr.d_seeds, None, fr.out, fr.ws)
        fr.oc.select_evict(wl.k, wl.w)
        kf.kf_select_evict(fr.gc, wl.k, wl.w, None, fr.ws)
        torch.cuda.synchronize()
        if first_div is None and not (host(fr.gc.pos)[..., : wl.k] == fr.oc.pos[..., : wl.k]).all():
            first_div = t
    print("tiny free-running first divergence step:", first_div)
    assert first_div is None      # well-separated scores: the sets stay identical for all 32 steps


SLICES = {
    # name: (slice kwargs, decode steps checked from t = 1, steps checked at the end of the schedule)
    "gptj": (dict(L=2, H=16, T=512), 512, 0),        # the whole generation: tau runs from tau_init to tau_end
    "mpt": (dict(L=1, B=2, H=8, T=1024), 256, 8),
    "batched": (dict(L=1, B=4, H=8, T=1024), 256, 8),
}


def late_steps(ls, late):
    """The last `late` iterations of the schedule (t = T-late+1 .. T, tau -> tau_end of Eq. 12) on the state
    the slice has reached: the generation in between is skipped, the query position jumps with t."""
    wl = ls.wl
    for t in range(wl.T - late + 1, wl.T + 1):
        ls.step(t, check_kv=(t == wl.T))
    assert kf.kf_tau(wl.T, wl.T, wl.tau_init, wl.tau_end) == wl.tau_end


@pytest.mark.parametrize("name", list(SLICES))
def test_config_slice_lockstep(name):
    kwargs, steps, late = SLICES[name]
    wl = kw.CONFIGS[name].slice(**kwargs)
    ls = LockStep(wl)
    ls.prefill()
    for t in range(1, steps + 1):
        ls.step(t, check_kv=(t == steps))
    late_steps(ls, late)
    assert ls.stats["steps"] == steps + late
    print(name, "slice lockstep", ls.stats)


def test_long_config_slice_lockstep():
    # full per-unit shape of the long-context configuration (n = 32768, k = 9830)
    wl = kw.CONFIGS["long"].slice(L=1, H=8, T=2048)
    ls = LockStep(wl)
    ls.prefill()
    for t in range(1, 129):
        ls.step(t, check_kv=(t == 128))
    late_steps(ls, 8)
    print("long slice lockstep", ls.stats)


def test_mpt_slice_free_running_with_position_bias():
    """No resynchronisation at all on an MPT-shaped slice (ALiBi, k = 2048): prompt scoring, first eviction and
    96 generation steps, each side following its own scores.  While the retained sets agree the GPU's
    self-accumulated scores are compared element by element; the step of the first difference, if any, is
    printed (a near-tie at the threshold may send the two apart for good)."""
    wl = kw.CONFIGS["mpt"].slice(L=1, B=2, H=4, T=1024)
    fr = LockStep(wl)
    fr.oc.prefill_score(fr.Q, wl.n, ko.tau(0, wl.T), wl.scale, fr.noise, fr.seeds, fr.slopes)
    kf.kf_prefill_score(fr.gc, dev(fr.Q), wl.n, kf.kf_tau(0, wl.T), wl.scale, fr.noise, fr.d_seeds, fr.d_slopes, fr.ws)
    fr.oc.select_evict(wl.k, wl.w)
    kf.kf_select_evict(fr.gc, wl.k, wl.w, None, fr.ws)
    torch.cuda.synchronize()
    first_div, steps, worst = None, 96, 0.0
    for t in range(1, steps + 1):
        q, kn, vn = kw.decode_inputs(wl, t)
        out_ref = fr.oc.decode_step(kw.to_oracle(q), kw.to_oracle(kn), kw.to_oracle(vn), wl.n + t - 1, ko.tau(t, wl.T),
                                    wl.scale, fr.noise, fr.seeds, fr.slopes)
        kf.kf_decode_select_step(fr.gc, q.cuda(), kn.cuda(), vn.cuda(), wl.n + t - 1, wl.k + 1, kf.kf_tau(t, wl.T), wl.scale,
                                 fr.noise, fr.d_seeds, fr.d_slopes, fr.out, k=wl.k, w=wl.w, workspace=fr.ws)
        fr.oc.select_evict(wl.k, wl.w)
        torch.cuda.synchronize()
        assert error_word(fr.ws) == 0
        if first_div is None:
            if (host(fr.gc.pos)[..., : wl.k] == fr.oc.pos[..., : wl.k]).all():
                assert_close_out(host(fr.out), out_ref, "free-running out step %d" % t)
                worst = max(worst, assert_close_score(host(fr.gc.score), fr.oc.score, fr.oc.len,
                                                      "free-running score step %d" % t, rtol=SCORE_RTOL_PREFILL))
            else:
                first_div = t
    print("mpt slice free-running: first divergence step:", first_div, "of", steps, "; worst score error", worst)
    assert first_div is None or first_div > 16


def test_gptj_full_size_in_bench_launch_shape_sampled_layers():
    """The workload bench.py times (all 28 layers x 16 heads = 448 units in one
    launch, cap = k+1 for decode), checked on three whole layers the oracle can
    compute: prompt scoring, first eviction, then decode steps in lock-step."""
    wl = kw.CONFIGS["gptj"]
    sample = [0, 13, 27]
    steps = 6
    seeds, d_seeds = kw.noise_seeds(wl), dev(kw.noise_seeds(wl))
    tau0 = kf.kf_tau(0, wl.T)
    # --- prompt phase on the GPU: every layer in one call
    stage = kf.Cache.allocate(wl.L, wl.B, wl.H, wl.d, wl.n, kf.BF16)
    Qg = torch.empty((wl.L, wl.B, wl.H, wl.n, wl.d), dtype=torch.bfloat16, device="cuda")
    ocs = {}
    for l in range(wl.L):
        Q, K, V = kw.prompt_layer(wl, l)              # CPU generator: the oracle sees the same bits
        Qg[l].copy_(Q)
        stage.K[l].copy_(K)
        stage.V[l].copy_(V)
        if l in sample:
            oc = ko.OracleCache(1, wl.B, wl.H, wl.d, wl.n, ko.BF16, layer0=l)
            oc.K[0], oc.V[0] = kw.to_oracle(K), kw.to_oracle(V)
            oc.prefill_score(kw.to_oracle(Q)[None], wl.n, ko.tau(0, wl.T), wl.scale, ko.NOISE_GUMBEL, seeds)
            ocs[l] = oc
    ws = kf.new_workspace(stage, wl.n)
    kf.kf_prefill_score(stage, Qg, wl.n, tau0, wl.scale, kf.NOISE_GUMBEL, d_seeds, None, ws)
    torch.cuda.synchronize()
    for l in sample:
        assert_close_score(host(stage.score[l:l + 1]), ocs[l].score, ocs[l].len, "prefill layer %d" % l, rtol=SCORE_RTOL_PREFILL)
        stage.score[l].copy_(dev(ocs[l].score)[0])    # lock-step: same scores before selection
    kept = torch.zeros((wl.L, wl.B, wl.H, wl.k), dtype=torch.int32, device="cuda")
    before = {l: (ocs[l].score.copy(), ocs[l].len.copy()) for l in sample}
    kf.kf_select_evict(stage, wl.k, wl.w, kept, ws)
    torch.cuda.synchronize()
    ties = 0
    for l in sample:
        kept_ref = ocs[l].select_evict(wl.k, wl.w)
        ties += compare_kept(host(kept[l:l + 1]), kept_ref, before[l][0], before[l][1], wl.k, wl.w)
    assert ties == 0
    # --- decode cache shaped as in bench.py: cap = k+1
    cache = kf.Cache.allocate(wl.L, wl.B, wl.H, wl.d, wl.k + 1, kf.BF16)
    cache.K[..., : wl.k, :].copy_(stage.K[..., : wl.k, :])
    cache.V[..., : wl.k, :].copy_(stage.V[..., : wl.k, :])
    cache.score[..., : wl.k].copy_(stage.score[..., : wl.k])
    cache.pos[..., : wl.k].copy_(stage.pos[..., : wl.k])
    cache.len.copy_(stage.len)
    del stage, Qg
    ws = kf.new_workspace(cache)
    out = torch.zeros((wl.L, wl.B, wl.H, wl.d), dtype=torch.float32, device="cuda")
    kept = torch.zeros((wl.L, wl.B, wl.H, wl.k), dtype=torch.int32, device="cuda")
    dec = {}
    for l in sample:                                   # the oracle continues in a cap = k+1 cache too
        o = ko.OracleCache(1, wl.B, wl.H, wl.d, wl.k + 1, ko.BF16, layer0=l)
        o.K[..., : wl.k, :], o.V[..., : wl.k, :] = ocs[l].K[..., : wl.k, :], ocs[l].V[..., : wl.k, :]
        o.score[..., : wl.k], o.pos[..., : wl.k] = ocs[l].score[..., : wl.k], ocs[l].pos[..., : wl.k]
        o.len[...] = ocs[l].len
        dec[l] = o
    for t in range(1, steps + 1):
        q, kn, vn = kw.decode_inputs(wl, t)
        q_pos = wl.n + t - 1
        kf.kf_decode_step(cache, q.cuda(), kn.cuda(), vn.cuda(), q_pos, wl.k + 1, kf.kf_tau(t, wl.T), wl.scale,
                          kf.NOISE_GUMBEL, d_seeds, None, out, ws)
        torch.cuda.synchronize()
        assert error_word(ws) == 0 and int(cache.len.min()) == wl.k + 1
        for l in sample:
            o = dec[l]
            out_ref = o.decode_step(kw.to_oracle(q[l:l + 1]), kw.to_oracle(kn[l:l + 1]), kw.to_oracle(vn[l:l + 1]),
                                    q_pos, ko.tau(t, wl.T), wl.scale, ko.NOISE_GUMBEL, seeds)
            assert_close_out(host(out[l:l + 1]), out_ref)
            assert_close_score(host(cache.score[l:l + 1]), o.score, o.len)
            cache.score[l].copy_(dev(o.score)[0])
            before[l] = (o.score.copy(), o.len.copy())
        kf.kf_select_evict(cache, wl.k, wl.w, kept, ws)
        torch.cuda.synchronize()
        for l in sample:
            kept_ref = dec[l].select_evict(wl.k, wl.w)
            ev = compare_kept(host(kept[l:l + 1]), kept_ref, before[l][0], before[l][1], wl.k, wl.w)
            assert ev == 0
            sub = kf.Cache(K=cache.K[l:l + 1], V=cache.V[l:l + 1], score=cache.score[l:l + 1], pos=cache.pos[l:l + 1],
                           len=cache.len[l:l + 1], L=1, B=wl.B, H=wl.H, d=wl.d, cap=wl.k + 1, dtype=kf.BF16)
            assert_state_equal(sub, dec[l], kv=(t == steps))
    assert int(cache.len.min()) == wl.k and int(cache.len.max()) == wl.k


@pytest.mark.parametrize("name", ["mpt", "long", "batched"])
def test_full_size_prompt_phase_in_bench_staging_shape_sampled_units(name):
    """Prompt scoring and the first eviction of the large configurations in the launch shapes bench.py
    stages them in (as many layers per call as kf_workloads.staging_layers allows, every sequence and head),
    for the first group of layers and for the last, smaller one.  Inputs are generated on the device; the
    oracle recomputes three single units per call -- first, middle, last -- from the rows copied back."""
    wl = kw.CONFIGS[name]
    Ls = kw.staging_layers(wl)
    assert Ls == {"mpt": 14, "long": 14, "batched": 3}[name]
    stage = kf.Cache.allocate(Ls, wl.B, wl.H, wl.d, wl.n, kf.BF16)
    Qs = torch.empty((Ls, wl.B, wl.H, wl.n, wl.d), dtype=torch.bfloat16, device="cuda")
    ws = kf.new_workspace(stage, wl.n)
    seeds, slopes = kw.noise_seeds(wl), kw.alibi_slopes(wl)
    d_seeds, d_slopes = dev(seeds), dev(slopes)
    tau0 = kf.kf_tau(0, wl.T, wl.tau_init, wl.tau_end)
    groups = [0] + ([wl.L // Ls * Ls] if wl.L % Ls else [])
    ties = 0
    for l0 in groups:
        nl = min(Ls, wl.L - l0)
        for i in range(nl):
            Q, K, V = kw.prompt_layer(wl, l0 + i, device="cuda")
            Qs[i].copy_(Q)
            stage.K[i].copy_(K)
            stage.V[i].copy_(V)
            del Q, K, V
        sub = stage if nl == Ls else kf.Cache(K=stage.K[:nl], V=stage.V[:nl], score=stage.score[:nl], pos=stage.pos[:nl],
                                              len=stage.len[:nl], L=nl, B=wl.B, H=wl.H, d=wl.d, cap=wl.n, dtype=kf.BF16)
        sub.layer0 = l0
        sub.score.fill_(-1.0)
        sub.len.fill_(0)
        gen = kf.Cache.allocate(nl, wl.B, wl.H, wl.d, wl.k + 1, kf.BF16)
        kept = torch.full((nl, wl.B, wl.H, wl.k), -7, dtype=torch.int32, device="cuda")
        kf.kf_prefill_score(sub, Qs[:nl], wl.n, tau0, wl.scale, kf.NOISE_GUMBEL, d_seeds, d_slopes, ws)
        kf.kf_select_evict_into(sub, gen, 0, wl.k, wl.w, kept, ws)
        torch.cuda.synchronize()
        assert error_word(ws) == 0
        assert int(sub.len.min()) == wl.n and int(sub.len.max()) == wl.n
        assert int(gen.len.min()) == wl.k and int(gen.len.max()) == wl.k
        assert bool((sub.score[..., : wl.n] > 0).all())          # every unit of the launch was scored
        for l, b, h in [(0, 0, 0), (nl // 2, wl.B // 2, wl.H // 2), (nl - 1, wl.B - 1, wl.H - 1)]:
            oc = ko.OracleCache(1, 1, 1, wl.d, wl.n, ko.BF16, layer0=l0 + l, head0=h)
            oc.K[0, 0, 0], oc.V[0, 0, 0] = host(stage.K[l, b, h]), host(stage.V[l, b, h])
            oc.prefill_score(host(Qs[l, b, h])[None, None, None], wl.n, ko.tau(0, wl.T, wl.tau_init, wl.tau_end), wl.scale,
                             ko.NOISE_GUMBEL, seeds[b:b + 1], slopes)
            what = "%s layers %d+%d unit (%d,%d,%d)" % (name, l0, nl, l, b, h)
            np.testing.assert_array_equal(host(sub.pos[l, b, h]), oc.pos[0, 0, 0])
            assert_close_score(host(sub.score[l, b, h])[None, None, None], oc.score, oc.len, what, rtol=SCORE_RTOL_PREFILL)
            before = (oc.score.copy(), oc.len.copy())
            kept_ref = oc.select_evict(wl.k, wl.w)
            ev = compare_kept(host(kept[l, b, h])[None, None, None], kept_ref, before[0], before[1], wl.k, wl.w)
            ties += ev
            if not ev:                                   # same survivors: rows gathered bit for bit
                np.testing.assert_array_equal(host(gen.pos[l, b, h, : wl.k]), oc.pos[0, 0, 0, : wl.k])
                np.testing.assert_array_equal(host(gen.K[l, b, h, : wl.k]), oc.K[0, 0, 0, : wl.k])
                np.testing.assert_array_equal(host(gen.V[l, b, h, : wl.k]), oc.V[0, 0, 0, : wl.k])
                assert_close_score(host(gen.score[l, b, h])[None, None, None], oc.score, oc.len, what + " after eviction",
                                   rtol=SCORE_RTOL_PREFILL)
        del gen, kept
    print(name, "full-size prompt phase: tie-band events", ties)


@pytest.mark.parametrize("name", ["mpt", "long", "batched"])
def test_full_size_decode_and_select_on_sampled_sequences(name):
    """The other configurations at their FULL size (all units in one launch, cap = k+1: the launch shape a
    bench run of that configuration uses), from a synthetic cache state, three generation steps in
    lock-step; the oracle computes three whole (layer, sequence) rows -- first, last and one in between."""
    wl = kw.CONFIGS[name]
    k, cap = wl.k, wl.k + 1
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    cache = kf.Cache.allocate(wl.L, wl.B, wl.H, wl.d, cap, kf.BF16)
    for l in range(wl.L):                       # layer by layer: no full-size temporaries
        cache.K[l].normal_(generator=g)
        cache.V[l].normal_(generator=g)
        cache.score[l].uniform_(0.0, 3.0, generator=g)
    cache.pos.copy_(torch.arange(wl.n - k, wl.n - k + cap, device="cuda", dtype=torch.int32).expand_as(cache.pos))
    cache.len.fill_(k)
    ws = kf.new_workspace(cache)
    seeds = kw.noise_seeds(wl)
    slopes = kw.alibi_slopes(wl)
    d_seeds, d_slopes = dev(seeds), dev(slopes)
    out = torch.zeros((wl.L, wl.B, wl.H, wl.d), dtype=torch.float32, device="cuda")
    kept = torch.zeros((wl.L, wl.B, wl.H, k), dtype=torch.int32, device="cuda")
    rows = [(0, 0), (wl.L // 2, wl.B // 2), (wl.L - 1, wl.B - 1)]
    ocs = {}
    for l, b in rows:
        oc = ko.OracleCache(1, 1, wl.H, wl.d, cap, ko.BF16, layer0=l)
        oc.K[0, 0], oc.V[0, 0] = host(cache.K[l, b]), host(cache.V[l, b])
        oc.score[0, 0], oc.pos[0, 0], oc.len[0, 0] = host(cache.score[l, b]), host(cache.pos[l, b]), host(cache.len[l, b])
        ocs[(l, b)] = oc
    ties = 0
    for t in range(1, 4):
        q, kn, vn = kw.decode_inputs(wl, t, device="cuda")
        q_pos = wl.n + t - 1
        kf.kf_decode_step(cache, q, kn, vn, q_pos, cap, kf.kf_tau(t, wl.T, wl.tau_init, wl.tau_end), wl.scale,
                          kf.NOISE_GUMBEL, d_seeds, d_slopes, out, ws)
        torch.cuda.synchronize()
        assert error_word(ws) == 0 and int(cache.len.min()) == cap
        before = {}
        for (l, b), oc in ocs.items():
            out_ref = oc.decode_step(host(q[l, b])[None, None], host(kn[l, b])[None, None], host(vn[l, b])[None, None],
                                     q_pos, ko.tau(t, wl.T, wl.tau_init, wl.tau_end), wl.scale, ko.NOISE_GUMBEL,
                                     seeds[b:b + 1], slopes)
            assert_close_out(host(out[l, b])[None, None], out_ref, "out (%d,%d)" % (l, b))
            assert_close_score(host(cache.score[l, b])[None, None], oc.score, oc.len, "score (%d,%d)" % (l, b))
            cache.score[l, b].copy_(dev(oc.score)[0, 0])          # lock-step: same scores before selection
            before[(l, b)] = (oc.score.copy(), oc.len.copy())
        kf.kf_select_evict(cache, k, wl.w, kept, ws)
        torch.cuda.synchronize()
        assert error_word(ws) == 0 and int(cache.len.max()) == k
        for (l, b), oc in ocs.items():
            kept_ref = oc.select_evict(k, wl.w)
            ev = compare_kept(host(kept[l, b])[None, None], kept_ref, before[(l, b)][0], before[(l, b)][1], k, wl.w)
            ties += ev
            sub = kf.Cache(K=cache.K[l:l + 1, b:b + 1], V=cache.V[l:l + 1, b:b + 1], score=cache.score[l:l + 1, b:b + 1],
                           pos=cache.pos[l:l + 1, b:b + 1], len=cache.len[l:l + 1, b:b + 1], L=1, B=1, H=wl.H, d=wl.d,
                           cap=cap, dtype=kf.BF16)
            if ev:                                  # adopt the oracle's choice inside the tie band and go on
                for nm in ("K", "V", "score", "pos", "len"):
                    getattr(cache, nm)[l, b].copy_(dev(getattr(oc, nm))[0, 0])
            else:
                assert_state_equal(sub, oc, kv=(t == 3))
    print(name, "full size: tie-band events", ties)


def test_layer_offset_draws_the_full_models_noise():
    # a cache holding only layer 5 (layer0 = 5) must reproduce layer 5 of a six-layer cache
    rng = np.random.default_rng(21)
    L, B, H, d, cap, n = 6, 1, 2, 64, 80, 60
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, n)
    q, kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    seeds = np.array([99], np.uint64)
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), 500, 0, 1.25, 0.125, kf.NOISE_GUMBEL, dev(seeds), None, out, ws)
    one = ko.OracleCache(1, B, H, d, cap, ko.BF16, layer0=5)
    for nm in ("K", "V", "score", "pos", "len"):
        getattr(one, nm)[...] = getattr(oc, nm)[5:6]
    g1 = upload(one)
    ws1 = kf.new_workspace(g1)
    out1 = torch.zeros((1, B, H, d), dtype=torch.float32, device="cuda")
    kf.kf_decode_step(g1, dev(q[5:6]), dev(kn[5:6]), dev(vn[5:6]), 500, 0, 1.25, 0.125, kf.NOISE_GUMBEL, dev(seeds),
                      None, out1, ws1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(g1.score), host(gc.score)[5:6])
    out_ref = one.decode_step(q[5:6], kn[5:6], vn[5:6], 500, 1.25, 0.125, ko.NOISE_GUMBEL, seeds)
    assert_close_out(host(out1), out_ref)
    assert_close_score(host(g1.score), one.score, one.len)


# ------------------------------------------------------------------ slot-replacement layout, fused step
@pytest.mark.parametrize("name,kwargs,steps", [("tiny", {}, 32), ("mpt", dict(L=1, B=2, H=4, T=1024), 16),
                                               ("gptj", dict(L=1, H=4, T=512), 24)])
def test_slot_layout_keeps_the_same_set_as_the_oracle(name, kwargs, steps):
    wl = kw.CONFIGS[name].slice(**kwargs) if kwargs else kw.CONFIGS[name]
    ls = LockStep(wl, layout=kf.LAYOUT_SLOT)
    ls.prefill()                       # n -> k is more than one eviction: done in the ordered layout
    unordered = False
    for t in range(1, steps + 1):
        ls.step(t, check_kv=(t % 8 == 0 or t == steps))
        # the GPU cache really leaves positional order (it may pass through it again: when the
        # evicted token is always the one that just left the window the slots behave as a ring)
        unordered |= bool((np.diff(host(ls.gc.pos)[..., : wl.k], axis=-1) < 0).any())
    assert unordered
    print(name, "slot layout lockstep", ls.stats)


def test_slot_layout_rejects_more_than_one_eviction():
    rng = np.random.default_rng(31)
    oc = random_cache(rng, 1, 1, 2, 64, 40, ko.BF16, 30)
    oc.pos[...] = np.arange(40)
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    kf.kf_select_evict(gc, 20, 4, None, ws, layout=kf.LAYOUT_SLOT)
    torch.cuda.synchronize()
    assert error_word(ws) == 2 and (host(gc.len) == 30).all()
    assert_state_equal(gc, oc)         # untouched


@pytest.mark.parametrize("dtype,d,cap,layout", [(ko.BF16, 256, 1025, 0), (ko.BF16, 128, 300, 0), (ko.F32, 64, 65, 0),
                                               (ko.BF16, 128, 2049, 1), (ko.BF16, 64, 131, 1)])
def test_fused_step_equals_the_two_calls(dtype, d, cap, layout):
    """kf_decode_select_step must leave exactly what kf_decode_step + kf_select_evict leave."""
    rng = np.random.default_rng(cap + d)
    L, B, H = 2, 2, 3            # 12 units: several splits at the larger caps, one split at the small ones
    k = cap - 1
    w = k // 5
    lens = np.full((L, B, H), k, np.int32)
    lens[0, 0, 0] = k // 2                       # under budget after the step: selection must not touch it
    oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
    oc.pos[...] = np.arange(cap)                 # consecutive positions (the slot layout's window rule)
    oc.score[0, 1, 0, 10:20] = 0.0               # tied minima
    q, kn, vn = (rnd(rng, (L, B, H, d), dtype) for _ in range(3))
    seeds = np.array([5, 6], np.uint64)
    results = []
    for fused in (False, True):
        gc = upload(oc)
        ws = kf.new_workspace(gc)
        out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
        kept = torch.full((L, B, H, k), -7, dtype=torch.int32, device="cuda")
        args = (dev(q), dev(kn), dev(vn), cap + 3, 0, 1.6, 0.11, kf.NOISE_GUMBEL, dev(seeds), None, out)
        if fused:
            kf.kf_decode_select_step(gc, *args, k=k, w=w, layout=layout, kept_idx=kept, workspace=ws)
        else:
            kf.kf_decode_step(gc, *args, ws)
            kf.kf_select_evict(gc, k, w, kept, ws, layout=layout)
        torch.cuda.synchronize()
        assert error_word(ws) == 0
        lens_now = host(gc.len)
        live = [host(t).copy() for t in (gc.K, gc.V, gc.score, gc.pos)]
        for l, b, h in np.ndindex(L, B, H):          # beyond a unit's length nothing is specified (a whole-step
            for t in live:                           # launch never appends the token it places directly)
                t[l, b, h, int(lens_now[l, b, h]):] = 0
        results.append([host(out).copy(), host(kept).copy(), lens_now.copy()] + live)
    for a, b in zip(*results):
        np.testing.assert_array_equal(a, b)
    # and the two-call path is the one checked against the oracle
    ref = oc.copy()
    out_ref = ref.decode_step(q, kn, vn, cap + 3, 1.6, 0.11, ko.NOISE_GUMBEL, seeds)
    assert_close_out(results[0][0], out_ref)


@pytest.mark.parametrize("sweep_seed", SWEEP_SEEDS)
def test_fused_step_on_random_shapes_equals_the_two_calls(sweep_seed):
    """Seeded sweep: kf_decode_select_step against kf_decode_step + kf_select_evict, bit for bit, over element
    types, head sizes, query heads per cached head, few and many units (every fused launch sequence: one
    launch, split + tail, decode + select, with and without the shared score), both layouts, ragged lengths."""
    rng = np.random.default_rng(20240310 if sweep_seed is None else 888000 + sweep_seed)
    combos = [(ko.BF16, 64), (ko.BF16, 128), (ko.BF16, 256), (ko.F32, 64), (ko.F32, 128), (ko.F16, 128), (ko.F16, 64),
              (ko.F16, 256)]
    for case in range(24):
        dtype, d = combos[case % len(combos)]
        G = int(rng.choice([1, 1, 2, 4, 8]))
        layout = int(rng.integers(0, 2))
        shared = bool(rng.integers(0, 4) == 0)
        if rng.integers(0, 2):
            L, B, H = 2, int(rng.integers(5, 9)), 32
            k = int(rng.integers(30, 400)) if case % 3 else int(rng.integers(800, 1200))
        else:
            L, B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 5))
            k = int(rng.integers(8, 5000))
        cap, w = k + 1, int(rng.integers(0, k // 2 + 1))
        lens = np.full((L, B, H), k, np.int32)
        if not shared:                                   # layers of a shared score must agree in length
            lens[0, 0, 0] = int(rng.integers(0, k))      # under budget after the step: not touched
        oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
        oc.pos[...] = np.arange(cap)                     # consecutive positions (the slot layout's window rule)
        if shared:
            oc.score[...] = oc.score[0:1]
        if layout == kf.LAYOUT_SLOT:                     # any slot order
            for l, b, h in np.ndindex(L, B, H):
                n_u = int(lens[l, b, h])
                perm = rng.permutation(n_u)
                if shared:
                    perm = np.arange(n_u)
                for nm in ("K", "V", "score", "pos"):
                    getattr(oc, nm)[l, b, h, :n_u] = getattr(oc, nm)[l, b, h, :n_u][perm]
        q = rnd(rng, (L, B, H * G, d), dtype)
        kn, vn = (rnd(rng, (L, B, H, d), dtype) for _ in range(2))
        seeds = rng.integers(0, 2 ** 63, B).astype(np.uint64)
        what = "case %d: dtype=%d d=%d G=%d L,B,H=%d,%d,%d k=%d w=%d layout=%d shared=%d" % (
            case, dtype, d, G, L, B, H, k, w, layout, shared)
        print(what, flush=True)
        mode = kf.SCORE_SHARED if shared else kf.SCORE_PER_LAYER
        results = []
        for fused in (False, True):
            gc = upload(oc, G)
            ws = kf.new_workspace(gc)
            out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
            kept = torch.full((L, B, H, k), -7, dtype=torch.int32, device="cuda")
            args = (dev(q), dev(kn), dev(vn), cap + 3, 0, 1.3, 0.09, kf.NOISE_GUMBEL, dev(seeds), None, out)
            if fused:
                kf.kf_decode_select_step(gc, *args, k=k, w=w, layout=layout, kept_idx=kept, workspace=ws, score_mode=mode)
            else:
                kf.kf_decode_step(gc, *args, ws, score_mode=mode)
                kf.kf_select_evict(gc, k, w, kept, ws, layout=layout)
            torch.cuda.synchronize()
            assert error_word(ws) == 0, what
            lens_now = host(gc.len)
            live = [host(t).copy() for t in (gc.K, gc.V, gc.score, gc.pos)]
            for l, b, h in np.ndindex(L, B, H):          # beyond a unit's length nothing is specified
                for t in live:
                    t[l, b, h, int(lens_now[l, b, h]):] = 0
            results.append([host(out).copy(), host(kept).copy(), lens_now.copy()] + live)
            del gc, ws, out, kept
        for i, (a_, b_) in enumerate(zip(*results)):
            np.testing.assert_array_equal(a_, b_, err_msg="%s tensor %d" % (what, i))


def test_steps_captured_in_a_hip_graph_replay_exactly():
    """A run of fused steps captured in a HIP graph must reproduce the eager run bit for bit on every
    replay (the library records no memset nodes; eager work and synchronisation sit between replays)."""
    wl = kw.CONFIGS["gptj"].slice(L=2, H=16, T=512)      # 32 units: several splits, merge in the tail kernel
    rng = np.random.default_rng(77)
    k, cap = wl.k, wl.k + 1
    oc = random_cache(rng, wl.L, wl.B, wl.H, wl.d, cap, ko.BF16, k)
    oc.pos[...] = np.arange(cap)
    state0 = upload(oc)
    seeds = dev(kw.noise_seeds(wl))
    steps = [tuple(t.cuda() for t in kw.decode_inputs(wl, t)) for t in range(1, 7)]
    out = torch.zeros((wl.L, wl.B, wl.H, wl.d), dtype=torch.float32, device="cuda")
    gc = upload(oc)
    ws = kf.new_workspace(gc)

    def restore():
        for nm in ("K", "V", "score", "pos", "len"):
            getattr(gc, nm).copy_(getattr(state0, nm))

    def run():
        for i, (q, kn, vn) in enumerate(steps):
            kf.kf_decode_select_step(gc, q, kn, vn, cap + i, cap, kf.kf_tau(i + 1, wl.T), wl.scale, kf.NOISE_GUMBEL,
                                     seeds, None, out, k=k, w=wl.w, layout=kf.LAYOUT_ORDERED, workspace=ws)

    def snapshot():
        torch.cuda.synchronize()
        return [host(t).copy() for t in (out, gc.K, gc.V, gc.score, gc.pos, gc.len)]

    run()                               # eager reference (also loads the kernels before capture)
    ref = snapshot()
    restore()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for rep in range(4):
        restore()
        (out * 0).sum().item()          # unrelated eager work + a synchronisation between replays
        g.replay()
        got = snapshot()
        for a, b in zip(got, ref):
            np.testing.assert_array_equal(a, b)
    assert error_word(ws) == 0


@pytest.mark.parametrize("cap", [90, 900])
def test_new_pos_mode_matches_oracle(cap):
    rng = np.random.default_rng(cap)
    L, B, H, d = 1, 2, 4, 128
    lens = rng.integers(cap // 2, cap, (L, B, H)).astype(np.int32)
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)      # positions with gaps
    q, kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    seeds = np.array([3, 4], np.uint64)
    slopes = np.array([0.5, 0.125, 0.03125, 0.0], np.float32)
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    q_pos = int(oc.pos.max()) + 1
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, 0, 1.3, 0.09, kf.NOISE_GUMBEL, dev(seeds), dev(slopes),
                      out, ws, pos_mode=kf.POS_NEW)
    torch.cuda.synchronize()
    org = oc.copy()
    out_ref = oc.decode_step(q, kn, vn, q_pos, 1.3, 0.09, ko.NOISE_GUMBEL, seeds, slopes, new_pos=True)
    assert_close_out(host(out), out_ref)
    assert_close_score(host(gc.score), oc.score, oc.len)
    out_org = org.decode_step(q, kn, vn, q_pos, 1.3, 0.09, ko.NOISE_GUMBEL, seeds, slopes)
    assert np.abs(out_org - out_ref).max() > 1e-3        # the two modes really differ on this cache


@pytest.mark.parametrize("dtype,d", [(ko.BF16, 256), (ko.BF16, 64), (ko.F32, 128)])
@pytest.mark.parametrize("n,k,w", [(600, 256, 51), (257, 256, 51), (100, 64, 0)])
def test_select_evict_into_another_cache(dtype, d, n, k, w):
    """Prompt-phase eviction gathered into the (smaller) generation cache: same survivors, same rows,
    as the in-place call checked against the oracle; the source stays as it was."""
    rng = np.random.default_rng(n + k + d)
    Ls, Ld, B, H = 2, 5, 1, 3
    lens = np.full((Ls, B, H), n, np.int32)
    lens[0, 0, 1] = k - 7                      # under budget: copied whole
    oc = random_cache(rng, Ls, B, H, d, n, dtype, lens)
    oc.score[1, 0, 0, : n // 2] = 1.0          # ties
    src = upload(oc)
    dst = kf.Cache.allocate(Ld, B, H, d, k + 1, dtype)
    dst.K.fill_(9.0)
    dst.len.fill_(-3)
    ws = kf.new_workspace(src, n)
    kept = torch.full((Ls, B, H, k), -5, dtype=torch.int32, device="cuda")
    kf.kf_select_evict_into(src, dst, 2, k, w, kept, ws)
    torch.cuda.synchronize()
    assert_state_equal(src, oc)                # the source is untouched
    ref = oc.copy()
    kept_ref = ref.select_evict(k, w)
    np.testing.assert_array_equal(host(kept), kept_ref)
    view = kf.Cache(K=dst.K[2:4], V=dst.V[2:4], score=dst.score[2:4], pos=dst.pos[2:4], len=dst.len[2:4],
                    L=Ls, B=B, H=H, d=d, cap=k + 1, dtype=dtype)
    got_len = host(view.len)
    np.testing.assert_array_equal(got_len, ref.len)
    gK, gV, gs, gp = host(view.K), host(view.V), host(view.score), host(view.pos)
    for l, b, h in itertools.product(range(Ls), range(B), range(H)):
        m = int(got_len[l, b, h])
        np.testing.assert_array_equal(gK[l, b, h, :m], ref.K[l, b, h, :m])
        np.testing.assert_array_equal(gV[l, b, h, :m], ref.V[l, b, h, :m])
        np.testing.assert_array_equal(gs[l, b, h, :m], ref.score[l, b, h, :m])
        np.testing.assert_array_equal(gp[l, b, h, :m], ref.pos[l, b, h, :m])
    assert (host(dst.len)[[0, 1, 4]] == -3).all()      # other layers of the destination untouched
    # without kept_idx
    dst2 = kf.Cache.allocate(Ld, B, H, d, k + 1, dtype)
    kf.kf_select_evict_into(src, dst2, 2, k, w, None, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(dst2.pos[2:4])[..., : k - 7], gp[..., : k - 7])
    with pytest.raises(kf.KeyformerError):
        kf.kf_select_evict_into(src, dst, 4, k, w, None, ws)      # layers 4,5 do not fit
    with pytest.raises(kf.KeyformerError):
        kf.kf_select_evict_into(src, src, 0, k, w, None, ws)      # must be another cache


# ------------------------------------------------------------------ shared (cross-layer) score function
@pytest.mark.parametrize("name,kwargs,steps,layout", [
    ("tiny", dict(L=3), 32, kf.LAYOUT_ORDERED),                     # one split per unit
    ("gptj", dict(L=3, H=4, T=512), 24, kf.LAYOUT_ORDERED),         # several splits: increments pass the merge
    ("tiny", dict(L=2), 32, kf.LAYOUT_SLOT)])
def test_shared_score_lockstep(name, kwargs, steps, layout):
    wl = kw.CONFIGS[name].slice(**kwargs)
    ls = LockStep(wl, shared=True, layout=layout)
    ls.prefill()
    for t in range(1, steps + 1):
        ls.step(t, check_kv=(t == steps))
    # all layers made the same decisions
    pos = host(ls.gc.pos)
    for l in range(1, wl.L):
        np.testing.assert_array_equal(np.sort(pos[l, ..., : wl.k], axis=-1), np.sort(pos[0, ..., : wl.k], axis=-1))
    print(name, "shared-score lockstep", ls.stats)


def test_shared_score_fused_step_and_disagreeing_layers():
    rng = np.random.default_rng(77)
    L, B, H, d, cap = 3, 2, 2, 128, 301
    lens = np.broadcast_to(rng.integers(250, 300, (1, B, H)), (L, B, H)).astype(np.int32)
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    oc.pos[...] = oc.pos[0]            # shared score: all layers hold the same tokens ...
    oc.score[...] = oc.score[0]        # ... with the same scores
    q, kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    seeds = np.array([5, 6], np.uint64)
    k, w = 240, 48
    a, b_ = upload(oc), upload(oc)
    ws = kf.new_workspace(a)
    out_a = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    out_b = torch.zeros_like(out_a)
    q_pos = int(oc.pos.max()) + 1
    kf.kf_decode_step(a, dev(q), dev(kn), dev(vn), q_pos, 0, 1.4, 0.09, kf.NOISE_GUMBEL, dev(seeds), None, out_a, ws,
                      score_mode=kf.SCORE_SHARED)
    kf.kf_select_evict(a, k, w, None, ws)
    kf.kf_decode_select_step(b_, dev(q), dev(kn), dev(vn), q_pos, 0, 1.4, 0.09, kf.NOISE_GUMBEL, dev(seeds), None, out_b,
                             k=k, w=w, workspace=ws, score_mode=kf.SCORE_SHARED)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    assert torch.equal(out_a, out_b)
    for nm in ("len", "pos", "score", "K", "V"):
        ta, tb = getattr(a, nm), getattr(b_, nm)
        assert torch.equal(ta[..., :k] if nm in ("pos", "score") else (ta[..., :k, :] if nm in ("K", "V") else ta),
                           tb[..., :k] if nm in ("pos", "score") else (tb[..., :k, :] if nm in ("K", "V") else tb)), nm
    out_ref = oc.decode_step(q, kn, vn, q_pos, 1.4, 0.09, ko.NOISE_GUMBEL, seeds, None, shared=True)
    oc.select_evict(k, w)
    assert_close_out(host(out_a), out_ref)
    np.testing.assert_array_equal(host(a.pos)[..., :k], oc.pos[..., :k])
    assert_close_score(host(a.score), oc.score, oc.len)

    # layers that disagree in length cannot share a score: reported, their scores left alone
    oc2 = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    oc2.len[1, 0, 1] -= 1
    c = upload(oc2)
    ws2 = kf.new_workspace(c)
    before = c.score.clone()
    kf.kf_decode_step(c, dev(q), dev(kn), dev(vn), q_pos + 99, 0, 1.4, 0.09, kf.NOISE_GUMBEL, dev(seeds), None, out_a,
                      ws2, score_mode=kf.SCORE_SHARED)
    torch.cuda.synchronize()
    assert error_word(ws2) == 1
    assert torch.equal(c.score[:, 0, 1, :200], before[:, 0, 1, :200])
    assert not torch.equal(c.score[:, 0, 0, :200], before[:, 0, 0, :200])


# ------------------------------------------------------------------ step number in device memory
@pytest.mark.parametrize("name,kwargs,shared", [("gptj", dict(L=2, H=8, T=12), False),   # splits + fused tail
                                                ("tiny", dict(T=12), False),             # one split per unit
                                                ("long", dict(L=1, H=2, T=6), False),    # splits, merge launch with the candidate minima
                                                ("tiny", dict(L=2, T=12), True)])
def test_one_captured_step_replays_as_successive_steps(name, kwargs, shared):
    """kf_decode_select_step_at reads t from device memory (q_pos = n+t-1, tau = tau_t) and advances it: ONE
    step captured in a HIP graph, replayed with refreshed inputs, must equal the eager host-driven steps
    bit for bit -- including the steps past T, which keep tau_end."""
    wl = kw.CONFIGS[name].slice(**kwargs)
    rng = np.random.default_rng(5)
    dt = ko.F32 if wl.dtype == "f32" else ko.BF16
    k, cap = wl.k, wl.k + 1
    oc = random_cache(rng, wl.L, wl.B, wl.H, wl.d, cap, dt, k)
    oc.pos[...] = np.arange(wl.n - k, wl.n - k + cap)       # the k most recent prompt positions
    if shared:
        oc.score[...] = oc.score[0]
    seeds = dev(kw.noise_seeds(wl))
    n_steps = wl.T + 3
    inputs = [tuple(t.cuda() for t in kw.decode_inputs(wl, t)) for t in range(1, n_steps + 1)]
    mode = kf.SCORE_SHARED if shared else kf.SCORE_PER_LAYER

    # eager, host-driven reference
    a = upload(oc)
    ws_a = kf.new_workspace(a)
    out_a = torch.zeros((wl.L, wl.B, wl.H, wl.d), dtype=torch.float32, device="cuda")
    ref = []
    for t in range(1, n_steps + 1):
        q, kn, vn = inputs[t - 1]
        kf.kf_decode_select_step(a, q, kn, vn, wl.n + t - 1, cap, kf.kf_tau(min(t, wl.T), wl.T, wl.tau_init, wl.tau_end),
                                 wl.scale, kf.NOISE_GUMBEL, seeds, None, out_a, k=k, w=wl.w, workspace=ws_a,
                                 score_mode=mode)
        torch.cuda.synchronize()
        ref.append([host(x).copy() for x in (out_a, a.score, a.pos, a.len)])
    assert error_word(ws_a) == 0

    # one captured step, replayed
    b_ = upload(oc)
    ws_b = kf.new_workspace(b_)
    out_b = torch.zeros_like(out_a)
    step = torch.ones(1, dtype=torch.int32, device="cuda")
    qb, kb, vb = (torch.empty_like(x) for x in inputs[0])

    def one():
        kf.kf_decode_select_step_at(b_, qb, kb, vb, wl.n, wl.T, wl.tau_init, wl.tau_end, step, cap, wl.scale,
                                    kf.NOISE_GUMBEL, seeds, None, out_b, k=k, w=wl.w, workspace=ws_b, score_mode=mode)

    for src, dst in zip(inputs[0], (qb, kb, vb)):
        dst.copy_(src)
    one()                                  # step 1 eagerly (loads the kernels before the capture)
    torch.cuda.synchronize()
    assert int(step.item()) == 2
    for x, y in zip([host(x) for x in (out_b, b_.score, b_.pos, b_.len)], ref[0]):
        np.testing.assert_array_equal(x, y)
    g = torch.cuda.CUDAGraph()
    state = [x.clone() for x in (b_.K, b_.V, b_.score, b_.pos, b_.len)]
    with torch.cuda.graph(g):
        one()
    # the capture did not execute anything: restore is not needed, but the counter must still say 2
    torch.cuda.synchronize()
    assert int(step.item()) == 2
    for x, y in zip((b_.K, b_.V, b_.score, b_.pos, b_.len), state):
        assert torch.equal(x, y)
    for t in range(2, n_steps + 1):
        for src, dst in zip(inputs[t - 1], (qb, kb, vb)):
            dst.copy_(src)
        (out_b * 0).sum().item()           # unrelated eager work + a synchronisation between replays
        g.replay()
        torch.cuda.synchronize()
        assert int(step.item()) == t + 1
        for x, y in zip([host(x) for x in (out_b, b_.score, b_.pos, b_.len)], ref[t - 1]):
            np.testing.assert_array_equal(x, y)
    assert error_word(ws_b) == 0


# ------------------------------------------------------------------ grouped-query attention
@pytest.mark.parametrize("dtype,d", DTYPES)
@pytest.mark.parametrize("G", [2, 4, 8])
@pytest.mark.parametrize("cap", [97, 1300])      # one split per unit; several splits (ragged last one) and a merge
def test_grouped_query_decode_matches_oracle(dtype, d, G, cap):
    rng = np.random.default_rng(7000 + d + cap + G)
    L, B, H = 2, 2, 2                              # cached heads; G query heads each
    lens = rng.integers(cap // 2, cap, (L, B, H)).astype(np.int32)
    lens[0, 0, 0] = 0
    lens[0, 0, 1] = cap - 1
    lens[1, 1, 1] = cap                            # full: skipped and reported
    oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
    gc = upload(oc, G)
    ws = kf.new_workspace(gc)
    q = rnd(rng, (L, B, H * G, d), dtype)
    kn, vn = (rnd(rng, (L, B, H, d), dtype) for _ in range(2))
    seeds = np.array([11, 2 ** 63 + 12], np.uint64)
    slopes = (0.7 ** np.arange(1, H * G + 1)).astype(np.float32)
    q_pos = int(oc.pos.max()) + 2
    tau, scale = 1.3125, float(1.0 / np.sqrt(np.float32(d)))
    out = torch.full((L, B, H * G, d), 7.0, dtype=torch.float32, device="cuda")
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, 0, tau, scale, kf.NOISE_GUMBEL, dev(seeds), dev(slopes),
                      out, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 1
    oc.len[1, 1, 1] = 0                            # the oracle refuses a full unit: run it emptied, skip it below
    out_ref = oc.decode_step(q, kn, vn, q_pos, tau, scale, ko.NOISE_GUMBEL, seeds, slopes, q_per_kv=G)
    ok = np.ones((L, B, H), bool)
    ok[1, 1, 1] = False
    okq = np.repeat(ok, G, axis=2)
    got_out, got_len = host(out), host(gc.len)
    assert (got_out[~okq] == 0).all() and got_len[1, 1, 1] == cap
    assert (got_len[ok] == oc.len[ok]).all()
    assert_close_out(got_out[okq], out_ref[okq])
    assert_close_score(host(gc.score), oc.score, np.where(ok, oc.len, 0))
    gK, gpos = host(gc.K), host(gc.pos)
    for l, b, h in itertools.product(range(L), range(B), range(H)):
        if ok[l, b, h]:
            m = int(oc.len[l, b, h])
            np.testing.assert_array_equal(gK[l, b, h, :m], oc.K[l, b, h, :m])
            np.testing.assert_array_equal(gpos[l, b, h, :m], oc.pos[l, b, h, :m])


@pytest.mark.parametrize("dtype,d,G", [(ko.BF16, 128, 4), (ko.BF16, 256, 2), (ko.F32, 64, 8)])
@pytest.mark.parametrize("n", [33, 300])
def test_grouped_query_prefill_matches_oracle(dtype, d, G, n):
    rng = np.random.default_rng(7100 + d + n)
    L, B, H = 1, 2, 2
    oc = random_cache(rng, L, B, H, d, n + 7, dtype, 0)
    Q = rnd(rng, (L, B, H * G, n, d), dtype)
    seeds = np.array([5, 6], np.uint64)
    slopes = (0.5 ** np.arange(1, H * G + 1)).astype(np.float32)
    gc = upload(oc, G)
    ws = kf.new_workspace(gc, n)
    scale = float(1.0 / np.sqrt(np.float32(d)))
    kf.kf_prefill_score(gc, dev(Q), n, 1.0, scale, kf.NOISE_GUMBEL, dev(seeds), dev(slopes), ws)
    torch.cuda.synchronize()
    oc.prefill_score(Q, n, 1.0, scale, ko.NOISE_GUMBEL, seeds, slopes, q_per_kv=G)
    np.testing.assert_array_equal(host(gc.len), oc.len)
    np.testing.assert_array_equal(host(gc.pos)[..., :n], oc.pos[..., :n])
    assert_close_score(host(gc.score), oc.score, oc.len, "grouped prefill score", rtol=SCORE_RTOL_PREFILL)


@pytest.mark.parametrize("G,shared,layout", [(4, False, kf.LAYOUT_ORDERED), (2, True, kf.LAYOUT_ORDERED),
                                            (8, False, kf.LAYOUT_SLOT)])
def test_grouped_query_lockstep(G, shared, layout):
    # mpt-like per-unit shape with position bias: 8 query heads on 8/G cached heads, prompt to generation
    wl = kw.CONFIGS["mpt"].slice(L=2 if shared else 1, B=2, H=8, T=1024, n=512, k=256, w=51)
    ls = LockStep(wl, q_per_kv=G, shared=shared, layout=layout)
    ls.prefill()
    for t in range(1, 25):
        ls.step(t, check_kv=(t == 24))
    print("grouped-query lockstep G=%d" % G, ls.stats)


def test_grouped_query_fused_and_device_step_equal_the_two_calls():
    rng = np.random.default_rng(7200)
    L, B, H, d, G, cap = 1, 2, 2, 128, 4, 701
    k, w = 700, 140
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, k)
    oc.pos[...] = np.arange(cap)
    q = rnd(rng, (L, B, H * G, d), ko.BF16)
    kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(2))
    seeds = dev(np.array([1, 2], np.uint64))
    n, T, t = 1000, 64, 9
    q_pos, tau = n + t - 1, kf.kf_tau(t, T, 1.0, 2.0)
    caches = [upload(oc, G) for _ in range(3)]
    wss = [kf.new_workspace(c) for c in caches]
    outs = [torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda") for _ in range(3)]
    kf.kf_decode_step(caches[0], dev(q), dev(kn), dev(vn), q_pos, 0, tau, 0.09, kf.NOISE_GUMBEL, seeds, None, outs[0],
                      wss[0])
    kf.kf_select_evict(caches[0], k, w, None, wss[0])
    kf.kf_decode_select_step(caches[1], dev(q), dev(kn), dev(vn), q_pos, 0, tau, 0.09, kf.NOISE_GUMBEL, seeds, None,
                             outs[1], k=k, w=w, workspace=wss[1])
    step = torch.full((1,), t, dtype=torch.int32, device="cuda")
    kf.kf_decode_select_step_at(caches[2], dev(q), dev(kn), dev(vn), n, T, 1.0, 2.0, step, 0, 0.09, kf.NOISE_GUMBEL,
                                seeds, None, outs[2], k=k, w=w, workspace=wss[2])
    torch.cuda.synchronize()
    assert int(step.item()) == t + 1
    for i in (1, 2):
        assert error_word(wss[i]) == 0
        assert torch.equal(outs[0], outs[i])
        assert torch.equal(caches[0].len, caches[i].len)
        for nm in ("score", "pos"):
            assert torch.equal(getattr(caches[0], nm)[..., :k], getattr(caches[i], nm)[..., :k]), nm
        for nm in ("K", "V"):
            assert torch.equal(getattr(caches[0], nm)[..., :k, :], getattr(caches[i], nm)[..., :k, :]), nm


def test_grouped_query_decode_at_the_largest_lds_footprint():
    # 1024 units fill the chip without splits: one workgroup per unit keeps 8 x 489 logit slots (twice) and
    # four 8 x 256 output rows in LDS -- the most the launch plan allows
    rng = np.random.default_rng(7300)
    L, B, H, d, G, cap = 4, 8, 32, 256, 8, 488
    c0 = kf.Cache(K=0x10000, V=0x20000, score=0x30000, pos=0x40000, len=0x50000, L=L, B=B, H=H, d=d, cap=cap,
                  dtype=kf.BF16, q_per_kv=G)
    assert kf.kf_decode_launch_shape(c0, cap) == (1, 488)
    lens = rng.integers(cap - 40, cap, (L, B, H)).astype(np.int32)
    lens[0, 0, 0] = cap - 1
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    gc = upload(oc, G)
    ws = kf.new_workspace(gc)
    q = rnd(rng, (L, B, H * G, d), ko.BF16)
    kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(2))
    seeds = np.arange(B).astype(np.uint64) + 77
    q_pos = int(oc.pos.max()) + 1
    out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, cap, 1.5, 0.0625, kf.NOISE_GUMBEL, dev(seeds), None, out, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    out_ref = oc.decode_step(q, kn, vn, q_pos, 1.5, 0.0625, ko.NOISE_GUMBEL, seeds, None, q_per_kv=G)
    assert_close_out(host(out), out_ref)
    assert_close_score(host(gc.score), oc.score, oc.len)


@pytest.mark.parametrize("dtype,d,G,noise,new_pos,cap", [
    (ko.BF16, 128, 8, ko.NOISE_GUMBEL, False, 2049), (ko.BF16, 64, 8, ko.NOISE_GAUSSIAN, True, 1500),
    (ko.BF16, 256, 8, ko.NOISE_NONE, False, 1500), (ko.BF16, 128, 4, ko.NOISE_GUMBEL, False, 4097),
    (ko.BF16, 64, 4, ko.NOISE_GUMBEL, True, 1500), (ko.BF16, 256, 4, ko.NOISE_CONSTANT, False, 900),
    (ko.F32, 64, 4, ko.NOISE_GUMBEL, False, 1100), (ko.F16, 128, 8, ko.NOISE_GUMBEL, False, 2049),
    (ko.F16, 64, 8, ko.NOISE_GUMBEL, True, 700), (ko.F16, 256, 4, ko.NOISE_GAUSSIAN, False, 1200)])
def test_grouped_query_one_eight_wave_workgroup_per_unit(dtype, d, G, noise, new_pos, cap):
    """4 or 8 query heads per cached head, a unit per compute unit and more than a few hundred tokens: one
    8-wave workgroup streams a whole unit (8 bf16 heads: logits on the matrix cores; partial outputs folded as a
    reduce-scatter into the logit area)."""
    rng = np.random.default_rng(7400 + d + G)
    L, B, H = 2, 8, 16
    c0 = kf.Cache(K=0x10000, V=0x20000, score=0x30000, pos=0x40000, len=0x50000, L=L, B=B, H=H, d=d, cap=cap,
                  dtype=dtype, q_per_kv=G)
    S, chunk = kf.kf_decode_launch_shape(c0, cap)
    assert S == 1 and chunk >= cap - 1
    lens = rng.integers(cap - 300, cap, (L, B, H)).astype(np.int32)
    lens[0, 0, 0] = 0            # the new token alone
    lens[0, 0, 1] = cap - 1      # fills the cache exactly
    lens[0, 0, 2] = 15           # less than one 16-row tile of one wave
    lens[0, 0, 3] = 129          # one row into the second sweep of the 8 waves
    lens[1, 7, 15] = cap         # no room: skipped and reported
    oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
    gc = upload(oc, G)
    ws = kf.new_workspace(gc)
    q = rnd(rng, (L, B, H * G, d), dtype)
    kn, vn = (rnd(rng, (L, B, H, d), dtype) for _ in range(2))
    seeds = (np.arange(B) * 7 + 1).astype(np.uint64)
    slopes = (0.5 ** (np.arange(1, H * G + 1) / 16.0)).astype(np.float32) * 0.05
    q_pos = int(oc.pos.max()) + 1
    out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
    scale = float(1.0 / np.sqrt(np.float32(d)))
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, cap, 1.5, scale, noise, dev(seeds), dev(slopes), out, ws,
                      pos_mode=kf.POS_NEW if new_pos else kf.POS_ORIGINAL)
    torch.cuda.synchronize()
    assert error_word(ws) == 1
    oc.len[1, 7, 15] = 0         # the oracle refuses the whole call for a full unit: let it skip that one
    out_ref = oc.decode_step(q, kn, vn, q_pos, 1.5, scale, noise, seeds, slopes, q_per_kv=G, new_pos=new_pos)
    g_out, g_len = host(out), host(gc.len)
    assert (g_out[1, 7, 15 * G:(15 + 1) * G] == 0).all() and g_len[1, 7, 15] == cap
    g_out[1, 7, 15 * G:(15 + 1) * G] = out_ref[1, 7, 15 * G:(15 + 1) * G]
    assert_close_out(g_out, out_ref)
    g_len[1, 7, 15] = oc.len[1, 7, 15]
    np.testing.assert_array_equal(g_len, oc.len)
    g_score = host(gc.score)
    g_score[1, 7, 15] = oc.score[1, 7, 15]
    assert_close_score(g_score, oc.score, oc.len)


@pytest.mark.parametrize("d,layout", [(128, kf.LAYOUT_ORDERED), (64, kf.LAYOUT_SLOT)])
def test_eight_wave_workgroup_on_units_of_a_few_tokens(d, layout):
    """8 query heads, a launch shaped for a 2048-token budget (one 8-wave workgroup per unit) on units that
    hold a few tokens only, as early in a generation or with a ragged batch: most waves of a workgroup find
    no rows of their own and must still wait for the softmax sums before they normalise the increments."""
    rng = np.random.default_rng(8800 + d)
    L, B, H, G, cap = 2, 8, 16, 8, 2049
    c0 = kf.Cache(K=0x10000, V=0x20000, score=0x30000, pos=0x40000, len=0x50000, L=L, B=B, H=H, d=d, cap=cap,
                  dtype=ko.BF16, q_per_kv=G)
    S, chunk = kf.kf_decode_launch_shape(c0, cap)
    assert S == 1 and chunk >= cap - 1
    lens = rng.integers(0, 40, (L, B, H)).astype(np.int32)
    lens[0, 0, :4] = [0, 1, 15, 17]
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    oc.pos[...] = np.arange(cap, dtype=np.int32) + 100          # consecutive: what the slot layout's window test expects
    gc = upload(oc, G)
    ws = kf.new_workspace(gc)
    seeds = (np.arange(B) * 5 + 3).astype(np.uint64)
    out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
    scale = float(1.0 / np.sqrt(np.float32(d)))
    for t in range(3):
        q = rnd(rng, (L, B, H * G, d), ko.BF16)
        kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(2))
        q_pos = 100 + cap + t
        kf.kf_decode_select_step(gc, dev(q), dev(kn), dev(vn), q_pos, cap, 1.25, scale, kf.NOISE_GUMBEL, dev(seeds), None,
                                 out, k=cap - 1, w=16, layout=layout, workspace=ws)
        torch.cuda.synchronize()
        assert error_word(ws) == 0
        out_ref = oc.decode_step(q, kn, vn, q_pos, 1.25, scale, ko.NOISE_GUMBEL, seeds, None, q_per_kv=G)
        assert_close_out(host(out), out_ref, "step %d" % t)
        np.testing.assert_array_equal(host(gc.len), oc.len)        # far under budget: nothing is evicted
        assert_close_score(host(gc.score), oc.score, oc.len, "step %d" % t)
        np.testing.assert_array_equal(host(gc.pos)[..., :40], oc.pos[..., :40])


@pytest.mark.parametrize("d,G,cap", [(64, 1, 10501), (128, 2, 5401)])
def test_long_units_one_eight_wave_workgroup_per_unit(d, G, cap):
    """Units whose logits no longer fit a compute unit's LDS twice (about 10 k tokens with one query head) but
    still fit it once stay one workgroup's, of 8 waves: no increments through memory, no merge launch."""
    rng = np.random.default_rng(7500 + d + G)
    L, B, H = 1, 10, 32
    c0 = kf.Cache(K=0x10000, V=0x20000, score=0x30000, pos=0x40000, len=0x50000, L=L, B=B, H=H, d=d, cap=cap,
                  dtype=kf.BF16, q_per_kv=G)
    S, chunk = kf.kf_decode_launch_shape(c0, cap)
    assert S == 1 and chunk >= cap - 1
    lens = rng.integers(cap - 2000, cap, (L, B, H)).astype(np.int32)
    lens[0, 0, 0] = cap - 1
    lens[0, 0, 1] = 3
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    gc = upload(oc, G)
    ws = kf.new_workspace(gc)
    q = rnd(rng, (L, B, H * G, d), ko.BF16)
    kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(2))
    seeds = (np.arange(B) * 11 + 5).astype(np.uint64)
    slopes = (0.5 ** (np.arange(1, H * G + 1) / 8.0)).astype(np.float32) * 0.01
    q_pos = int(oc.pos.max()) + 1
    out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
    scale = float(1.0 / np.sqrt(np.float32(d)))
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, cap, 1.25, scale, kf.NOISE_GUMBEL, dev(seeds), dev(slopes), out, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    out_ref = oc.decode_step(q, kn, vn, q_pos, 1.25, scale, ko.NOISE_GUMBEL, seeds, slopes, q_per_kv=G)
    assert_close_out(host(out), out_ref)
    np.testing.assert_array_equal(host(gc.len), oc.len)
    assert_close_score(host(gc.score), oc.score, oc.len)


@pytest.mark.parametrize("H,G,cap", [(1, 1, 20001), (2, 2, 12001)])
def test_one_long_unit_in_more_than_64_splits(H, G, cap):
    """One or two long units are cut into more splits than a wave has lanes: the merge then holds two
    partial records per lane.  Decode call, and the whole step against the two calls."""
    rng = np.random.default_rng(9100 + G)
    L, B, d = 1, 1, 128
    c0 = kf.Cache(K=0x10000, V=0x20000, score=0x30000, pos=0x40000, len=0x50000, L=L, B=B, H=H, d=d, cap=cap,
                  dtype=kf.BF16, q_per_kv=G)
    S, chunk = kf.kf_decode_launch_shape(c0, cap)
    assert S > 64
    lens = np.full((L, B, H), cap - 1, np.int32)
    lens[0, 0, H - 1] = cap - 1 - 3 * chunk - 5  # the last splits of this unit are empty
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    gc, g2 = upload(oc, G), upload(oc, G)
    ws, ws2 = kf.new_workspace(gc), kf.new_workspace(g2)
    q = rnd(rng, (L, B, H * G, d), ko.BF16)
    kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(2))
    seeds = np.array([77], np.uint64)
    q_pos = int(oc.pos.max()) + 1
    out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
    scale = float(1.0 / np.sqrt(np.float32(d)))
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, cap, 1.5, scale, kf.NOISE_GUMBEL, dev(seeds), None, out, ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    out_ref = oc.decode_step(q, kn, vn, q_pos, 1.5, scale, ko.NOISE_GUMBEL, seeds, None, q_per_kv=G)
    assert_close_out(host(out), out_ref)
    np.testing.assert_array_equal(host(gc.len), oc.len)
    assert_close_score(host(gc.score), oc.score, oc.len)
    # the whole step on a second copy equals the two calls on the first
    k, w = cap - 1, (cap - 1) // 5
    out2 = torch.zeros_like(out)
    kf.kf_select_evict(gc, k, w, None, ws, layout=kf.LAYOUT_ORDERED)
    kf.kf_decode_select_step(g2, dev(q), dev(kn), dev(vn), q_pos, cap, 1.5, scale, kf.NOISE_GUMBEL, dev(seeds), None, out2,
                             k=k, w=w, layout=kf.LAYOUT_ORDERED, workspace=ws2)
    torch.cuda.synchronize()
    assert error_word(ws) == 0 and error_word(ws2) == 0
    np.testing.assert_array_equal(host(out2), host(out))
    ln = host(gc.len)
    np.testing.assert_array_equal(host(g2.len), ln)
    for h in range(H):
        n = int(ln[0, 0, h])
        np.testing.assert_array_equal(host(g2.pos)[0, 0, h, :n], host(gc.pos)[0, 0, h, :n])
        np.testing.assert_array_equal(host(g2.score)[0, 0, h, :n], host(gc.score)[0, 0, h, :n])


@pytest.mark.parametrize("G,layout,k", [(1, 0, 6000), (1, 1, 6000), (2, 1, 6000), (4, 0, 6000),
                                        (1, 0, 1500), (1, 1, 1500), (8, 1, 1500), (2, 0, 1500)])
def test_fused_step_of_few_split_units_equals_the_two_calls(G, layout, k):
    """Few units in splits: in the fused step the merge, which has every final score in a register once,
    also finds the smallest eviction candidate -- per slice in the merge launch of units of several
    thousand tokens (the selection's own scan launch is skipped), for the whole unit where the merge rides
    in the selection launch.  One unit is under budget, one is full: the decode refuses it and reports it,
    the selection still evicts from it -- in both forms."""
    rng = np.random.default_rng(4400 + 10 * G + layout + k)
    L, B, H, d = 1, 2, 3, 128
    cap, w = k + 1, k // 8
    lens = np.full((L, B, H), k, np.int32)
    lens[0, 0, 1] = k - 5
    lens[0, 1, 2] = cap
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    oc.pos[...] = np.arange(cap)
    oc.score[0, 1, 0, 17] = oc.score[0, 1, 0, 2 * k // 3] = -1.0  # two far-apart slices hold the smallest scores
    if layout == kf.LAYOUT_SLOT:
        for l, b, h in np.ndindex(L, B, H):
            n_u = int(lens[l, b, h])
            perm = rng.permutation(n_u)
            if n_u == cap:
                perm[n_u - 1:] = n_u - 1                   # the newest entry of a unit over budget sits in the last slot
                perm[:n_u - 1] = rng.permutation(n_u - 1)
            for nm in ("K", "V", "score", "pos"):
                getattr(oc, nm)[l, b, h, :n_u] = getattr(oc, nm)[l, b, h, :n_u][perm]
    q = rnd(rng, (L, B, H * G, d), ko.BF16)
    kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(2))
    seeds = rng.integers(0, 2 ** 63, B).astype(np.uint64)
    results = []
    for fused in (False, True):
        gc = upload(oc, G)
        S, _ = kf.kf_decode_launch_shape(gc, cap)
        assert S > 1
        ws = kf.new_workspace(gc)
        out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
        kept = torch.full((L, B, H, k), -7, dtype=torch.int32, device="cuda")
        args = (dev(q), dev(kn), dev(vn), cap + 3, 0, 1.3, 0.09, kf.NOISE_GUMBEL, dev(seeds), None, out)
        if fused:
            kf.kf_decode_select_step(gc, *args, k=k, w=w, layout=layout, kept_idx=kept, workspace=ws)
        else:
            kf.kf_decode_step(gc, *args, ws)
            kf.kf_select_evict(gc, k, w, kept, ws, layout=layout)
        torch.cuda.synchronize()
        assert error_word(ws) == 1                      # the full unit
        lens_now = host(gc.len)
        assert lens_now[0, 0, 1] == k - 4 and lens_now[0, 1, 2] == k and lens_now[0, 0, 0] == k
        live = [host(t).copy() for t in (gc.K, gc.V, gc.score, gc.pos)]
        for l, b, h in np.ndindex(L, B, H):
            for t in live:
                t[l, b, h, int(lens_now[l, b, h]):] = 0
        kept_h = host(kept).copy()
        kept_h[0, 0, 1] = 0                             # under budget: no survivor list
        results.append([host(out).copy(), kept_h, lens_now.copy()] + live)
    for i, (a_, b_) in enumerate(zip(*results)):
        np.testing.assert_array_equal(a_, b_, err_msg="tensor %d" % i)


@pytest.mark.parametrize("sweep_seed", SWEEP_SEEDS)
def test_decode_step_on_random_shapes_matches_oracle(sweep_seed):
    """Seeded sweep over the decode call's shape space: element types, head sizes, query heads per cached
    head, few and many units (one workgroup per unit or splits, 4- and 8-wave workgroups), ragged lengths,
    every logit adjustment, both position modes, with and without a position bias (30 shapes)."""
    rng = np.random.default_rng(20240309 if sweep_seed is None else 777000 + sweep_seed)
    combos = [(ko.BF16, 64), (ko.BF16, 128), (ko.BF16, 256), (ko.F32, 64), (ko.F32, 128), (ko.F16, 128), (ko.F16, 64),
              (ko.F16, 256)]
    seen = set()
    for case in range(30):
        dtype, d = combos[case % len(combos)]
        G = int(rng.choice([1, 2, 4, 8]))
        many = bool(rng.integers(0, 2))
        if many:                                    # enough units for the one-workgroup-per-unit shapes
            L, B, H = 2, int(rng.integers(5, 9)), 32
            cap = int(rng.integers(40, 420)) if case % 3 else int(rng.integers(900, 1300))
        else:
            L, B, H = 1, int(rng.integers(1, 4)), int(rng.integers(1, 5))
            cap = int(rng.integers(2, 3000))
        lens = rng.integers(0, cap, (L, B, H)).astype(np.int32)
        lens.flat[0] = cap - 1
        lens.flat[-1] = 0
        noise = int(rng.choice([ko.NOISE_GUMBEL, ko.NOISE_GUMBEL, ko.NOISE_NONE, ko.NOISE_GAUSSIAN, ko.NOISE_CONSTANT]))
        new_pos = bool(rng.integers(0, 2))
        slopes = (rng.random(H * G) * 0.05).astype(np.float32) if rng.integers(0, 2) else None
        tau = float(np.float32(rng.uniform(0.7, 2.5)))
        oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
        gc = upload(oc, G)
        seen.add((G, kf.kf_decode_launch_shape(gc, cap)[0] == 1))
        ws = kf.new_workspace(gc)
        q = rnd(rng, (L, B, H * G, d), dtype)
        kn, vn = (rnd(rng, (L, B, H, d), dtype) for _ in range(2))
        seeds = rng.integers(0, 2 ** 63, B).astype(np.uint64)
        q_pos = int(oc.pos.max()) + int(rng.integers(1, 5))
        out = torch.full((L, B, H * G, d), 3.0, dtype=torch.float32, device="cuda")
        scale = float(1.0 / np.sqrt(np.float32(d)))
        what = "case %d: dtype=%d d=%d G=%d L,B,H=%d,%d,%d cap=%d noise=%d new_pos=%d slopes=%s" % (
            case, dtype, d, G, L, B, H, cap, noise, new_pos, slopes is not None)
        print(what, flush=True)
        kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, 0, tau, scale, noise, dev(seeds),
                          None if slopes is None else dev(slopes), out, ws,
                          pos_mode=kf.POS_NEW if new_pos else kf.POS_ORIGINAL)
        torch.cuda.synchronize()
        assert error_word(ws) == 0, what
        out_ref = oc.decode_step(q, kn, vn, q_pos, tau, scale, noise, seeds, slopes, q_per_kv=G, new_pos=new_pos)
        assert_close_out(host(out), out_ref, what)
        np.testing.assert_array_equal(host(gc.len), oc.len)
        assert_close_score(host(gc.score), oc.score, oc.len, what)
        gpos = host(gc.pos)
        for l, b, h in np.ndindex(L, B, H):
            m = int(oc.len[l, b, h])
            np.testing.assert_array_equal(gpos[l, b, h, :m], oc.pos[l, b, h, :m])
        del gc, ws, out
    if sweep_seed is None:
        assert len(seen) >= 7, seen                 # both launch shapes for (nearly) every group size


# ------------------------------------------------------------------ sequences at different steps
@pytest.mark.parametrize("cap,layout", [(120, kf.LAYOUT_ORDERED), (1500, kf.LAYOUT_ORDERED), (300, kf.LAYOUT_SLOT)])
def test_per_sequence_position_and_temperature(cap, layout):
    rng = np.random.default_rng(cap)
    L, B, H, d = 2, 3, 4, 128
    k, w = cap - 1, (cap - 1) // 5
    lens = np.broadcast_to(np.array([k, k - 7, k // 2], np.int32)[None, :, None], (L, B, H)).copy()
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    q, kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(3))
    seeds = np.array([1, 2, 3], np.uint64)
    slopes = np.array([0.5, 0.25, 0.0, 0.01], np.float32)
    oc.pos[...] = np.arange(cap)           # consecutive positions, as a generation leaves them at the recent end
    q_pos = lens[0, :, 0].copy()           # every sequence appends its own next position
    taus = np.array([1.0, 1.5, 1.96875], np.float32)
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    kept = torch.zeros((L, B, H, k), dtype=torch.int32, device="cuda")
    kf.kf_decode_select_step(gc, dev(q), dev(kn), dev(vn), 0, 0, 1.0, 0.09, kf.NOISE_GUMBEL, dev(seeds), dev(slopes), out,
                             k=k, w=w, layout=layout, kept_idx=kept, workspace=ws, seq_q_pos=dev(q_pos), seq_tau=dev(taus))
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    out_ref = oc.decode_step(q, kn, vn, 0, 1.0, 0.09, ko.NOISE_GUMBEL, seeds, slopes, q_pos_seq=q_pos, tau_seq=taus)
    assert_close_out(host(out), out_ref)
    before_score, before_len = oc.score.copy(), oc.len.copy()
    kept_ref = oc.select_evict(k, w)
    np.testing.assert_array_equal(host(gc.len), oc.len)          # only the sequence that was full lost a token
    if layout == kf.LAYOUT_ORDERED:
        assert compare_kept(host(kept), kept_ref, before_score, before_len, k, w) == 0
        assert_state_equal(gc, oc, kv=True, score_exact=False)
        assert_close_score(host(gc.score), oc.score, oc.len)
    else:
        assert_set_equal(gc, oc, kv=True, score_exact=False)


# ------------------------------------------------------------------ beam search: one cache per beam
@pytest.mark.parametrize("dtype,d,cap", [(ko.BF16, 128, 700), (ko.BF16, 256, 65), (ko.F32, 64, 130)])
def test_beam_fork_matches_oracle(dtype, d, cap):
    rng = np.random.default_rng(8100 + d)
    L, B, H = 3, 6, 4
    lens = rng.integers(0, cap + 1, (L, B, H)).astype(np.int32)
    lens[0, 0, 0] = cap
    lens[0, 0, 1] = 0
    oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
    gc = upload(oc)
    ws = kf.new_workspace(gc)
    before = oc.copy()
    parent = np.array([0, 0, 2, 0, 2, 5], np.int32)          # beams 1, 3 continue beam 0; beam 4 continues beam 2
    kf.kf_beam_fork(gc, dev(parent), ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 0
    oc.beam_fork(parent)
    assert_state_equal(gc, oc, kv=True, score_exact=True)
    # beyond the copied entries a row keeps what it had
    gK = host(gc.K)
    for l, b, h in np.ndindex(L, B, H):
        m = int(oc.len[l, b, h])
        np.testing.assert_array_equal(gK[l, b, h, m:], before.K[l, b, h, m:])
    # parents that do not continue themselves, or lie outside the batch: those rows are left alone and counted
    bad = np.array([1, 0, 2, 7, -1, 5], np.int32)
    ref = oc.copy()
    kf.kf_beam_fork(gc, dev(bad), ws)
    torch.cuda.synchronize()
    assert error_word(ws) == 4 * L * H
    assert_state_equal(gc, ref, kv=True, score_exact=True)


def test_beam_search_steps_in_lockstep_with_the_oracle():
    """Four beams of one prompt (Sec. 4): after every step some beams are replaced by continuations of
    others; forked beams then answer exactly like a cache that had lived that hypothesis from the start."""
    rng = np.random.default_rng(8200)
    wl = kw.CONFIGS["tiny"].slice(B=1)
    L, H, d, n, k, w = wl.L, wl.H, wl.d, wl.n, wl.k, wl.w
    B = 4
    dtype = ko.F32 if wl.dtype == "f32" else ko.BF16
    oc = ko.OracleCache(L, B, H, d, n, dtype)
    K1 = rnd(rng, (L, 1, H, n, d), dtype)
    V1 = rnd(rng, (L, 1, H, n, d), dtype)
    Q1 = rnd(rng, (L, 1, H, n, d), dtype)
    oc.K[...] = np.repeat(K1, B, axis=1)                     # the beams share the prompt
    oc.V[...] = np.repeat(V1, B, axis=1)
    Q = np.repeat(Q1, B, axis=1)
    seeds = np.full(B, 77, np.uint64)                        # one sequence: one noise stream for all its beams
    T = 12
    gc = upload(oc)
    ws = kf.new_workspace(gc, n)
    kf.kf_prefill_score(gc, dev(Q), n, kf.kf_tau(0, T), wl.scale, kf.NOISE_GUMBEL, dev(seeds), None, ws)
    oc.prefill_score(Q, n, ko.tau(0, T), wl.scale, ko.NOISE_GUMBEL, seeds)
    kf.kf_select_evict(gc, k, w, None, ws)
    oc.select_evict(k, w)
    out = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    parents = [[0, 0, 2, 3], [0, 1, 1, 1], [0, 1, 2, 3], [3, 3, 3, 3], [0, 0, 2, 2]]
    for t in range(1, T + 1):
        q, kn, vn = (rnd(rng, (L, B, H, d), dtype) for _ in range(3))   # every beam appends its own token
        kf.kf_decode_select_step(gc, dev(q), dev(kn), dev(vn), n + t - 1, k + 1, kf.kf_tau(t, T), wl.scale,
                                 kf.NOISE_GUMBEL, dev(seeds), None, out, k=k, w=w, layout=kf.LAYOUT_ORDERED, workspace=ws)
        out_ref = oc.decode_step(q, kn, vn, n + t - 1, ko.tau(t, T), wl.scale, ko.NOISE_GUMBEL, seeds)
        oc.select_evict(k, w)
        torch.cuda.synchronize()
        assert_close_out(host(out), out_ref, "out step %d" % t)
        np.testing.assert_array_equal(host(gc.pos)[..., :k], oc.pos[..., :k])
        parent = np.array(parents[t % len(parents)], np.int32)
        kf.kf_beam_fork(gc, dev(parent), ws)
        oc.beam_fork(parent)
        torch.cuda.synchronize()
        assert error_word(ws) == 0
        assert_state_equal(gc, oc, kv=True, score_exact=False)
        upload_into(gc, oc, kv=False)                        # scores: continue from the oracle's bits
    assert_close_score(host(gc.score), oc.score, oc.len)


# ------------------------------------------------------------------ IEEE half caches
@pytest.mark.parametrize("name,layout", [("gptj", kf.LAYOUT_ORDERED), ("mpt", kf.LAYOUT_SLOT)])
def test_half_precision_cache_lockstep(name, layout):
    """The gptj- and mpt-shaped slices with K, V and Q held as IEEE half instead of bf16: prompt scoring,
    first eviction and generation steps in lock-step with the oracle."""
    import dataclasses
    wl = dataclasses.replace(kw.CONFIGS[name].slice(L=1, B=1 if name == "gptj" else 2, H=4, n=512, k=256, w=51, T=64),
                             dtype="f16")
    ls = LockStep(wl, layout=layout)
    ls.prefill()
    for t in range(1, 17):
        ls.step(t, check_kv=(t == 16))
    print("half lockstep", name, ls.stats)


# ------------------------------------------------------------------ the C ABI without Python
def test_standalone_cpp_user_of_the_c_abi():
    """examples/generate_loop.cpp: hipMalloc'ed buffers, prompt scoring, eviction into the generation cache,
    then 30 steps replayed from one captured HIP-graph step; it checks Algorithm 1's invariants itself."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(kf.lib_path()), "examples", "generate_loop")
    if not os.path.exists(exe):
        pytest.skip("examples/generate_loop is not built (python -m paper_2403_09054_amd.build builds it)")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, r.stderr
    assert "all invariants hold" in r.stdout


# ------------------------------------------------------------------ whole step in one launch (slot layout, one split)
@pytest.mark.parametrize("dtype,d,G,w,k", [
    (ko.BF16, 64, 1, 26, 129), (ko.BF16, 128, 1, 0, 129), (ko.F32, 64, 1, 26, 129), (ko.BF16, 128, 2, 26, 129),
    (ko.BF16, 64, 4, 129, 129), (ko.BF16, 128, 8, 26, 129), (ko.BF16, 64, 8, 0, 129), (ko.BF16, 256, 8, 50, 129),
    (ko.BF16, 64, 1, 2000, 10500),       # a unit too long for two workgroups per CU: one 8-wave workgroup
    (ko.BF16, 128, 4, 300, 1500)])       # 4 query heads in the 8-wave workgroup
def test_single_launch_slot_step_equals_the_two_calls(dtype, d, G, w, k):
    """With at least 320 units of a length that fits LDS, kf_decode_select_step in the slot layout is ONE
    launch: the workgroup that scored a unit evicts for it and stores the new token straight into the freed
    slot.  Same results, bit for bit, as kf_decode_step + kf_select_evict (which the oracle checks)."""
    rng = np.random.default_rng(9000 + d + G + w)
    L, B, H = 4, 4, 20
    cap = k + 2
    c0 = kf.Cache(K=0x10000, V=0x20000, score=0x30000, pos=0x40000, len=0x50000, L=L, B=B, H=H, d=d, cap=cap,
                  dtype=dtype, q_per_kv=G)
    assert kf.kf_decode_launch_shape(c0, k + 1)[0] == 1
    lens = np.full((L, B, H), k, np.int32)
    lens[0, 0, :5] = [k - 1, k - 40, 0, k + 1, k]        # room left (no eviction), empty, two over budget (reported)
    oc = random_cache(rng, L, B, H, d, cap, dtype, lens)
    oc.pos[...] = np.arange(cap)                          # consecutive positions, then shuffled slots
    for l, b, h in np.ndindex(L, B, H):
        n_u = int(lens[l, b, h])
        perm = rng.permutation(n_u)
        for nm in ("K", "V", "score", "pos"):
            getattr(oc, nm)[l, b, h, :n_u] = getattr(oc, nm)[l, b, h, :n_u][perm]
    oc.score[1, 1, 1, :k] = 0.25                          # all scores equal: the tie-break through pos decides
    seeds = dev(np.arange(B).astype(np.uint64) + 9)
    a, b_ = upload(oc, G), upload(oc, G)
    ws_a, ws_b = kf.new_workspace(a), kf.new_workspace(b_)
    out_a = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
    out_b = torch.zeros_like(out_a)
    kept_a = torch.zeros((L, B, H, k), dtype=torch.int32, device="cuda")
    kept_b = torch.zeros_like(kept_a)
    seq_pos = torch.from_numpy(np.full(B, k, np.int32)).cuda()
    for t in range(1, 4 if k < 1000 else 2):
        q = dev(rnd(rng, (L, B, H * G, d), dtype))
        kn, vn = (dev(rnd(rng, (L, B, H, d), dtype)) for _ in range(2))
        q_pos = k + t - 1
        tau = kf.kf_tau(t, 8)
        kf.kf_decode_step(a, q, kn, vn, q_pos, k + 1, tau, 0.11, kf.NOISE_GUMBEL, seeds, None, out_a, ws_a)
        kf.kf_select_evict(a, k, w, kept_a, ws_a, layout=kf.LAYOUT_SLOT)
        kf.kf_decode_select_step(b_, q, kn, vn, q_pos, k + 1, tau, 0.11, kf.NOISE_GUMBEL, seeds, None, out_b, k=k, w=w,
                                 layout=kf.LAYOUT_SLOT, kept_idx=kept_b, workspace=ws_b)
        torch.cuda.synchronize()
        # the unit two over budget: refused by the selection in step 1; from step 2 on it is full, so the
        # decode part skips it and the selection refuses it again -- the same count on both paths
        assert error_word(ws_a) == error_word(ws_b) == 2 * t - 1
        assert torch.equal(out_a, out_b)
        assert torch.equal(a.len, b_.len)
        la = host(a.len)
        ok = la <= k                                               # every unit but the reported one
        for nm in ("score", "pos", "K", "V"):
            xa, xb = host(getattr(a, nm)), host(getattr(b_, nm))
            for l, b, h in np.ndindex(L, B, H):
                n_u = int(la[l, b, h])
                np.testing.assert_array_equal(xa[l, b, h, :n_u], xb[l, b, h, :n_u], err_msg="%s (%d,%d,%d) step %d" % (nm, l, b, h, t))
        np.testing.assert_array_equal(host(kept_a)[ok], host(kept_b)[ok])
    assert int(a.len[1, 1, 1]) == k


@pytest.mark.parametrize("layout", [kf.LAYOUT_SLOT, kf.LAYOUT_ORDERED])
def test_single_launch_step_from_the_device_counter_and_in_a_graph(layout):
    rng = np.random.default_rng(9100)
    L, B, H, d, k, w = 4, 4, 20, 64, 129, 26
    cap = k + 1
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, k)
    oc.pos[...] = np.arange(cap)
    seeds = dev(np.arange(B).astype(np.uint64) + 3)
    n, T, steps = k, 6, 8
    inputs = [tuple(dev(rnd(rng, (L, B, H, d), ko.BF16)) for _ in range(3)) for _ in range(steps)]
    a, b_ = upload(oc), upload(oc)
    ws_a, ws_b = kf.new_workspace(a), kf.new_workspace(b_)
    out_a = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    out_b = torch.zeros_like(out_a)
    ref = []
    for t in range(1, steps + 1):
        q, kn, vn = inputs[t - 1]
        kf.kf_decode_select_step(a, q, kn, vn, n + t - 1, cap, kf.kf_tau(min(t, T), T), 0.125, kf.NOISE_GUMBEL, seeds, None,
                                 out_a, k=k, w=w, layout=layout, workspace=ws_a)
        torch.cuda.synchronize()
        ref.append([host(x).copy() for x in (out_a, a.score[..., :k], a.pos[..., :k], a.len)])
    step = torch.ones(1, dtype=torch.int32, device="cuda")
    qb, kb, vb = (torch.empty_like(x) for x in inputs[0])

    def one():
        kf.kf_decode_select_step_at(b_, qb, kb, vb, n, T, 1.0, 2.0, step, cap, 0.125, kf.NOISE_GUMBEL, seeds, None, out_b,
                                    k=k, w=w, layout=layout, workspace=ws_b)

    for src, dst in zip(inputs[0], (qb, kb, vb)):
        dst.copy_(src)
    one()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one()
    for t in range(1, steps + 1):
        if t > 1:
            for src, dst in zip(inputs[t - 1], (qb, kb, vb)):
                dst.copy_(src)
            (out_b * 0).sum().item()
            g.replay()
            torch.cuda.synchronize()
        assert int(step.item()) == t + 1
        for x, y in zip([host(x) for x in (out_b, b_.score[..., :k], b_.pos[..., :k], b_.len)], ref[t - 1]):
            np.testing.assert_array_equal(x, y)
    assert error_word(ws_b) == 0


# ------------------------------------------------------------------ temperature away from the schedule's range
@pytest.mark.parametrize("G", [1, 8])
@pytest.mark.parametrize("tau", [0.05, 0.5, 8.0, 1000.0])
def test_decode_at_extreme_temperatures(tau, G):
    """Sec. 3.3.1: small tau sharpens the score distribution towards one-hot, large tau flattens it towards
    uniform; the kernels keep everything in the base-2 domain with running maxima, so neither end overflows."""
    rng = np.random.default_rng(int(tau * 100))
    L, B, H, d, cap = 1, 2, 3, 128, 900
    lens = rng.integers(600, cap, (L, B, H)).astype(np.int32)
    oc = random_cache(rng, L, B, H, d, cap, ko.BF16, lens)
    q = rnd(rng, (L, B, H * G, d), ko.BF16)
    kn, vn = (rnd(rng, (L, B, H, d), ko.BF16) for _ in range(2))
    seeds = np.array([21, 22], np.uint64)
    gc = upload(oc, G)
    ws = kf.new_workspace(gc)
    out = torch.zeros((L, B, H * G, d), dtype=torch.float32, device="cuda")
    q_pos = int(oc.pos.max()) + 1
    before = oc.score.copy()
    kf.kf_decode_step(gc, dev(q), dev(kn), dev(vn), q_pos, 0, tau, 0.0884, kf.NOISE_GUMBEL, dev(seeds), None, out, ws)
    torch.cuda.synchronize()
    out_ref, _, df = oc.decode_step(q, kn, vn, q_pos, tau, 0.0884, ko.NOISE_GUMBEL, seeds, None, debug=True, q_per_kv=G)
    df = df.reshape(L, B, H, G, cap).sum(axis=3)      # a cached head's score takes the sum of its query heads' increments
    assert_close_out(host(out), out_ref)
    # increments: 2e-3 relative where they matter, plus an absolute floor of 1e-7 of the step's unit mass
    # (at tau = 0.05 most increments are far below fp32's resolution next to the scores they are added to)
    got = host(gc.score).astype(np.float64) - np.where(np.arange(cap) < lens[..., None], before, 0.0)
    for l, b, h in np.ndindex(L, B, H):
        m = int(lens[l, b, h]) + 1
        g, r = got[l, b, h, :m], df[l, b, h, :m]
        assert np.all(np.abs(g - r) <= 2e-3 * np.abs(r) + 2e-7 * (1.0 + np.abs(before[l, b, h, :m]))), (tau, l, b, h)
        assert abs(g.sum() - G) < 1e-3 * G
    if tau <= 0.05:
        assert df.max(axis=-1).min() > 0.5 / (G ** 0.5)    # nearly one-hot (per query head)
    if tau >= 1000.0:
        assert df[0, 0, 0, : lens[0, 0, 0] + 1].max() < 2.0 * G / lens[0, 0, 0]   # nearly uniform


# ------------------------------------------------------------------ free-running on a bf16 slice (informational)
def test_gptj_slice_free_running_reports_first_divergence():
    """No resynchronisation at all on a GPT-J-shaped slice: GPU and oracle each follow their own scores.  A
    near-tie at the eviction threshold may eventually send them apart (then every later step differs), so only
    the start is asserted; the step of the first difference, if any, is printed."""
    wl = kw.CONFIGS["gptj"].slice(L=1, H=4, T=512)
    fr = LockStep(wl)
    fr.oc.prefill_score(fr.Q, wl.n, ko.tau(0, wl.T), wl.scale, fr.noise, fr.seeds, fr.slopes)
    kf.kf_prefill_score(fr.gc, dev(fr.Q), wl.n, kf.kf_tau(0, wl.T), wl.scale, fr.noise, fr.d_seeds, None, fr.ws)
    fr.oc.select_evict(wl.k, wl.w)
    kf.kf_select_evict(fr.gc, wl.k, wl.w, None, fr.ws)
    first_div = None
    steps = 128
    for t in range(1, steps + 1):
        q, kn, vn = kw.decode_inputs(wl, t)
        fr.oc.decode_step(kw.to_oracle(q), kw.to_oracle(kn), kw.to_oracle(vn), wl.n + t - 1, ko.tau(t, wl.T), wl.scale,
                          fr.noise, fr.seeds)
        kf.kf_decode_select_step(fr.gc, q.cuda(), kn.cuda(), vn.cuda(), wl.n + t - 1, wl.k + 1, kf.kf_tau(t, wl.T), wl.scale,
                                 fr.noise, fr.d_seeds, None, fr.out, k=wl.k, w=wl.w, workspace=fr.ws)
        fr.oc.select_evict(wl.k, wl.w)
        torch.cuda.synchronize()
        if first_div is None and not (host(fr.gc.pos)[..., : wl.k] == fr.oc.pos[..., : wl.k]).all():
            first_div = t
    print("gptj slice free-running: first divergence step:", first_div, "of", steps)
    assert first_div is None or first_div > 16
