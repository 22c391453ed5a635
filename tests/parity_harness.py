"""Shared helpers of the GPU parity tests: move state between the oracle's numpy
caches and the library's torch caches, compare with the tolerances the build
target states, and run the lock-step protocol.

Tolerances (from the build target): attention outputs and accumulated scores
within 2e-3 relative (fp32 accumulation over bf16 K/V); retained index sets
bit-exact except at tokens whose oracle score lies within 1e-5 relative of the
(k-w)-th largest candidate score.
"""
from __future__ import annotations

import numpy as np
import torch

import kf_workloads as kw
import paper_2403_09054_amd as kf
from oracle import kf_oracle as ko

RTOL = 2e-3
TIE_BAND = 1e-5


def dev(a):
    """numpy (oracle format) -> cuda tensor in the library's format."""
    if a is None:
        return None
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64).copy()).cuda()
    return kw.from_oracle(a).cuda()


def upload(oc: ko.OracleCache, q_per_kv=1) -> kf.Cache:
    return kf.Cache(K=dev(oc.K), V=dev(oc.V), score=dev(oc.score), pos=dev(oc.pos), len=dev(oc.len),
                    L=oc.L, B=oc.B, H=oc.H, d=oc.d, cap=oc.cap, dtype=oc.dtype, layer0=oc.layer0,
                    q_per_kv=q_per_kv)


def upload_into(gc: kf.Cache, oc: ko.OracleCache, kv=True):
    if kv:
        gc.K.copy_(dev(oc.K))
        gc.V.copy_(dev(oc.V))
    gc.score.copy_(dev(oc.score))
    gc.pos.copy_(dev(oc.pos))
    gc.len.copy_(dev(oc.len))


def host(t):
    return kw.to_oracle(t)


def assert_close_out(got, ref, what="out"):
    """|got-ref| <= 2e-3*|ref| + 1e-5*max|ref| per unit (last axis = head dim)."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    atol = 1e-5 * np.abs(ref).max(axis=-1, keepdims=True) + 1e-30
    bad = np.abs(got - ref) > RTOL * np.abs(ref) + atol
    assert not bad.any(), "%s: %d elements off, worst abs err %g" % (
        what, bad.sum(), np.abs(got - ref).max())
    return float((np.abs(got - ref) / (np.abs(ref) + atol)).max())


def assert_close_score(got, ref, lens, what="score"):
    """Accumulated scores of the live slots, relative 2e-3 element by element."""
    worst = 0.0
    L, B, H = lens.shape
    for l in range(L):
        for b in range(B):
            for h in range(H):
                m = int(lens[l, b, h])
                g = got[l, b, h, :m].astype(np.float64)
                r = ref[l, b, h, :m].astype(np.float64)
                err = np.abs(g - r) / (np.abs(r) + 1e-30)
                assert (err <= RTOL).all(), "%s unit (%d,%d,%d): worst rel err %g at slot %d" % (
                    what, l, b, h, err.max(), int(err.argmax()))
                worst = max(worst, float(err.max()) if m else 0.0)
    return worst


def compare_kept(kept_gpu, kept_ref, score_before, len_before, k, w):
    """Exact match of the survivor lists, or a difference confined to the tie band.
    Returns the number of units that needed the tie-band rule."""
    events = 0
    L, B, H = len_before.shape
    for l in range(L):
        for b in range(B):
            for h in range(H):
                g, r = kept_gpu[l, b, h], kept_ref[l, b, h]
                if (g == r).all():
                    continue
                n = int(len_before[l, b, h])
                assert n > k, "untouched unit must report identity"
                f = score_before[l, b, h, : n - w].astype(np.float64)
                thr = np.sort(f)[::-1][k - w - 1]
                gs, rs = set(g.tolist()), set(r.tolist())
                assert len(gs) == k and (np.diff(g) > 0).all(), "GPU survivors not a sorted k-set"
                assert set(range(n - w, n)) <= gs, "recent window not retained"
                for slot in gs ^ rs:
                    assert slot < n - w
                    assert abs(f[slot] - thr) <= TIE_BAND * abs(thr), (
                        "unit (%d,%d,%d) slot %d score %r differs outside the tie band of threshold %r"
                        % (l, b, h, slot, f[slot], thr))
                events += 1
    return events


def assert_state_equal(gc: kf.Cache, oc: ko.OracleCache, kv=True, score_exact=True):
    """Bit-exact comparison of the live part of both caches."""
    lens = host(gc.len)
    np.testing.assert_array_equal(lens, oc.len)
    pos, score = host(gc.pos), host(gc.score)
    K = host(gc.K) if kv else None
    V = host(gc.V) if kv else None
    for l in range(oc.L):
        for b in range(oc.B):
            for h in range(oc.H):
                m = int(lens[l, b, h])
                np.testing.assert_array_equal(pos[l, b, h, :m], oc.pos[l, b, h, :m])
                if score_exact:
                    np.testing.assert_array_equal(score[l, b, h, :m], oc.score[l, b, h, :m])
                if kv:
                    np.testing.assert_array_equal(K[l, b, h, :m], oc.K[l, b, h, :m])
                    np.testing.assert_array_equal(V[l, b, h, :m], oc.V[l, b, h, :m])


def sort_by_pos(gc: kf.Cache):
    """Host copy of a cache with every unit's live entries sorted by original
    position (what an unordered, slot-replacement cache means as a set).
    Returns (K, V, score, pos, len, order) numpy arrays; order[l,b,h,:m] is the
    slot of the i-th entry in position order."""
    K, V, score, pos, lens = host(gc.K).copy(), host(gc.V).copy(), host(gc.score).copy(), host(gc.pos).copy(), host(gc.len)
    order = np.zeros(pos.shape, np.int64)
    L, B, H = lens.shape
    for l in range(L):
        for b in range(B):
            for h in range(H):
                m = int(lens[l, b, h])
                o = np.argsort(pos[l, b, h, :m], kind="stable")
                order[l, b, h, :m] = o
                K[l, b, h, :m] = K[l, b, h, o]
                V[l, b, h, :m] = V[l, b, h, o]
                score[l, b, h, :m] = score[l, b, h, o]
                pos[l, b, h, :m] = pos[l, b, h, o]
    return K, V, score, pos, lens, order


def assert_set_equal(gc: kf.Cache, oc: ko.OracleCache, kv=True, score_exact=True):
    """The unordered GPU cache holds exactly the oracle's entries (keyed by pos), bit for bit."""
    K, V, score, pos, lens, _ = sort_by_pos(gc)
    np.testing.assert_array_equal(lens, oc.len)
    for l in range(oc.L):
        for b in range(oc.B):
            for h in range(oc.H):
                m = int(lens[l, b, h])
                np.testing.assert_array_equal(pos[l, b, h, :m], oc.pos[l, b, h, :m])
                if score_exact:
                    np.testing.assert_array_equal(score[l, b, h, :m], oc.score[l, b, h, :m])
                if kv:
                    np.testing.assert_array_equal(K[l, b, h, :m], oc.K[l, b, h, :m])
                    np.testing.assert_array_equal(V[l, b, h, :m], oc.V[l, b, h, :m])


def error_word(ws) -> int:
    return int(ws[:4].view(torch.int32)[0].item())


class LockStep:
    """Oracle and GPU advance together over a workload; before every call both
    hold the same state (scores are re-uploaded from the oracle after each
    decode step, everything after a tie-band event)."""

    def __init__(self, wl: kw.Workload, noise=ko.NOISE_GUMBEL, cap=None, layout=kf.LAYOUT_ORDERED,
                 shared=False, q_per_kv=1):
        self.wl, self.noise, self.layout = wl, noise, layout
        self.G = G = q_per_kv           # grouped queries: wl.H counts QUERY heads, the caches hold wl.H // G
        self.shared = shared            # one score function for all layers (the paper's "Shared" ablation)
        self.score_mode = kf.SCORE_SHARED if shared else kf.SCORE_PER_LAYER
        self.cap = cap or wl.n
        dt = {"f32": ko.F32, "bf16": ko.BF16, "f16": ko.F16}[wl.dtype]
        assert wl.H % G == 0
        self.oc = ko.OracleCache(wl.L, wl.B, wl.H // G, wl.d, self.cap, dt)
        self.Q = np.zeros((wl.L, wl.B, wl.H, wl.n, wl.d), self.oc.K.dtype)
        for l in range(wl.L):
            Q, K, V = kw.prompt_layer(wl, l)
            self.Q[l] = kw.to_oracle(Q)
            self.oc.K[l, :, :, : wl.n] = kw.to_oracle(K)[:, ::G]
            self.oc.V[l, :, :, : wl.n] = kw.to_oracle(V)[:, ::G]
        self.seeds = kw.noise_seeds(wl)
        self.slopes = kw.alibi_slopes(wl)
        self.gc = upload(self.oc, G)
        self.ws = kf.new_workspace(self.gc, wl.n)
        self.d_seeds, self.d_slopes = dev(self.seeds), dev(self.slopes)
        self.out = torch.zeros((wl.L, wl.B, wl.H, wl.d), dtype=torch.float32, device="cuda")
        self.kept = torch.zeros((wl.L, wl.B, wl.H // G, wl.k), dtype=torch.int32, device="cuda")
        self.stats = dict(out_err=0.0, score_err=0.0, tie_events=0, steps=0)

    def prefill(self):
        wl = self.wl
        tau_o, tau_g = ko.tau(0, wl.T, wl.tau_init, wl.tau_end), kf.kf_tau(0, wl.T, wl.tau_init, wl.tau_end)
        assert tau_o == tau_g
        self.oc.prefill_score(self.Q, wl.n, tau_o, wl.scale, self.noise, self.seeds, self.slopes, shared=self.shared,
                              q_per_kv=self.G)
        kf.kf_prefill_score(self.gc, dev(self.Q), wl.n, tau_g, wl.scale, self.noise, self.d_seeds,
                            self.d_slopes, self.ws, score_mode=self.score_mode)
        torch.cuda.synchronize()
        lens = host(self.gc.len)
        np.testing.assert_array_equal(lens, self.oc.len)
        np.testing.assert_array_equal(host(self.gc.pos)[..., : wl.n], self.oc.pos[..., : wl.n])
        e = assert_close_score(host(self.gc.score), self.oc.score, lens, "prefill score")
        self.stats["prefill_err"] = e
        self.gc.score.copy_(dev(self.oc.score))
        self.select()

    def select(self):
        wl = self.wl
        before_score, before_len = self.oc.score.copy(), self.oc.len.copy()
        kept_ref = self.oc.select_evict(wl.k, wl.w)
        slot = self.layout == kf.LAYOUT_SLOT and int(before_len.max()) <= wl.k + 1
        if slot:
            order_before = sort_by_pos(self.gc)[5]
        kf.kf_select_evict(self.gc, wl.k, wl.w, self.kept, self.ws,
                           layout=kf.LAYOUT_SLOT if slot else kf.LAYOUT_ORDERED)
        torch.cuda.synchronize()
        assert error_word(self.ws) == 0
        if slot:
            # survivors as ranks in position order = the ordered layout's slot numbers
            kept_slots = host(self.kept)
            kept_g = np.full_like(kept_ref, -1)
            for l, b, h in np.ndindex(*before_len.shape):
                n_u = int(before_len[l, b, h])
                rank = np.empty(n_u, np.int64)
                rank[order_before[l, b, h, :n_u]] = np.arange(n_u)
                kk = kept_slots[l, b, h]
                kk = kk[kk >= 0]
                kept_g[l, b, h, : len(kk)] = np.sort(rank[kk])
        else:
            kept_g = host(self.kept)
        ev = compare_kept(kept_g, kept_ref, before_score, before_len, wl.k, wl.w)
        self.stats["tie_events"] += ev
        if ev:
            upload_into(self.gc, self.oc)       # adopt the oracle's choice and go on
        return ev

    def step(self, t, check_kv=False):
        wl = self.wl
        q, kn, vn = kw.decode_inputs(wl, t)
        kn, vn = kn[:, :, ::self.G].contiguous(), vn[:, :, ::self.G].contiguous()
        q_pos = wl.n + t - 1
        tau_o, tau_g = ko.tau(t, wl.T, wl.tau_init, wl.tau_end), kf.kf_tau(t, wl.T, wl.tau_init, wl.tau_end)
        assert tau_o == tau_g
        out_ref = self.oc.decode_step(kw.to_oracle(q), kw.to_oracle(kn), kw.to_oracle(vn), q_pos, tau_o,
                                      wl.scale, self.noise, self.seeds, self.slopes, shared=self.shared,
                                      q_per_kv=self.G)
        kf.kf_decode_step(self.gc, q.cuda(), kn.cuda(), vn.cuda(), q_pos, min(wl.k + 1, self.cap), tau_g,
                          wl.scale, self.noise, self.d_seeds, self.d_slopes, self.out, self.ws,
                          score_mode=self.score_mode)
        torch.cuda.synchronize()
        assert error_word(self.ws) == 0
        lens = host(self.gc.len)
        np.testing.assert_array_equal(lens, self.oc.len)
        if self.shared:                 # one function: every layer holds the same copy, bit for bit
            g = host(self.gc.score)
            for l in range(1, wl.L):
                for b, h in np.ndindex(wl.B, wl.H // self.G):
                    np.testing.assert_array_equal(g[l, b, h, : lens[l, b, h]], g[0, b, h, : lens[0, b, h]])
        self.stats["out_err"] = max(self.stats["out_err"], assert_close_out(host(self.out), out_ref))
        if self.layout == kf.LAYOUT_SLOT:
            _, _, g_score, g_pos, _, order = sort_by_pos(self.gc)
            for l, b, h in np.ndindex(*lens.shape):
                np.testing.assert_array_equal(g_pos[l, b, h, : lens[l, b, h]], self.oc.pos[l, b, h, : lens[l, b, h]])
            self.stats["score_err"] = max(self.stats["score_err"], assert_close_score(g_score, self.oc.score, lens))
            new_score = host(self.gc.score).copy()       # oracle scores, scattered to the GPU's slots
            for l, b, h in np.ndindex(*lens.shape):
                m = int(lens[l, b, h])
                new_score[l, b, h, order[l, b, h, :m]] = self.oc.score[l, b, h, :m]
            self.gc.score.copy_(dev(new_score))
        else:
            self.stats["score_err"] = max(self.stats["score_err"],
                                          assert_close_score(host(self.gc.score), self.oc.score, lens))
            self.gc.score.copy_(dev(self.oc.score))     # lock-step: same scores before selection
        ev = self.select()
        if self.layout == kf.LAYOUT_SLOT:
            if ev:    # the oracle's (ordered) state was adopted: it is a valid unordered state as well
                pass
            assert_set_equal(self.gc, self.oc, kv=check_kv)
        else:
            assert_state_equal(self.gc, self.oc, kv=check_kv)
        self.stats["steps"] += 1
