"""The allocation-free entry point (kf_decode_select_step_noalloc: scratch built into the library's
device code, no workspace argument) against kf_decode_select_step on a caller's workspace: same kernels,
so every output must agree bit for bit, and both must agree with the oracle within the parity tolerances.
Two calls in a row on the same GPU, the second on a smaller input, share the built-in buffer."""
import numpy as np
import pytest
import torch

import paper_2403_09054_amd as kf
from oracle import kf_oracle as ko
from parity_harness import assert_close_out, assert_close_score, dev, error_word, host, upload

pytestmark = pytest.mark.gpu


def bf16_round(a):
    b = a.astype(np.float32).view(np.uint32).astype(np.uint64)
    return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)


def one_case(rng, L, B, H, d, cap, w, layout, full_unit):
    k = cap - 1
    oc = ko.OracleCache(L, B, H, d, cap, ko.BF16)
    oc.K[...] = bf16_round(rng.standard_normal(oc.K.shape))
    oc.V[...] = bf16_round(rng.standard_normal(oc.V.shape))
    oc.score[...] = (rng.random(oc.score.shape) * 3).astype(np.float32)
    oc.pos[...] = np.arange(cap, dtype=np.int32) + 50
    oc.len[...] = k                                  # a full budget: the step appends one token and evicts one
    oc.len[0, 0, 0] = k - 37                         # under budget: appended, nothing leaves
    if full_unit:
        oc.len[-1, -1, -1] = cap                     # no room: skipped and counted
    q, kn, vn = (bf16_round(rng.standard_normal((L, B, H, d))) for _ in range(3))
    seeds = (np.arange(B) + 77).astype(np.uint64)
    slopes = (0.5 ** np.arange(1, H + 1)).astype(np.float32) * 0.01
    q_pos, tau, scale = 50 + cap + 3, 1.375, float(1.0 / np.sqrt(np.float32(d)))

    c_ref, c_new = upload(oc), upload(oc)
    assert kf.kf_workspace_bytes(c_ref) <= kf.NOALLOC_SCRATCH_BYTES
    S, _ = kf.kf_decode_launch_shape(c_ref, cap)
    ws = kf.new_workspace(c_ref)
    out_ref = torch.zeros((L, B, H, d), dtype=torch.float32, device="cuda")
    out_new = torch.full((L, B, H, d), 3.0, dtype=torch.float32, device="cuda")
    kept_ref = torch.zeros((L, B, H, k), dtype=torch.int32, device="cuda")
    kept_new = torch.full((L, B, H, k), -5, dtype=torch.int32, device="cuda")
    skipped = torch.zeros(1, dtype=torch.int32, device="cuda")
    args = (dev(q), dev(kn), dev(vn), q_pos, cap, tau, scale, kf.NOISE_GUMBEL, dev(seeds), dev(slopes))
    kf.kf_decode_select_step(c_ref, *args, out_ref, k=k, w=w, layout=layout, kept_idx=kept_ref, workspace=ws)
    kf.kf_decode_select_step_noalloc(c_new, *args, out_new, k=k, w=w, layout=layout, kept_idx=kept_new, skipped=skipped)
    torch.cuda.synchronize()
    # the existing entry point is the reference: bit for bit
    assert int(skipped.item()) == error_word(ws) == (1 if full_unit else 0)
    assert torch.equal(out_new, out_ref)
    assert torch.equal(kept_new, kept_ref)
    for nm in ("len", "pos", "score", "K", "V"):
        a, b = getattr(c_new, nm), getattr(c_ref, nm)
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b), nm
    # and both follow the oracle (the unit without room is left out: the oracle refuses it)
    if full_unit:
        oc.len[-1, -1, -1] = 0
    o = oc.decode_step(q, kn, vn, q_pos, tau, scale, ko.NOISE_GUMBEL, seeds, slopes)
    oc.select_evict(k, w)
    ok = np.ones((L, B, H), bool)
    if full_unit:
        ok[-1, -1, -1] = False
    assert_close_out(host(out_new)[ok], o[ok])
    if layout == kf.LAYOUT_ORDERED:
        lens = np.where(ok, oc.len, 0)
        np.testing.assert_array_equal(host(c_new.len)[ok], oc.len[ok])
        assert_close_score(host(c_new.score), oc.score, lens)
    return S


def test_step_on_built_in_scratch_equals_step_on_a_workspace_twice_in_a_row():
    rng = np.random.default_rng(424)
    # few units of 1024 tokens: the decode launch is split, partial records and increments go through scratch
    S1 = one_case(rng, L=1, B=2, H=8, d=128, cap=1025, w=205, layout=kf.LAYOUT_ORDERED, full_unit=True)
    # right after it, a smaller input on the same buffer (which still holds the first call's records)
    S2 = one_case(rng, L=1, B=1, H=4, d=64, cap=300, w=30, layout=kf.LAYOUT_SLOT, full_unit=False)
    assert S1 > 1 and S2 >= 1
