"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, mirrors the oracle's tau schedule and noise
hash bit for bit, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2403_09054_amd as kf
from paper_2403_09054_amd import binding
from oracle import kf_oracle as ko

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "keyformer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kf_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(binding.SYMBOLS)
    raw = ctypes.CDLL(kf.lib_path())
    for n in names:
        assert getattr(raw, n) is not None
    assert kf.kf_version() == 1


def test_tau_matches_oracle_bits():
    for T in (1, 32, 512, 1024, 2048):
        for t in range(0, T + 1, max(1, T // 37)):
            assert kf.kf_tau(t, T, 1.0, 2.0) == ko.tau(t, T, 1.0, 2.0)
    assert kf.kf_tau(0, 512) == 1.0 and abs(kf.kf_tau(512, 512) - 2.0) < 1e-6


def test_noise_bits_match_golden_and_oracle():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "noise_bits.txt")) if not l.startswith("#")]
    for r in rows:
        args = list(map(int, r[:5]))
        assert kf.kf_noise_bits(*args) == int(r[5])
    rng = np.random.default_rng(0)
    for _ in range(2000):
        seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        a = [int(rng.integers(0, 64)), int(rng.integers(0, 64)), int(rng.integers(0, 2 ** 31)),
             int(rng.integers(0, 2 ** 31))]
        assert kf.kf_noise_bits(seed, *a) == ko.noise_bits(seed, *a)


def fake_cache(**over):
    # addresses are never dereferenced: validation fails (or is all that is tested) first
    kw = dict(K=0x10000, V=0x20000, score=0x30000, pos=0x40000, len=0x50000, L=2, B=1, H=4, d=128,
              cap=1025, dtype=kf.BF16)
    kw.update(over)
    return kf.Cache(**kw)


WS = (0x100000, 1 << 40)


def expect(status, fn, *a, **k):
    with pytest.raises(kf.KeyformerError) as e:
        fn(*a, **k)
    assert e.value.status == status, e.value
    assert len(str(e.value)) > 20


def test_workspace_size_query():
    c = fake_cache()
    small = kf.kf_workspace_bytes(c, 0)
    big = kf.kf_workspace_bytes(c, 1 << 20)
    assert 0 < small <= big
    assert kf.kf_workspace_bytes(fake_cache(d=96), 0) == 0
    assert kf.kf_workspace_bytes(fake_cache(dtype=kf.F32, d=256), 0) == 0


def test_select_argument_validation():
    c = fake_cache()
    expect(binding.KF_EINVAL, kf.kf_select_evict, c, 0, 0, None, WS, 0)
    expect(binding.KF_EINVAL, kf.kf_select_evict, c, 8, 9, None, WS, 0)
    expect(binding.KF_EINVAL, kf.kf_select_evict, c, 8, -1, None, WS, 0)
    expect(binding.KF_EINVAL, kf.kf_select_evict, c, 1026, 3, None, WS, 0)
    expect(binding.KF_EWORKSPACE, kf.kf_select_evict, c, 8, 2, None, (0x100000, 64), 0)
    expect(binding.KF_EWORKSPACE, kf.kf_select_evict, c, 8, 2, None, None, 0)
    expect(binding.KF_EWORKSPACE, kf.kf_select_evict, c, 8, 2, None, (0x100004, 1 << 40), 0)
    expect(binding.KF_EINVAL, kf.kf_select_evict, fake_cache(K=None), 8, 2, None, WS, 0)
    expect(binding.KF_EINVAL, kf.kf_select_evict, fake_cache(K=0x10004), 8, 2, None, WS, 0)
    expect(binding.KF_EUNSUPPORTED, kf.kf_select_evict, fake_cache(d=96), 8, 2, None, WS, 0)
    expect(binding.KF_EINVAL, kf.kf_select_evict, fake_cache(dtype=7), 8, 2, None, WS, 0)
    expect(binding.KF_EINVAL, kf.kf_select_evict, fake_cache(L=0), 8, 2, None, WS, 0)


def test_decode_argument_validation():
    c = fake_cache()
    good = dict(q=0x1000, k_new=0x2000, v_new=0x3000, q_pos=10, m_hint=0, tau=1.5, scale=0.1,
                noise=kf.NOISE_GUMBEL, seeds=0x4000, slopes=None, out=0x5000, workspace=WS, stream=0)

    def call(**over):
        a = dict(good)
        a.update(over)
        kf.kf_decode_step(c, a["q"], a["k_new"], a["v_new"], a["q_pos"], a["m_hint"], a["tau"], a["scale"],
                          a["noise"], a["seeds"], a["slopes"], a["out"], a["workspace"], a["stream"])

    for bad in (dict(q=None), dict(k_new=None), dict(v_new=None), dict(out=None), dict(q=0x1008),
                dict(q_pos=-1), dict(m_hint=-1), dict(m_hint=1026), dict(tau=0.0), dict(tau=-1.0),
                dict(tau=float("inf")), dict(tau=float("nan")), dict(scale=float("nan")), dict(noise=9),
                dict(seeds=None), dict(noise=kf.NOISE_GAUSSIAN, seeds=None)):
        expect(binding.KF_EINVAL, call, **bad)
    expect(binding.KF_EWORKSPACE, call, workspace=(0x100000, 1000))


def test_prefill_argument_validation():
    c = fake_cache(cap=4096)
    cfg = dict(tau=1.0, scale=0.1, noise=kf.NOISE_GUMBEL, seeds=0x4000, slopes=None, workspace=WS, stream=0)
    expect(binding.KF_EINVAL, kf.kf_prefill_score, c, None, 128, **cfg)
    expect(binding.KF_EINVAL, kf.kf_prefill_score, c, 0x1000, 0, **cfg)
    expect(binding.KF_EINVAL, kf.kf_prefill_score, c, 0x1000, 4097, **cfg)
    expect(binding.KF_EINVAL, kf.kf_prefill_score, c, 0x1004, 128, **cfg)
    expect(binding.KF_EINVAL, kf.kf_prefill_score, c, 0x1000, 128, **dict(cfg, tau=0.0))
    expect(binding.KF_EINVAL, kf.kf_prefill_score, c, 0x1000, 128, **dict(cfg, seeds=None))
    expect(binding.KF_EWORKSPACE, kf.kf_prefill_score, c, 0x1000, 128, **dict(cfg, workspace=(0x100000, 4096)))


def test_decode_launch_shape_covers_the_rows_and_balances_the_chip():
    # (L, B, H, d, cap, dtype, m_hint): the five workload shapes plus odd ones
    shapes = [(1, 1, 2, 64, 65, kf.F32, 65), (28, 1, 16, 256, 1025, kf.BF16, 1025), (32, 8, 32, 128, 2049, kf.BF16, 2049),
              (32, 1, 32, 128, 9831, kf.BF16, 9831), (32, 64, 32, 128, 1025, kf.BF16, 1025),
              (1, 1, 1, 128, 600000, kf.BF16, 0), (3, 1, 5, 64, 777, kf.BF16, 500), (1, 1, 1, 64, 1, kf.F32, 1)]
    for (L, B, H, d, cap, dt, hint) in shapes:
        c = fake_cache(L=L, B=B, H=H, d=d, cap=cap, dtype=dt)
        S, chunk = kf.kf_decode_launch_shape(c, hint)
        rows = (hint or cap) - 1
        assert 1 <= S <= 256 and 1 <= chunk <= (20480 if S == 1 else 4096)     # LDS: up to 158 KB single, 64 KB split
        assert S * chunk >= rows                      # every cache row belongs to a split
        assert (S - 1) * chunk < max(rows, 1) or S == 1   # no split is entirely beyond the rows
    # more than one unit per compute unit and the logits fit LDS: one workgroup per unit, nothing to merge
    assert kf.kf_decode_launch_shape(fake_cache(L=28, B=1, H=16, d=256, cap=1025), 1025) == (1, 1024)
    assert kf.kf_decode_launch_shape(fake_cache(L=32, B=64, H=32, d=128, cap=1025), 1025) == (1, 1024)
    assert kf.kf_decode_launch_shape(fake_cache(L=32, B=1, H=32, d=128, cap=9831), 9831) == (1, 9840)
    # too few units to fill the chip that way: 256 units -> 4 splits of 256 rows = 1024 workgroups
    assert kf.kf_decode_launch_shape(fake_cache(L=16, B=1, H=16, d=256, cap=1025), 1025) == (4, 256)
    # logits beyond what two workgroups per compute unit can hold in LDS, but within one's reach: still one per unit
    S, chunk = kf.kf_decode_launch_shape(fake_cache(L=32, B=1, H=32, d=128, cap=16385), 16385)
    assert S == 1 and chunk >= 16384
    # beyond that: splits of at most 4096 rows
    S, chunk = kf.kf_decode_launch_shape(fake_cache(L=32, B=1, H=32, d=128, cap=24000), 24000)
    assert S >= 6 and chunk <= 4096
    # 8 bf16 query heads per cached head: one workgroup per unit while 2 x 8 logit rows fit a compute
    # unit's LDS (about 2500 tokens) and there is a unit per compute unit; splits of at most 1024 rows otherwise
    assert kf.kf_decode_launch_shape(fake_cache(L=32, B=8, H=8, d=128, cap=2049, q_per_kv=8), 2049) == (1, 2048)
    S, chunk = kf.kf_decode_launch_shape(fake_cache(L=32, B=8, H=8, d=128, cap=4097, q_per_kv=8), 4097)
    assert S >= 4 and chunk <= 1024
    # 4 query heads: the same up to about 5000 tokens
    assert kf.kf_decode_launch_shape(fake_cache(L=32, B=8, H=8, d=128, cap=4097, q_per_kv=4), 4097) == (1, 4096)
    S, chunk = kf.kf_decode_launch_shape(fake_cache(L=32, B=8, H=8, d=128, cap=8193, q_per_kv=4), 8193)
    assert S >= 4 and chunk <= 2048
    S, chunk = kf.kf_decode_launch_shape(fake_cache(L=2, B=8, H=8, d=128, cap=2049, q_per_kv=8), 2049)
    assert S >= 2 and chunk <= 1024
    S, chunk = kf.kf_decode_launch_shape(fake_cache(L=32, B=8, H=8, d=128, cap=2049, q_per_kv=8, dtype=kf.F32), 2049)
    assert S >= 4 and chunk <= 512
    expect(binding.KF_EINVAL, kf.kf_decode_launch_shape, fake_cache(), 2000)
    expect(binding.KF_EUNSUPPORTED, kf.kf_decode_launch_shape, fake_cache(d=96), 0)


def test_decode_launch_plan_is_consistent_with_workspace():
    # the workspace a cache asks for must cover the decode plan at every hint:
    # probe through the public size query on a grid of shapes
    for (L, B, H, d, cap, dt) in [(1, 1, 1, 64, 128, kf.F32), (28, 1, 16, 256, 1025, kf.BF16),
                                  (32, 8, 32, 128, 2049, kf.BF16), (32, 1, 32, 128, 9831, kf.BF16),
                                  (1, 1, 1, 128, 600000, kf.BF16)]:
        c = fake_cache(L=L, B=B, H=H, d=d, cap=cap, dtype=dt)
        nbytes = kf.kf_workspace_bytes(c, 0)
        U = L * B * H
        assert nbytes >= U * cap * 4 + U * 4          # at least the increments and the counters


def test_step_from_device_memory_argument_validation():
    c = fake_cache()
    good = dict(n=64, T=32, tau_init=1.0, tau_end=2.0, step=0x6000, score_mode=kf.SCORE_PER_LAYER, k=8, w=2)

    def call(**over):
        a = dict(good)
        a.update(over)
        kf.kf_decode_select_step_at(c, 0x1000, 0x2000, 0x3000, a["n"], a["T"], a["tau_init"], a["tau_end"], a["step"],
                                    0, 0.1, kf.NOISE_GUMBEL, 0x4000, None, 0x5000, k=a["k"], w=a["w"], workspace=WS,
                                    stream=0, score_mode=a["score_mode"])

    for bad in (dict(step=None), dict(n=-1), dict(T=0), dict(tau_init=0.0), dict(tau_end=float("nan")),
                dict(tau_end=float("inf")), dict(score_mode=5), dict(k=0), dict(w=9)):
        expect(binding.KF_EINVAL, call, **bad)


def test_unknown_score_mode_is_rejected():
    c = fake_cache()
    expect(binding.KF_EINVAL, kf.kf_decode_step, c, 0x1000, 0x2000, 0x3000, 10, 0, 1.5, 0.1, kf.NOISE_GUMBEL, 0x4000,
           None, 0x5000, WS, 0, score_mode=2)


def test_query_group_validation_and_sizes():
    for g in (3, 5, 16):
        expect(binding.KF_EUNSUPPORTED, kf.kf_select_evict, fake_cache(q_per_kv=g), 8, 2, None, WS, 0)
        assert kf.kf_workspace_bytes(fake_cache(q_per_kv=g), 0) == 0
    expect(binding.KF_EINVAL, kf.kf_select_evict, fake_cache(q_per_kv=-1), 8, 2, None, WS, 0)
    sizes = [kf.kf_workspace_bytes(fake_cache(q_per_kv=g), 2048) for g in (0, 1, 2, 4, 8)]
    assert sizes[0] == sizes[1] and sizes[1] < sizes[2] < sizes[3] < sizes[4]
    # a workgroup keeps G logit rows in LDS: its chunk shrinks with G, and the splits cover the rows
    for g in (1, 2, 4, 8):
        for cap in (1025, 9831, 40000):
            S, chunk = kf.kf_decode_launch_shape(fake_cache(L=4, B=2, H=8, cap=cap, q_per_kv=g), cap)
            lim = 8192 if g >= 4 else 4096            # 4 and 8 heads: splits for 8-wave workgroups
            assert (chunk * g <= lim or S == 1) and S * chunk >= cap - 1 and 1 <= S <= 256, (g, cap, S, chunk)


def test_launches_beyond_the_grid_limit_are_refused():
    # 2^24 units of a million tokens would need 2^32 decode workgroups; 2^24 units of 2^20 prompt rows 2^37
    huge = fake_cache(L=256, B=256, H=256, d=64, cap=1 << 20)
    expect(binding.KF_EUNSUPPORTED, kf.kf_decode_step, huge, 0x1000, 0x2000, 0x3000, 10, 0, 1.5, 0.1, kf.NOISE_GUMBEL,
           0x4000, None, 0x5000, (0x100000, 1 << 62), 0)
    expect(binding.KF_EUNSUPPORTED, kf.kf_prefill_score, huge, 0x1000, 1 << 20, 1.0, 0.1, kf.NOISE_GUMBEL, 0x4000, None,
           (0x100000, 1 << 62), 0)


def test_beam_fork_argument_validation():
    expect(binding.KF_EINVAL, kf.kf_beam_fork, fake_cache(), None, WS)
    expect(binding.KF_EWORKSPACE, kf.kf_beam_fork, fake_cache(), 0x60000, (0x100000, 4))
    expect(binding.KF_EINVAL, kf.kf_beam_fork, fake_cache(K=None), 0x60000, WS)


def test_element_types_and_head_sizes():
    for dt, ds in ((kf.F32, (64, 128)), (kf.BF16, (64, 128, 256)), (kf.F16, (64, 128, 256))):
        for d in ds:
            assert kf.kf_decode_launch_shape(fake_cache(dtype=dt, d=d), 0)[0] >= 1
    expect(binding.KF_EUNSUPPORTED, kf.kf_decode_launch_shape, fake_cache(dtype=kf.F32, d=256), 0)
    expect(binding.KF_EUNSUPPORTED, kf.kf_decode_launch_shape, fake_cache(dtype=3), 0)
    expect(binding.KF_EINVAL, kf.kf_beam_fork, fake_cache(dtype=3), 0x60000, WS)


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_built_in_scratch_rejects_shapes_it_cannot_hold():
    # the allocation-free step refuses, on the host and before any device call, a cache whose scratch
    # does not fit the buffer built into the library
    big = fake_cache(L=32, B=8, H=32, cap=2049)
    assert kf.kf_workspace_bytes(big) > kf.NOALLOC_SCRATCH_BYTES
    with pytest.raises(kf.KeyformerError) as e:
        kf.kf_decode_select_step_noalloc(big, 0x1000, 0x2000, 0x3000, 5000, 0, 1.5, 0.09, kf.NOISE_NONE, None, None,
                                         0x4000, k=2048, w=410)
    assert e.value.status == binding.KF_EWORKSPACE and "built-in" in str(e.value)
    assert kf.kf_workspace_bytes(fake_cache()) <= kf.NOALLOC_SCRATCH_BYTES
