"""ctypes front end of the CPU oracle (oracle/kf_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this.  It shares no code with the GPU
library and never calls it.

All state lives in numpy arrays laid out as the paper's per-layer, per-head
caches (Fig. 5 caption: the score accumulates "for each layer and head"):
K, V [L,B,H,cap,d] (float32, float16, or uint16 holding bf16 bits), score [L,B,H,cap]
float32, pos [L,B,H,cap] int32, len [L,B,H] int32.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kf_oracle.c")
_LIB = os.path.join(_HERE, "libkf_oracle.so")

F32, BF16, F16 = 0, 1, 2
NOISE_NONE, NOISE_GUMBEL, NOISE_GAUSSIAN, NOISE_CONSTANT = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE double arithmetic, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.kfo_tau.restype = C.c_float
        L.kfo_tau.argtypes = [C.c_int, C.c_int, C.c_float, C.c_float]
        L.kfo_noise_bits.restype = C.c_uint32
        L.kfo_noise_bits.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.kfo_gumbel.restype = C.c_double
        L.kfo_gumbel.argtypes = [C.c_uint32]
        L.kfo_zeta.restype = C.c_double
        L.kfo_zeta.argtypes = [C.c_int, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        vp = C.c_void_p
        L.kfo_prefill_score.restype = C.c_int
        L.kfo_prefill_score.argtypes = [vp, vp, vp, vp, vp] + [C.c_int] * 9 + [
            C.c_float, C.c_float, C.c_int, vp, vp, C.c_int, C.c_int]
        L.kfo_decode_step.restype = C.c_int
        L.kfo_decode_step.argtypes = [vp, vp, vp, vp, vp] + [C.c_int] * 8 + [
            vp, vp, vp, C.c_int32, C.c_float, C.c_float, C.c_int, vp, vp, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp]
        L.kfo_select_evict.restype = C.c_int
        L.kfo_select_evict.argtypes = [vp, vp, vp, vp, vp] + [C.c_int] * 8 + [vp]
        _lib = L
    return _lib


def tau(t: int, T: int, tau_init: float = 1.0, tau_end: float = 2.0) -> float:
    return float(lib().kfo_tau(t, T, tau_init, tau_end))


def noise_bits(seed: int, layer: int, head: int, q_pos: int, k_pos: int) -> int:
    return int(lib().kfo_noise_bits(seed, layer, head, q_pos, k_pos))


def gumbel(bits: int) -> float:
    return float(lib().kfo_gumbel(bits))


def zeta(noise: int, seed: int, layer: int, head: int, q_pos: int, k_pos: int) -> float:
    return float(lib().kfo_zeta(noise, seed, layer, head, q_pos, k_pos))


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float16:
        return F16
    raise TypeError("K/V must be float32, float16 or uint16 (bf16 bits), got %s" % a.dtype)


class OracleCache:
    """Per-unit KV caches + accumulated scores, on the host."""

    def __init__(self, L, B, H, d, cap, dtype=F32, layer0=0, head0=0):
        self.L, self.B, self.H, self.d, self.cap, self.dtype = L, B, H, d, cap, dtype
        self.layer0 = layer0    # model-wide index of the first layer held (noise key)
        self.head0 = head0      # ... and of the first cached head (noise key, and index into `slopes`)
        et = {F32: np.float32, BF16: np.uint16, F16: np.float16}[dtype]
        self.K = np.zeros((L, B, H, cap, d), et)
        self.V = np.zeros((L, B, H, cap, d), et)
        self.score = np.zeros((L, B, H, cap), np.float32)
        self.pos = np.zeros((L, B, H, cap), np.int32)
        self.len = np.zeros((L, B, H), np.int32)

    def copy(self):
        o = OracleCache.__new__(OracleCache)
        o.L, o.B, o.H, o.d, o.cap, o.dtype = self.L, self.B, self.H, self.d, self.cap, self.dtype
        o.layer0, o.head0 = self.layer0, self.head0
        for nm in ("K", "V", "score", "pos", "len"):
            setattr(o, nm, getattr(self, nm).copy())
        return o

    def _dims(self):
        return [self.L, self.B, self.H, self.d, self.cap, self.dtype]

    def _check(self, *arrs):
        for a in arrs:
            if a is not None:
                assert a.flags["C_CONTIGUOUS"]

    def prefill_score(self, Q, n, tau_, scale, noise=NOISE_GUMBEL, seeds=None, slopes=None, shared=False,
                      q_per_kv=1, n_seq=None):
        """Q: [L,B,H*q_per_kv,n,d] same element type as K; K rows 0..n-1 must be filled.
        shared: one score function for all layers (the sum of the layers' scores).
        q_per_kv: query heads per cached head (grouped-query attention).
        n_seq: [B] prompt length of every sequence of a batch padded to n rows: a sequence is
        scored on its own first n_seq[b] rows, by itself, exactly as if the padding did not exist."""
        assert Q.shape == (self.L, self.B, self.H * q_per_kv, n, self.d) and _dtype_code(Q) == self.dtype
        if n_seq is not None:
            assert len(n_seq) == self.B
            for b in range(self.B):
                nb = int(n_seq[b])
                assert 1 <= nb <= n
                one = OracleCache(self.L, 1, self.H, self.d, self.cap, self.dtype, self.layer0, self.head0)
                for nm in ("K", "V", "score", "pos", "len"):
                    setattr(one, nm, np.ascontiguousarray(getattr(self, nm)[:, b:b + 1]))
                one.prefill_score(np.ascontiguousarray(Q[:, b:b + 1, :, :nb]), nb, tau_, scale, noise,
                                  None if seeds is None else np.asarray(seeds)[b:b + 1], slopes, shared, q_per_kv)
                for nm in ("score", "pos", "len"):
                    getattr(self, nm)[:, b:b + 1] = getattr(one, nm)
            return
        seeds = None if seeds is None else np.ascontiguousarray(seeds, np.uint64)
        slopes = None if slopes is None else np.ascontiguousarray(slopes, np.float32)
        Q = np.ascontiguousarray(Q)
        rc = lib().kfo_prefill_score(_p(Q), _p(self.K), _p(self.score), _p(self.pos), _p(self.len),
                                     *self._dims(), self.layer0, self.head0, n, tau_, scale, noise, _p(seeds), _p(slopes),
                                     int(shared), int(q_per_kv))
        if rc:
            raise ValueError("kfo_prefill_score rc=%d" % rc)

    def decode_step(self, q, k_new, v_new, q_pos, tau_, scale, noise=NOISE_GUMBEL,
                    seeds=None, slopes=None, debug=False, new_pos=False, shared=False,
                    q_per_kv=1, q_pos_seq=None, tau_seq=None):
        """k_new, v_new: [L,B,H,d]; q: [L,B,H*q_per_kv,d].  Returns out [L,B,H*q_per_kv,d]
        float32 (and, with debug, every query head's attention probabilities and score
        increment as float64 [L,B,H*q_per_kv,cap]).  q_pos_seq / tau_seq: [B] per-sequence
        query position and temperature, replacing the scalars."""
        shp = (self.L, self.B, self.H, self.d)
        qshp = (self.L, self.B, self.H * q_per_kv, self.d)
        q, k_new, v_new = (np.ascontiguousarray(a) for a in (q, k_new, v_new))
        for a, sh_ in ((q, qshp), (k_new, shp), (v_new, shp)):
            assert a.shape == sh_ and _dtype_code(a) == self.dtype
        seeds = None if seeds is None else np.ascontiguousarray(seeds, np.uint64)
        slopes = None if slopes is None else np.ascontiguousarray(slopes, np.float32)
        q_pos_seq = None if q_pos_seq is None else np.ascontiguousarray(q_pos_seq, np.int32)
        tau_seq = None if tau_seq is None else np.ascontiguousarray(tau_seq, np.float32)
        for a in (q_pos_seq, tau_seq):
            assert a is None or a.shape == (self.B,)
        out = np.zeros(qshp, np.float32)
        dshape = (self.L, self.B, self.H * q_per_kv, self.cap)
        dp = np.zeros(dshape, np.float64) if debug else None
        df = np.zeros(dshape, np.float64) if debug else None
        rc = lib().kfo_decode_step(_p(self.K), _p(self.V), _p(self.score), _p(self.pos), _p(self.len),
                                   *self._dims(), self.layer0, self.head0, _p(q), _p(k_new), _p(v_new), q_pos, tau_, scale,
                                   noise, _p(seeds), _p(slopes), int(new_pos), int(shared), int(q_per_kv), _p(q_pos_seq), _p(tau_seq),
                                   _p(out), _p(dp), _p(df))
        if rc:
            raise ValueError("kfo_decode_step rc=%d" % rc)
        return (out, dp, df) if debug else out

    def select_evict(self, k, w, want_idx=True):
        kept = np.full((self.L, self.B, self.H, k), -1, np.int32) if want_idx else None
        rc = lib().kfo_select_evict(_p(self.K), _p(self.V), _p(self.score), _p(self.pos), _p(self.len),
                                    *self._dims(), k, w, _p(kept))
        if rc:
            raise ValueError("kfo_select_evict rc=%d" % rc)
        return kept

    def beam_fork(self, parent):
        """Beam search with one cache per beam (Sec. 4: every evaluation uses 4 beams; Sec. 6: tokens are
        discarded across heads, layers and beams): row b of the batch continues the hypothesis that row
        parent[b] held before this step.  Rows that continue themselves keep their state; every other
        row receives a copy of its parent's live entries (K, V, score, pos, len).  A parent must continue
        itself -- the caller numbers the new beams so -- because its row is read while others are written."""
        parent = np.asarray(parent, np.int64)
        assert parent.shape == (self.B,)
        for b in range(self.B):
            pb = int(parent[b])
            if not (0 <= pb < self.B) or int(parent[pb]) != pb:
                raise ValueError("beam %d: parent %d does not continue itself" % (b, pb))
        for b in range(self.B):
            pb = int(parent[b])
            if pb == b:
                continue
            for l in range(self.L):
                for h in range(self.H):
                    m = int(self.len[l, pb, h])
                    for nm in ("K", "V", "score", "pos"):
                        getattr(self, nm)[l, b, h, :m] = getattr(self, nm)[l, pb, h, :m]
                    self.len[l, b, h] = m

