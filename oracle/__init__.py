"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this package.  It
compiles ``orthrus_oracle.c`` with gcc on first use (plain -O2, no fast-math, OpenMP over
independent outputs) and exposes the two oracle entry points on numpy arrays.  It imports
nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "orthrus_oracle.c")
_LIB = os.path.join(_HERE, "liborthrus_oracle.so")
# sanitizer builds (CPU test suite): the same source under AddressSanitizer + UndefinedBehaviorSanitizer as a
# library (selected with ORTHRUS_ORACLE_SANITIZE=1; load it with ASAN_OPTIONS=verify_asan_link_order=0) and
# as a self-contained driver executable (sanitize_selftest.c)
_LIB_SAN = os.path.join(_HERE, "liborthrus_oracle_asan.so")
_SELFTEST_SRC = os.path.join(_HERE, "sanitize_selftest.c")
_SELFTEST = os.path.join(_HERE, "sanitize_selftest")
_SAN_FLAGS = ["-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
              "-fno-omit-frame-pointer", "-Wall", "-Wextra"]

VIEW_DIFFUSION = 0
VIEW_AR_VERIFY = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle's C source into a shared library next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized() -> str:
    """The oracle as a shared library under ASan + UBSan (gcc's shared sanitizer runtimes)."""
    tmp = _LIB_SAN + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc"] + _SAN_FLAGS + ["-fPIC", "-shared", "-o", tmp, _SRC, "-lm"], check=True)
    os.replace(tmp, _LIB_SAN)
    return _LIB_SAN


def build_selftest() -> str:
    """The sanitizer driver executable: oracle + sanitize_selftest.c under ASan + UBSan."""
    tmp = _SELFTEST + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc"] + _SAN_FLAGS + ["-o", tmp, _SRC, _SELFTEST_SRC, "-lm"], check=True)
    os.replace(tmp, _SELFTEST)
    return _SELFTEST


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_sanitized() if os.environ.get("ORTHRUS_ORACLE_SANITIZE") == "1" else build())
        i32, i64, f64 = ctypes.c_int, ctypes.c_int64, ctypes.c_double
        p = ctypes.c_void_p
        lib.orthrus_oracle_num_threads.restype = ctypes.c_int
        lib.orthrus_oracle_dual_view_attn.restype = ctypes.c_int
        lib.orthrus_oracle_dual_view_attn.argtypes = [
            i32, i32, i32, i32, i32, i32, i32, i64, i32, f64,
            p, p, p, p, p, i64, i64, i64, p, p, p, p]
        lib.orthrus_oracle_consensus_commit.restype = ctypes.c_int
        lib.orthrus_oracle_consensus_commit.argtypes = [
            i32, i32, i32, i32, i32, i32, i32, i32, i64,
            p, p, p, p, p, p, i64, i64, i64, i64, p, p, p, p, p, p]
        lib.orthrus_oracle_sampling_consensus_commit.restype = ctypes.c_int
        lib.orthrus_oracle_sampling_consensus_commit.argtypes = [
            i32, i32, i32, f64, i32, i32, i32, i32, i32, i64,
            p, p, p, p, p, p, p, p, p, i64, i64, i64, i64, p, p, p, p, p, p, p, p]
        lib.orthrus_oracle_prefill_attn.restype = ctypes.c_int
        lib.orthrus_oracle_prefill_attn.argtypes = [
            i32, i32, i32, i32, i32, i32, i32, i64, f64,
            p, p, p, p, p, p, i64, i64, i64, p, p, p]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().orthrus_oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(a: np.ndarray, dtype, name: str) -> np.ndarray:
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("%s must be a C-contiguous %s array" % (name, np.dtype(dtype).name))
    return a


def _pool_strides(pool: np.ndarray):
    """Element strides (page, head, token) of a [pages, H_kv, P, d] pool."""
    if pool.ndim != 4:
        raise ValueError("pool must be [pages, H_kv, P, d]")
    es = pool.itemsize
    return pool.strides[0] // es, pool.strides[1] // es, pool.strides[2] // es


def dual_view_attn(view: int, sm_scale: float, q: np.ndarray, k_blk: np.ndarray, v_blk: np.ndarray,
                   k_pool: np.ndarray, v_pool: np.ndarray, page_table: np.ndarray,
                   seq_lens: np.ndarray, want_lse: bool = False):
    """Eq. 4 of the paper on bf16-bit inputs; returns fp64 ``out[B,K,H_q,d]`` (and ``lse[B,H_q,K]``)."""
    lib = _load()
    B, K, Hq, d = q.shape
    Hkv = k_blk.shape[2]
    _check(q, np.uint16, "q"); _check(k_blk, np.uint16, "k_blk"); _check(v_blk, np.uint16, "v_blk")
    _check(k_pool, np.uint16, "k_pool"); _check(v_pool, np.uint16, "v_pool")
    _check(page_table, np.int32, "page_table"); _check(seq_lens, np.int32, "seq_lens")
    if k_blk.shape != (B, K, Hkv, d) or v_blk.shape != k_blk.shape:
        raise ValueError("block K/V shape mismatch")
    if k_pool.shape != v_pool.shape or k_pool.shape[1] != Hkv or k_pool.shape[3] != d:
        raise ValueError("pool shape mismatch")
    sp, sh, st = _pool_strides(k_pool)
    out = np.empty((B, K, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq, K), dtype=np.float64) if want_lse else None
    rc = lib.orthrus_oracle_dual_view_attn(
        B, Hq, Hkv, d, K, k_pool.shape[2], page_table.shape[1], k_pool.shape[0], int(view),
        float(sm_scale), _ptr(q), _ptr(k_blk), _ptr(v_blk), _ptr(k_pool), _ptr(v_pool),
        sp, sh, st, _ptr(page_table), _ptr(seq_lens), _ptr(out), _ptr(lse))
    if rc != 0:
        raise RuntimeError("orthrus_oracle_dual_view_attn failed with status %d" % rc)
    return (out, lse) if want_lse else out


def prefill_attn(sm_scale: float, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, new_lens: np.ndarray,
                 k_pool: np.ndarray, v_pool: np.ndarray, page_table: np.ndarray, seq_lens: np.ndarray,
                 allow_capacity_error: bool = False):
    """AR prefill of one layer: appends the new tokens' K/V, causal attention of each over the cache.

    ``q`` is ``[B,T,H_q,d]``, ``k_new``/``v_new`` ``[B,T,H_kv,d]`` (bf16 bits), ``new_lens[b] <= T``;
    pools and ``seq_lens`` are updated in place.  Returns fp64 ``out[B,T,H_q,d]`` (rows past
    ``new_lens[b]`` are NaN) and the status (0, or -4 when allowed).
    """
    lib = _load()
    B, T, Hq, d = q.shape
    Hkv = k_new.shape[2]
    for a, n in ((q, "q"), (k_new, "k_new"), (v_new, "v_new"), (k_pool, "k_pool"), (v_pool, "v_pool")):
        _check(a, np.uint16, n)
    _check(page_table, np.int32, "page_table"); _check(seq_lens, np.int32, "seq_lens")
    _check(new_lens, np.int32, "new_lens")
    if k_new.shape != (B, T, Hkv, d) or v_new.shape != k_new.shape:
        raise ValueError("new K/V shape mismatch")
    if k_pool.shape != v_pool.shape or k_pool.shape[1] != Hkv or k_pool.shape[3] != d:
        raise ValueError("pool shape mismatch")
    sp, sh, st = _pool_strides(k_pool)
    out = np.full((B, T, Hq, d), np.nan, dtype=np.float64)
    rc = lib.orthrus_oracle_prefill_attn(
        B, T, Hq, Hkv, d, k_pool.shape[2], page_table.shape[1], k_pool.shape[0], float(sm_scale),
        _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(new_lens), _ptr(k_pool), _ptr(v_pool), sp, sh, st,
        _ptr(page_table), _ptr(seq_lens), _ptr(out))
    if rc != 0 and not (rc == -4 and allow_capacity_error):
        raise RuntimeError("orthrus_oracle_prefill_attn failed with status %d" % rc)
    return out, rc


def consensus_commit(ar_logits: np.ndarray, draft_tokens: np.ndarray,
                     k_blk_ar: Optional[np.ndarray] = None, v_blk_ar: Optional[np.ndarray] = None,
                     k_pool: Optional[np.ndarray] = None, v_pool: Optional[np.ndarray] = None,
                     page_table: Optional[np.ndarray] = None, seq_lens: Optional[np.ndarray] = None,
                     allow_capacity_error: bool = False) -> Dict[str, np.ndarray]:
    """Eq. 8 consensus plus in-place commit.

    ``k_blk_ar``/``v_blk_ar`` are ``[layers,B,K,H_kv,d]`` (or ``[B,K,H_kv,d]`` for one layer);
    pools are ``[layers,pages,H_kv,P,d]`` or ``[pages,H_kv,P,d]``; both pools and ``seq_lens``
    are updated in place.  With the K/V arguments omitted only the consensus outputs are made.
    """
    lib = _load()
    B, K, V = ar_logits.shape
    _check(ar_logits, np.float32, "ar_logits"); _check(draft_tokens, np.int32, "draft_tokens")
    accept_len = np.empty(B, np.int32); num_committed = np.empty(B, np.int32)
    out_tokens = np.empty((B, K), np.int32); next_anchor = np.empty(B, np.int32)
    if k_blk_ar is None:
        rc = lib.orthrus_oracle_consensus_commit(
            B, K, V, 0, 0, 0, 0, 0, 0, _ptr(ar_logits), _ptr(draft_tokens), None, None, None, None,
            0, 0, 0, 0, None, None, _ptr(accept_len), _ptr(num_committed), _ptr(out_tokens),
            _ptr(next_anchor))
    else:
        kb = k_blk_ar if k_blk_ar.ndim == 5 else k_blk_ar[None]
        vb = v_blk_ar if v_blk_ar.ndim == 5 else v_blk_ar[None]
        kp = k_pool if k_pool.ndim == 5 else k_pool[None]
        vp = v_pool if v_pool.ndim == 5 else v_pool[None]
        for a, n in ((kb, "k_blk_ar"), (vb, "v_blk_ar"), (kp, "k_pool"), (vp, "v_pool")):
            _check(a, np.uint16, n)
        _check(page_table, np.int32, "page_table"); _check(seq_lens, np.int32, "seq_lens")
        layers, _, _, Hkv, d = kb.shape
        if kb.shape != (layers, B, K, Hkv, d) or vb.shape != kb.shape:
            raise ValueError("block K/V shape mismatch")
        if kp.shape != vp.shape or kp.shape[0] != layers or kp.shape[2] != Hkv or kp.shape[4] != d:
            raise ValueError("pool shape mismatch")
        es = kp.itemsize
        sl, sp, sh, st = (kp.strides[0] // es, kp.strides[1] // es, kp.strides[2] // es,
                          kp.strides[3] // es)
        rc = lib.orthrus_oracle_consensus_commit(
            B, K, V, layers, Hkv, d, kp.shape[3], page_table.shape[1], kp.shape[1],
            _ptr(ar_logits), _ptr(draft_tokens), _ptr(kb), _ptr(vb), _ptr(kp), _ptr(vp),
            sl, sp, sh, st, _ptr(page_table), _ptr(seq_lens), _ptr(accept_len),
            _ptr(num_committed), _ptr(out_tokens), _ptr(next_anchor))
    if rc != 0 and not (rc == -4 and allow_capacity_error):
        raise RuntimeError("orthrus_oracle_consensus_commit failed with status %d" % rc)
    return dict(accept_len=accept_len, num_committed=num_committed, out_tokens=out_tokens,
                next_anchor=next_anchor, status=rc)


def sampling_consensus_commit(ar_logits: np.ndarray, diff_logits: np.ndarray, draft_tokens: np.ndarray,
                              accept_u: np.ndarray, gumbel: np.ndarray, temperature: float,
                              k_blk_ar: Optional[np.ndarray] = None, v_blk_ar: Optional[np.ndarray] = None,
                              k_pool: Optional[np.ndarray] = None, v_pool: Optional[np.ndarray] = None,
                              page_table: Optional[np.ndarray] = None, seq_lens: Optional[np.ndarray] = None,
                              allow_capacity_error: bool = False) -> Dict[str, np.ndarray]:
    """Temperature > 0 consensus (speculative-sampling accept/replace rule) plus in-place commit.

    Shapes as in ``consensus_commit``; ``diff_logits`` like ``ar_logits``; ``accept_u`` is ``[B,K]``
    fp32 in [0,1), ``gumbel`` is ``[B,V]`` fp32 standard Gumbel noise.  Also returns the decision
    margins the oracle reports (``margin_accept [B,K]``, ``margin_draw [B]``).
    """
    lib = _load()
    B, K, V = ar_logits.shape
    for a, n in ((ar_logits, "ar_logits"), (diff_logits, "diff_logits"), (accept_u, "accept_u"), (gumbel, "gumbel")):
        _check(a, np.float32, n)
    _check(draft_tokens, np.int32, "draft_tokens")
    if diff_logits.shape != (B, K, V) or accept_u.shape != (B, K) or gumbel.shape != (B, V):
        raise ValueError("sampling input shape mismatch")
    accept_len = np.empty(B, np.int32); num_committed = np.empty(B, np.int32)
    out_tokens = np.empty((B, K), np.int32); next_anchor = np.empty(B, np.int32)
    m_acc = np.empty((B, K), np.float64); m_draw = np.empty(B, np.float64)
    if k_blk_ar is None:
        rc = lib.orthrus_oracle_sampling_consensus_commit(
            B, K, V, float(temperature), 0, 0, 0, 0, 0, 0, _ptr(ar_logits), _ptr(diff_logits),
            _ptr(draft_tokens), _ptr(accept_u), _ptr(gumbel), None, None, None, None, 0, 0, 0, 0, None, None,
            _ptr(accept_len), _ptr(num_committed), _ptr(out_tokens), _ptr(next_anchor), _ptr(m_acc), _ptr(m_draw))
    else:
        kb = k_blk_ar if k_blk_ar.ndim == 5 else k_blk_ar[None]
        vb = v_blk_ar if v_blk_ar.ndim == 5 else v_blk_ar[None]
        kp = k_pool if k_pool.ndim == 5 else k_pool[None]
        vp = v_pool if v_pool.ndim == 5 else v_pool[None]
        for a, n in ((kb, "k_blk_ar"), (vb, "v_blk_ar"), (kp, "k_pool"), (vp, "v_pool")):
            _check(a, np.uint16, n)
        _check(page_table, np.int32, "page_table"); _check(seq_lens, np.int32, "seq_lens")
        layers, _, _, Hkv, d = kb.shape
        es = kp.itemsize
        sl, sp, sh, st = (kp.strides[0] // es, kp.strides[1] // es, kp.strides[2] // es, kp.strides[3] // es)
        rc = lib.orthrus_oracle_sampling_consensus_commit(
            B, K, V, float(temperature), layers, Hkv, d, kp.shape[3], page_table.shape[1], kp.shape[1],
            _ptr(ar_logits), _ptr(diff_logits), _ptr(draft_tokens), _ptr(accept_u), _ptr(gumbel),
            _ptr(kb), _ptr(vb), _ptr(kp), _ptr(vp), sl, sp, sh, st, _ptr(page_table), _ptr(seq_lens),
            _ptr(accept_len), _ptr(num_committed), _ptr(out_tokens), _ptr(next_anchor), _ptr(m_acc), _ptr(m_draw))
    if rc != 0 and not (rc == -4 and allow_capacity_error):
        raise RuntimeError("orthrus_oracle_sampling_consensus_commit failed with status %d" % rc)
    return dict(accept_len=accept_len, num_committed=num_committed, out_tokens=out_tokens,
                next_anchor=next_anchor, status=rc, margin_accept=m_acc, margin_draw=m_draw)


def block_mask_attn(sm_scale: float, block_k: int, anchors: np.ndarray, q_diff: np.ndarray,
                    k_ar: np.ndarray, v_ar: np.ndarray, k_diff: np.ndarray, v_diff: np.ndarray) -> np.ndarray:
    """Diffusion-view attention under the training block mask M_diff (Section 3.2, Eq. 6), evaluated literally.

    The key axis is the L clean AR keys followed by the NB*K diffusion keys of all blocks.  For the diffusion
    query at index qi (block nb = qi // K, anchor a = anchors[nb]) and key index k:
        allowed  <=>  (k < L and k <= a - 1)  or  (k >= L and qi // K == (k - L) // K)
    Dense scores over the whole key axis, the mask, a softmax and the weighted sum, in fp64 with numpy
    (one query head at a time).  ``q_diff`` [NB*K,H_q,d], ``k_ar``/``v_ar`` [L,H_kv,d],
    ``k_diff``/``v_diff`` [NB*K,H_kv,d] as bf16 bit patterns; returns fp64 [NB*K,H_q,d].
    """
    from orthrus_inputs import bf16_bits_to_f32
    f = lambda a: bf16_bits_to_f32(a).astype(np.float64)
    Q, KA, VA, KD, VD = f(q_diff), f(k_ar), f(v_ar), f(k_diff), f(v_diff)
    NQ, Hq, d = Q.shape
    L, Hkv, _ = KA.shape
    K = int(block_k)
    if NQ % K or KD.shape[0] != NQ or len(anchors) != NQ // K:
        raise ValueError("shape mismatch")
    G = Hq // Hkv
    qi = np.arange(NQ)[:, None]
    kk = np.arange(L + NQ)[None, :]
    a_of_q = np.asarray(anchors, dtype=np.int64)[qi // K]
    allowed = ((kk < L) & (kk <= a_of_q - 1)) | ((kk >= L) & (qi // K == (kk - L) // K))
    out = np.empty((NQ, Hq, d), dtype=np.float64)
    for h in range(Hq):
        g = h // G
        keys = np.concatenate([KA[:, g], KD[:, g]])
        vals = np.concatenate([VA[:, g], VD[:, g]])
        s = (Q[:, h] @ keys.T) * float(sm_scale)
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        out[:, h] = p @ vals
    return out
