"""Double-precision CPU oracle for the ATOMO encoder/decoder (arXiv 1806.04090).

TEST INFRASTRUCTURE ONLY: imported by the test-suite, by the smoke check and by
the benchmark's cpu_baseline leg.  The HIP library never imports or calls it,
and this package imports nothing from the HIP side.

The arithmetic lives in ``atomo_oracle.c`` (plain C, fp64); this module only
marshals numpy arrays and chains the stages in the order of Section 3:
decomposition -> Algorithm 1 probabilities -> Bernoulli(p) -> lambda/p -> sum.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "atomo_oracle.c")
# ATOMO_ORACLE_SANITIZE=undefined builds and loads a second library with gcc's undefined-behaviour sanitizer
# (traps abort the process), which loads into a running interpreter as it is; the address sanitizer needs its
# runtime first in the process and is run on sanitize_driver.c instead (tests/test_oracle_sanitizers.py).
_SANITIZE = os.environ.get("ATOMO_ORACLE_SANITIZE", "")
_LIB = os.path.join(_HERE, "libatomo_oracle_ubsan.so" if _SANITIZE == "undefined" else "libatomo_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (a second or two).  Returns the library path."""
    if _SANITIZE not in ("", "undefined"):
        raise RuntimeError("ATOMO_ORACLE_SANITIZE supports only 'undefined'")
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        flags = ["-O2"] if not _SANITIZE else ["-O1", "-g", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
        subprocess.check_call(["gcc", *flags, "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c = ctypes
        dp, fp = c.POINTER(c.c_double), c.POINTER(c.c_float)
        u8p, i64p, u32p = c.POINTER(c.c_uint8), c.POINTER(c.c_int64), c.POINTER(c.c_uint32)
        lib.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_uniforms.argtypes = [c.c_uint64, c.c_uint64, c.c_int64, c.c_int64, fp]
        lib.oracle_uniforms.restype = None
        lib.oracle_bernoulli_mask.argtypes = [fp, c.c_int64, c.c_uint64, c.c_uint64, u8p]
        lib.oracle_bernoulli_mask.restype = None
        lib.oracle_probabilities.argtypes = [dp, c.c_int64, c.c_double, dp]
        lib.oracle_probabilities.restype = c.c_int64
        lib.oracle_svd.argtypes = [c.c_int32, c.c_int32, dp, dp, dp, dp]
        lib.oracle_svd.restype = c.c_int
        lib.oracle_pack_weights.argtypes = [dp, dp, u8p, c.c_int64, i64p, dp]
        lib.oracle_pack_weights.restype = c.c_int64
        lib.oracle_decode_svd_accumulate.argtypes = [c.c_int32, c.c_int32, c.c_int64, dp, dp, dp, c.c_double, dp]
        lib.oracle_decode_svd_accumulate.restype = None
        lib.oracle_decode_entrywise_accumulate.argtypes = [c.c_int64, i64p, dp, c.c_double, dp]
        lib.oracle_decode_entrywise_accumulate.restype = None
        lib.oracle_lq_norm.argtypes = [dp, c.c_int64, c.c_double, c.c_int]
        lib.oracle_lq_norm.restype = c.c_double
        lib.oracle_lq_probabilities.argtypes = [dp, c.c_int64, c.c_double, c.c_int, dp]
        lib.oracle_lq_probabilities.restype = c.c_double
        lib.oracle_decode_lq_accumulate.argtypes = [c.c_int64, i64p, c.POINTER(c.c_int8), c.c_double, c.c_double, dp]
        lib.oracle_decode_lq_accumulate.restype = None
        _lib = lib
    return _lib


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


# ---------------------------------------------------------------- stages ----

def philox4x32_10(ctr, key):
    """One Philox4x32-10 block: 4 counter words, 2 key words -> 4 output words."""
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _L().oracle_philox4x32_10(_ptr(ctr, ctypes.c_uint32), _ptr(key, ctypes.c_uint32), _ptr(out, ctypes.c_uint32))
    return out


def uniforms(seed: int, stream: int, n: int, first: int = 0):
    """u_i in [0,1) for atoms first..first+n of (seed, stream); float32, exact multiples of 2^-24."""
    u = np.empty(n, dtype=np.float32)
    _L().oracle_uniforms(seed, stream, first, n, _ptr(u, ctypes.c_float))
    return u


def bernoulli_mask(p32, seed: int, stream: int):
    """t_i = [u_i < p_i], compared in float32 on the float32 p handed in."""
    p32 = np.ascontiguousarray(p32, dtype=np.float32)
    mask = np.empty(p32.size, dtype=np.uint8)
    _L().oracle_bernoulli_mask(_ptr(p32, ctypes.c_float), p32.size, seed, stream, _ptr(mask, ctypes.c_uint8))
    return mask.astype(bool)


def probabilities(lam, s: float, return_forced: bool = False):
    """Algorithm 1 on lambda in any order; p comes back in the same order (float64)."""
    lam = np.ascontiguousarray(lam, dtype=np.float64)
    p = np.empty_like(lam)
    forced = _L().oracle_probabilities(_ptr(lam, ctypes.c_double), lam.size, float(s), _ptr(p, ctypes.c_double))
    return (p, int(forced)) if return_forced else p


def svd(G):
    """Thin SVD of a 2-D array (upcast to float64): (sigma desc, U m x r, V n x r), columns are atoms."""
    G = np.ascontiguousarray(G, dtype=np.float64)
    m, n = G.shape
    r = min(m, n)
    sigma = np.empty(r)
    U = np.empty((r, m))            # C column-major m x r  ==  numpy (r, m) row-major
    V = np.empty((r, n))
    sweeps = _L().oracle_svd(m, n, _ptr(G, ctypes.c_double), _ptr(sigma, ctypes.c_double),
                             _ptr(U, ctypes.c_double), _ptr(V, ctypes.c_double))
    if sweeps < 0:
        raise RuntimeError("oracle Jacobi SVD did not converge")
    return sigma, U.T, V.T


def pack_weights(lam, p, mask):
    """Kept atoms (ascending index) and their weights lambda_i / p_i."""
    lam = np.ascontiguousarray(lam, dtype=np.float64)
    p = np.ascontiguousarray(p, dtype=np.float64)
    m8 = np.ascontiguousarray(mask, dtype=np.uint8)
    idx = np.empty(lam.size, dtype=np.int64)
    w = np.empty(lam.size, dtype=np.float64)
    k = _L().oracle_pack_weights(_ptr(lam, ctypes.c_double), _ptr(p, ctypes.c_double), _ptr(m8, ctypes.c_uint8),
                                 lam.size, _ptr(idx, ctypes.c_int64), _ptr(w, ctypes.c_double))
    return idx[:k].copy(), w[:k].copy()


def decode_svd(messages, m: int, n: int, scale: float = 1.0):
    """Dense m x n float64 sum of the messages' kept rank-1 atoms, times scale.

    Each message is a dict with 'w' (k,), 'U' (m, k), 'V' (n, k); 'w' None marks the folded form, whose U
    columns are the weighted singular vectors (sigma / p) u (Section 6)."""
    out = np.zeros((m, n))
    for msg in messages:
        k = np.asarray(msg["U"]).shape[1] if np.asarray(msg["U"]).ndim == 2 else 0
        w = np.ones(k) if msg["w"] is None else np.ascontiguousarray(msg["w"], dtype=np.float64)
        k = w.size
        if k == 0:
            continue
        Uc = np.ascontiguousarray(np.asarray(msg["U"], dtype=np.float64).T)   # (k, m) == column-major m x k
        Vc = np.ascontiguousarray(np.asarray(msg["V"], dtype=np.float64).T)
        assert Uc.shape == (k, m) and Vc.shape == (k, n)
        _L().oracle_decode_svd_accumulate(m, n, k, _ptr(w, ctypes.c_double), _ptr(Uc, ctypes.c_double),
                                          _ptr(Vc, ctypes.c_double), float(scale), _ptr(out, ctypes.c_double))
    return out


def decode_entrywise(messages, n: int, scale: float = 1.0):
    """Dense length-n float64 sum of the messages' (idx, val) pairs, times scale."""
    out = np.zeros(n)
    for msg in messages:
        idx = np.ascontiguousarray(msg["idx"], dtype=np.int64)
        val = np.ascontiguousarray(msg["val"], dtype=np.float64)
        if idx.size:
            assert idx.min() >= 0 and idx.max() < n
            _L().oracle_decode_entrywise_accumulate(idx.size, _ptr(idx, ctypes.c_int64), _ptr(val, ctypes.c_double),
                                                    float(scale), _ptr(out, ctypes.c_double))
    return out


def lq_probabilities(g, q: float):
    """(p, ||g||_q) of l_q quantisation, p_i = |g_i| / ||g||_q (Section 4); q = float('inf') is the maximum norm."""
    g = np.ascontiguousarray(np.asarray(g, dtype=np.float64).ravel())
    p = np.empty_like(g)
    is_inf = 1 if np.isinf(q) else 0
    norm = _L().oracle_lq_probabilities(_ptr(g, ctypes.c_double), g.size, 0.0 if is_inf else float(q), is_inf,
                                        _ptr(p, ctypes.c_double))
    return p, float(norm)


def decode_lq(messages, n: int, scale: float = 1.0):
    """Dense length-n float64 sum of l_q messages {'idx', 'sign', 'norm'}, times scale."""
    out = np.zeros(n)
    for msg in messages:
        idx = np.ascontiguousarray(msg["idx"], dtype=np.int64)
        sign = np.ascontiguousarray(msg["sign"], dtype=np.int8)
        if idx.size:
            assert idx.min() >= 0 and idx.max() < n and set(np.unique(sign)) <= {-1, 1}
            _L().oracle_decode_lq_accumulate(idx.size, _ptr(idx, ctypes.c_int64), _ptr(sign, ctypes.c_int8),
                                             float(msg["norm"]), float(scale), _ptr(out, ctypes.c_double))
    return out


# ----------------------------------------------------------------- chains ----

def encode_svd(G, s: float, seed: int, stream: int, sigma_UV=None, p32=None):
    """Spectral-ATOMO encode of one matrix.  Optional sigma_UV / p32 splice in another
    implementation's decomposition / float32 probabilities."""
    sigma, U, V = svd(G) if sigma_UV is None else sigma_UV
    sigma = np.asarray(sigma, dtype=np.float64)
    p = probabilities(sigma, s)
    p_used32 = p.astype(np.float32) if p32 is None else np.asarray(p32, dtype=np.float32)
    mask = bernoulli_mask(p_used32, seed, stream)
    p_for_w = p if p32 is None else p_used32.astype(np.float64)
    idx, w = pack_weights(sigma, p_for_w, mask)
    return {"sigma": sigma, "p": p, "mask": mask, "idx": idx, "w": w,
            "U": np.asarray(U)[:, idx], "V": np.asarray(V)[:, idx]}


def fold_svd_message(msg):
    """The same message with the weight inside U: columns (sigma / p) u, no separate weights; rows + cols reals
    per kept atom, the communication cost s(n + m) of Table "matrix_sparse"."""
    out = dict(msg)
    out["U"] = np.asarray(msg["U"], dtype=np.float64) * np.asarray(msg["w"], dtype=np.float64)[None, :]
    out["w"] = None
    return out


def ps_update(params, worker_messages, gamma: float):
    """The parameter server's step of Section 2, w <- w - gamma * g_hat, with g_hat the average over the P
    workers of their decoded messages (Section 6).  params: list of m x n arrays, one per layer;
    worker_messages[l]: the P messages of layer l.  Returns the new float64 parameters."""
    out = []
    for w, msgs in zip(params, worker_messages):
        w = np.asarray(w, dtype=np.float64)
        g_hat = decode_svd(msgs, w.shape[0], w.shape[1], 1.0 / len(msgs))
        out.append(w - gamma * g_hat)
    return out


def encode_entrywise(g, s: float, seed: int, stream: int, p32=None):
    """Entry-wise ATOMO encode of a flat gradient: atoms e_i, lambda_i = g_i."""
    g = np.asarray(g, dtype=np.float64).ravel()
    p = probabilities(g, s)
    p_used32 = p.astype(np.float32) if p32 is None else np.asarray(p32, dtype=np.float32)
    mask = bernoulli_mask(p_used32, seed, stream)
    p_for_w = p if p32 is None else p_used32.astype(np.float64)
    idx, val = pack_weights(g, p_for_w, mask)
    return {"p": p, "mask": mask, "idx": idx, "val": val}


def encode_lq(g, q: float, seed: int, stream: int, p32=None):
    """l_q quantisation of a flat gradient (Section 4): kept coordinates (ascending), their signs, ||g||_q."""
    g = np.asarray(g, dtype=np.float64).ravel()
    p, norm = lq_probabilities(g, q)
    p_used32 = p.astype(np.float32) if p32 is None else np.asarray(p32, dtype=np.float32)
    mask = bernoulli_mask(p_used32, seed, stream)
    idx = np.flatnonzero(mask)
    return {"p": p, "mask": mask, "idx": idx, "sign": np.sign(g[idx]).astype(np.int8), "norm": norm}

