"""ctypes/numpy front end of the CPU oracle (TEST INFRASTRUCTURE, not product code).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the HIP package.
The arithmetic lives in ``kvq_oracle.c``; this file marshals numpy arrays and
chains the C calls (quantize -> dequantize -> attention) per head.  One step is
done here: the sign vector of the randomised rotation is applied by multiplying
the inputs (and the cached part of the output) by +-1 in numpy, which is exact.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvq_oracle.c")
_LIB = os.path.join(_HERE, "libkvq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile kvq_oracle.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    dp = ctypes.POINTER(ctypes.c_double)
    fp = ctypes.POINTER(ctypes.c_float)
    bp = ctypes.POINTER(ctypes.c_uint8)
    i64, ci, cd = ctypes.c_int64, ctypes.c_int, ctypes.c_double
    lib.kvqo_diagnostics.argtypes = [ci, ci, i64, i64, i64, dp, dp, dp, dp, dp, dp, dp, dp, cd, ci, ci, dp, dp]
    lib.kvqo_num_threads.restype = ci
    lib.kvqo_hadamard.argtypes = [ci, dp, dp]
    lib.kvqo_quantize_rows.argtypes = [i64, ci, ci, ci, ci, dp, bp, fp, fp]
    lib.kvqo_quantize_cols.argtypes = [i64, ci, ci, ci, dp, bp, fp, fp]
    lib.kvqo_quantize_rows_fp8meta.argtypes = [i64, ci, ci, ci, ci, dp, bp, fp, fp, bp]
    lib.kvqo_e4m3_ceil.argtypes = [cd, bp]
    lib.kvqo_e4m3_ceil.restype = cd
    lib.kvqo_bf16_round.argtypes = [cd]
    lib.kvqo_bf16_round.restype = cd
    lib.kvqo_dequantize_rows.argtypes = [i64, ci, ci, bp, fp, fp, dp]
    lib.kvqo_log_sinhc.argtypes = [cd]
    lib.kvqo_log_sinhc.restype = cd
    lib.kvqo_correction.argtypes = [ci, ci, dp, dp, cd, ci]
    lib.kvqo_correction.restype = cd
    lib.kvqo_attention.argtypes = [ci, ci, i64, i64, i64, dp, dp, dp, dp, dp, dp, cd, ci, ci, dp, dp]
    lib.kvqo_attention_masked.argtypes = [ci, ci, i64, i64, i64, dp, dp, dp, dp, dp, dp, cd, ci, ci, ci, dp, dp, dp]
    _lib = lib
    return lib


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def num_threads() -> int:
    return int(_load().kvqo_num_threads())


def hadamard(x) -> np.ndarray:
    """Unnormalised H_d x for one vector."""
    x = _d(x)
    u = np.empty_like(x)
    if _load().kvqo_hadamard(x.shape[0], _p(x, ctypes.c_double), _p(u, ctypes.c_double)):
        raise ValueError("hadamard: size must be a power of two")
    return u


def _signs(signs, d: int) -> Optional[np.ndarray]:
    if signs is None:
        return None
    s = _d(signs).reshape(d)
    if not np.all(np.abs(s) == 1.0):
        raise ValueError("signs must be +1 / -1")
    return s


def quantize(x, bits: int, group: Optional[int] = None, rotate: bool = True, fp8_meta: bool = False,
             signs=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """x [rows][d] -> codes uint8 [rows][d], scale float32 [rows][G], zero float32 [rows][G].

    fp8_meta: the stored scale is an FP8 E4M3 value and the stored zero-point a BF16 value.
    signs [d] of +1/-1 (with rotate): randomised Hadamard rotation, x -> Hn (signs * x)."""
    x = _d(x)
    if signs is not None and rotate:
        x = np.ascontiguousarray(x * _signs(signs, x.shape[1])[None, :])   # exact: entries are +-1
    rows, d = x.shape
    group = d if group is None else group
    codes = np.empty((rows, d), dtype=np.uint8)
    scale = np.empty((rows, d // group), dtype=np.float32)
    zero = np.empty((rows, d // group), dtype=np.float32)
    if fp8_meta:
        rc = _load().kvqo_quantize_rows_fp8meta(rows, d, bits, group, int(rotate), _p(x, ctypes.c_double),
                                                _p(codes, ctypes.c_uint8), _p(scale, ctypes.c_float),
                                                _p(zero, ctypes.c_float), None)
    else:
        rc = _load().kvqo_quantize_rows(rows, d, bits, group, int(rotate), _p(x, ctypes.c_double),
                                        _p(codes, ctypes.c_uint8), _p(scale, ctypes.c_float),
                                        _p(zero, ctypes.c_float))
    if rc:
        raise ValueError("quantize: bad arguments")
    return codes, scale, zero


def quantize_per_channel(x, bits: int, rotate: bool = True, signs=None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One block of tokens x [rows][d] -> codes uint8 [rows][d], scale float32 [d], zero float32 [d]: one
    (scale, zero-point) per channel of the (rotated) vectors, shared by all tokens of the block."""
    x = _d(x)
    rows, d = x.shape
    if signs is not None and rotate:
        x = np.ascontiguousarray(x * _signs(signs, d)[None, :])
    codes = np.empty((rows, d), dtype=np.uint8)
    scale = np.empty((d,), dtype=np.float32)
    zero = np.empty((d,), dtype=np.float32)
    if _load().kvqo_quantize_cols(rows, d, bits, int(rotate), _p(x, ctypes.c_double), _p(codes, ctypes.c_uint8),
                                  _p(scale, ctypes.c_float), _p(zero, ctypes.c_float)):
        raise ValueError("quantize_per_channel: bad arguments")
    return codes, scale, zero


def e4m3_ceil(x: float) -> Tuple[float, int]:
    """Smallest FP8 E4M3 value >= x (x > 0) and its encoding."""
    b = ctypes.c_uint8(0)
    v = float(_load().kvqo_e4m3_ceil(float(x), ctypes.byref(b)))
    return v, int(b.value)


def bf16_round(x: float) -> float:
    return float(_load().kvqo_bf16_round(float(x)))


def dequantize(codes, scale, zero) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    zero = np.ascontiguousarray(zero, dtype=np.float32)
    rows, d = codes.shape
    group = d // scale.shape[1]
    out = np.empty((rows, d), dtype=np.float64)
    if _load().kvqo_dequantize_rows(rows, d, group, _p(codes, ctypes.c_uint8), _p(scale, ctypes.c_float),
                                    _p(zero, ctypes.c_float), _p(out, ctypes.c_double)):
        raise ValueError("dequantize: bad arguments")
    return out


def log_sinhc(a: float) -> float:
    return float(_load().kvqo_log_sinhc(float(a)))


def correction(qv, step, sigma: float, mode: int) -> float:
    """b for one (query, key): qv [d] in the key's basis, step [G]; mode 0 off, 1 Taylor, 2 exact."""
    qv, step = _d(qv), _d(np.atleast_1d(step))
    d = qv.shape[0]
    return float(_load().kvqo_correction(d, d // step.shape[0], _p(qv, ctypes.c_double),
                                         _p(step, ctypes.c_double), float(sigma), int(mode)))


def attention(q, khat, kstep, vhat, kr, vr, sigma: Optional[float] = None, correction: int = 1,
              rotate: bool = True, causal: bool = False, signs=None) -> Tuple[np.ndarray, np.ndarray]:
    """One head.  q [m][d]; khat, vhat [ns][d]; kstep [ns][G]; kr, vr [nr][d] -> (out [m][d], P_S [m]).
    causal: current key j is visible to query r only if j <= r + nr - m.
    signs [d] of +1/-1: the cache basis is the randomised rotation x -> Hn (signs * x)."""
    q = _d(q)
    m, d = q.shape
    khat = _d(khat).reshape(-1, d)
    vhat = _d(vhat).reshape(-1, d)
    kr = _d(kr).reshape(-1, d)
    vr = _d(vr).reshape(-1, d)
    ns, nr = khat.shape[0], kr.shape[0]
    kstep = _d(kstep).reshape(ns, -1) if ns else np.zeros((0, 1))
    G = kstep.shape[1] if ns else 1
    sigma = 1.0 / np.sqrt(d) if sigma is None else float(sigma)
    out = np.empty((m, d), dtype=np.float64)
    mass = np.empty((m,), dtype=np.float64)
    sg = _signs(signs, d) if rotate else None
    rc = _load().kvqo_attention_masked(d, d // G, m, ns, nr, _p(q, ctypes.c_double), _p(khat, ctypes.c_double),
                                       _p(kstep, ctypes.c_double), _p(vhat, ctypes.c_double),
                                       _p(kr, ctypes.c_double), _p(vr, ctypes.c_double), sigma,
                                       int(correction), int(rotate), int(causal),
                                       None if sg is None else _p(sg, ctypes.c_double), _p(out, ctypes.c_double),
                                       _p(mass, ctypes.c_double))
    if rc:
        raise ValueError("attention: bad arguments")
    return out, mass


def chunk_attention(q, k_cached, v_cached, k_cur, v_cur, bits: int, correction: int = 1,
                    sigma: Optional[float] = None, group: Optional[int] = None, rotate: bool = True,
                    fp8_meta: bool = False, causal: bool = False, signs=None, key_blocks=None):
    """Whole path for [token][head][d] inputs: quantize the cached K/V per head, then attention.

    q may have a multiple of the K/V head count (grouped-query attention): query head h uses
    key/value head h // (q_heads // kv_heads).
    Returns (out [m][q_heads][d], P_S [q_heads][m], quantized) where quantized holds the
    per-KV-head codes / scales / zeros of K and V for parity checks.
    key_blocks: list of block lengths that add up to the cached tokens; the keys of each block are then
    quantized per channel (one scale / zero-point per channel, shared by the block's tokens), the values
    per token as always, and k_scale / k_zero are [tokens][d] (each token carries its block's values).
    """
    q = np.asarray(q)
    m, heads, d = q.shape
    kv_heads = np.asarray(k_cached).shape[1] if np.asarray(k_cached).shape[0] else np.asarray(k_cur).shape[1]
    assert heads % kv_heads == 0
    ratio = heads // kv_heads
    out = np.empty((m, heads, d), dtype=np.float64)
    mass = np.empty((heads, m), dtype=np.float64)
    quantized = []
    for g in range(kv_heads):
        if key_blocks is None:
            kc, ks, kz = quantize(np.asarray(k_cached)[:, g, :], bits, group, rotate, fp8_meta, signs)
        else:
            assert sum(key_blocks) == np.asarray(k_cached).shape[0]
            parts, t0 = [], 0
            for n in key_blocks:
                c_, s_, z_ = quantize_per_channel(np.asarray(k_cached)[t0:t0 + n, g, :], bits, rotate, signs)
                parts.append((c_, np.repeat(s_[None, :], n, axis=0), np.repeat(z_[None, :], n, axis=0)))
                t0 += n
            kc, ks, kz = (np.concatenate([p_[i] for p_ in parts]) if parts else np.zeros((0, d), dt)
                          for i, dt in ((0, np.uint8), (1, np.float32), (2, np.float32)))
        vc, vs, vz = quantize(np.asarray(v_cached)[:, g, :], bits, group, rotate, fp8_meta, signs)
        khat, vhat = dequantize(kc, ks, kz), dequantize(vc, vs, vz)
        for h in range(g * ratio, (g + 1) * ratio):
            o, p = attention(q[:, h, :], khat, ks, vhat, np.asarray(k_cur)[:, g, :], np.asarray(v_cur)[:, g, :],
                             sigma, correction, rotate, causal, signs)
            out[:, h, :] = o
            mass[h] = p
        quantized.append(dict(k_codes=kc, k_scale=ks, k_zero=kz, v_codes=vc, v_scale=vs, v_zero=vz))
    return out, mass, quantized


def diagnostics(q, khat, kstep, vhat, kref, vref, kr, vr, sigma: Optional[float] = None, correction: int = 1,
                rotate: bool = True, signs=None) -> np.ndarray:
    """One head.  Quantized (optionally corrected) attention against attention over the unquantized
    cache kref, vref [ns][d]: returns [m][4] = (P_S, P^_S, JSD(p, p^) in nats over all keys, output MSE)."""
    q = _d(q)
    m, d = q.shape
    khat, vhat = _d(khat).reshape(-1, d), _d(vhat).reshape(-1, d)
    kref, vref = _d(kref).reshape(-1, d), _d(vref).reshape(-1, d)
    kr, vr = _d(kr).reshape(-1, d), _d(vr).reshape(-1, d)
    ns, nr = khat.shape[0], kr.shape[0]
    assert kref.shape[0] == ns and vref.shape[0] == ns and vhat.shape[0] == ns
    kstep = _d(kstep).reshape(ns, -1) if ns else np.zeros((0, 1))
    G = kstep.shape[1] if ns else 1
    sigma = 1.0 / np.sqrt(d) if sigma is None else float(sigma)
    sg = _signs(signs, d) if rotate else None
    diag = np.empty((m, 4), dtype=np.float64)
    dp = ctypes.c_double
    rc = _load().kvqo_diagnostics(d, d // G, m, ns, nr, _p(q, dp), _p(khat, dp), _p(kstep, dp), _p(vhat, dp),
                                  _p(kref, dp), _p(vref, dp), _p(kr, dp), _p(vr, dp), sigma, int(correction),
                                  int(rotate), None if sg is None else _p(sg, dp), _p(diag, dp))
    if rc:
        raise ValueError("diagnostics: bad arguments")
    return diag


def chunk_diagnostics(q, k_cached, v_cached, k_cur, v_cur, bits: int, correction: int = 1,
                      sigma: Optional[float] = None, group: Optional[int] = None, rotate: bool = True,
                      fp8_meta: bool = False, signs=None) -> np.ndarray:
    """[token][head][d] inputs: quantize the cached K/V per head, then diagnostics -> [heads][m][4]."""
    q = np.asarray(q)
    m, heads, d = q.shape
    out = np.empty((heads, m, 4), dtype=np.float64)
    for h in range(heads):
        kc, ks, kz = quantize(np.asarray(k_cached)[:, h, :], bits, group, rotate, fp8_meta, signs)
        vc, vs, vz = quantize(np.asarray(v_cached)[:, h, :], bits, group, rotate, fp8_meta, signs)
        out[h] = diagnostics(q[:, h, :], dequantize(kc, ks, kz), ks, dequantize(vc, vs, vz),
                             np.asarray(k_cached)[:, h, :], np.asarray(v_cached)[:, h, :],
                             np.asarray(k_cur)[:, h, :], np.asarray(v_cur)[:, h, :], sigma, correction, rotate, signs)
    return out
