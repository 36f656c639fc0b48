"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run the library
through its C ABI (via the ctypes binding), and run the CPU oracle on the same inputs."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2605_26266_amd import binding as B
from paper_2605_26266_amd import workloads as wl

DEV = "cuda:0"

# Tolerances of the parity bar (floating point): outputs within 2e-2 max-abs for BF16 I/O,
# 1e-4 for the fp32 path; attention masses within 1e-3 relative (compared where the mass is
# at least 1e-6).
TOL_OUT_BF16 = 2e-2
TOL_OUT_FP32 = 1e-4
TOL_MASS_REL = 1e-3
MASS_FLOOR = 1e-6


def to_dev(x: np.ndarray, io_dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV)
    return t.to(torch.bfloat16) if io_dtype == "bf16" else t


def make_cache(w: wl.Workload, capacity: int, heads: int = None, group: int = None, fp8_meta: bool = False,
               per_channel_keys: bool = False) -> B.Cache:
    io = B.KVQ_BF16 if w.io_dtype == "bf16" else B.KVQ_FP32
    meta = B.KVQ_META_FP8_BF16 if fp8_meta else B.KVQ_META_FP32
    axis = B.KVQ_KEYS_PER_CHANNEL if per_channel_keys else B.KVQ_KEYS_PER_TOKEN
    return B.Cache(B.make_desc(w.num_heads if heads is None else heads, w.head_dim, w.bits, capacity, io,
                               group_size=group, meta_format=meta, key_axis=axis), DEV)


def export_np(cache: B.Cache, which: int, start: int = 0, count: int = None):
    codes, scales, zeros = B.export_all(cache, which, start, count)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), scales.cpu().numpy(), zeros.cpu().numpy()


def assert_quantized_equal(cache: B.Cache, k: np.ndarray, v: np.ndarray, heads=None, start: int = 0, signs=None):
    """Bit-exact comparison of the exported cache rows [start, start+n) with the oracle's quantizer.

    k, v: float32 [n][heads_in_k][d] holding exactly the appended values for `heads` (default all)."""
    n = k.shape[0]
    hs = list(range(cache.desc.num_heads)) if heads is None else list(heads)
    bits = cache.desc.bits
    fp8_meta = cache.desc.meta_format == B.KVQ_META_FP8_BF16
    group = cache.desc.group_size
    for which, x in ((0, k), (1, v)):
        codes, scales, zeros = export_np(cache, which, start, n)
        scales, zeros = scales.reshape(scales.shape[0], n, -1), zeros.reshape(zeros.shape[0], n, -1)
        for j, h in enumerate(hs):
            oc, osc, oz = oracle.quantize(x[:, j, :].astype(np.float64), bits, group, True, fp8_meta, signs)
            assert np.array_equal(codes[h], oc), "codes differ: tensor %d head %d (%d elements)" % (
                which, h, int(np.sum(codes[h] != oc)))
            bad = np.nonzero(np.any(scales[h].view(np.uint32) != osc.view(np.uint32), axis=1))[0]
            assert bad.size == 0, "scales differ: tensor %d head %d rows %s: %s vs %s" % (
                which, h, bad[:8], scales[h][bad[:8]], osc[bad[:8]])
            # zero-points are integers; +0 and -0 are the same zero-point
            bad = np.nonzero(np.any(zeros[h] != oz, axis=1))[0]
            assert bad.size == 0, "zero-points differ at rows %s: %s vs %s" % (bad[:8], zeros[h][bad[:8]], oz[bad[:8]])


def run_gpu_attention(cache, q, k_cur, v_cur, io_dtype, cache_start=0, cache_len=None, correction=1,
                      softmax_scale=0.0, fp32_kernel=False, causal=None):
    """q/k_cur/v_cur: float32 numpy [tokens][H][d].  Returns (out float64 [m][H][d], mass float64 [H][m]).
    causal not None: the extended entry point (grouped query heads, optional causal current block)."""
    cache_len = len(cache) - cache_start if cache_len is None else cache_len
    qd = to_dev(q, io_dtype)
    kd = to_dev(k_cur, io_dtype) if k_cur is not None and k_cur.shape[0] else None
    vd = to_dev(v_cur, io_dtype) if v_cur is not None and v_cur.shape[0] else None
    out = torch.full_like(qd, float("nan"))
    mass = torch.full((q.shape[1], q.shape[0]), float("nan"), dtype=torch.float32, device=DEV)
    if causal is not None:
        B.kvq_chunk_attention_ex(cache, cache_start, cache_len, qd, kd, vd, out, mass, softmax_scale, correction,
                                 causal=causal)
        torch.cuda.synchronize()
        return out.float().cpu().numpy().astype(np.float64), mass.cpu().numpy().astype(np.float64)
    fn = B.kvq_chunk_attention_fp32 if fp32_kernel else B.kvq_chunk_attention
    fn(cache, cache_start, cache_len, qd, kd, vd, out, mass, softmax_scale, correction)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), mass.cpu().numpy().astype(np.float64)


def assert_attention_close(out_gpu, mass_gpu, out_ref, mass_ref, tol_out, what="", mass_floor=None):
    """mass_floor: smallest probability the relative bar is applied to (default MASS_FLOOR).  P_R is
    derived from the fp32 P_S that the call returns, which resolves 6e-8 near 1: rows that see one or two
    current keys under a causal mask need a higher floor for the bar to measure the kernel, not the format."""
    mass_floor = MASS_FLOOR if mass_floor is None else mass_floor
    assert np.all(np.isfinite(out_gpu)), what + ": non-finite output"
    err = float(np.max(np.abs(out_gpu - out_ref)))
    assert err <= tol_out, "%s: max |O - O_oracle| = %.3e > %.1e" % (what, err, tol_out)
    for got, ref, name in ((mass_gpu, mass_ref, "P_S"), (1.0 - mass_gpu, 1.0 - mass_ref, "P_R")):
        sel = ref >= mass_floor
        if np.any(sel):
            rel = float(np.max(np.abs(got[sel] - ref[sel]) / ref[sel]))
            assert rel <= TOL_MASS_REL, "%s: %s relative error %.3e > %.0e" % (what, name, rel, TOL_MASS_REL)
    return err
