"""GPU parity of per-channel key quantization (appendix "Per-Channel Quantization Correction"): codes,
per-channel scales and zero-points bit-exact against the oracle for every appended block, values per
token as always, and attention with one correction scalar per query and block."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import parity
    return parity


def _assert_key_blocks_equal(P, cache, k, blocks, start=0):
    import oracle
    codes, scales, zeros = P.export_np(cache, 0, start, k.shape[0])
    t0 = 0
    for n in blocks:
        for h in range(k.shape[1]):
            oc, osc, oz = oracle.quantize_per_channel(k[t0:t0 + n, h, :].astype(np.float64), cache.desc.bits)
            assert np.array_equal(codes[h, t0:t0 + n], oc), "codes differ: block at %d head %d" % (t0, h)
            assert np.array_equal(scales[h, t0:t0 + n].view(np.uint32), np.repeat(osc[None, :], n, 0).view(np.uint32))
            assert np.all(zeros[h, t0:t0 + n] == oz[None, :])
        t0 += n


@pytest.mark.parametrize("name,io,bits", [("small", "bf16", 2), ("small", "bf16", 4), ("tiny", "fp32", 2)])
def test_per_channel_keys(P, name, io, bits):
    import oracle
    from dataclasses import replace
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = replace(wl.WORKLOADS[name], io_dtype=io, bits=bits)
    heads = min(2, w.num_heads)
    blocks = [min(200, w.chunk_tokens), 37, min(96, w.chunk_tokens), 1]       # ragged: blocks start inside tiles
    cache = P.make_cache(w, sum(blocks) + 10, heads=heads, per_channel_keys=True)
    ks, vs = [], []
    for i, n in enumerate(blocks):
        k, v = wl.chunk_kv(w, i, heads=range(heads), n_tokens=n)
        B.kvq_quantize_append(cache, P.to_dev(k, io), P.to_dev(v, io))
        ks.append(k); vs.append(v)
    kc, vc = np.concatenate(ks), np.concatenate(vs)
    _assert_key_blocks_equal(P, cache, kc, blocks)
    # values are quantized per token exactly as in a per-token cache
    vcodes, vscale, vzero = P.export_np(cache, 1)
    for h in range(heads):
        oc, osc, oz = oracle.quantize(vc[:, h, :].astype(np.float64), bits)
        assert np.array_equal(vcodes[h], oc) and np.array_equal(vscale[h], osc[:, 0]) and np.all(vzero[h] == oz[:, 0])
    q = wl.chunk_q(w, heads=range(heads))[:50]
    kr, vr = wl.chunk_kv(w, 9, heads=range(heads), n_tokens=min(70, w.chunk_tokens))
    tol = P.TOL_OUT_BF16 if io == "bf16" else P.TOL_OUT_FP32
    for correction in (0, 1, 2):
        ref, mass_ref, _ = oracle.chunk_attention(q, kc, vc, kr, vr, bits, correction, key_blocks=blocks)
        # default dispatch (BF16, d = 128, Taylor or no correction: matrix cores, one pass per key block) and the vector kernel
        for fp32_kernel in (False, True):
            out, mass = P.run_gpu_attention(cache, q, kr, vr, io, correction=correction, fp32_kernel=fp32_kernel)
            P.assert_attention_close(out, mass, ref, mass_ref, tol, "per-channel keys, correction %d" % correction)
    # a window that starts inside the first block and ends inside the third
    s0 = 150 if blocks[0] > 150 else 10
    ln = sum(blocks[:2]) + 20 - s0
    # the oracle quantizes whole blocks: take its dequantized keys for the window from the full call
    ref_full = oracle.chunk_attention(q, kc, vc, kr, vr, bits, 1, key_blocks=blocks)[2]
    out, mass = P.run_gpu_attention(cache, q, kr, vr, io, cache_start=s0, cache_len=ln)
    refs = []
    for h in range(heads):
        qd = ref_full[h]
        khat = oracle.dequantize(qd["k_codes"][s0:s0 + ln], qd["k_scale"][s0:s0 + ln], qd["k_zero"][s0:s0 + ln])
        vhat = oracle.dequantize(qd["v_codes"][s0:s0 + ln], qd["v_scale"][s0:s0 + ln], qd["v_zero"][s0:s0 + ln])
        refs.append(oracle.attention(q[:, h, :], khat, qd["k_scale"][s0:s0 + ln], vhat, kr[:, h, :], vr[:, h, :]))
    ref = np.stack([r[0] for r in refs], axis=1)
    mass_ref = np.stack([r[1] for r in refs])
    P.assert_attention_close(out, mass, ref, mass_ref, tol, "per-channel keys, window")


def test_per_channel_keys_many_tiles(P):
    """Five blocks of 1000 tokens (none of them a whole number of tiles), 300 query rows, outlier channels:
    the block-by-block matrix-core path over several stages per block, with a window that cuts two blocks."""
    import oracle
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["small"]
    heads, nblk, blen = 2, 5, 1000
    cache = P.make_cache(w, nblk * blen + 24, heads=heads, per_channel_keys=True)
    ks, vs = [], []
    for i in range(nblk):
        k, v = wl.chunk_kv(w, i, heads=range(heads), n_tokens=blen)
        B.kvq_quantize_append(cache, P.to_dev(k, "bf16"), P.to_dev(v, "bf16"))
        ks.append(k); vs.append(v)
    kc, vc = np.concatenate(ks), np.concatenate(vs)
    q = wl.chunk_q(w, heads=range(heads))[:300]
    kr, vr = wl.chunk_kv(w, 9, heads=range(heads), n_tokens=500)
    for correction in (1, 0):
        ref, mass_ref, qds = oracle.chunk_attention(q, kc, vc, kr, vr, 2, correction, key_blocks=[blen] * nblk)
        if correction == 1:
            full = qds
        out, mass = P.run_gpu_attention(cache, q, kr, vr, "bf16", correction=correction)
        P.assert_attention_close(out, mass, ref, mass_ref, P.TOL_OUT_BF16, "per-channel, 5 x 1000 tokens, correction %d" % correction)
    s0, ln = 700, 2900                                   # from inside block 0 to inside block 3
    refs = []
    for h in range(heads):
        qd = full[h]
        khat = oracle.dequantize(qd["k_codes"][s0:s0 + ln], qd["k_scale"][s0:s0 + ln], qd["k_zero"][s0:s0 + ln])
        vhat = oracle.dequantize(qd["v_codes"][s0:s0 + ln], qd["v_scale"][s0:s0 + ln], qd["v_zero"][s0:s0 + ln])
        refs.append(oracle.attention(q[:, h, :], khat, qd["k_scale"][s0:s0 + ln], vhat, kr[:, h, :], vr[:, h, :]))
    out, mass = P.run_gpu_attention(cache, q, kr, vr, "bf16", cache_start=s0, cache_len=ln)
    P.assert_attention_close(out, mass, np.stack([r[0] for r in refs], axis=1), np.stack([r[1] for r in refs]),
                             P.TOL_OUT_BF16, "per-channel, window over four blocks")


def test_per_channel_partly_evicted_block_and_grouped_heads(P):
    """A block that has lost its first tokens keeps the parameters of the whole block; grouped query heads and
    the causal current block work on the block-by-block path as on the others."""
    import oracle
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["small"]
    heads, blocks = 2, [100, 100, 60]
    cache = P.make_cache(w, 288, heads=heads, per_channel_keys=True)
    ks, vs = [], []
    for i, n in enumerate(blocks):
        k, v = wl.chunk_kv(w, i, heads=range(heads), n_tokens=n)
        B.kvq_quantize_append(cache, P.to_dev(k, "bf16"), P.to_dev(v, "bf16"))
        ks.append(k); vs.append(v)
    kc, vc = np.concatenate(ks), np.concatenate(vs)
    B.kvq_cache_evict(cache, 32)
    q4 = wl.chunk_q(w, heads=range(2 * heads))[:64]               # two query heads per key/value head
    kr, vr = wl.chunk_kv(w, 9, heads=range(heads), n_tokens=64)
    full = oracle.chunk_attention(q4[:, :heads], kc, vc, kr, vr, 2, 1, key_blocks=blocks)[2]
    for causal in (False, True):
        refs = []
        for qh in range(2 * heads):
            qd = full[qh // 2]
            khat = oracle.dequantize(qd["k_codes"][32:], qd["k_scale"][32:], qd["k_zero"][32:])
            vhat = oracle.dequantize(qd["v_codes"][32:], qd["v_scale"][32:], qd["v_zero"][32:])
            refs.append(oracle.attention(q4[:, qh, :], khat, qd["k_scale"][32:], vhat, kr[:, qh // 2, :], vr[:, qh // 2, :],
                                         causal=causal))
        ref, mass_ref = np.stack([r[0] for r in refs], axis=1), np.stack([r[1] for r in refs])
        out, mass = P.run_gpu_attention(cache, q4, kr, vr, "bf16", causal=causal)
        P.assert_attention_close(out, mass, ref, mass_ref, P.TOL_OUT_BF16, "per-channel, evicted head of a block, causal %s" % causal,
                                 mass_floor=1e-4 if causal else None)


def test_per_channel_ring_and_block_limit(P):
    """Blocks are evicted with their tokens; slots are reused; more live blocks than the storage has slots
    for is refused."""
    import oracle
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["small"]
    heads, chunk = 2, 64
    cache = P.make_cache(w, 3 * chunk, heads=heads, per_channel_keys=True)     # 6 tiles -> 8 block slots
    live = []
    q = wl.chunk_q(w, heads=range(heads))[:40]
    kr, vr = wl.chunk_kv(w, 30, heads=range(heads), n_tokens=33)
    for c in range(14):
        k, v = wl.chunk_kv(w, c, heads=range(heads), n_tokens=chunk)
        if len(live) == 3:
            B.kvq_cache_evict(cache, chunk)
            live.pop(0)
        B.kvq_quantize_append(cache, P.to_dev(k, "bf16"), P.to_dev(v, "bf16"))
        live.append((k, v))
        if c in (2, 5, 9, 13):
            kc, vc = np.concatenate([x[0] for x in live]), np.concatenate([x[1] for x in live])
            _assert_key_blocks_equal(P, cache, kc, [chunk] * len(live))
            ref, mass_ref, _ = oracle.chunk_attention(q, kc, vc, kr, vr, 2, 1, key_blocks=[chunk] * len(live))
            out, mass = P.run_gpu_attention(cache, q, kr, vr, "bf16")
            P.assert_attention_close(out, mass, ref, mass_ref, P.TOL_OUT_BF16, "per-channel ring %d" % c)
    B.kvq_cache_reset(cache)
    one_k, one_v = wl.chunk_kv(w, 0, heads=range(heads), n_tokens=1)
    for i in range(8):                                   # eight one-token blocks fill the slots
        B.kvq_quantize_append(cache, P.to_dev(one_k, "bf16"), P.to_dev(one_v, "bf16"))
    with pytest.raises(B.KvqError) as e:
        B.kvq_quantize_append(cache, P.to_dev(one_k, "bf16"), P.to_dev(one_v, "bf16"))
    assert e.value.status == B.KVQ_ERR_CAPACITY
    B.kvq_cache_truncate(cache, 7)                       # dropping the newest block frees its slot
    B.kvq_quantize_append(cache, P.to_dev(one_k, "bf16"), P.to_dev(one_v, "bf16"))
    assert len(cache) == 8


def test_per_channel_needs_fp32_metadata(P):
    from paper_2605_26266_amd import binding as B
    d = B.make_desc(2, 128, 2, 64, B.KVQ_BF16, group_size=32, meta_format=B.KVQ_META_FP8_BF16, key_axis=B.KVQ_KEYS_PER_CHANNEL)
    assert B.kvq_cache_bytes(d) == 0 and B.kvq_cache_create_status(d) == B.KVQ_ERR_UNSUPPORTED
