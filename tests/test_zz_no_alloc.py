"""kvq_quantize_append_static (the entry point that allocates nothing and keeps the per-channel work space of an
append in the library's static device array) against kvq_quantize_append: bit-identical caches and attention
outputs, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import parity
    return parity


@pytest.mark.parametrize("bits", [2, 4])
def test_static_work_space_gives_the_same_cache(P, bits):
    from dataclasses import replace
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = replace(wl.WORKLOADS["small"], bits=bits)
    heads = 4
    blocks = [300, 70]                                   # two appends in a row, the second smaller
    ref_cache = P.make_cache(w, sum(blocks) + 32, heads=heads, per_channel_keys=True)
    new_cache = P.make_cache(w, sum(blocks) + 32, heads=heads, per_channel_keys=True)
    # the work space inside the new cache's storage must not be what makes it work: poison the whole storage
    new_cache.storage.fill_(0xFF)
    for i, n in enumerate(blocks):
        k, v = wl.chunk_kv(w, i, heads=range(heads), n_tokens=n)
        kd, vd = P.to_dev(k, "bf16"), P.to_dev(v, "bf16")
        B.kvq_quantize_append(ref_cache, kd, vd)
        held = torch.cuda.memory_allocated()
        B.kvq_quantize_append_static(new_cache, kd, vd)
        assert torch.cuda.memory_allocated() == held     # nothing went through torch's allocator
        for which in (0, 1):
            a = B.export_all(ref_cache, which)
            b = B.export_all(new_cache, which)
            torch.cuda.synchronize()
            for x, y, name in zip(a, b, ("codes", "scales", "zero-points")):
                assert torch.equal(x, y), "%s differ after append %d (tensor %d)" % (name, i, which)
    q = P.to_dev(wl.chunk_q(w, heads=range(heads))[:96], "bf16")
    kr, vr = (P.to_dev(x, "bf16") for x in wl.chunk_kv(w, 5, heads=range(heads), n_tokens=64))
    outs = []
    for cache in (ref_cache, new_cache):
        out = torch.empty_like(q)
        mass = torch.empty((heads, q.shape[0]), dtype=torch.float32, device=q.device)
        B.kvq_chunk_attention(cache, 0, len(cache), q, kr, vr, out, mass)
        torch.cuda.synchronize()
        outs.append((out, mass))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    # and the whole thing matches the oracle, block by block, like the existing entry point
    import oracle
    ks = np.concatenate([wl.chunk_kv(w, i, heads=range(heads), n_tokens=n)[0] for i, n in enumerate(blocks)])
    codes, scales, zeros = P.export_np(new_cache, 0)
    t0 = 0
    for n in blocks:
        for h in range(heads):
            oc, osc, oz = oracle.quantize_per_channel(ks[t0:t0 + n, h, :].astype(np.float64), bits)
            assert np.array_equal(codes[h, t0:t0 + n], oc)
            assert np.all(zeros[h, t0:t0 + n] == oz[None, :])
        t0 += n


def test_static_work_space_limits_and_per_token_caches(P):
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["small"]
    # 72 heads x 128 channels = 9216 > 8192: refused with a clear status, nothing enqueued, cache unchanged
    big = B.Cache(B.make_desc(72, 128, 2, 64, B.KVQ_BF16, key_axis=B.KVQ_KEYS_PER_CHANNEL), P.DEV)
    k = torch.zeros((32, 72, 128), dtype=torch.bfloat16, device=P.DEV)
    with pytest.raises(B.KvqError) as err:
        B.kvq_quantize_append_static(big, k, k)
    assert err.value.status == B.KVQ_ERR_CAPACITY and len(big) == 0
    B.kvq_quantize_append(big, k, k)                      # the existing entry point serves it
    assert len(big) == 32
    # a per-token cache has no work space: the new entry point is the old one
    heads = 2
    a, b = P.make_cache(w, 128, heads=heads), P.make_cache(w, 128, heads=heads)
    kk, vv = wl.chunk_kv(w, 0, heads=range(heads), n_tokens=100)
    B.kvq_quantize_append(a, P.to_dev(kk, "bf16"), P.to_dev(vv, "bf16"))
    B.kvq_quantize_append_static(b, P.to_dev(kk, "bf16"), P.to_dev(vv, "bf16"))
    for which in (0, 1):
        for x, y in zip(B.export_all(a, which), B.export_all(b, which)):
            assert torch.equal(x, y)
