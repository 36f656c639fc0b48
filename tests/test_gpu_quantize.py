"""GPU parity of kvq_quantize_append against the oracle's quantizer: bit-exact codes, scales, zero-points."""
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


@pytest.mark.parametrize("name,bits", [("tiny", 2), ("tiny", 4), ("small", 2), ("small", 4)])
def test_whole_config_in_chunks(P, name, bits):
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS[name].with_bits(bits)
    cache = P.make_cache(w, w.cached_tokens)
    ks, vs = [], []
    for c in range(w.cached_chunks):
        k, v = wl.chunk_kv(w, c)
        B.kvq_quantize_append(cache, P.to_dev(k, w.io_dtype), P.to_dev(v, w.io_dtype))
        ks.append(k)
        vs.append(v)
    assert len(cache) == w.cached_tokens
    P.assert_quantized_equal(cache, np.concatenate(ks), np.concatenate(vs))


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("name", ["tiny", "small"])
def test_ragged_appends_merge_partial_tiles(P, name, bits):
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS[name].with_bits(bits)
    heads = [0, w.num_heads - 1] if w.num_heads > 1 else [0]
    sizes = [1, 30, 1, 32, 33, 7, 64, 5, 100, 31]
    total = sum(sizes)
    k, v = wl.chunk_kv(w, 0, heads=range(w.num_heads))
    reps = -(-total // k.shape[0])
    k, v = np.concatenate([k] * reps)[:total], np.concatenate([v] * reps)[:total]
    cache = P.make_cache(w, total + 3)
    pos = 0
    kd, vd = P.to_dev(k, w.io_dtype), P.to_dev(v, w.io_dtype)
    for n in sizes:
        B.kvq_quantize_append(cache, kd[pos:pos + n], vd[pos:pos + n])
        pos += n
    assert len(cache) == total
    P.assert_quantized_equal(cache, k[:, heads], v[:, heads], heads=heads)
    # truncate into the middle of a tile and append again: earlier tokens must survive
    B.kvq_cache_truncate(cache, 45)
    B.kvq_quantize_append(cache, kd[100:150], vd[100:150])
    kk, vv = np.concatenate([k[:45], k[100:150]]), np.concatenate([v[:45], v[100:150]])
    P.assert_quantized_equal(cache, kk[:, heads], vv[:, heads], heads=heads)


def test_degenerate_and_one_signed_rows(P):
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["small"]
    k, v = wl.chunk_kv(w, 0, n_tokens=40)
    k, v = k.copy(), v.copy()
    k[0] = 0.0                       # all-zero vectors: step 0
    v[1] = 2.5                       # nonzero constant
    k[2] = -0.75
    k[3, :, 0] = 4096.0              # huge DC term: rotated vector is one-signed, zero-point far outside [0, 3]
    v[4] = wl.round_to_bf16(np.abs(v[4]) + np.float32(100.0))
    k[5, :, 1:] = 0.0                # single nonzero channel: rotated vector is +-c everywhere
    v[6] = v[6] * np.float32(2.0 ** -100)   # tiny magnitudes (exact power-of-two scaling)
    k[7] = k[7] * np.float32(2.0 ** 100)    # huge magnitudes
    cache = P.make_cache(w, 64)
    B.kvq_quantize_append(cache, P.to_dev(k, "bf16"), P.to_dev(v, "bf16"))
    P.assert_quantized_equal(cache, k, v)
    _, ks, kz = P.export_np(cache, 0)
    assert ks[0, 0] == 0 and kz[0, 0] == 0
    assert kz[0, 3] < -10


def test_mid_shape_chunks_not_multiple_of_tile(P):
    from paper_2605_26266_amd import binding as B, workloads as wl
    for bits in (2, 4):
        w = wl.WORKLOADS["mid"].with_bits(bits)
        heads = [0, 11, 23]
        cache = P.make_cache(w, 2 * w.chunk_tokens)
        ks, vs = [], []
        for c in range(2):
            k, v = wl.chunk_kv(w, c)
            B.kvq_quantize_append(cache, P.to_dev(k, "bf16"), P.to_dev(v, "bf16"))
            ks.append(k[:, heads])
            vs.append(v[:, heads])
        P.assert_quantized_equal(cache, np.concatenate(ks), np.concatenate(vs), heads=heads)


def test_large_shape_sampled_heads(P):
    """Full Large-config append (4096 tokens x 48 heads) as the benchmark launches it; oracle on 3 heads."""
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["large"]
    heads = [0, 17, 47]
    cache = P.make_cache(w, 2 * w.chunk_tokens)
    k, v = wl.chunk_kv(w, 0)
    for _ in range(2):
        B.kvq_quantize_append(cache, P.to_dev(k, "bf16"), P.to_dev(v, "bf16"))
    P.assert_quantized_equal(cache, k[:, heads], v[:, heads], heads=heads, start=w.chunk_tokens)


def test_capacity_and_argument_errors(P):
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["small"]
    cache = P.make_cache(w, 48)
    k, v = wl.chunk_kv(w, 0, n_tokens=40)
    kd, vd = P.to_dev(k, "bf16"), P.to_dev(v, "bf16")
    B.kvq_quantize_append(cache, kd, vd)
    with pytest.raises(B.KvqError) as e:
        B.kvq_quantize_append(cache, kd, vd)
    assert e.value.status == B.KVQ_ERR_CAPACITY and len(cache) == 40
    B.kvq_quantize_append(cache, kd[:0], vd[:0])          # empty append is a no-op
    assert len(cache) == 40
    with pytest.raises(B.KvqError) as e:                 # misaligned base pointer
        B.kvq_quantize_append(cache, kd.view(-1)[1:1 + 8 * 128].view(1, 8, 128), vd[:1])
    assert e.value.status == B.KVQ_ERR_INVALID_ARG
    with pytest.raises(B.KvqError):
        B.kvq_cache_truncate(cache, 41)
    B.kvq_cache_reset(cache)
    assert len(cache) == 0


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("group", [32, 64, 128])
def test_fp8_metadata_groups_bit_exact(P, bits, group):
    """Group-wise quantization with FP8-E4M3 scales and BF16 zero-points: codes, stored scales and stored
    zero-points equal the oracle's, for appends that start and end inside a tile."""
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["small"].with_bits(bits)
    heads = 3
    cache = P.make_cache(w, 300, heads=heads, group=group, fp8_meta=True)
    assert B.kvq_cache_bytes(cache.desc) == 2 * heads * 320 * (128 * bits // 8 + 3 * (128 // group)) + 256
    k, v = wl.chunk_kv(w, 0, heads=range(heads), n_tokens=300)
    # widen the dynamic range so that scales land in many binades, including E4M3 subnormals
    k = wl.round_to_bf16(k * np.exp2(np.arange(300) % 19 - 12).astype(np.float32)[:, None, None])
    pos = 0
    for n in (45, 1, 130, 124):
        B.kvq_quantize_append(cache, P.to_dev(k[pos:pos + n], "bf16"), P.to_dev(v[pos:pos + n], "bf16"))
        pos += n
    P.assert_quantized_equal(cache, k, v)


def test_fp8_metadata_head_dim_64(P):
    from paper_2605_26266_amd import binding as B, workloads as wl
    w = wl.WORKLOADS["tiny"]
    cache = P.make_cache(w, 256, group=32, fp8_meta=True)
    k, v = wl.chunk_kv(w, 0, n_tokens=256)
    B.kvq_quantize_append(cache, P.to_dev(k, w.io_dtype), P.to_dev(v, w.io_dtype))
    P.assert_quantized_equal(cache, k, v)


def test_fp8_metadata_descriptor_errors(P):
    from paper_2605_26266_amd import binding as B
    bad = [B.make_desc(2, 128, 2, 64, group_size=32),                                    # groups need the FP8 format
           B.make_desc(2, 128, 2, 64, group_size=16, meta_format=B.KVQ_META_FP8_BF16),
           B.make_desc(2, 64, 2, 64, group_size=128, meta_format=B.KVQ_META_FP8_BF16),
           B.make_desc(2, 128, 2, 64, meta_format=7)]
    for d in bad:
        assert B.kvq_cache_bytes(d) == 0
