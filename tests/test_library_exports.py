"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, validates arguments."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2605_26266_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_26266_amd import build
        build.build()
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "kvq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(kvq_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTED), declared ^ set(B.EXPORTED)
    for name in declared:
        assert hasattr(B.lib(), name), name


def test_status_strings_and_version(B):
    assert B.kvq_status_string(B.KVQ_OK) == "ok"
    assert len({B.kvq_status_string(i) for i in range(5)}) == 5
    assert B.kvq_status_string(99) == "unknown status"
    assert re.fullmatch(r"\d+\.\d+", B.kvq_version())


def test_cache_bytes_accounting(B):
    # 2 tensors x heads x capacity rounded to 32 tokens x (d*bits/8 code bytes + 8 metadata bytes), plus one
    # status block of 256 bytes per cache (the sticky "zero-point outside the matrix-core domain" word)
    for heads, d, bits, cap in [(48, 128, 2, 69632), (24, 128, 4, 28080), (1, 64, 2, 256), (3, 128, 2, 33)]:
        cap32 = -(-cap // 32) * 32
        assert B.kvq_cache_bytes(B.make_desc(heads, d, bits, cap)) == 2 * heads * cap32 * (d * bits // 8 + 8) + 256
    # effective bits per cached element with 64 metadata bits per token: 2 + 64/128 = 2.5 at d = 128
    n = B.kvq_cache_bytes(B.make_desc(8, 128, 2, 4096)) - 256
    assert n * 8 / (2 * 8 * 4096 * 128) == 2.5


def test_description_validation(B):
    ok = B.make_desc(8, 128, 2, 1024)
    assert B.kvq_cache_create_status(ok) == B.KVQ_ERR_INVALID_ARG          # valid description, null storage
    for bad in [B.make_desc(8, 96, 2, 1024), B.make_desc(8, 128, 3, 1024), B.make_desc(8, 128, 8, 1024),
                B.make_desc(8, 128, 2, 1024, group_size=32), B.make_desc(8, 128, 2, 1024, rotate=0)]:
        assert B.kvq_cache_bytes(bad) == 0
        assert B.kvq_cache_create_status(bad) == B.KVQ_ERR_UNSUPPORTED
    for bad in [B.make_desc(0, 128, 2, 1024), B.make_desc(8, 128, 2, 0), B.make_desc(8, 128, 2, 10, io_dtype=7)]:
        assert B.kvq_cache_bytes(bad) == 0
        assert B.kvq_cache_create_status(bad) == B.KVQ_ERR_INVALID_ARG


def test_null_handles_are_rejected_not_dereferenced(B):
    L = B.lib()
    assert L.kvq_cache_len(None) == -1
    assert L.kvq_cache_reset(None) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_cache_truncate(None, 0) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_cache_evict(None, 0) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_cache_set_rotation_signs(None, None) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_quantize_append(None, None, None, 4, 128, 128, None) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_chunk_attention(None, 0, 0, None, None, None, 1, 1, 128, 128, 0.0, 1, None, None, None) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_cache_export(None, 0, 0, 0, None, None, None, None) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_attention_diagnostics(None, 0, 0, None, None, None, None, None, 1, 1, 128, 128, 0.0, 1, None, None) == B.KVQ_ERR_INVALID_ARG
    L.kvq_cache_destroy(None)


def test_host_side_cache_object_without_a_gpu(B):
    """create/len/truncate/destroy only touch host memory: a fake, aligned device address is enough."""
    L = B.lib()
    desc = B.make_desc(2, 128, 2, 100)
    handle = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x10000000)
    assert L.kvq_cache_create(ctypes.byref(desc), fake, B.kvq_cache_bytes(desc), ctypes.byref(handle)) == B.KVQ_OK
    assert L.kvq_cache_len(handle) == 0
    assert L.kvq_cache_truncate(handle, 1) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_cache_evict(handle, 1) == B.KVQ_ERR_INVALID_ARG       # nothing to evict
    assert L.kvq_cache_evict(handle, 0) == B.KVQ_OK
    assert L.kvq_cache_set_rotation_signs(handle, bytes([1, 0] * 64)) == B.KVQ_OK
    assert L.kvq_cache_set_rotation_signs(handle, None) == B.KVQ_OK
    assert L.kvq_cache_create(ctypes.byref(desc), ctypes.c_void_p(0x10000010), 1 << 20, ctypes.byref(ctypes.c_void_p())) \
        == B.KVQ_ERR_INVALID_ARG                                         # storage not 256-byte aligned
    assert L.kvq_cache_create(ctypes.byref(desc), fake, 16, ctypes.byref(ctypes.c_void_p())) == B.KVQ_ERR_INVALID_ARG
    # capacity is checked before anything is launched
    assert L.kvq_quantize_append(handle, fake, fake, 101, 256, 128, None) == B.KVQ_ERR_CAPACITY
    assert L.kvq_quantize_append(handle, fake, fake, 0, 256, 128, None) == B.KVQ_OK
    assert L.kvq_quantize_append(handle, ctypes.c_void_p(0x10000002), fake, 1, 256, 128, None) == B.KVQ_ERR_INVALID_ARG
    assert L.kvq_quantize_append(handle, fake, fake, 1, 250, 128, None) == B.KVQ_ERR_INVALID_ARG  # stride not 16-byte
    L.kvq_cache_destroy(handle)


def test_binding_rejects_tensors_that_do_not_fit_the_cache(B):
    """The kernels index tensors by the cache's head count and head_dim; the binding refuses any other shape before
    anything is launched (checked here on a cache object whose storage is host memory: no call reaches a kernel)."""
    import pytest
    import torch
    desc = B.make_desc(4, 128, 2, 64)
    storage_ok = torch.empty(B.kvq_cache_bytes(desc) + 256, dtype=torch.uint8)
    if storage_ok.data_ptr() % 256 != 0:      # the host allocator gives 64-byte alignment: take an aligned view
        off = 256 - storage_ok.data_ptr() % 256
        storage_ok = storage_ok[off:]
    cache = object.__new__(B.Cache)
    cache.desc, cache.storage, cache.torch_dtype = desc, storage_ok, torch.bfloat16
    handle = ctypes.c_void_p()
    assert B.lib().kvq_cache_create(ctypes.byref(desc), storage_ok.data_ptr(), B.kvq_cache_bytes(desc), ctypes.byref(handle)) == B.KVQ_OK
    cache.handle = handle

    def t(n, h, d):
        return torch.zeros((n, h, d), dtype=torch.bfloat16)

    with pytest.raises(ValueError):
        B.kvq_quantize_append(cache, t(8, 3, 128), t(8, 3, 128))          # fewer heads than the cache
    with pytest.raises(ValueError):
        B.kvq_quantize_append(cache, t(8, 4, 64), t(8, 4, 64))            # head_dim 64 against a 128 cache
    q, out = t(16, 4, 128), t(16, 4, 128)
    with pytest.raises(ValueError):
        B.kvq_chunk_attention(cache, 0, 0, t(16, 2, 128), t(8, 4, 128), t(8, 4, 128), out)
    with pytest.raises(ValueError):
        B.kvq_chunk_attention(cache, 0, 0, q, t(8, 4, 128), t(8, 4, 128), t(15, 4, 128))
    with pytest.raises(ValueError):
        B.kvq_chunk_attention(cache, 0, 0, q, t(8, 2, 128), t(8, 2, 128), out)
    with pytest.raises(ValueError):
        B.kvq_chunk_attention(cache, 0, 0, q, t(8, 4, 128), t(7, 4, 128), out)
    with pytest.raises(ValueError):
        B.kvq_chunk_attention(cache, 0, 0, q, t(8, 4, 128), t(8, 4, 128), out, torch.zeros(4 * 15))
    with pytest.raises(ValueError):
        B.kvq_chunk_attention_ex(cache, 0, 0, t(16, 8, 64), t(16, 4, 128), t(16, 4, 128), t(16, 8, 64), causal=True)
    cache.close()


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N above 1 exits with a message before anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
