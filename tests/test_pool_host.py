"""The size-keyed memory pool and the name-keyed cache (section "Caching and Pooling"), host-backed so that the
bookkeeping runs without a GPU: the behaviour the paper states -- a pointer returned to the pool is handed out again
for the same size, and from the second iteration of a repeating request sequence nothing is allocated."""
import ctypes

import pytest

from paper_2409_11600_amd import binding as B


@pytest.fixture
def pool():
    p = B.Pool(B.NSK_POOL_HOST)
    yield p
    p.destroy()


def test_a_returned_pointer_is_reused_for_its_size_only(pool):
    a = pool.get(512 * 4)
    b = pool.get(512 * 4)
    assert a != b and a % 256 == 0 and b % 256 == 0
    pool.put(a)
    c = pool.get(1024 * 4)                 # another size: its list is empty, so a new buffer
    assert c not in (a, b)
    d = pool.get(512 * 4)                  # the figure's case: a 512-float tensor sampled from the pool
    assert d == a
    s = pool.stats()
    assert s == {"bytes_allocated": 2 * 2048 + 4096, "allocations": 3, "requests": 4, "hits": 1}


def test_sizes_are_rounded_up_to_256_bytes(pool):
    a = pool.get(1)
    pool.put(a)
    assert pool.get(256) == a              # same bucket
    assert pool.stats()["bytes_allocated"] == 256


def test_no_allocation_after_the_first_iteration(pool):
    sizes = [4096, 100, 4096, 65536, 300, 100, 4096]
    for it in range(4):
        held = [pool.get(n) for n in sizes]
        assert len(set(held)) == len(held)                      # live buffers are distinct
        for k, p in enumerate(held):                            # and writable over their whole length
            ctypes.memset(p, it + k, sizes[k])
        for p in reversed(held):
            pool.put(p)
        if it == 0:
            first = pool.stats()["allocations"]
            assert first == len(sizes)
        assert pool.stats()["allocations"] == first             # the second iteration onwards allocates nothing
    s = pool.stats()
    assert s["requests"] == 4 * len(sizes) and s["hits"] == 3 * len(sizes)


def test_cache_keeps_one_buffer_per_name(pool):
    p0, created0 = pool.cached("conv1.weight.grad", 64 * 3 * 7 * 7 * 4)
    p1, created1 = pool.cached("conv1.weight.grad", 64 * 3 * 7 * 7 * 4)
    q, created2 = pool.cached("fc.bias.grad", 40)
    assert created0 and not created1 and created2 and p0 == p1 and q != p0
    with pytest.raises(B.NskError):
        pool.cached("fc.bias.grad", 4000)                       # same name, another size
    assert pool.stats()["allocations"] == 2 and pool.stats()["requests"] == 0


def test_errors(pool):
    L = B.lib()
    a = pool.get(100)
    pool.put(a)
    with pytest.raises(B.NskError):
        pool.put(a)                                             # returned twice
    with pytest.raises(B.NskError):
        pool.put(a + 256)                                       # not from this pool
    with pytest.raises(B.NskError):
        pool.get(0)
    h = ctypes.c_void_p()
    assert L.nsk_pool_create(7, ctypes.byref(h)) == B.NSK_ERR_BAD_DESC
    assert L.nsk_pool_create(B.NSK_POOL_HOST, None) == B.NSK_ERR_NULL
    assert L.nsk_pool_get(None, 16, ctypes.byref(h)) == B.NSK_ERR_NULL
    assert L.nsk_pool_destroy(None) == B.NSK_ERR_NULL
