"""Page bookkeeping of the paged memory manager (paper Sec. 4.1).  The oracle's free list is pinned by
invariants that hold for any correct allocator plus the documented order; the library's host-side
functions are then compared with it call by call on seeded random sequences (no GPU involved)."""
import random

import pytest

import oracle as orc
from paper_2602_02108_amd import api


def test_oracle_pool_invariants_and_order():
    pool = orc.PagePool(10)
    assert pool.alloc(3) == [0, 1, 2] and pool.alloc(2) == [3, 4]          # ascending after a reset
    pool.release([1, 3])
    assert pool.alloc(3) == [3, 1, 5]                                      # last released first, then fresh pages
    assert pool.n_free == 4
    with pytest.raises(MemoryError):
        pool.alloc(5)
    assert pool.n_free == 4                                                # a failed call changes nothing
    for bad in ([10], [-1], [6], [0, 0]):                                  # out of range, free already, listed twice
        with pytest.raises(ValueError):
            pool.release(bad)
    assert pool.n_free == 4
    assert pool.alloc(0) == []


def test_oracle_pool_conserves_pages_on_random_sequences():
    rng = random.Random(5)
    n = 37
    pool = orc.PagePool(n)
    held = []
    for _ in range(2000):
        if rng.random() < 0.55 and pool.n_free:
            got = pool.alloc(rng.randint(0, min(6, pool.n_free)))
            assert not set(got) & set(held)                                # never handed out twice
            held += got
        elif held:
            rng.shuffle(held)
            k = rng.randint(0, min(5, len(held)))
            pool.release(held[:k])
            held = held[k:]
        assert sorted(held + pool.free) == list(range(n))                  # every page is either held or free


def test_library_pool_matches_the_oracle_call_by_call():
    rng = random.Random(11)
    n = 53
    ref, pool = orc.PagePool(n), api.PagePool(n)
    held = []
    for step in range(3000):
        r = rng.random()
        if r < 0.5:
            k = rng.randint(0, 9)
            if k > ref.n_free:
                with pytest.raises(MemoryError):
                    ref.alloc(k)
                with pytest.raises(api.OombError) as e:
                    pool.alloc(k)
                assert e.value.status == api.ERR_OUT_OF_PAGES
            else:
                want = ref.alloc(k)
                assert pool.alloc(k) == want, step
                held += want
        elif r < 0.9:
            rng.shuffle(held)
            k = rng.randint(0, min(7, len(held)))
            ref.release(held[:k])
            pool.release(held[:k])
            held = held[k:]
        else:  # an invalid release: refused by both, state unchanged
            bad = rng.choice([[n], [-1], [held[0], held[0]] if held else [n + 1], [ref.free[0]] if ref.free else [-2]])
            with pytest.raises(ValueError):
                ref.release(bad)
            with pytest.raises(api.OombError) as e:
                pool.release(bad)
            assert e.value.status == api.ERR_INVALID_ARG
        assert pool.n_free == ref.n_free, step
    # drain both: same pages in the same order
    assert pool.alloc(pool.n_free) == ref.alloc(ref.n_free)


def test_library_pool_argument_errors():
    import ctypes
    l = api.lib()
    nf = ctypes.c_int64(0)
    stack = (ctypes.c_int32 * 4)()
    assert l.oomb_page_pool_reset(4, None, ctypes.byref(nf)) == api.ERR_INVALID_ARG
    assert l.oomb_page_pool_reset(-1, stack, ctypes.byref(nf)) == api.ERR_INVALID_ARG
    assert l.oomb_page_pool_reset(4, stack, ctypes.byref(nf)) == api.OK and nf.value == 4
    out = (ctypes.c_int32 * 4)()
    assert l.oomb_page_pool_alloc(stack, ctypes.byref(nf), -1, out) == api.ERR_INVALID_ARG
    assert l.oomb_page_pool_alloc(stack, ctypes.byref(nf), 2, None) == api.ERR_INVALID_ARG
    assert l.oomb_page_pool_alloc(stack, ctypes.byref(nf), 5, out) == api.ERR_OUT_OF_PAGES and nf.value == 4
    assert l.oomb_page_pool_release(4, stack, ctypes.byref(nf), out, 1) == api.ERR_INVALID_ARG   # nothing is in use
