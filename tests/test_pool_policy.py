"""On-demand swapping, host side (no GPU): the residency policy oracle against what the textbook fixes, and the
library's dry-run pool (bookkeeping only) against the oracle, request by request."""
import ctypes
import random

import pytest

from oracle.pool_oracle import LruPool

try:
    import paper_2406_09041_amd as mes
    from paper_2406_09041_amd import binding as B
    HAVE_LIB = True
except ImportError:                                   # the library is built by __graft_entry__.build()
    HAVE_LIB = False

needs_lib = pytest.mark.skipif(not HAVE_LIB, reason="libmes.so not built")


# ---------------------------------------------------------------- the oracle against textbook facts

def test_lru_compulsory_misses_only_when_everything_fits():
    p = LruPool(6)
    rng = random.Random(1)
    for _ in range(200):
        p.acquire(rng.sample(range(6), rng.randint(1, 6)))
    assert p.misses == 6                               # one compulsory miss per expert, never an eviction


def test_lru_cyclic_scan_over_one_more_than_fits_always_misses():
    """The classic worst case: n + 1 items touched round-robin through n slots never hit."""
    p = LruPool(4)
    for i in range(50):
        p.acquire([i % 5])
    assert p.hits == 0 and p.misses == 50


def test_lru_evicts_the_least_recently_used_and_keeps_the_request_together():
    p = LruPool(3)
    p.acquire([0]); p.acquire([1]); p.acquire([2])
    p.acquire([0])                                      # 1 is now the oldest
    slots, loaded = p.acquire([3])
    assert loaded == [3] and p.slot_of(1) == -1 and p.slot_of(0) >= 0 and p.slot_of(2) >= 0
    slots, loaded = p.acquire([1, 2, 4])                # 2 is resident: 0 and 3 have to go, 2 may not
    assert sorted(loaded) == [1, 4] and p.slot_of(2) >= 0 and p.slot_of(0) == -1 and p.slot_of(3) == -1
    assert len(set(slots)) == 3


def test_lru_inclusion_property():
    """LRU is a stack algorithm: with single-expert requests a larger pool never misses more."""
    rng = random.Random(7)
    seq = [rng.randrange(12) for _ in range(400)]
    misses = []
    for n in (2, 4, 6, 8, 12):
        p = LruPool(n)
        for e in seq:
            p.acquire([e])
        misses.append(p.misses)
    assert misses == sorted(misses, reverse=True) and misses[-1] == len(set(seq))


def test_prefetch_spares_the_slots_of_the_latest_acquire():
    p = LruPool(4)
    p.acquire([0, 1])                                   # slots 0, 1; two slots free
    assert p.prefetch([2, 3, 4]) == [2, 3]              # the free slots go; nothing else may: 4 is skipped
    assert p.slot_of(0) >= 0 and p.slot_of(1) >= 0 and p.slot_of(4) == -1
    slots, loaded = p.acquire([2, 3])                   # both prefetched: hits
    assert loaded == [] and p.hits == 2 and p.misses == 2
    assert p.prefetch([4]) == [4] and p.slot_of(0) == -1     # 0 and 1 are older than the latest acquire now: 0 is the oldest
    assert p.prefetch([5]) == [5] and p.slot_of(1) == -1
    assert p.prefetch([6]) == []                             # 2, 3 belong to the latest acquire, 4, 5 were just prefetched
    assert p.prefetched == 4


def test_prefetch_of_the_next_request_turns_its_misses_into_hits():
    """With twice as many slots as a request needs, prefetching request i + 1 right after acquiring request i
    leaves the acquires nothing to load but the very first request."""
    rng = random.Random(3)
    p = LruPool(8)
    reqs = [rng.sample(range(30), 4) for _ in range(100)]
    for i, r in enumerate(reqs):
        p.acquire(r)
        if i + 1 < len(reqs):
            p.prefetch(reqs[i + 1])
    assert p.misses == 4


# ---------------------------------------------------------------- the library's bookkeeping against the oracle

@needs_lib
@pytest.mark.parametrize("n_slots,n_experts,seed", [(4, 9, 0), (16, 40, 1), (3, 3, 2), (1, 5, 3)])
def test_dry_run_pool_follows_the_oracle(n_slots, n_experts, seed):
    d_in, d_out, k, bits = 264, 72, 5, 3
    pool = mes.ExpertPool(d_in, d_out, k, bits, 0, n_slots, n_experts, dry_run=True)
    for e in range(n_experts):
        pool.register_raw(e, 4096 + e * 16, 4096, 4096, 4096)      # fake pinned addresses: never dereferenced
    ref = LruPool(n_slots)
    rng = random.Random(seed)
    slot_bytes = B.lib.mes_pool_slot_bytes(d_in, d_out, k, bits)
    codes_b, sal_b = B.codes_bytes(d_in, d_out, bits), B.salient_bytes(d_out, k)
    up = lambda v: (v + 255) // 256 * 256
    assert slot_bytes == up(up(up(up(codes_b) + 4 * d_out) + sal_b) + 4 * k)
    copied = 0
    for _ in range(300):
        req = rng.sample(range(n_experts), rng.randint(1, n_slots))
        slots, loaded = ref.acquire(req)
        desc = pool.acquire(req)
        copied += len(loaded) * (codes_b + 4 * d_out + sal_b + 4 * k)
        for i, e in enumerate(req):
            assert pool.slot_of(e) == slots[i]
            base = 256 + slots[i] * slot_bytes                      # the dry-run arena starts at address 256
            assert desc[i].codes == base and desc[i].step == base + up(codes_b)
            assert desc[i].salient == base + up(up(codes_b) + 4 * d_out)
            assert (desc[i].d_in, desc[i].d_out, desc[i].k, desc[i].bits, desc[i].grid) == (d_in, d_out, k, bits, 0)
        for e in range(n_experts):
            assert pool.slot_of(e) == ref.slot_of(e)
    assert pool.stats() == (ref.hits, ref.misses, copied)


@needs_lib
@pytest.mark.parametrize("n_slots,n_experts,seed", [(6, 20, 0), (16, 40, 1), (2, 7, 2)])
def test_dry_run_pool_with_prefetches_follows_the_oracle(n_slots, n_experts, seed):
    """A pool over three linear layers, acquires and prefetches interleaved at random: residency, slots, counters and
    the descriptors' addresses against the oracle and the documented slot layout."""
    d_in, d_out, k, bits = [264, 264, 520], [72, 136, 264], [5, 0, 16], 2
    pool = mes.ExpertPool(d_in, d_out, k, bits, 0, n_slots, n_experts, dry_run=True)
    for e in range(n_experts):
        B._check(B.lib.mes_pool_register_blob(pool.handle, e, 4096 + e * 16))   # fake pinned address: never dereferenced
    up = lambda v: (v + 255) // 256 * 256
    lin_bytes = [B.lib.mes_pool_slot_bytes(d_in[l], d_out[l], k[l], bits) for l in range(3)]
    assert pool.slot_bytes == sum(lin_bytes)
    assert [B.lib.mes_pool_linear_offset(pool.handle, l) for l in range(3)] == [0, lin_bytes[0], lin_bytes[0] + lin_bytes[1]]
    payload = sum(B.codes_bytes(d_in[l], d_out[l], bits) + 4 * d_out[l] + (B.salient_bytes(d_out[l], k[l]) + 4 * k[l] if k[l] else 0)
                  for l in range(3))
    ref = LruPool(n_slots)
    rng = random.Random(seed)
    copied = 0
    for _ in range(400):
        req = rng.sample(range(n_experts), rng.randint(1, n_slots))
        if rng.random() < 0.4:
            loaded = ref.prefetch(req)
            assert pool.prefetch(req) == len(loaded)
        else:
            slots, loaded = ref.acquire(req)
            desc = pool.acquire(req)
            for l in range(3):
                for i, e in enumerate(req):
                    base = 256 + slots[i] * pool.slot_bytes + sum(lin_bytes[:l])
                    d = desc[l][i]
                    assert d.codes == base and d.step == base + up(B.codes_bytes(d_in[l], d_out[l], bits))
                    assert (d.d_in, d.d_out, d.k, d.bits) == (d_in[l], d_out[l], k[l], bits)
                    assert (d.salient is None) == (k[l] == 0)
        copied += len(loaded) * payload
        for e in range(n_experts):
            assert pool.slot_of(e) == ref.slot_of(e)
    assert pool.stats() == (ref.hits, ref.misses, copied) and pool.prefetched() == ref.prefetched


@needs_lib
def test_pool_argument_errors():
    lib = B.lib
    h = ctypes.c_void_p()
    mk = lambda **kw: lib.mes_pool_create(*[kw.get(n, v) for n, v in
                                            (("d_in", 256), ("d_out", 256), ("k", 8), ("bits", 2), ("grid", 0), ("n_slots", 4),
                                             ("n_experts", 8), ("arena", 256), ("bytes", 1 << 30), ("dry", 1))], ctypes.byref(h))
    assert mk() == 0
    pool = ctypes.c_void_p(h.value)
    assert mk(bits=5) == 3 and mk(bits=1, grid=1) == 3
    assert mk(k=300) == 4
    assert mk(n_slots=0) == 2 and mk(n_slots=65) == 2 and mk(d_in=7) == 2
    assert mk(arena=None) == 1 and mk(arena=8) == 6
    assert mk(bytes=1000) == 7 and b"needed" in lib.mes_last_error()
    assert lib.mes_pool_register(pool, 9, 256, 256, 256, 256) == 2
    assert lib.mes_pool_register(pool, 0, None, 256, 256, 256) == 1
    assert lib.mes_pool_register(pool, 0, 256, 256, 256, 256) == 0
    ids = (ctypes.c_int32 * 5)(0, 0, 1, 2, 3)
    out = (B.mes_delta * 5)()
    assert lib.mes_pool_acquire(pool, ids, 5, out, None, None) == 2          # more than the pool has slots
    assert lib.mes_pool_acquire(pool, ids, 2, out, None, None) == 2          # the same expert twice
    ids = (ctypes.c_int32 * 2)(0, 1)
    assert lib.mes_pool_acquire(pool, ids, 2, out, None, None) == 1          # expert 1 was never registered
    assert lib.mes_pool_acquire(pool, ids, 1, out, None, None) == 0
    assert lib.mes_pool_slot_of(pool, 0) == 0 and lib.mes_pool_slot_of(pool, 1) == -1
    assert lib.mes_pool_prefetch(pool, ids, 2, None, None) == 1              # expert 1 was never registered
    assert lib.mes_pool_prefetch(pool, ids, 1, None, None) == 0
    assert lib.mes_pool_register_blob(pool, 1, None) == 1 and lib.mes_pool_register_blob(pool, 1, 264) == 6
    assert lib.mes_pool_register_blob(pool, 1, 512) == 0
    lib.mes_pool_destroy(pool)
    assert lib.mes_pool_slot_bytes(256, 256, 8, 5) == 0
    three = (ctypes.c_int32 * 3)(256, 256, 256)
    ks = (ctypes.c_int32 * 3)(8, 0, 300)
    assert lib.mes_pool_create_multi(3, three, three, ks, 2, 0, 4, 8, 256, 1 << 30, 1, ctypes.byref(h)) == 4
    assert lib.mes_pool_create_multi(9, three, three, ks, 2, 0, 4, 8, 256, 1 << 30, 1, ctypes.byref(h)) == 2
    ks[2] = 16
    assert lib.mes_pool_create_multi(3, three, three, ks, 2, 0, 4, 8, 256, 1 << 30, 1, ctypes.byref(h)) == 0
    multi = ctypes.c_void_p(h.value)
    assert lib.mes_pool_register(multi, 0, 256, 256, 256, 256) == 2          # four-buffer registration is for single-linear pools
    assert lib.mes_pool_acquire(multi, ids, 1, out, None, None) == 2
    lib.mes_pool_destroy(multi)
