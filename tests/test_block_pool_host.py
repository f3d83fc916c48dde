"""Host-side block pool (Sec. 3.1 "Block Pool with Per-Agent Isolation"): ownership bookkeeping checked against a
plain Python model and against the invariants isolation means -- no block in two lists, free + owned = all.
No GPU needed."""
import random
import threading

import pytest

from paper_2603_04428_amd import binding as b


def check_invariants(pool, num_blocks, agents):
    owned = {}
    for a in agents:
        for blk in pool.blocks(a):
            assert blk not in owned, f"block {blk} in two lists"
            owned[blk] = a
    assert len(owned) + pool.free_blocks() == num_blocks
    for blk in range(num_blocks):
        assert pool.owner(blk) == owned.get(blk, -1)


def test_reserve_grows_in_place_lowest_ids_first():
    p = b.BlockPool(10)
    assert p.free_blocks() == 10 and p.lru_victim() == -1
    assert p.reserve(7, 1) == 1 and p.blocks(7) == [0]
    assert p.reserve(3, 600) == 3 and p.blocks(3) == [1, 2, 3]          # ceil(600 / 256)
    assert p.reserve(7, 256) == 1 and p.blocks(7) == [0]                 # still one block
    assert p.reserve(7, 257) == 2 and p.blocks(7) == [0, 4]              # grows at the end, old block stays first
    assert p.reserve(7, 10) == 2                                         # never shrinks
    assert p.reserve(9, 0) == 0 and p.blocks(9) == []                    # known, empty
    assert p.table_row(7, 4, fill=-1) == [0, 4, -1, -1]
    assert p.table_row(3, 3, fill=9) == [1, 2, 3]
    with pytest.raises(b.Q4KVError) as e:
        p.table_row(3, 2)
    assert e.value.code == -3
    assert p.release(3) == 3 and p.free_blocks() == 8
    assert p.reserve(5, 512) == 2 and p.blocks(5) == [1, 2]              # freed ids are reused, lowest first
    check_invariants(p, 10, [7, 5, 9])


def test_no_space_changes_nothing():
    p = b.BlockPool(4)
    p.reserve(1, 700)
    before = (p.blocks(1), p.free_blocks())
    with pytest.raises(b.Q4KVError) as e:
        p.reserve(2, 600)                                                # needs 3, one is free
    assert e.value.code == b.BlockPool.ENOSPACE
    with pytest.raises(b.Q4KVError):
        p.blocks(2)                                                      # the failed call did not create the agent
    with pytest.raises(b.Q4KVError) as e:
        p.reserve(1, 2000)                                               # growth that does not fit: nothing taken
    assert e.value.code == b.BlockPool.ENOSPACE
    assert (p.blocks(1), p.free_blocks()) == before
    with pytest.raises(b.Q4KVError):
        p.reserve(1, 256 * 5)                                            # more than the pool has at all
    assert p.reserve(2, 256) == 1


def test_least_recently_used_victim_and_pins():
    p = b.BlockPool(8)
    for a in (10, 11, 12):
        p.reserve(a, 300)
    assert p.lru_victim() == 10
    p.touch(10)
    assert p.lru_victim() == 11
    p.reserve(11, 600)                                                   # growing counts as use
    assert p.lru_victim() == 12
    p.pin(12)
    assert p.lru_victim() == 10
    p.pin(10)
    p.pin(11)
    assert p.lru_victim() == -1                                          # everything is in the running batch
    p.pin(12, False)
    assert p.lru_victim() == 12
    p.reserve(13, 0)                                                     # an agent without blocks frees nothing: never a victim
    p.release(12)
    p.pin(10, False)
    assert p.lru_victim() == 10
    # the eviction sequence: victim's blocks go back, the newcomer gets them
    p.pin(11, False)
    assert p.free_blocks() == 3
    with pytest.raises(b.Q4KVError):
        p.reserve(14, 256 * 4)
    victim = p.lru_victim()
    freed = p.blocks(victim)
    p.release(victim)
    assert p.reserve(14, 256 * 4) == 4 and set(freed) <= set(p.blocks(14))


def test_random_operations_against_a_model():
    rng = random.Random(5)
    N = 64
    p = b.BlockPool(N)
    model, free, stamp, clock = {}, set(range(N)), {}, 0
    for step in range(4000):
        op = rng.random()
        a = rng.randrange(12)
        if op < 0.55:
            tokens = rng.randrange(0, 256 * 12)
            need = (tokens + 255) // 256
            have = len(model.get(a, []))
            if need - have > len(free):
                with pytest.raises(b.Q4KVError):
                    p.reserve(a, tokens)
            else:
                clock += 1
                lst = model.setdefault(a, [])
                for _ in range(max(0, need - have)):
                    blk = min(free)
                    free.remove(blk)
                    lst.append(blk)
                stamp[a] = clock
                assert p.reserve(a, tokens) == len(lst)
        elif op < 0.75:
            if a in model:
                assert p.release(a) == len(model[a])
                free |= set(model.pop(a))
                stamp.pop(a)
            else:
                with pytest.raises(b.Q4KVError):
                    p.release(a)
        elif op < 0.9:
            if a in model:
                clock += 1
                stamp[a] = clock
                p.touch(a)
        else:
            cands = [x for x in model if model[x]]
            want = min(cands, key=lambda x: stamp[x]) if cands else -1
            assert p.lru_victim() == want
        if step % 200 == 0:
            for x in model:
                assert p.blocks(x) == model[x]
            check_invariants(p, N, list(model))
    check_invariants(p, N, list(model))


def test_concurrent_callers_keep_the_invariants():
    N = 256
    p = b.BlockPool(N)
    errors = []

    def worker(base):
        rng = random.Random(base)
        try:
            for _ in range(1500):
                a = base * 100 + rng.randrange(4)
                try:
                    if rng.random() < 0.6:
                        p.reserve(a, rng.randrange(0, 256 * 20))
                    else:
                        p.release(a)
                except b.Q4KVError as e:
                    if e.code not in (-1, -6):
                        raise
        except Exception as e:          # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i + 1,)) for i in range(6)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors
    agents = [(i + 1) * 100 + j for i in range(6) for j in range(4)]
    known = []
    for a in agents:
        try:
            p.blocks(a)
            known.append(a)
        except b.Q4KVError:
            pass
    check_invariants(p, N, known)


def test_argument_errors():
    l = b.lib()
    assert not l.q4kv_block_pool_create(0) and not l.q4kv_block_pool_create(-3)
    assert l.q4kv_block_pool_reserve(None, 1, 1) == -1
    assert l.q4kv_block_pool_lru_victim(None) == -1 and l.q4kv_block_pool_owner(None, 0) == -1
    p = b.BlockPool(2)
    with pytest.raises(b.Q4KVError):
        p.reserve(-1, 10)
    with pytest.raises(b.Q4KVError):
        p.reserve(1, -10)
    with pytest.raises(b.Q4KVError):
        p.touch(99)
    with pytest.raises(b.Q4KVError):
        p.pin(99)
    assert p.owner(-1) == -1 and p.owner(2) == -1
    p.close()
    p.close()                                                            # idempotent
