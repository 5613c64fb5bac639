"""The host-side free list of K/V block numbers (sqa_block_pool): no block is handed out twice, what is given
back comes out again, bad calls change nothing.  Checked against a plain Python set model under a random
sequence of sequences joining and leaving with different budgets."""
import ctypes as C
import random

import pytest

from paper_2404_04793_amd import binding as sqa


def test_take_and_give_against_a_set_model():
    rng = random.Random(7)
    n_blocks = 257
    pool = sqa.BlockPool(n_blocks)
    free, held = set(range(n_blocks)), {}
    for step in range(2000):
        if held and (rng.random() < 0.45 or len(free) < 12):
            seq = rng.choice(sorted(held))
            ids = held.pop(seq)
            rng.shuffle(ids)
            pool.give(ids)
            free |= set(ids)
        else:
            budget = rng.choice([17, 35, 143, 368, 571])               # tokens -> 16-row blocks
            need = (budget + sqa.SQA_BLOCK_SLOTS - 1) // sqa.SQA_BLOCK_SLOTS
            if need > len(free):
                with pytest.raises(sqa.SqaError) as e:
                    pool.take(need)
                assert e.value.code == 6                                    # all or nothing
            else:
                ids = pool.take(need)
                assert len(set(ids)) == need and set(ids) <= free, (step, ids)
                free -= set(ids)
                held[step] = ids
        assert pool.free_count() == len(free)
    for ids in held.values():
        pool.give(ids)
    assert pool.free_count() == n_blocks
    assert sorted(pool.take(n_blocks)) == list(range(n_blocks))           # every block exists exactly once
    assert pool.free_count() == 0
    pool.close()


def test_fresh_blocks_go_first_and_returned_ones_last_in_first_out():
    pool = sqa.BlockPool(8)
    assert pool.take(3) == [0, 1, 2]
    pool.give([1])
    assert pool.take(2) == [3, 4]                                          # never-used blocks before the returned one
    pool.give([0, 4])
    assert pool.take(3) == [5, 6, 7]
    assert pool.take(3) == [4, 0, 1]
    assert pool.free_count() == 0


def test_bad_calls_change_nothing():
    pool = sqa.BlockPool(6)
    ids = pool.take(4)
    for bad in ([4], [-1], [6], [0, 0], [1, 2, 9]):                         # free block, out of range, named twice
        with pytest.raises(sqa.SqaError) as e:
            pool.give(bad)
        assert e.value.code == 2
        assert pool.free_count() == 2
    pool.give(ids)                                                          # the blocks named in the failed calls are still in use
    assert pool.free_count() == 6
    with pytest.raises(sqa.SqaError) as e:
        pool.take(7)
    assert e.value.code == 6 and pool.free_count() == 6
    assert pool.take(0) == []
    lib = sqa._lib
    assert lib.sqa_block_pool_create(0) is None
    assert lib.sqa_block_pool_free_count(None) == -1
    assert lib.sqa_block_pool_take(None, 1, (C.c_int32 * 1)()) == 1
    assert lib.sqa_block_pool_take(pool._p, 1, None) == 1
    assert lib.sqa_block_pool_take(pool._p, -1, (C.c_int32 * 1)()) == 2
    assert lib.sqa_block_pool_give(pool._p, None, 1) == 1
    lib.sqa_block_pool_destroy(None)
    with pytest.raises(ValueError):
        sqa.BlockPool(0)
