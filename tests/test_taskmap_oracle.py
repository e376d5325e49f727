"""Pins for the pure-Python task-mapping definitions (Section 5.1 of the paper)."""
import json
import os
import random

import pytest

from oracle.taskmap import compose, repeat, spatial


def _build(expr):
    fs = [{"repeat": repeat, "spatial": spatial}[name](*dims) for name, dims in expr]
    f = fs[0]
    for g in fs[1:]:
        f = f * g
    return f


@pytest.fixture(scope="module")
def golden(golden_dir):
    with open(os.path.join(golden_dir, "taskmap_examples.json")) as fh:
        return json.load(fh)


def test_basic_mappings():
    r = repeat(2, 2)
    assert r.num_workers == 1 and r.task_shape == (2, 2)
    assert r(0) == [(0, 0), (0, 1), (1, 0), (1, 1)]
    s = spatial(2, 2)
    assert s.num_workers == 4 and s.task_shape == (2, 2)
    assert [s(w) for w in range(4)] == [[(0, 0)], [(0, 1)], [(1, 0)], [(1, 1)]]
    assert spatial(2, 3, 4)(17) == [(1, 1, 1)]


def test_cooperative_load_example(golden):
    ex = golden["cooperative_load"]
    f = _build(ex["expr"])
    assert f.num_workers == ex["num_workers"] and list(f.task_shape) == ex["task_shape"]
    gh, gw = ex["group_shape"]
    for w in range(f.num_workers):
        tasks = f(w)
        assert len(tasks) == ex["tasks_per_worker"]
        # one task per group of 16x8, groups visited in order
        assert [t[0] // gh for t in tasks] == list(range(ex["num_groups"]))
        assert tasks == [(gh * r + w // gw, w % gw) for r in range(ex["num_groups"])]
    # each group is executed by all 128 threads, one element each
    for r in range(ex["num_groups"]):
        assert sorted(f(w)[r] for w in range(128)) == [(gh * r + i, k) for i in range(gh) for k in range(gw)]


def test_cuda_core_matmul_example(golden):
    ex = golden["cuda_core_matmul"]
    f = _build(ex["expr"])
    assert f.num_workers == ex["num_workers"] and list(f.task_shape) == ex["task_shape"]
    seen = set()
    for w in range(f.num_workers):
        tasks = f(w)
        assert len(tasks) == ex["tasks_per_worker"]
        seen.update(tasks)
    assert len(seen) == 128 * 128
    # worker 0 = warp (0,0), lane (0,0): its first repeat covers a 4x4 patch at the origin
    assert f(0)[:16] == [(i, j) for i in range(4) for j in range(4)]
    # thread 1 of warp 0 sits one 4-wide patch to the right (threads in a warp are laid out 4x8)
    assert f(1)[0] == (0, 4)
    # warp 1 (workers 32..63) sits one warp tile to the right: 2 repeats * 8 threads * 4 elements = 64 columns
    assert f(32)[0] == (0, 64)


def test_block_mma_example(golden):
    ex = golden["block_mma"]
    # 4 warps as 2x2, each repeating 2x2 MMA tiles: the only composition of the two basic mappings that gives
    # every warp a contiguous 2x2 patch of the 4x4 MMA grid
    f = spatial(2, 2) * repeat(2, 2)
    assert f.num_workers == ex["num_workers"] and list(f.task_shape) == ex["task_shape"]
    allt = []
    for w in range(4):
        assert len(f(w)) == ex["tasks_per_worker"]
        allt += f(w)
    assert sorted(allt) == [(i, j) for i in range(4) for j in range(4)]


def _random_mapping(rnd, dim):
    d = [rnd.choice([1, 2, 3]) for _ in range(dim)]
    return rnd.choice([repeat, spatial])(*d)


def _table(f):
    return [f(w) for w in range(f.num_workers)]


def test_composition_is_associative_including_order():
    rnd = random.Random(0)
    for _ in range(200):
        dim = rnd.choice([1, 2, 3])
        f1, f2, f3 = (_random_mapping(rnd, dim) for _ in range(3))
        left, right = (f1 * f2) * f3, f1 * (f2 * f3)
        assert left.num_workers == right.num_workers and left.task_shape == right.task_shape
        assert _table(left) == _table(right)


def test_composition_is_not_commutative():
    a, b = repeat(1, 2), spatial(2, 1)
    c, d = spatial(2, 2), repeat(2, 2)
    assert _table(c * d) != _table(d * c)
    ab, ba = a * b, b * a
    assert ab.task_shape == ba.task_shape
    # same shapes here, but spatial-of-repeat and repeat-of-spatial interleave differently in general:
    f, g = repeat(2, 1) * spatial(2, 1), spatial(2, 1) * repeat(2, 1)
    assert _table(f) == [[(0, 0), (2, 0)], [(1, 0), (3, 0)]]
    assert _table(g) == [[(0, 0), (1, 0)], [(2, 0), (3, 0)]]


def test_column_major_assignment_by_composition():
    # spatial(1,n) composed over spatial(m,1) walks workers down the columns first
    f = spatial(1, 3) * spatial(2, 1)
    assert [f(w)[0] for w in range(6)] == [(0, 0), (1, 0), (0, 1), (1, 1), (0, 2), (1, 2)]


def test_compositions_partition_the_task_domain():
    rnd = random.Random(1)
    for _ in range(100):
        dim = rnd.choice([1, 2, 3])
        f = _random_mapping(rnd, dim)
        for _ in range(rnd.choice([0, 1, 2, 3])):
            f = f * _random_mapping(rnd, dim)
        tasks = [t for w in range(f.num_workers) for t in f(w)]
        total = 1
        for d in f.task_shape:
            total *= d
        assert len(tasks) == total == len(set(tasks))
        assert all(0 <= t[i] < f.task_shape[i] for t in tasks for i in range(dim))


def test_compose_rejects_mismatched_dimensions():
    with pytest.raises(ValueError):
        compose(repeat(2), spatial(2, 2))
