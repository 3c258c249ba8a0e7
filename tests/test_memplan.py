"""Static memory plan (tvg_plan_arena): host-only tests.  Several plans are valid for one
problem, so the checks are the properties every valid plan has, the bounds that hold for any
plan, and the exact optimum on the two network bodies, where the lower bound is attained."""
import ctypes
import itertools
import random

import pytest

import paper_1802_04799_amd as tvg
import tvg_inputs as ti


def rounded(b):
    return (b + 255) // 256 * 256


def check_plan(lives, offs, arena):
    n = len(lives)
    assert len(offs) == n
    for (b, f, l), o in zip(lives, offs):
        assert o % 256 == 0 and o + rounded(b) <= arena
    assert arena == max(o + rounded(b) for (b, _, _), o in zip(lives, offs))
    for i, j in itertools.combinations(range(n), 2):
        (bi, fi, li), (bj, fj, lj) = lives[i], lives[j]
        if fi <= lj and fj <= li:                                  # alive together
            assert offs[i] + rounded(bi) <= offs[j] or offs[j] + rounded(bj) <= offs[i], (i, j)
    steps = max(l for _, _, l in lives) + 1
    peak = max(sum(rounded(b) for b, f, l in lives if f <= s <= l) for s in range(steps))
    assert peak <= arena <= sum(rounded(b) for b, _, _ in lives)
    return peak


@pytest.mark.parametrize("seed", range(40))
def test_random_lifetimes_give_valid_plans(seed):
    rng = random.Random(9100 + seed)
    n = rng.randint(1, 60)
    steps = rng.randint(1, 40)
    lives = []
    for _ in range(n):
        f = rng.randrange(steps)
        lives.append((rng.choice([1, 255, 256, 257, 1000, 4096, rng.randint(1, 1 << 20)]), f,
                      rng.randint(f, steps - 1)))
    offs, arena = tvg.tvg_plan_arena(lives)
    check_plan(lives, offs, arena)
    assert (offs, arena) == tvg.tvg_plan_arena(lives)              # deterministic


def test_special_cases():
    # never alive together: everything at offset 0, the arena is the largest tensor
    lives = [(1000 * (i + 1), i, i) for i in range(10)]
    offs, arena = tvg.tvg_plan_arena(lives)
    assert offs == [0] * 10 and arena == rounded(10000)
    # all alive together: nothing shares, the arena is the sum
    lives = [(300, 0, 5)] * 7
    offs, arena = tvg.tvg_plan_arena(lives)
    assert sorted(offs) == [512 * i for i in range(7)] and arena == 7 * 512
    # a chain x0 -> x1 -> x2 -> ...: two buffers suffice (ping-pong)
    lives = [(4096, i, i + 1) for i in range(12)]                  # written at i, read at i + 1
    offs, arena = tvg.tvg_plan_arena(lives)
    check_plan(lives, offs, arena)
    assert arena == 2 * 4096


@pytest.mark.parametrize("network", ["resnet18", "mobilenet"])
def test_network_bodies_reach_the_lower_bound(network):
    steps = ti.resnet18_body(32) if network == "resnet18" else ti.mobilenet_body(32)
    lives = ti.tensor_lives(steps)
    ids = list(lives)
    offs, arena = tvg.tvg_plan_arena([lives[t] for t in ids])
    peak = check_plan([lives[t] for t in ids], offs, arena)
    assert arena == peak                       # no plan can be smaller than the peak of live bytes
    total = sum(b for b, _, _ in lives.values())
    assert arena * 2 < total                   # 64 of 181 MB, 77 of 332 MB
    # an operator's output never overlaps its inputs
    off = dict(zip(ids, offs))
    for st in steps:
        for t in (st.src, st.residual):
            if t is not None:
                a, b = (off[t], off[t] + lives[t][0]), (off[st.dst], off[st.dst] + lives[st.dst][0])
                assert a[1] <= b[0] or b[1] <= a[0], st.name


def test_lifetimes_of_the_resnet_body():
    steps = ti.resnet18_body(2)
    lives = ti.tensor_lives(steps)
    assert len(lives) == 22 and lives[0] == (2 * 3 * 224 * 224 * 2, 0, 0)
    assert lives[1] == (2 * 64 * 112 * 112 * 2, 0, 1)             # stem output, read by the pool
    # the pooled map is read by conv1 of the first block and, as the shortcut, by its conv2
    assert lives[2] == (2 * 64 * 56 * 56 * 2, 1, 3)
    assert lives[steps[-1].dst] == (2 * 512 * 7 * 7 * 2, len(steps) - 1, len(steps) - 1)


def test_rejects_bad_arguments():
    lib = tvg.load()
    one = (tvg.TensorLife * 1)(tvg.TensorLife(16, 0, 0))
    offs = (ctypes.c_uint64 * 1)()
    total = ctypes.c_uint64()
    assert lib.tvg_plan_arena(None, 1, offs, ctypes.byref(total)) == 1
    assert lib.tvg_plan_arena(one, 1, None, ctypes.byref(total)) == 1
    assert lib.tvg_plan_arena(one, 1, offs, None) == 1
    assert lib.tvg_plan_arena(one, 0, offs, ctypes.byref(total)) == 2
    assert lib.tvg_plan_arena(one, 5000, offs, ctypes.byref(total)) == 2
    for bad in [(0, 0, 0), (16, -1, 0), (16, 3, 2)]:
        with pytest.raises(tvg.TvgError) as e:
            tvg.tvg_plan_arena([bad])
        assert e.value.status == 2
