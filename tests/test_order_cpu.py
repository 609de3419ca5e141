"""The connection-ordering routine of the weight set-up (csrc/spdnn_order.h), run
through its host build: it must place every connection exactly once, one per
lane and step, and bring the LDS bank cost close to its lower bound."""
import ctypes

import numpy as np
import pytest

import synth
from paper_2007_14152_amd import build as hip_build


@pytest.fixture(scope="module")
def lib():
    L = ctypes.CDLL(hip_build.ORDER_HOST_LIB)
    L.spdnn_order_group_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
    L.spdnn_order_cost_host.argtypes = [ctypes.c_void_p]
    return L


def order(lib, quads, nsteps=32):
    quads = np.ascontiguousarray(quads, dtype=np.uint8)
    step_of = np.zeros((16, 32), dtype=np.uint8)
    cost = lib.spdnn_order_group_host(quads.ctypes.data, step_of.ctypes.data, nsteps)
    return cost, step_of


def brute_cost(quads, step_of):
    total = 0
    for s in range(32):
        q = [quads[l, np.nonzero(step_of[l] == s)[0][0]] for l in range(16) if (step_of[l] == s).any()]
        q = [x for x in q if x < 16]
        total += np.bincount(q, minlength=16).max() if q else 0
    return int(total)


def test_every_connection_placed_once_and_cost_reported_correctly(lib):
    rng = np.random.default_rng(0)
    for _ in range(50):
        quads = rng.integers(0, 16, size=(16, 32)).astype(np.uint8)
        cost, step_of = order(lib, quads)
        assert np.array_equal(np.sort(step_of, axis=1), np.tile(np.arange(32), (16, 1)))
        assert cost == brute_cost(quads, step_of)
        assert cost >= max(32, np.bincount(quads.ravel(), minlength=16).max())


def test_latin_square_input_reaches_the_ideal(lib):
    # every lane has 2 connections in every quad: a conflict-free schedule exists
    rng = np.random.default_rng(1)
    quads = np.stack([rng.permutation(np.repeat(np.arange(16), 2)) for _ in range(16)])
    cost, _ = order(lib, quads)
    assert cost == 32


def test_all_same_quad_costs_sixteen_per_step(lib):
    cost, step_of = order(lib, np.full((16, 32), 5))
    assert cost == 16 * 32
    assert np.array_equal(np.sort(step_of, axis=1), np.tile(np.arange(32), (16, 1)))


def test_absent_lanes_are_skipped(lib):
    rng = np.random.default_rng(2)
    quads = rng.integers(0, 16, size=(16, 32)).astype(np.uint8)
    quads[5:] = 255
    cost, step_of = order(lib, quads)
    assert np.all(step_of[5:] == 255)
    assert np.array_equal(np.sort(step_of[:5], axis=1), np.tile(np.arange(32), (5, 1)))
    assert cost >= 32


def test_fewer_connections_than_steps(lib):
    """Lanes with 0..16 connections placed in 16 steps: each connection once, no lane
    twice in a step, and lanes with slack avoid collisions where they can."""
    rng = np.random.default_rng(3)
    for trial in range(30):
        quads = np.full((16, 32), 255, dtype=np.uint8)
        counts = rng.integers(0, 17, size=16)
        for l in range(16):
            quads[l, :counts[l]] = rng.integers(0, 16, size=counts[l])
        cost, step_of = order(lib, quads, nsteps=16)
        for l in range(16):
            used = step_of[l, :counts[l]]
            assert np.all(used < 16) and len(set(used.tolist())) == counts[l]
            assert np.all(step_of[l, counts[l]:] == 255)
        assert cost == brute_cost(quads, step_of)
    # 8 connections per lane, all lanes the same 8 quads, 16 steps: slack lets every step be conflict-free
    quads = np.full((16, 32), 255, dtype=np.uint8)
    for l in range(16):
        quads[l, :8] = np.arange(8)
    cost, _ = order(lib, quads, nsteps=16)
    assert cost <= 16


def test_benchmark_patterns_get_close_to_the_bound(lib):
    c = synth.config(4)
    idx = synth.gen_layer(c["N"], 0, c["seed"], c["window"])[:2048]
    quads = ((idx - (idx.min() // 4) * 4) % 16).astype(np.uint8).reshape(-1, 16, 32)
    cost, nat, lb = [], [], []
    for g in quads:
        cst, _ = order(lib, g)
        cost.append(cst)
        nat.append(lib.spdnn_order_cost_host(np.ascontiguousarray(g).ctypes.data))
        lb.append(max(32, np.bincount(g.ravel(), minlength=16).max()))
    assert np.mean(nat) > 90            # random order: about three lanes per quad in the worst quad
    assert np.mean(cost) < 1.12 * np.mean(lb)
    assert np.mean(cost) < 0.5 * np.mean(nat)


# ---- groups of 32 lanes and 32 bank pairs (the two-rows-per-entry kernel) ----

def order32(lib, pairs):
    lib.spdnn_order_group32_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    pairs = np.ascontiguousarray(pairs, dtype=np.uint8)
    step_of = np.full((32, 32), 255, dtype=np.uint8)
    cost = lib.spdnn_order_group32_host(pairs.ctypes.data, step_of.ctypes.data)
    return cost, step_of


def brute_cost32(pairs, step_of):
    total = 0
    for s in range(32):
        q = [pairs[l, np.nonzero(step_of[l] == s)[0][0]] for l in range(32)]
        total += int(np.bincount(q, minlength=32).max())
    return total


def test_group32_places_every_connection_once(lib):
    rng = np.random.default_rng(1)
    for _ in range(30):
        pairs = rng.integers(0, 32, size=(32, 32)).astype(np.uint8)
        cost, step_of = order32(lib, pairs)
        assert cost > 0
        for l in range(32):
            assert sorted(step_of[l].tolist()) == list(range(32))     # one connection per lane and step
        assert cost == brute_cost32(pairs, step_of)
        assert cost >= max(32, int(np.bincount(pairs.ravel(), minlength=32).max()))


def test_group32_latin_square_and_worst_case(lib):
    latin = (np.arange(32)[:, None] + np.arange(32)[None, :]) % 32     # any order is conflict-free... if steps align
    rng = np.random.default_rng(2)
    shuffled = np.stack([rng.permutation(latin[l]) for l in range(32)])
    cost, _ = order32(lib, shuffled)
    assert cost == 32, cost
    cost, _ = order32(lib, np.full((32, 32), 7))
    assert cost == 32 * 32


def test_group32_uniform_patterns_close_to_the_bound(lib):
    """Uniform columns at N = 16384 (the benchmark's 16384-neuron configuration): the cost stays within
    15 % of the lower bound max(32, busiest pair)."""
    c = synth.config(3)
    cols = synth.gen_layer(c["N"], 0, c["seed"])[:32 * 24]
    tot = lb = 0
    for g in range(24):
        pairs = ((cols[32 * g:32 * g + 32] >> 2) & 31).astype(np.uint8)
        cost, _ = order32(lib, pairs)
        tot += cost
        lb += max(32, int(np.bincount(pairs.ravel(), minlength=32).max()))
    assert tot <= 1.15 * lb, (tot, lb)
