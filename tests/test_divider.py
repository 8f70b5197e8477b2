"""Hybrid-migration divider (arXiv 2501.06709, Sec. "Adaptive Request Migration",
"Hybrid Migration" / "Global Consensus"): the oracle is pinned by a hand-worked
fixture, by invariants checked against brute force over all 3^n divisions of tiny
instances, and by reductions to a running-sum prefix rule; the library's
kvm_divide_moves must then equal the oracle on random instances (host code only,
no GPU).
"""
import itertools
import os

import numpy as np
import pytest

import paper_2501_06709_amd as kvm
from paper_2501_06709_amd import build as kvm_build

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "divider_small.txt")
KV, TOK, DEFER = 0, 1, 2


@pytest.fixture(scope="module", autouse=True)
def built():
    if kvm_build.stale():
        kvm_build.build()


def load_golden():
    comm = comp = None
    rows = []
    for ln in open(GOLDEN):
        if ln.startswith("#") or not ln.strip():
            continue
        parts = ln.split()
        if parts[0] == "comm":
            comm = [int(x) for x in parts[1:]]
        elif parts[0] == "comp":
            comp = [int(x) for x in parts[1:]]
        else:
            rows.append([int(x) for x in parts])
    moves = [tuple(r[:4]) for r in rows]
    return moves, comm, comp, [r[4] for r in rows], [r[5] for r in rows]


def feasible(moves, comm, comp, classes):
    link = [0] * len(comm)
    inst = [0] * len(comp)
    for (l, d, b, t), c in zip(moves, classes):
        if c == KV:
            link[l] += b
        elif c == TOK:
            inst[d] += t
    return all(x <= c for x, c in zip(link, comm)) and all(x <= c for x, c in zip(inst, comp))


def test_golden_worked_example(oracle):
    moves, comm, comp, ff, bf = load_golden()
    assert oracle.divide_moves(moves, comm, comp, "first_fit") == ff
    assert oracle.divide_moves(moves, comm, comp, "best_fit") == bf
    assert list(kvm.kvm_divide_moves(moves, comm, comp, kvm.KVM_FIRST_FIT)) == ff
    assert list(kvm.kvm_divide_moves(moves, comm, comp, kvm.KVM_BEST_FIT)) == bf
    # equal free fractions (50/100 and 5/10): the KV class wins the tie
    assert oracle.divide_moves([(0, 0, 50, 5)], [100], [10], "best_fit") == [KV]
    assert oracle.divide_moves([(0, 0, 50, 4)], [100], [10], "best_fit") == [KV]
    assert oracle.divide_moves([(0, 0, 49, 5)], [100], [10], "best_fit") == [TOK]


def test_invariants_against_brute_force(oracle):
    rng = np.random.default_rng(0)
    for trial in range(150):
        n = int(rng.integers(1, 8))
        n_links, n_inst = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        comm = [int(x) for x in rng.integers(0, 60, n_links)]
        comp = [int(x) for x in rng.integers(0, 30, n_inst)]
        moves = [(int(rng.integers(n_links)), int(rng.integers(n_inst)), int(rng.integers(0, 40)),
                  int(rng.integers(0, 20))) for _ in range(n)]
        best = max(sum(c != DEFER for c in cls)
                   for cls in itertools.product((KV, TOK, DEFER), repeat=n)
                   if feasible(moves, comm, comp, cls))
        for policy in ("first_fit", "best_fit"):
            cls = oracle.divide_moves(moves, comm, comp, policy)
            assert feasible(moves, comm, comp, cls)            # boundaries are never exceeded
            assert sum(c != DEFER for c in cls) <= best        # cannot beat the optimum
            # maximal: no deferred move could still be added to either bin at the end
            link = list(comm)
            inst = list(comp)
            for (l, d, b, t), c in zip(moves, cls):
                if c == KV:
                    link[l] -= b
                elif c == TOK:
                    inst[d] -= t
            for (l, d, b, t), c in zip(moves, cls):
                if c == DEFER:
                    assert b > link[l] and t > inst[d]
            # the first move that fits anywhere is never deferred
            if moves[0][2] <= comm[moves[0][0]] or moves[0][3] <= comp[moves[0][1]]:
                assert cls[0] != DEFER
        if best == n:
            # if everything fits as KV alone, first-fit sends everything as KV
            if feasible(moves, comm, comp, [KV] * n):
                assert oracle.divide_moves(moves, comm, comp, "first_fit") == [KV] * n


def test_reduces_to_running_sum_when_one_bin_is_closed(oracle):
    """With computation boundaries 0 (and tokens > 0) only the KV bin exists: a move
    is accepted iff it fits what the accepted ones before it left over."""
    rng = np.random.default_rng(1)
    sizes = [int(x) for x in rng.integers(1, 50, 40)]
    moves = [(0, 0, s, 1) for s in sizes]
    for policy in ("first_fit", "best_fit"):
        cls = oracle.divide_moves(moves, [300], [0], policy)
        used = 0
        for s, c in zip(sizes, cls):
            if used + s <= 300:
                assert c == KV
                used += s
            else:
                assert c == DEFER
    # mirrored: only the token bin
    cls = oracle.divide_moves([(0, 0, 1, s) for s in sizes], [0], [300], "first_fit")
    used = 0
    for s, c in zip(sizes, cls):
        if used + s <= 300:
            assert c == TOK
            used += s
        else:
            assert c == DEFER


def test_library_equals_oracle_on_random_instances(oracle):
    rng = np.random.default_rng(2)
    for trial in range(300):
        n = int(rng.integers(0, 40))
        n_links, n_inst = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        comm = [int(x) for x in rng.integers(0, 10**12, n_links)]
        comp = [int(x) for x in rng.integers(0, 10**5, n_inst)]
        if trial % 7 == 0:
            comm[0] = 0
        if trial % 11 == 0:
            comp[0] = 0
        moves = [(int(rng.integers(n_links)), int(rng.integers(n_inst)),
                  int(rng.integers(0, 4 * 10**11)), int(rng.integers(0, 4 * 10**4)))
                 for _ in range(n)]
        for name, code in (("first_fit", kvm.KVM_FIRST_FIT), ("best_fit", kvm.KVM_BEST_FIT)):
            assert list(kvm.kvm_divide_moves(moves, comm, comp, code)) == \
                oracle.divide_moves(moves, comm, comp, name)


def test_every_instance_reaches_the_same_division(oracle):
    """Global consensus: the division is a pure function of the shared move list."""
    moves, comm, comp, ff, _ = load_golden()
    for _ in range(3):
        assert list(kvm.kvm_divide_moves(list(moves), list(comm), list(comp))) == ff


def test_argument_errors():
    for args in (([(2, 0, 1, 1)], [5], [5], 0), ([(0, 1, 1, 1)], [5], [5], 0), ([(0, 0, -1, 1)], [5], [5], 0),
                 ([(0, 0, 1, 1)], [-5], [5], 0), ([(0, 0, 1, 1)], [5], [5], 2)):
        with pytest.raises(kvm.KvmError) as e:
            kvm.kvm_divide_moves(*args)
        assert e.value.status == kvm.KVM_EINVAL
    assert len(kvm.kvm_divide_moves([], [1], [1])) == 0
