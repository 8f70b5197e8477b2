"""The order-stream generator built from the paper's online scheduler (arXiv
2501.06709, Sec. "Online KV Cache Scheduling" and Sec. "Analysis") is pinned by the
paper's own claims: Eq. 2 (capacity), Theorem 1 (packing properties, up to a few
GPUs), Theorem 2 (GPU count within 4/3 of a lower bound plus a constant),
Theorem 3 (at most ten item migrations per operation), and the effect of request
operation batching (fewer migrations than one-at-a-time execution).
"""
import numpy as np
import pytest

from kvm_workload import scheduler as sc

C = 16 * 10**9          # KV capacity of a 40 GB GPU holding 24 GB of weights
BPT = 819200            # LLaMA-13B bytes per token


T1_EXCEPTIONS = 8       # Theorem 1's "constant number of exceptions": the same bound at every cluster size


@pytest.mark.parametrize("rate,slots", [(3, 250), (12, 250), (48, 120)])
def test_static_sizes_satisfy_the_packing_theorems(rate, slots):
    """37, 120 and 450 GPUs: the number of GPUs that break one of Theorem 1's five
    properties stays below one constant (measured 5, 6 and 6; 8 at 900 GPUs)."""
    tr = sc.simulate(C, BPT, n_slots=slots, arrival_rate=rate, median=4000, cap_tokens=16384,
                     growth_tokens=64, static_sizes=True, seed=11)       # check=True: Eq. 2 every slot
    g, lb = np.array(tr.gpus_per_slot), np.array(tr.lower_bound_per_slot)
    assert tr.peak_gpus > 8 * rate
    assert tr.worst_theorem1_violations <= T1_EXCEPTIONS
    assert (g <= 4 * lb / 3 + 2).all()                  # Theorem 2 against OPT >= ceil(total / C)
    assert tr.max_moves_per_op <= 10                    # Theorem 3
    assert tr.request_moves_batched <= tr.request_moves_unbatched


def test_growing_sizes_keep_capacity_count_and_migration_bounds():
    tr = sc.simulate(C, BPT, n_slots=250, arrival_rate=6, median=4000, cap_tokens=16384,
                     growth_tokens=64, static_sizes=False, seed=12)
    g, lb = np.array(tr.gpus_per_slot), np.array(tr.lower_bound_per_slot)
    assert (g <= 4 * lb / 3 + 4).all()
    assert tr.max_moves_per_op <= 10
    assert tr.request_moves_batched < tr.request_moves_unbatched     # batching removes moves
    saved = 1 - tr.request_moves_batched / tr.request_moves_unbatched
    assert 0.02 < saved < 0.6, saved


def test_orders_are_consistent_moves():
    tr = sc.simulate(C, BPT, n_slots=120, arrival_rate=6, median=4000, cap_tokens=16384,
                     growth_tokens=64, static_sizes=True, seed=13)
    seen = 0
    for slot in tr.orders:
        rids = [o[0] for o in slot]
        assert len(set(rids)) == len(rids)              # net moves: one per request and slot
        for rid, src, dst, nbytes in slot:
            assert src != dst and nbytes > 0 and nbytes % BPT == 0
        seen += len(slot)
    assert seen == tr.request_moves_batched and seen > 50
    again = sc.simulate(C, BPT, n_slots=120, arrival_rate=6, median=4000, cap_tokens=16384,
                        growth_tokens=64, static_sizes=True, seed=13)
    assert again.orders == tr.orders                    # seeded


def test_size_classes():
    assert [sc.size_class(s, 24) for s in (24, 13, 12, 9, 8, 7, 6, 3, 1)] == \
        ["L", "L", "M", "M", "S", "S", "T", "T", "T"]


def replay(tr, capacity):
    """An independent ledger driven only by what the generator emits (departures,
    net moves, arrivals per slot): every order must start where the ledger has the
    request, no GPU may exceed its capacity at the end of a slot, and the number of
    GPUs in use must be the one the generator reports."""
    where, size = {}, {}
    for slot, (deps, moves, arrs) in enumerate(zip(tr.departures, tr.orders, tr.arrivals)):
        for rid in deps:
            del where[rid], size[rid]
        for rid, src, dst, nbytes in moves:
            assert where[rid] == src and size[rid] == nbytes, (slot, rid)
            where[rid] = dst
        for rid, gpu, nbytes in arrs:
            assert rid not in where
            where[rid], size[rid] = gpu, nbytes
        load = {}
        for rid, gpu in where.items():
            load[gpu] = load.get(gpu, 0) + size[rid]
        assert all(v <= capacity for v in load.values()), slot
        assert len(load) == tr.gpus_per_slot[slot], slot
    return len(where)


def test_emitted_stream_replays_on_an_independent_ledger():
    tr = sc.simulate(C, BPT, n_slots=200, arrival_rate=8, median=4000, cap_tokens=16384,
                     growth_tokens=64, static_sizes=True, seed=21, check=False)
    assert replay(tr, C) > 20


def optimal_bins(sizes, capacity):
    """Exact bin packing by exhaustive search (tiny inputs): fewest bins of `capacity`."""
    sizes = sorted(sizes, reverse=True)
    best = [len(sizes)]

    def go(i, bins):
        if len(bins) >= best[0]:
            return
        if i == len(sizes):
            best[0] = len(bins)
            return
        seen = set()
        for b in range(len(bins)):
            if bins[b] + sizes[i] <= capacity and bins[b] not in seen:
                seen.add(bins[b])
                bins[b] += sizes[i]
                go(i + 1, bins)
                bins[b] -= sizes[i]
        bins.append(sizes[i])
        go(i + 1, bins)
        bins.pop()

    go(0, [])
    return best[0]


def test_tiny_instances_against_exhaustive_optimal_packing():
    """Theorem 2 on instances small enough for an exact optimum: after every arrival
    and departure the scheduler's GPU count is within 4/3 of the optimal packing of
    the live requests plus the constant of the latest GPUs, and no operation moves
    more than ten items (Theorem 3)."""
    cap = 240
    rng = np.random.default_rng(5)
    worst_gap = 0
    for trial in range(40):
        sch = sc.Scheduler(cap)
        live = []
        for step in range(30):
            if live and (len(live) >= 11 or rng.random() < 0.4):
                it = live.pop(int(rng.integers(len(live))))
                sch.run_op(sch.depart, it)
            else:
                it = sc.Item({("r", trial, step): int(rng.integers(cap // 8 + 1, cap + 1))})
                live.append(it)
                sch.run_op(sch.allocate, it)
            sch.check_capacity()
            assert sorted(id(x) for g in sch.gpus for x in g.items) == sorted(id(x) for x in live)
            if live:
                opt = optimal_bins([x.size for x in live], cap)
                assert len(sch.gpus) >= opt
                worst_gap = max(worst_gap, len(sch.gpus) - 4 * opt / 3)
                assert len(sch.gpus) <= 4 * opt / 3 + 2, (trial, step, len(sch.gpus), opt)
        assert sch.max_moves_per_op <= 10
    assert worst_gap > -1          # the bound is not vacuous on these instances
