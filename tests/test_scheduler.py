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


@pytest.mark.parametrize("rate", [3, 12])
def test_static_sizes_satisfy_the_packing_theorems(rate):
    tr = sc.simulate(C, BPT, n_slots=250, arrival_rate=rate, median=4000, cap_tokens=16384,
                     growth_tokens=64, static_sizes=True, seed=11)       # check=True: Eq. 2 every slot
    g, lb = np.array(tr.gpus_per_slot), np.array(tr.lower_bound_per_slot)
    assert tr.peak_gpus > 25
    assert tr.worst_theorem1_violations <= max(10, 0.05 * tr.peak_gpus)
    assert (g <= 4 * lb / 3 + 4).all()                  # Theorem 2 against OPT >= ceil(total / C)
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
