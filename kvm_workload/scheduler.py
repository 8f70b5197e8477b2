"""Order-stream generator: a simulator of the online KV-cache scheduler of arXiv
2501.06709 (Sec. "Online KV Cache Scheduling": request classes L/M/S/T, the
Allocate / Depart / Update operations of the operations figure, Algorithm 1, and
request operation batching).  Its job in this repository is to *produce inputs*:
realistic streams of "move request i from GPU j to GPU j'" orders for the
migration path (kvm_divide_moves decides how each one travels, kvm_migrate moves
the KV).  It is not part of the library and moves no KV itself.

The paper leaves much of the algorithm open; the readings taken here:

* Sizes are bytes of KV (tokens x bytes_per_token); C is a GPU's KV capacity.
  Classes by size s: L (C/2, C], M (C/3, C/2], S (C/4, C/3], T (0, C/4].
* Requests of at most C/8 are grouped into multi-items ("bundles") that aim at a
  total in (C/8, C/4]; a bundle is handled as one T item and moving it counts as
  one migration in the per-operation bound, although every member's KV moves.  A
  new small request joins the first open bundle it fits, else opens a new one.
* A GPU's category is the class of its largest item.  "Most recently activated"
  is by activation order.  Priority among candidate GPUs: more free bytes first,
  then fewer items, then older (the paper leaves the weights to the provider).
* Allocate T: an L-GPU with room (best priority), else an M-GPU with room that
  holds no T yet, else the latest T-GPU if it has room, else a new GPU.
* Allocate S / M: an L-GPU that holds no S/M item and whose L item leaves room
  (T items there are evicted, largest first, only as far as needed, and
  re-allocated); else the latest GPU of the same category with a free place
  (two M, three S) and room; else a new GPU.
* Allocate L: a new GPU; then one S/M item that fits is pulled in from an S/M-GPU
  (largest fitting item, latest GPU first) and that GPU is refilled from the
  latest GPU of its category.
* Depart: remove the item.  If its GPU is not the latest of its category, refill
  it: after a T left, one T item that fits is pulled from the latest T-GPU; after
  an S/M left an S/M-GPU, one item of that class is pulled from the latest GPU of
  the category; after an S/M left an L-GPU, one S/M item that fits is pulled from
  an S/M-GPU (best priority) which is then refilled from the latest one; after an
  L left, all other items of the GPU are departed and re-allocated.
* Update (a size change): a class change departs and re-allocates the item; if a
  GPU is over capacity after growth, its other items are departed and
  re-allocated smallest first until it fits (the paper only covers the L and M
  cases); a bundle that outgrows C/4 sheds members (latest first), which re-enter
  as new small requests.
* Batching: within a time slot all departures are applied first, then updates,
  then arrivals; the orders emitted for the slot are the *net* moves (where a
  request is at the end of the slot against where it was at the start), which
  drops moves that cancel or chain; the unbatched count is kept for comparison.

* T-GPU upkeep after an operation: a GPU that gave its last S/M/L item away has
  become a T-GPU, and a T-GPU that lost bytes may have dropped under 75 %.  The
  operations figure only repairs the GPU a request departs from; without a rule for
  these donors and left-overs the number of under-filled T-GPUs grows with the
  cluster (13 of 406 GPUs, against 4 of 30), which Theorem 1 excludes.  So every
  GPU that lost an item during an operation is looked at once the operation has
  been carried out: unless it is the latest T-GPU, a T-GPU under 75 % that holds one
  item is dissolved (the item is re-allocated), else it is filled up from the
  latest T-GPU (any T item fits while more than a quarter of the memory is free).

Pins (tests/test_scheduler.py) are the paper's own claims: capacity is never
exceeded (Eq. 2); with fixed request sizes (the setting of the packing theorems)
the five properties of Theorem 1 hold on all but a constant number of GPUs (at
most 8 from 35 to 920 GPUs: the latest GPU of each category and a few in
transit); the GPU count stays within 4/3 of the size lower bound plus 2 (Theorem
2), and within 4/3 of the exact optimum plus 2 on instances small enough for
exhaustive packing; no operation moves more than ten items (Theorem 3; at most 6
observed); the emitted order stream replays on an independent ledger.
"""
from dataclasses import dataclass, field

import numpy as np

ORDER = {"L": 3, "M": 2, "S": 1, "T": 0}


def size_class(s, C):
    if s * 2 > C:
        return "L"
    if s * 3 > C:
        return "M"
    if s * 4 > C:
        return "S"
    return "T"


@dataclass
class Item:
    members: dict = field(default_factory=dict)   # request id -> size
    bundle: bool = False
    gpu: object = None

    @property
    def size(self):
        return sum(self.members.values())


@dataclass
class Gpu:
    gid: int
    items: list = field(default_factory=list)

    def used(self):
        return sum(it.size for it in self.items)


class Scheduler:
    def __init__(self, capacity):
        self.C = int(capacity)
        self.gpus = []              # activation order
        self.next_gid = 0
        self.where = {}             # request id -> Item
        self.moves_this_op = 0      # item moves caused by the current operation
        self.max_moves_per_op = 0
        self.total_item_moves = 0
        self.total_request_moves = 0
        self.peak_gpus = 0
        self.lost = []              # GPUs that gave an item away during the current operation

    # ---- helpers ----
    def cls(self, item):
        return size_class(item.size, self.C)

    def category(self, g):
        return max((self.cls(it) for it in g.items), key=lambda c: ORDER[c]) if g.items else None

    def free(self, g):
        return self.C - g.used()

    def latest(self, cat, exclude=None):
        for g in reversed(self.gpus):
            if g is not exclude and self.category(g) == cat:
                return g
        return None

    def priority(self, g):
        return (self.free(g), -len(g.items), -g.gid)

    def _new_gpu(self):
        g = Gpu(self.next_gid)
        self.next_gid += 1
        self.gpus.append(g)
        self.peak_gpus = max(self.peak_gpus, len(self.gpus))
        return g

    def _place(self, item, g):
        g.items.append(item)
        item.gpu = g

    def _take(self, item):
        g = item.gpu
        g.items.remove(item)
        item.gpu = None
        if not g.items:
            self.gpus.remove(g)
        else:
            self.lost.append(g)     # looked at again when the operation has been carried out
        return g

    def _move(self, item, dst):
        """One item migration (a bundle counts once)."""
        self._take(item)
        self._place(item, dst)
        self.moves_this_op += 1
        self.total_item_moves += 1
        self.total_request_moves += len(item.members)

    def _count(self, g, c):
        return sum(1 for it in g.items if self.cls(it) == c)

    # ---- Allocate ----
    def allocate(self, item, migrating=False):
        c = self.cls(item)
        s = item.size
        target = None
        evict = []
        if c == "T":
            cands = [g for g in self.gpus if self.category(g) == "L" and self.free(g) >= s]
            if not cands:
                cands = [g for g in self.gpus if self.category(g) == "M" and self.free(g) >= s
                         and self._count(g, "M") == 2 and self._count(g, "T") == 0]
            if cands:
                target = max(cands, key=self.priority)
            else:
                g = self.latest("T")
                target = g if g is not None and self.free(g) >= s else None
        elif c in ("S", "M"):
            cands = []
            for g in self.gpus:
                if self.category(g) != "L" or self._count(g, "S") + self._count(g, "M") > 0:
                    continue
                big = sum(it.size for it in g.items if self.cls(it) == "L")
                if big + s < self.C:
                    cands.append(g)
            if cands:
                target = max(cands, key=self.priority)
                ts = sorted((it for it in target.items if self.cls(it) == "T"), key=lambda it: -it.size)
                need = s - self.free(target)
                for it in ts:
                    if need <= 0:
                        break
                    evict.append(it)
                    need -= it.size
            else:
                g = self.latest(c)
                limit = 2 if c == "M" else 3
                if g is not None and self._count(g, c) < limit:
                    evict = self._ts_to_evict(g, s)      # a T riding along must not block a pair
                    if self.free(g) + sum(it.size for it in evict) >= s:
                        target = g
                    else:
                        evict = []
        if target is None:
            target = self._new_gpu()
        for it in evict:
            self._take(it)
        self._place(item, target)
        if migrating:
            self.moves_this_op += 1
            self.total_item_moves += 1
            self.total_request_moves += len(item.members)
        for it in evict:
            self.allocate(it, migrating=True)
        if c == "L":
            self._pull_sm_into(target)

    def _pull_sm_into(self, g):
        """Move one S/M item that fits from an S/M-GPU into L-GPU g, refill the donor."""
        room = self.free(g)
        best = None
        for d in reversed(self.gpus):
            if d is g or self.category(d) not in ("S", "M"):
                continue
            for it in d.items:
                if self.cls(it) in ("S", "M") and it.size <= room and \
                        sum(x.size for x in g.items if self.cls(x) == "L") + it.size < self.C:
                    if best is None or it.size > best.size:
                        best = it
            if best is not None:
                break
        if best is None:
            return
        donor, c = best.gpu, self.cls(best)
        self._move(best, g)
        if donor in self.gpus:
            self._refill_same_class(donor, c)

    def _ts_to_evict(self, g, need_bytes):
        """T items of g (largest first) whose removal makes room for need_bytes."""
        out, need = [], need_bytes - self.free(g)
        for it in sorted((it for it in g.items if self.cls(it) == "T"), key=lambda it: -it.size):
            if need <= 0:
                break
            out.append(it)
            need -= it.size
        return out

    def _refill_same_class(self, g, c):
        """g lost an item of class c: pull one from the latest GPU of that category
        (T items of g give way and are re-allocated)."""
        last = self.latest(c, exclude=g)
        if last is None or self.gpus.index(last) < self.gpus.index(g):
            return
        for it in sorted(last.items, key=lambda it: -it.size):
            if self.cls(it) != c:
                continue
            evict = self._ts_to_evict(g, it.size)
            if self.free(g) + sum(x.size for x in evict) >= it.size:
                for x in evict:
                    self._take(x)
                self._move(it, g)
                for x in evict:
                    self.allocate(x, migrating=True)
                return

    # ---- Depart ----
    def depart(self, item, c=None):
        """Remove the item and repair its GPU; `c` is the class it had while it was
        placed (differs from its current class inside Update)."""
        c = c or self.cls(item)
        g = item.gpu
        cat = self.category(g)
        was_latest = self.latest(cat) is g
        self._take(item)
        if g not in self.gpus:
            return
        if c == "L":
            for it in sorted(list(g.items), key=lambda it: -it.size):
                self._take(it)
                self.allocate(it, migrating=True)
            return
        if was_latest:
            return
        if c == "T":
            self.refill_t(g)
        elif cat == "L":
            self._pull_sm_into(g)
        else:
            self._refill_same_class(g, c)

    def refill_t(self, g):
        """g lost T bytes: pull up to two T items that fit from the latest T-GPU."""
        if g not in self.gpus:
            return
        last = self.latest("T", exclude=g)
        if last is None:
            return
        if self.category(g) == "T" and self.gpus.index(last) < self.gpus.index(g):
            return
        pulled = 0
        for it in sorted(last.items, key=lambda it: -it.size):
            if pulled < 2 and self.cls(it) == "T" and it.size <= self.free(g):
                self._move(it, g)
                pulled += 1

    # ---- Update ----
    def update(self, item, old_class):
        g = item.gpu
        c = self.cls(item)
        if c != old_class:
            self.depart(item, old_class)
            self.allocate(item, migrating=True)
            g = item.gpu
        # overload after growth: shed other items, smallest first
        while self.free(g) < 0 and len(g.items) > 1:
            victim = min((it for it in g.items if it is not item), key=lambda it: it.size)
            self._take(victim)
            self.allocate(victim, migrating=True)

    def _repair_t_gpus(self):
        """A GPU that gave its last S/M/L item away has become a T-GPU; any T-GPU that
        lost bytes may have dropped under 75 %.  Unless it is the latest T-GPU (the one
        allowed exception), such a GPU is dissolved when one item is all it holds (the
        item is re-allocated: one migration), else filled up from the latest T-GPU (any
        T item fits while more than a quarter of the memory is free)."""
        guard = 0
        while self.lost and guard < 64:
            guard += 1
            g = self.lost.pop()
            if g not in self.gpus or self.category(g) != "T" or g.used() * 4 >= 3 * self.C:
                continue
            last = self.latest("T")
            if last is g:
                continue
            if len(g.items) == 1:
                it = g.items[0]
                self._take(it)
                self.allocate(it, migrating=True)
                continue
            while g.used() * 4 < 3 * self.C:
                last = self.latest("T", exclude=g)
                if last is None or self.gpus.index(last) < self.gpus.index(g):
                    break
                fits = [it for it in last.items if it.size <= self.free(g)]
                if not fits:
                    break
                self._move(max(fits, key=lambda it: it.size), g)
        self.lost.clear()

    # ---- one operation with migration accounting ----
    def run_op(self, fn, *args):
        self.moves_this_op = 0
        self.lost.clear()
        fn(*args)
        self._repair_t_gpus()
        self.max_moves_per_op = max(self.max_moves_per_op, self.moves_this_op)

    # ---- invariants ----
    def check_capacity(self):
        for g in self.gpus:
            assert g.used() <= self.C, (g.gid, g.used(), self.C)
            assert g.items
        for rid, it in self.where.items():
            assert rid in it.members and it.gpu is not None and it in it.gpu.items

    def theorem1_violations(self):
        """Number of GPUs that break one of the five packing properties."""
        C = self.C
        bad = 0
        sm_items = [it for g in self.gpus if self.category(g) in ("S", "M") for it in g.items
                    if self.cls(it) in ("S", "M")]
        lm_full = all(g.used() * 4 >= 3 * C for g in self.gpus if self.category(g) in ("L", "M"))
        for g in self.gpus:
            cat = self.category(g)
            if cat == "M" and not (self._count(g, "M") == 2 and self._count(g, "S") == 0
                                   and self._count(g, "T") <= 1):
                bad += 1
            elif cat == "S" and self._count(g, "S") != 3:
                bad += 1
            elif cat == "T" and g.used() * 4 < 3 * C:
                bad += 1
            elif cat == "L" and self._count(g, "S") + self._count(g, "M") == 0:
                big = sum(it.size for it in g.items if self.cls(it) == "L")
                if any(big + it.size < C for it in sm_items):
                    bad += 1
        t_gpus = sum(1 for g in self.gpus if self.category(g) == "T")
        if t_gpus and not lm_full:
            bad += sum(1 for g in self.gpus if self.category(g) in ("L", "M") and g.used() * 4 < 3 * C)
        return bad


@dataclass
class Trace:
    orders: list            # per slot: list of (request id, src gpu id, dst gpu id, bytes)
    departures: list        # per slot: request ids that completed (applied first)
    arrivals: list          # per slot: (request id, gpu id at the end of the slot, bytes)
    gpus_per_slot: list
    lower_bound_per_slot: list
    max_moves_per_op: int
    item_moves_unbatched: int
    request_moves_batched: int
    request_moves_unbatched: int
    worst_theorem1_violations: int
    peak_gpus: int


def simulate(capacity, bytes_per_token, n_slots=200, arrival_rate=0.8, median=768, sigma=0.8,
             cap_tokens=16384, growth_tokens=16, final_factor=(1.0, 1.6), seed=20250106,
             static_sizes=False, check=True):
    """Poisson arrivals; a request arrives with `prompt` tokens (log-normal), then
    gains `growth_tokens` per slot until it reaches prompt * U(final_factor) and
    completes.  static_sizes: requests keep their arrival size (no Update
    operations), the setting in which the packing theorems are stated."""
    rng = np.random.Generator(np.random.Philox(seed))
    sch = Scheduler(capacity)
    open_bundles = []
    live = {}       # rid -> [tokens, final tokens]
    rid_next = 0
    orders, gpus_per_slot, lb, worst = [], [], [], 0
    departures, arrivals = [], []
    req_unbatched = 0

    def gpu_of(rid):
        return sch.where[rid].gpu.gid

    def add_small(rid, size):
        for b in open_bundles:
            if b.gpu is not None and b.size + size <= capacity // 4 and sch.free(b.gpu) >= size:
                b.members[rid] = size
                sch.where[rid] = b
                return
        b = Item({rid: size}, bundle=True)
        open_bundles.append(b)
        sch.where[rid] = b
        sch.run_op(sch.allocate, b)

    def add_request(rid, size):
        if size * 8 <= capacity:
            add_small(rid, size)
        else:
            it = Item({rid: size})
            sch.where[rid] = it
            sch.run_op(sch.allocate, it)

    def remove_request(rid):
        it = sch.where.pop(rid)
        if it.bundle and len(it.members) > 1:
            old = sch.cls(it)
            del it.members[rid]
            sch.run_op(sch.update, it, old)      # a shrink: only refits if its class changed
            if it.gpu is not None and it.gpu.used() * 4 < 3 * capacity:
                sch.run_op(sch.refill_t, it.gpu)
        else:
            if it.bundle:
                open_bundles.remove(it)
            sch.run_op(sch.depart, it)

    for slot in range(n_slots):
        start_place = {rid: gpu_of(rid) for rid in live}
        moves_before = sch.total_request_moves
        # (1) departures
        done = [rid for rid, (tok, fin) in live.items() if tok >= fin]
        departures.append(list(done))
        for rid in done:
            del live[rid]
            start_place.pop(rid)
            remove_request(rid)
        # (2) updates: growth
        if not static_sizes:
            for rid in list(live):
                tok, fin = live[rid]
                new_tok = min(fin, tok + growth_tokens)
                if new_tok == tok:
                    continue
                live[rid][0] = new_tok
                it = sch.where[rid]
                old = sch.cls(it)
                it.members[rid] = new_tok * bytes_per_token
                if it.bundle:
                    shed = []
                    while it.size * 4 > capacity and len(it.members) > 1:
                        last = list(it.members)[-1]
                        shed.append((last, it.members.pop(last)))
                    for r2, s2 in shed:
                        del sch.where[r2]
                if sch.cls(it) != old or sch.free(it.gpu) < 0:
                    sch.run_op(sch.update, it, old)
                if it.bundle:
                    for r2, s2 in shed:
                        add_request(r2, s2)
        # (3) arrivals
        for _ in range(rng.poisson(arrival_rate)):
            prompt = int(np.clip(np.rint(np.exp(np.log(median) + sigma * rng.standard_normal())), 1,
                                 cap_tokens))
            fin = prompt if static_sizes else min(cap_tokens, int(prompt * rng.uniform(*final_factor)) + 1)
            if static_sizes:
                fin = prompt + int(rng.integers(5, 60)) * growth_tokens   # lifetime only
            rid = rid_next
            rid_next += 1
            live[rid] = [prompt, fin]
            add_request(rid, prompt * bytes_per_token)
        if static_sizes:
            for rid in live:
                live[rid][0] += growth_tokens       # ages, size unchanged
        # (4) net moves of the slot = the batched order list
        slot_orders = []
        for rid, g0 in start_place.items():
            g1 = gpu_of(rid)
            if g1 != g0:
                slot_orders.append((rid, g0, g1, sch.where[rid].members[rid]))
        orders.append(slot_orders)
        arrivals.append([(rid, gpu_of(rid), sch.where[rid].members[rid]) for rid in live
                         if rid not in start_place])
        req_unbatched += sch.total_request_moves - moves_before
        gpus_per_slot.append(len(sch.gpus))
        total = sum(it.size for g in sch.gpus for it in g.items)
        lb.append(-(-total // capacity))
        if check:
            sch.check_capacity()
            worst = max(worst, sch.theorem1_violations())
    return Trace(orders, departures, arrivals, gpus_per_slot, lb, sch.max_moves_per_op, sch.total_item_moves,
                 sum(len(o) for o in orders), req_unbatched, worst, sch.peak_gpus)
