"""Input generator for the multi-LLM mixed-pool scenario: one HBM arena carved
into three model regions (7B-shaped fp16, 8B-GQA-shaped bf16, 13B-shaped fp16),
each split into two halves that act as source and destination pools, a live set
of requests spread over them, and a seeded stream of migration orders.

Input generation only: the scenario says which request moves and how far
(`u`, the fraction of its tokens that is transferred as KV); carrying the order
out (allocation, copy, release) is the job of the code under test.

Stands in for the multi-model serving setting of arXiv 2501.06709 (Sec.
"Introduction": requests of several LLMs share the GPUs); lengths are seeded
log-normal instead of the chat datasets' conversation lengths.
"""
from dataclasses import dataclass

import numpy as np

from . import LLAMA2_7B, LLAMA2_13B, LLAMA3_8B, Model, lognormal_lengths

ALIGN = 2 << 20
SEED = 20250106 + 4
STREAM_BASE = 16  # value stream of (model i, half h) = STREAM_BASE + 2*i + h


@dataclass
class Request:
    model: int          # index into Scenario.models
    half: int           # 0 or 1: which half of the model's region holds it now
    length: int         # tokens currently cached
    table: np.ndarray   # int32 block ids in that half
    origin: list        # [(half, block id)] the logical blocks' first home: content identity


@dataclass
class Scenario:
    models: list
    half_blocks: list       # blocks per half, per model
    half_offset: list       # [model][half] byte offset into the arena
    arena_bytes: int
    requests: list
    orders: list            # (request index, u in [0.5, 1])
    seed: int

    def stream(self, model, half):
        return STREAM_BASE + 2 * model + half


def make(n_requests=512, n_orders=200, median=768, sigma=0.8, cap=16384, mix=(0.20, 0.65, 0.15),
         capacity_factor=1.5, models=None, seed=SEED):
    """capacity_factor: both halves of a model together hold this many times the
    model's live blocks, so a half is about 1/capacity_factor*... full and a move
    into it finds a fragmented free list."""
    rng = np.random.Generator(np.random.Philox(seed))
    models = list(models) if models is not None else [LLAMA2_7B, LLAMA3_8B, LLAMA2_13B]
    which = rng.choice(len(models), size=n_requests, p=np.asarray(mix) / np.sum(mix))
    lens = lognormal_lengths(rng, n_requests, median, sigma, cap)
    half_blocks, half_offset, off = [], [], 0
    loads = [[0, 0] for _ in models]
    assign = []
    for r in range(n_requests):
        mi = int(which[r])
        nb = -(-int(lens[r]) // models[mi].B)
        h = 0 if loads[mi][0] <= loads[mi][1] else 1
        loads[mi][h] += nb
        assign.append(h)
    for mi, m in enumerate(models):
        live = loads[mi][0] + loads[mi][1]
        n = max(int(np.ceil(capacity_factor * live / 2.0)), max(loads[mi]) + 1, 4)
        half_blocks.append(n)
        offs = []
        for _ in range(2):
            offs.append(off)
            off += -(-(n * m.block_bytes) // ALIGN) * ALIGN
        half_offset.append(offs)
    perms = [[rng.permutation(half_blocks[mi]).astype(np.int32) for _ in range(2)]
             for mi in range(len(models))]
    used = [[0, 0] for _ in models]
    requests = []
    for r in range(n_requests):
        mi, h = int(which[r]), assign[r]
        nb = -(-int(lens[r]) // models[mi].B)
        tab = perms[mi][h][used[mi][h]:used[mi][h] + nb].copy()
        used[mi][h] += nb
        requests.append(Request(mi, h, int(lens[r]), tab, [(h, int(b)) for b in tab]))
    orders = [(int(rng.integers(n_requests)), float(rng.uniform(0.5, 1.0))) for _ in range(n_orders)]
    return Scenario(models, half_blocks, half_offset, off, requests, orders, seed)


def occupancy(sc, model, half):
    """uint8 [half_blocks]: 1 where a live request holds the block."""
    occ = np.zeros(sc.half_blocks[model], dtype=np.uint8)
    for rq in sc.requests:
        if rq.model == model and rq.half == half:
            occ[rq.table] = 1
    return occ


def small_models():
    """The three layouts with fewer layers, for cases the CPU oracle must finish
    in seconds (heads, head_dim, dtype and grouping as in the full shapes)."""
    return [Model("llama2_7b_L2", 2, 32, 32, 128, 16, "f16"),
            Model("llama3_8b_gqa_L2", 2, 8, 32, 128, 16, "bf16"),
            Model("llama2_13b_L2", 2, 40, 40, 128, 16, "f16")]
