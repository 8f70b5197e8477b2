"""The library allocates nothing and never synchronises, so a sequence of its
calls can be captured into a HIP graph and replayed: the launch-bound tiny config
(four kernels of ~10 us) is where that pays.  Each replay is checked against the
eager result, with eager work and synchronisation between replays and with the
source pool's contents changed in between.
"""
import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm
from kvm_workload import device as wl_device

from gpu_util import DEV, Side, to_host

pytestmark = pytest.mark.gpu


def test_captured_path_replays_like_eager(oracle):
    w = wl.make("tiny")
    m = w.model
    h_src = wl.gen_pool_host(w.seed, wl.STREAM_SRC, m, w.n_blocks_src)
    h_dst = wl.gen_pool_host(w.seed, wl.STREAM_DST, m, w.n_blocks_dst)
    fl = kvm.FreeList(w.n_blocks_dst, w.dst_occupied)
    d_tabs = [fl.alloc(n) for n in w.n_dst_blocks()]
    src = Side(m, w.n_blocks_src, h_src, [w.src_tables[i] for i in w.migrate_ids], w.k)
    dst = Side(m, w.n_blocks_dst, h_dst, d_tabs, w.k)
    n_stage = kvm.kvm_staging_bytes(src.layout, src.batch)
    stage = torch.zeros(n_stage, dtype=torch.uint8, device=DEV)
    q = wl.gen_q(w.seed, m, len(w.k))
    q_dev = torch.from_numpy(q.view(np.int16)).to(DEV)
    out = torch.zeros(q.shape, dtype=torch.float32, device=DEV)

    def path():
        kvm.kvm_pack(src.pool, src.batch, stage, staging_bytes=n_stage)
        kvm.kvm_unpack(stage, dst.pool, dst.batch, staging_bytes=n_stage)
        kvm.kvm_migrate(src.pool, src.batch, dst.pool, dst.batch)
        kvm.kvm_paged_decode(dst.pool, dst.batch, q_dev, out)

    path()                      # eager warm-up before capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for seed in (101, 102, 103, 104):
        # new source contents (eager fill kernel), destination reset, then one replay
        wl_device.fill_pool(src.dev, m, w.n_blocks_src, seed, wl.STREAM_SRC)
        wl_device.fill_pool(dst.dev, m, w.n_blocks_dst, seed, wl.STREAM_DST)
        out.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_dst, got_out = to_host(dst.dev).copy(), out.cpu().numpy().copy()
        wl_device.fill_pool(dst.dev, m, w.n_blocks_dst, seed, wl.STREAM_DST)
        out.fill_(-1.0)
        path()                  # the same work eagerly
        torch.cuda.synchronize()
        assert np.array_equal(got_dst, to_host(dst.dev)), "replay differs from eager (seed %d)" % seed
        assert np.array_equal(got_out, out.cpu().numpy())
        # and both equal the oracle for this seed
        hs = wl.gen_pool_host(seed, wl.STREAM_SRC, m, w.n_blocks_src)
        hd = wl.gen_pool_host(seed, wl.STREAM_DST, m, w.n_blocks_dst)
        oracle.migrate(hs, src.st, hd, dst.st, m.L, m.H, m.D, m.B, src.off, src.blk, dst.off, dst.blk, w.k)
        assert np.array_equal(got_dst, hd)
    # timing: replay against eager launches of the same four kernels
    def timed(fn, reps=50):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    print("tiny path: eager %.1f us per pass, graph replay %.1f us" % (1e3 * timed(path), 1e3 * timed(graph.replay)))
