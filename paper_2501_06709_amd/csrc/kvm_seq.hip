// Order sequencing around the data path: allocate, upload the tables, copy, decode,
// release the source only after the copy has finished.
//
// An order moves tokens [0,k) of one request from its pool into another pool of
// the same model (arXiv 2501.06709, Sec. "Adaptive Request Migration").  The
// scheduler hands over a time slot's move list at once (Sec. "Online KV Cache
// Scheduling", request operation batching), so orders are staged and then enqueued
// together: one host-to-device copy carries the tables of all staged orders, and
// the staged orders that share a (source pool, destination pool) pair become one
// kvm_migrate and one kvm_paged_decode_rows call.  The source blocks of an order go
// back to the source free list only when the event recorded behind its flush has
// completed ("Boundary Profiling": source memory is held until the transfer is
// complete); at most `depth` flushes are in flight before the host waits for the
// oldest one, so the stream never drains between flushes.
//
// Host code only: the data movement is kvm_migrate's and kvm_paged_decode_rows'.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <deque>
#include <map>
#include <memory>
#include <utility>
#include <vector>

#include "kvm_internal.h"

namespace {

using namespace kvm;

struct Side {
  kvm_pool pool;      // copied: the caller's struct need not outlive the call
  kvm_freelist* fl;
};

struct Order {
  std::vector<int32_t> table, ids;
  int32_t k;
  Side src, dst;
  const void* q;
  void* out;
  int32_t row;
};

struct Flight {
  std::shared_ptr<hipEvent_t> ev;
  std::vector<std::pair<kvm_freelist*, std::vector<int32_t>>> released;
};

struct CopyMark {
  hipEvent_t e0, e1;
  int64_t bytes;
};

}  // namespace

struct kvm_sequencer {
  int32_t max_blocks, max_staged, depth;
  int32_t* pin;
  int32_t* dev;
  int64_t region_ints;
  int32_t n_regions, region = 0;
  std::vector<std::shared_ptr<hipEvent_t>> region_event;
  std::vector<Order> staged;
  std::deque<Flight> pending;
  // blocks that a staged, not yet enqueued order will write, per pool (by base address)
  std::map<const void*, std::vector<uint8_t>> staged_writes;
  void* ws;
  int64_t ws_bytes;
  int64_t launches = 0;
  bool timing = false;
  std::vector<CopyMark> marks;
  std::vector<hipEvent_t> spare_events;

  std::shared_ptr<hipEvent_t> new_event(int* rc) {
    hipEvent_t ev = nullptr;
    if (!spare_events.empty()) {
      ev = spare_events.back();
      spare_events.pop_back();
    } else {
      const hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
      if (e != hipSuccess) {
        *rc = fail(KVM_EHIP, std::string("hipEventCreate: ") + hipGetErrorString(e));
        return nullptr;
      }
    }
    // the last holder hands the event back for reuse
    return std::shared_ptr<hipEvent_t>(new hipEvent_t(ev), [this](hipEvent_t* p) {
      spare_events.push_back(*p);
      delete p;
    });
  }
};

namespace {

int wait_event(const std::shared_ptr<hipEvent_t>& ev) {
  if (!ev) return KVM_OK;
  const hipError_t e = hipEventSynchronize(*ev);
  return e == hipSuccess ? KVM_OK : fail(KVM_EHIP, std::string("hipEventSynchronize: ") + hipGetErrorString(e));
}

int retire_oldest(kvm_sequencer* s) {
  Flight f = std::move(s->pending.front());
  s->pending.pop_front();
  int rc = wait_event(f.ev);
  // the blocks are released even if the wait reports an error of some earlier launch:
  // nothing reads them any more once the stream has stopped
  for (auto& r : f.released) {
    const int rc2 = kvm_freelist_free(r.first, (int32_t)r.second.size(), r.second.data());
    if (rc == KVM_OK) rc = rc2;
  }
  return rc;
}

std::vector<uint8_t>& write_mask(kvm_sequencer* s, const kvm_pool& pool) {
  std::vector<uint8_t>& m = s->staged_writes[pool.base];
  if ((int64_t)m.size() < pool.n_blocks) m.resize((size_t)pool.n_blocks, 0);
  return m;
}

int flush(kvm_sequencer* s, hipStream_t st) {
  if (s->staged.empty()) return KVM_OK;
  std::vector<Order> staged;
  staged.swap(s->staged);
  for (const Order& o : staged) {
    std::vector<uint8_t>& m = write_mask(s, o.dst.pool);
    for (int32_t id : o.ids) m[(size_t)id] = 0;
  }
  // groups: orders with the same (source pool, destination pool), in order of first appearance
  std::vector<std::vector<const Order*>> groups;
  for (const Order& o : staged) {
    bool placed = false;
    for (auto& g : groups)
      if (g[0]->src.pool.base == o.src.pool.base && g[0]->dst.pool.base == o.dst.pool.base) {
        g.push_back(&o);
        placed = true;
        break;
      }
    if (!placed) groups.push_back({&o});
  }
  // the region's previous readers must be done before it is rewritten
  int rc = wait_event(s->region_event[s->region]);
  s->region_event[s->region].reset();
  const int64_t lo = (int64_t)s->region * s->region_ints;
  int64_t at = lo;
  struct Plan {
    std::vector<int32_t> s_off, d_off, s_blk, d_blk, k;
    int64_t s_at, d_at;
  };
  std::vector<Plan> plans(groups.size());
  for (size_t g = 0; g < groups.size(); ++g) {
    Plan& p = plans[g];
    p.s_off.push_back(0);
    p.d_off.push_back(0);
    for (const Order* o : groups[g]) {
      p.s_blk.insert(p.s_blk.end(), o->table.begin(), o->table.end());
      p.d_blk.insert(p.d_blk.end(), o->ids.begin(), o->ids.end());
      p.s_off.push_back((int32_t)p.s_blk.size());
      p.d_off.push_back((int32_t)p.d_blk.size());
      p.k.push_back(o->k);
    }
    p.s_at = at;
    p.d_at = at + (int64_t)p.s_blk.size();
    if (!p.s_blk.empty()) memcpy(s->pin + p.s_at, p.s_blk.data(), p.s_blk.size() * 4);
    if (!p.d_blk.empty()) memcpy(s->pin + p.d_at, p.d_blk.data(), p.d_blk.size() * 4);
    at = p.d_at + (int64_t)p.d_blk.size();
  }
  if (rc == KVM_OK && at > lo) {
    const hipError_t e = hipMemcpyAsync(s->dev + lo, s->pin + lo, (size_t)(at - lo) * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) rc = fail(KVM_EHIP, std::string("hipMemcpyAsync: ") + hipGetErrorString(e));
  }
  Flight flight;
  size_t enqueued = 0;   // groups whose copy is in flight
  for (size_t g = 0; g < groups.size() && rc == KVM_OK; ++g) {
    const Plan& p = plans[g];
    const Order& first = *groups[g][0];
    kvm_batch sb{(int32_t)p.k.size(), p.s_off.data(), s->dev + p.s_at, p.s_blk.data(), p.k.data(), nullptr};
    kvm_batch db{(int32_t)p.k.size(), p.d_off.data(), s->dev + p.d_at, p.d_blk.data(), p.k.data(), nullptr};
    CopyMark mark{nullptr, nullptr, 0};
    bool timed = s->timing && hipEventCreate(&mark.e0) == hipSuccess && hipEventCreate(&mark.e1) == hipSuccess &&
                 hipEventRecord(mark.e0, st) == hipSuccess;
    rc = kvm_migrate(&first.src.pool, &sb, &first.dst.pool, &db, st);
    if (timed && hipEventRecord(mark.e1, st) == hipSuccess) {
      int64_t tokens = 0;
      for (int32_t k : p.k) tokens += k;
      mark.bytes = 2 * tokens * kvm_bytes_per_token(&first.src.pool.layout);
      s->marks.push_back(mark);
    }
    if (rc != KVM_OK) break;
    ++s->launches;
    // from here on the group's copy is in flight: its sources are released after the
    // flush's event, whatever happens to the decode call
    enqueued = g + 1;
    for (const Order* o : groups[g]) flight.released.emplace_back(o->src.fl, o->table);
    // decode of the group's requests over the destination: one call per distinct
    // (q, out) buffer pair, normally one
    std::vector<std::pair<const void*, void*>> bufs;
    for (const Order* o : groups[g])
      if (o->q && o->k > 0 && std::find(bufs.begin(), bufs.end(), std::make_pair(o->q, o->out)) == bufs.end())
        bufs.emplace_back(o->q, o->out);
    for (const auto& b : bufs) {
      std::vector<int32_t> rows(p.k.size(), 0), ks(p.k.size(), 0);   // requests without this decode: k = 0, skipped
      for (size_t i = 0; i < groups[g].size(); ++i) {
        const Order* o = groups[g][i];
        if (o->q == b.first && o->out == b.second && o->k > 0) {
          rows[i] = o->row;
          ks[i] = o->k;
        }
      }
      kvm_batch qb{(int32_t)ks.size(), p.d_off.data(), s->dev + p.d_at, p.d_blk.data(), ks.data(), nullptr};
      rc = kvm_paged_decode_rows(&first.dst.pool, &qb, rows.data(), b.first, b.second, 1, 0.f, s->ws, s->ws_bytes, st);
      if (rc != KVM_OK) break;
      ++s->launches;
    }
  }
  // groups that were not enqueued give their destination blocks back at once; their
  // sources stay allocated
  const std::string why = kvm_last_error();
  for (size_t g = enqueued; g < groups.size(); ++g)
    for (const Order* o : groups[g]) kvm_freelist_free(o->dst.fl, (int32_t)o->ids.size(), o->ids.data());
  int rc_ev = KVM_OK;
  std::shared_ptr<hipEvent_t> ev = s->new_event(&rc_ev);
  if (ev) {
    const hipError_t e = hipEventRecord(*ev, st);
    if (e != hipSuccess) rc_ev = fail(KVM_EHIP, std::string("hipEventRecord: ") + hipGetErrorString(e));
  }
  flight.ev = ev;
  if (!flight.released.empty()) s->pending.push_back(std::move(flight));
  s->region_event[s->region] = ev;
  s->region = (s->region + 1) % s->n_regions;
  if (rc != KVM_OK) return fail(rc, why);
  return rc_ev;
}

}  // namespace

extern "C" {

int64_t kvm_sequencer_table_ints(int32_t max_blocks_per_request, int32_t max_staged, int32_t depth) {
  if (max_blocks_per_request <= 0 || max_staged <= 0 || depth <= 0) return -1;
  return (int64_t)(depth + 2) * 2 * max_blocks_per_request * max_staged;
}

kvm_sequencer* kvm_sequencer_create(int32_t max_blocks_per_request, int32_t max_staged, int32_t depth,
                                    int32_t* tables_host_pinned, int32_t* tables_dev, int64_t table_ints,
                                    void* decode_workspace_dev, int64_t decode_workspace_bytes) {
  clear_error();
  const int64_t need = kvm_sequencer_table_ints(max_blocks_per_request, max_staged, depth);
  if (need < 0 || !tables_host_pinned || !tables_dev || table_ints < need) {
    fail(KVM_EINVAL, "kvm_sequencer_create: bad sizes, NULL table buffers or too few table ints");
    return nullptr;
  }
  kvm_sequencer* s = new kvm_sequencer;
  s->max_blocks = max_blocks_per_request;
  s->max_staged = max_staged;
  s->depth = depth;
  s->pin = tables_host_pinned;
  s->dev = tables_dev;
  s->region_ints = (int64_t)2 * max_blocks_per_request * max_staged;
  s->n_regions = depth + 2;
  s->region_event.resize((size_t)s->n_regions);
  s->ws = decode_workspace_dev;
  s->ws_bytes = decode_workspace_dev ? decode_workspace_bytes : 0;
  return s;
}

int kvm_sequencer_flush(kvm_sequencer* s, void* hip_stream) {
  if (!s) return fail(KVM_EINVAL, "kvm_sequencer_flush: sequencer is NULL");
  clear_error();
  return flush(s, (hipStream_t)hip_stream);
}

int kvm_sequencer_drain(kvm_sequencer* s, void* hip_stream) {
  if (!s) return fail(KVM_EINVAL, "kvm_sequencer_drain: sequencer is NULL");
  clear_error();
  int rc = flush(s, (hipStream_t)hip_stream);
  while (!s->pending.empty()) {
    const int rc2 = retire_oldest(s);
    if (rc == KVM_OK) rc = rc2;
  }
  return rc;
}

int kvm_sequencer_stage(kvm_sequencer* s, const kvm_pool* src, kvm_freelist* src_free, const kvm_pool* dst,
                        kvm_freelist* dst_free, const int32_t* src_table, int32_t n_src_blocks, int32_t k,
                        const void* q_dev, void* out_dev, int32_t row, int32_t* dst_table_out,
                        void* hip_stream) {
  clear_error();
  if (!s || !src || !dst || !src_free || !dst_free || n_src_blocks < 0 || (n_src_blocks > 0 && !src_table))
    return fail(KVM_EINVAL, "kvm_sequencer_stage: NULL argument");
  const int B = src->layout.block_tokens;
  if (B <= 0 || k < 0 || (int64_t)k > (int64_t)n_src_blocks * B || n_src_blocks > s->max_blocks)
    return fail(KVM_EINVAL, "kvm_sequencer_stage: k or table length out of range");
  if (q_dev && (!out_dev || row < 0)) return fail(KVM_EINVAL, "kvm_sequencer_stage: decode needs out_dev and a row >= 0");
  const int32_t nb = (int32_t)ceil_div(k, B);
  if (nb > 0 && !dst_table_out) return fail(KVM_EINVAL, "kvm_sequencer_stage: dst_table_out is NULL");
  for (int32_t j = 0; j < n_src_blocks; ++j)
    if (src_table[j] < 0 || src_table[j] >= src->n_blocks)
      return fail(KVM_EINVAL, "kvm_sequencer_stage: source block id outside the pool");
  const hipStream_t st = (hipStream_t)hip_stream;
  // an order whose source is written by a staged order (the same request moved twice)
  // cannot share a launch with it
  bool hazard = false;
  {
    const std::vector<uint8_t>& m = write_mask(s, *src);
    for (int32_t j = 0; j < n_src_blocks && !hazard; ++j) hazard = m[(size_t)src_table[j]] != 0;
  }
  int rc = KVM_OK;
  if ((int32_t)s->staged.size() >= s->max_staged || hazard) rc = flush(s, st);
  while (rc == KVM_OK && (int32_t)s->pending.size() >= s->depth) rc = retire_oldest(s);
  if (rc != KVM_OK) return rc;
  std::vector<int32_t> ids((size_t)nb);
  rc = kvm_freelist_alloc(dst_free, nb, ids.data());
  if (rc == KVM_ENOMEM) {
    // blocks may be waiting for the release of orders that are still staged or in flight
    rc = kvm_sequencer_drain(s, hip_stream);
    if (rc != KVM_OK) return rc;
    rc = kvm_freelist_alloc(dst_free, nb, ids.data());
  }
  if (rc != KVM_OK) return rc;
  std::vector<uint8_t>& wm = write_mask(s, *dst);
  for (int32_t id : ids) wm[(size_t)id] = 1;
  if (nb > 0) memcpy(dst_table_out, ids.data(), (size_t)nb * 4);
  Order o;
  o.table.assign(src_table, src_table + n_src_blocks);
  o.ids = std::move(ids);
  o.k = k;
  o.src = Side{*src, src_free};
  o.dst = Side{*dst, dst_free};
  o.q = q_dev;
  o.out = out_dev;
  o.row = row;
  s->staged.push_back(std::move(o));
  return KVM_OK;
}

int64_t kvm_sequencer_launches(const kvm_sequencer* s) { return s ? s->launches : -1; }

int kvm_sequencer_timing(kvm_sequencer* s, int enable) {
  if (!s) return fail(KVM_EINVAL, "kvm_sequencer_timing: sequencer is NULL");
  s->timing = enable != 0;
  for (CopyMark& m : s->marks) {
    (void)hipEventDestroy(m.e0);
    (void)hipEventDestroy(m.e1);
  }
  s->marks.clear();
  return KVM_OK;
}

int kvm_sequencer_copy_stats(kvm_sequencer* s, double* ms_out, int64_t* bytes_out, int64_t* launches_out) {
  if (!s || !ms_out || !bytes_out || !launches_out) return fail(KVM_EINVAL, "kvm_sequencer_copy_stats: NULL argument");
  double ms = 0;
  int64_t bytes = 0;
  for (const CopyMark& m : s->marks) {
    hipError_t e = hipEventSynchronize(m.e1);
    float t = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, m.e0, m.e1);
    if (e != hipSuccess) return fail(KVM_EHIP, std::string("copy timing: ") + hipGetErrorString(e));
    ms += t;
    bytes += m.bytes;
  }
  *ms_out = ms;
  *bytes_out = bytes;
  *launches_out = (int64_t)s->marks.size();
  return KVM_OK;
}

void kvm_sequencer_destroy(kvm_sequencer* s) {
  if (!s) return;
  // orders that were never enqueued give their destination blocks back
  for (const Order& o : s->staged) kvm_freelist_free(o.dst.fl, (int32_t)o.ids.size(), o.ids.data());
  s->staged.clear();
  while (!s->pending.empty()) retire_oldest(s);
  for (auto& ev : s->region_event) ev.reset();
  for (CopyMark& m : s->marks) {
    (void)hipEventDestroy(m.e0);
    (void)hipEventDestroy(m.e1);
  }
  for (hipEvent_t ev : s->spare_events) (void)hipEventDestroy(ev);
  delete s;
}

}  // extern "C"
