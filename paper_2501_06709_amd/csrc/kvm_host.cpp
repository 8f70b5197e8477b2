// Host-only part of libkvm: size helpers, argument validation, the free-list
// allocator and diagnostics.  No HIP call is made from this file.
#include <cstdio>
#include <cstring>

#include "kvm_internal.h"

namespace kvm {

static thread_local std::string g_last_error;

int fail(int status, const std::string& msg) {
  g_last_error = msg;
  return status;
}
void clear_error() { g_last_error.clear(); }

Options& options() {
  static Options o;
  return o;
}

bool layout_ok(const kvm_layout* l, std::string* why) {
  auto bad = [&](const char* m) {
    if (why) *why = m;
    return false;
  };
  if (!l) return bad("layout is NULL");
  if (l->n_layers <= 0 || l->n_kv_heads <= 0 || l->n_q_heads <= 0 || l->head_dim <= 0 ||
      l->block_tokens <= 0)
    return bad("layout sizes must be positive");
  if (l->dtype != KVM_F16 && l->dtype != KVM_BF16) return bad("unknown dtype");
  if (l->n_q_heads % l->n_kv_heads) return bad("n_q_heads is not a multiple of n_kv_heads");
  if ((l->head_dim * 2) % 16) return bad("head_dim*2 bytes is not a multiple of 16");
  const int64_t st[5] = {l->stride_layer, l->stride_kv, l->stride_block, l->stride_head,
                         l->stride_slot};
  for (int64_t s : st) {
    if (s <= 0) return bad("strides must be positive");
    if ((s * 2) % 16) return bad("a stride is not a multiple of 16 bytes");
  }
  if (l->stride_slot < l->head_dim) return bad("stride_slot is smaller than head_dim");
  // the kernels keep a lane's offset inside one block in 32 bits (bytes)
  const __int128 inner = (__int128)(l->n_kv_heads - 1) * l->stride_head +
                         (__int128)(l->block_tokens - 1) * l->stride_slot + l->head_dim;
  if (inner > INT32_MAX) return bad("one block spans more than 2^32 bytes of head and slot strides");
  return true;
}

static int64_t span_elems(const kvm_layout* l, int64_t n_blocks) {
  return (int64_t)(l->n_layers - 1) * l->stride_layer + l->stride_kv +
         (n_blocks - 1) * l->stride_block + (int64_t)(l->n_kv_heads - 1) * l->stride_head +
         (int64_t)(l->block_tokens - 1) * l->stride_slot + l->head_dim;
}

int validate_side(const char* what, const kvm_pool* pool, const kvm_batch* batch, bool writing,
                  BatchView* out) {
  std::string why;
  const std::string w(what);
  if (!pool) return fail(KVM_EINVAL, w + ": pool is NULL");
  if (!batch) return fail(KVM_EINVAL, w + ": batch is NULL");
  if (!layout_ok(&pool->layout, &why)) return fail(KVM_EINVAL, w + ": " + why);
  if (!pool->base) return fail(KVM_EINVAL, w + ": pool base is NULL");
  if ((uintptr_t)pool->base % 16) return fail(KVM_EINVAL, w + ": pool base is not 16-byte aligned");
  if (pool->n_blocks <= 0 || pool->n_blocks > INT32_MAX)
    return fail(KVM_EINVAL, w + ": n_blocks out of range");
  if (batch->n_req < 0) return fail(KVM_EINVAL, w + ": n_req is negative");
  out->n_req = batch->n_req;
  out->bt_off.assign(batch->n_req, 0);
  out->k.assign(batch->n_req, 0);
  out->start.assign(batch->n_req, 0);
  out->jb.assign(batch->n_req, 0);
  out->nb.assign(batch->n_req, 0);
  out->total_tokens = out->total_blocks = 0;
  if (batch->n_req == 0) return KVM_OK;
  if (!batch->bt_offsets || !batch->k) return fail(KVM_EINVAL, w + ": bt_offsets or k is NULL");
  if (batch->bt_offsets[0] != 0) return fail(KVM_EINVAL, w + ": bt_offsets[0] must be 0");
  const int B = pool->layout.block_tokens;
  for (int r = 0; r < batch->n_req; ++r) {
    const int64_t lo = batch->bt_offsets[r], hi = batch->bt_offsets[r + 1];
    if (hi < lo) return fail(KVM_EINVAL, w + ": bt_offsets is not non-decreasing");
    const int64_t k = batch->k[r];
    char buf[96];
    if (k < 0 || k > (hi - lo) * B) {
      snprintf(buf, sizeof buf, ": k[%d]=%lld outside [0, %lld]", r, (long long)k,
               (long long)((hi - lo) * B));
      return fail(KVM_EINVAL, w + buf);
    }
    const int64_t st = batch->start ? batch->start[r] : 0;
    if (st < 0 || st > k) {
      snprintf(buf, sizeof buf, ": start[%d]=%lld outside [0, k=%lld]", r, (long long)st, (long long)k);
      return fail(KVM_EINVAL, w + buf);
    }
    out->bt_off[r] = (int32_t)lo;
    out->k[r] = (int32_t)k;
    out->start[r] = (int32_t)st;
    out->jb[r] = (int32_t)(st / B);
    out->nb[r] = k > st ? (int32_t)ceil_div(k, B) : out->jb[r];
    out->total_tokens += k - st;
    out->total_blocks += out->nb[r] - out->jb[r];
  }
  if (out->total_blocks > 0 && !batch->bt_blocks_dev)
    return fail(KVM_EINVAL, w + ": bt_blocks_dev is NULL");
  if (batch->bt_blocks_host) {
    std::vector<uint64_t> seen;
    if (writing) seen.assign((size_t)ceil_div(pool->n_blocks, 64), 0);
    for (int r = 0; r < batch->n_req; ++r)
      for (int j = out->jb[r]; j < out->nb[r]; ++j) {
        const int64_t id = batch->bt_blocks_host[out->bt_off[r] + j];
        char buf[96];
        if (id < 0 || id >= pool->n_blocks) {
          snprintf(buf, sizeof buf, ": request %d entry %d: block id %lld outside [0, %lld)", r, j,
                   (long long)id, (long long)pool->n_blocks);
          return fail(KVM_EINVAL, w + buf);
        }
        if (writing) {
          uint64_t& word = seen[(size_t)id >> 6];
          const uint64_t bit = 1ull << (id & 63);
          if (word & bit) {
            snprintf(buf, sizeof buf, ": block id %lld is written twice (request %d entry %d)",
                     (long long)id, r, j);
            return fail(KVM_EINVAL, w + buf);
          }
          word |= bit;
        }
      }
  }
  return KVM_OK;
}

}  // namespace kvm

using namespace kvm;

extern "C" {

int64_t kvm_bytes_per_token(const kvm_layout* l) {
  if (!layout_ok(l, nullptr)) return -1;
  return (int64_t)l->n_layers * 2 * l->n_kv_heads * l->head_dim * 2;
}

int64_t kvm_block_bytes(const kvm_layout* l) {
  const int64_t bpt = kvm_bytes_per_token(l);
  return bpt < 0 ? -1 : bpt * l->block_tokens;
}

int64_t kvm_staging_bytes(const kvm_layout* l, const kvm_batch* b) {
  const int64_t bpt = kvm_bytes_per_token(l);
  if (bpt < 0 || !b || b->n_req < 0 || (b->n_req > 0 && !b->k)) return -1;
  int64_t tokens = 0;
  for (int r = 0; r < b->n_req; ++r) {
    const int64_t st = b->start ? b->start[r] : 0;
    if (b->k[r] < 0 || st < 0 || st > b->k[r]) return -1;
    tokens += b->k[r] - st;
  }
  return tokens * bpt;
}

int kvm_layout_canonical(kvm_layout* out, int32_t n_layers, int32_t n_kv_heads, int32_t n_q_heads,
                         int32_t head_dim, int32_t block_tokens, int32_t dtype, int64_t n_blocks) {
  if (!out) return fail(KVM_EINVAL, "kvm_layout_canonical: out is NULL");
  if (n_blocks <= 0) return fail(KVM_EINVAL, "kvm_layout_canonical: n_blocks must be positive");
  kvm_layout l;
  l.n_layers = n_layers;
  l.n_kv_heads = n_kv_heads;
  l.n_q_heads = n_q_heads;
  l.head_dim = head_dim;
  l.block_tokens = block_tokens;
  l.dtype = dtype;
  l.stride_slot = head_dim;
  l.stride_head = (int64_t)block_tokens * l.stride_slot;
  l.stride_block = (int64_t)n_kv_heads * l.stride_head;
  l.stride_kv = n_blocks * l.stride_block;
  l.stride_layer = 2 * l.stride_kv;
  std::string why;
  if (!layout_ok(&l, &why)) return fail(KVM_EINVAL, "kvm_layout_canonical: " + why);
  *out = l;
  return KVM_OK;
}

int64_t kvm_pool_span_bytes(const kvm_layout* l, int64_t n_blocks) {
  if (!layout_ok(l, nullptr) || n_blocks <= 0) return -1;
  return span_elems(l, n_blocks) * 2;
}

// ---- free list: one bit per block, lowest id first --------------------------
struct kvm_freelist {
  int64_t n_blocks;
  int64_t n_free;
  int64_t hint;                 // no free bit below word index `hint`
  std::vector<uint64_t> bits;   // 1 = free
};

kvm_freelist* kvm_freelist_create(int64_t n_blocks, const uint8_t* occupied) {
  if (n_blocks <= 0 || n_blocks > INT32_MAX) return nullptr;
  kvm_freelist* fl = new kvm_freelist;
  fl->n_blocks = n_blocks;
  fl->n_free = 0;
  fl->hint = 0;
  fl->bits.assign((size_t)ceil_div(n_blocks, 64), 0);
  for (int64_t b = 0; b < n_blocks; ++b)
    if (!occupied || !occupied[b]) {
      fl->bits[(size_t)b >> 6] |= 1ull << (b & 63);
      ++fl->n_free;
    }
  return fl;
}

void kvm_freelist_destroy(kvm_freelist* fl) { delete fl; }

int64_t kvm_freelist_available(const kvm_freelist* fl) { return fl ? fl->n_free : -1; }

int kvm_freelist_alloc(kvm_freelist* fl, int32_t n, int32_t* out_ids) {
  if (!fl || n < 0 || (n > 0 && !out_ids)) return fail(KVM_EINVAL, "kvm_freelist_alloc: bad argument");
  if (n > fl->n_free) return fail(KVM_ENOMEM, "kvm_freelist_alloc: not enough free blocks");
  int32_t got = 0;
  size_t w = (size_t)fl->hint;
  while (got < n) {
    uint64_t word = fl->bits[w];
    while (word && got < n) {
      const int bit = __builtin_ctzll(word);
      out_ids[got++] = (int32_t)(w * 64 + bit);
      word &= word - 1;
    }
    fl->bits[w] = word;
    if (got < n) ++w;
  }
  fl->hint = (int64_t)w;
  fl->n_free -= n;
  return KVM_OK;
}

int kvm_freelist_free(kvm_freelist* fl, int32_t n, const int32_t* ids) {
  if (!fl || n < 0 || (n > 0 && !ids)) return fail(KVM_EINVAL, "kvm_freelist_free: bad argument");
  // first pass: validate without changing anything (set bits as a duplicate
  // detector, roll them back on failure)
  int32_t done = 0;
  bool ok = true;
  for (; done < n; ++done) {
    const int64_t id = ids[done];
    if (id < 0 || id >= fl->n_blocks) { ok = false; break; }
    uint64_t& word = fl->bits[(size_t)id >> 6];
    const uint64_t bit = 1ull << (id & 63);
    if (word & bit) { ok = false; break; }  // already free, or repeated in ids
    word |= bit;
  }
  if (!ok) {
    for (int32_t i = 0; i < done; ++i) fl->bits[(size_t)ids[i] >> 6] &= ~(1ull << (ids[i] & 63));
    return fail(KVM_EINVAL, "kvm_freelist_free: id out of range, already free, or repeated");
  }
  for (int32_t i = 0; i < n; ++i)
    if ((ids[i] >> 6) < fl->hint) fl->hint = ids[i] >> 6;
  fl->n_free += n;
  return KVM_OK;
}

int kvm_freelist_reserve(kvm_freelist* fl, int32_t n, const int32_t* ids) {
  if (!fl || n < 0 || (n > 0 && !ids)) return fail(KVM_EINVAL, "kvm_freelist_reserve: bad argument");
  int32_t done = 0;
  bool ok = true;
  for (; done < n; ++done) {
    const int64_t id = ids[done];
    if (id < 0 || id >= fl->n_blocks) { ok = false; break; }
    uint64_t& word = fl->bits[(size_t)id >> 6];
    const uint64_t bit = 1ull << (id & 63);
    if (!(word & bit)) { ok = false; break; }  // in use, or repeated in ids
    word &= ~bit;
  }
  if (!ok) {
    for (int32_t i = 0; i < done; ++i) fl->bits[(size_t)ids[i] >> 6] |= 1ull << (ids[i] & 63);
    return fail(KVM_EINVAL, "kvm_freelist_reserve: id out of range, not free, or repeated");
  }
  fl->n_free -= n;
  return KVM_OK;
}

int kvm_divide_moves(const kvm_move* moves, int32_t n_moves, const int64_t* comm_boundary,
                     int32_t n_links, const int64_t* comp_boundary, int32_t n_instances,
                     int32_t policy, int32_t* out_class) {
  if (n_moves < 0 || n_links < 0 || n_instances < 0)
    return fail(KVM_EINVAL, "kvm_divide_moves: negative count");
  if ((n_moves > 0 && (!moves || !out_class)) || (n_links > 0 && !comm_boundary) ||
      (n_instances > 0 && !comp_boundary))
    return fail(KVM_EINVAL, "kvm_divide_moves: NULL pointer");
  if (policy != KVM_FIRST_FIT && policy != KVM_BEST_FIT)
    return fail(KVM_EINVAL, "kvm_divide_moves: unknown policy");
  for (int32_t l = 0; l < n_links; ++l)
    if (comm_boundary[l] < 0) return fail(KVM_EINVAL, "kvm_divide_moves: negative boundary");
  for (int32_t j = 0; j < n_instances; ++j)
    if (comp_boundary[j] < 0) return fail(KVM_EINVAL, "kvm_divide_moves: negative boundary");
  for (int32_t i = 0; i < n_moves; ++i) {
    const kvm_move& mv = moves[i];
    if (mv.link < 0 || mv.link >= n_links || mv.dst < 0 || mv.dst >= n_instances)
      return fail(KVM_EINVAL, "kvm_divide_moves: link or dst out of range");
    if (mv.kv_bytes < 0 || mv.tokens < 0) return fail(KVM_EINVAL, "kvm_divide_moves: negative size");
  }
  std::vector<int64_t> link_left(comm_boundary, comm_boundary + n_links);
  std::vector<int64_t> inst_left(comp_boundary, comp_boundary + n_instances);
  for (int32_t i = 0; i < n_moves; ++i) {
    const kvm_move& mv = moves[i];
    const bool fits_kv = mv.kv_bytes <= link_left[mv.link];
    const bool fits_tok = mv.tokens <= inst_left[mv.dst];
    int cls = KVM_CLASS_DEFER;
    if (fits_kv && fits_tok && policy == KVM_BEST_FIT) {
      // compare free fractions (left - size) / boundary without division:
      // a/b <= c/d  <=>  a*d <= c*b for positive b, d; an empty bin (boundary 0,
      // size 0) counts as fraction 0
      const __int128 a = link_left[mv.link] - mv.kv_bytes, b = comm_boundary[mv.link];
      const __int128 c = inst_left[mv.dst] - mv.tokens, d = comp_boundary[mv.dst];
      const __int128 lhs = b == 0 ? 0 : a * (d == 0 ? 1 : d);
      const __int128 rhs = d == 0 ? 0 : c * (b == 0 ? 1 : b);
      cls = lhs <= rhs ? KVM_CLASS_KV : KVM_CLASS_TOKENS;
    } else if (fits_kv) {
      cls = KVM_CLASS_KV;
    } else if (fits_tok) {
      cls = KVM_CLASS_TOKENS;
    }
    if (cls == KVM_CLASS_KV) link_left[mv.link] -= mv.kv_bytes;
    if (cls == KVM_CLASS_TOKENS) inst_left[mv.dst] -= mv.tokens;
    out_class[i] = cls;
  }
  return KVM_OK;
}

const char* kvm_strerror(int status) {
  switch (status) {
    case KVM_OK: return "ok";
    case KVM_EINVAL: return "invalid argument";
    case KVM_ENOMEM: return "free list exhausted";
    case KVM_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* kvm_last_error(void) { return g_last_error.c_str(); }

int kvm_set_option(const char* name, int64_t value) {
  if (!name) return fail(KVM_EINVAL, "kvm_set_option: name is NULL");
  Options& o = options();
  if (!strcmp(name, "reset")) {
    o = Options();
  } else if (!strcmp(name, "copy.nontemporal")) {
    if (value != 0 && value != 1) return fail(KVM_EINVAL, "copy.nontemporal must be 0 or 1");
    o.copy_nontemporal = (int)value;
  } else if (!strcmp(name, "copy.order")) {
    if (value < -1 || value > 1) return fail(KVM_EINVAL, "copy.order must be -1, 0 or 1");
    o.copy_order = (int)value;
  } else if (!strcmp(name, "copy.stage_linear")) {
    if (value < -1 || value > 3) return fail(KVM_EINVAL, "copy.stage_linear must be in [-1,3]");
    o.stage_linear = (int)value;
  } else if (!strcmp(name, "decode.cap_waves")) {
    if (value < -1 || value > 1) return fail(KVM_EINVAL, "decode.cap_waves must be -1, 0 or 1");
    o.decode_cap_waves = (int)value;
  } else if (!strcmp(name, "decode.mfma")) {
    if (value < -1 || value > 1) return fail(KVM_EINVAL, "decode.mfma must be -1, 0 or 1");
    o.decode_mfma = (int)value;
  } else if (!strcmp(name, "decode.spread")) {
    if (value < -1 || value > 6) return fail(KVM_EINVAL, "decode.spread must be in [-1,6]");
    o.decode_spread = (int)value;
  } else if (!strcmp(name, "decode.split_target")) {
    if (value < 1 || value > (1 << 20)) return fail(KVM_EINVAL, "decode.split_target must be in [1, 2^20]");
    o.decode_split_target = (int)value;
  } else if (!strcmp(name, "decode.max_splits")) {
    if (value < 1 || value > 64) return fail(KVM_EINVAL, "decode.max_splits must be in [1,64]");
    o.decode_max_splits = (int)value;
  } else if (!strcmp(name, "decode.force_splits")) {
    if (value < 0 || value > 64) return fail(KVM_EINVAL, "decode.force_splits must be in [0,64]");
    o.decode_force_splits = (int)value;
  } else {
    return fail(KVM_EINVAL, std::string("kvm_set_option: unknown option ") + name);
  }
  return KVM_OK;
}

}  // extern "C"
