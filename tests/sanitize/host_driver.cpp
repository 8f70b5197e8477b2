// Seeded random driver over the host-only part of libkvm (free list, divider,
// validation, size helpers, launch-splitting arithmetic), built by
// tests/test_sanitizers.py with -fsanitize=address,undefined.  Any out-of-bounds
// access, leak, overflow or failed check ends the run with a non-zero status.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "kvm.h"
#include "kvm_internal.h"

#define CHECK(x)                                                      \
  do {                                                                \
    if (!(x)) {                                                       \
      fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #x); \
      exit(1);                                                        \
    }                                                                 \
  } while (0)

static void free_list(std::mt19937& rng) {
  for (int trial = 0; trial < 300; ++trial) {
    const int n = 1 + rng() % 300;
    std::vector<uint8_t> occ(n);
    int64_t n_free = 0;
    for (auto& o : occ) n_free += !(o = rng() % 3 == 0);
    kvm_freelist* fl = kvm_freelist_create(n, occ.data());
    CHECK(fl && kvm_freelist_available(fl) == n_free);
    std::vector<std::vector<int32_t>> held;
    for (int it = 0; it < 100; ++it) {
      if (!held.empty() && rng() % 2) {
        auto ids = held.back();
        held.pop_back();
        CHECK(kvm_freelist_free(fl, (int)ids.size(), ids.data()) == KVM_OK);
        n_free += (int64_t)ids.size();
        if (!ids.empty()) {   // a second free is refused, a reserve takes the id back
          CHECK(kvm_freelist_free(fl, 1, ids.data()) == KVM_EINVAL);
          CHECK(kvm_freelist_reserve(fl, 1, ids.data()) == KVM_OK);
          CHECK(kvm_freelist_reserve(fl, 1, ids.data()) == KVM_EINVAL);
          CHECK(kvm_freelist_free(fl, 1, ids.data()) == KVM_OK);
        }
      } else {
        const int want = rng() % (n / 2 + 2);
        std::vector<int32_t> ids(want, -7);
        const int rc = kvm_freelist_alloc(fl, want, ids.data());
        if (rc == KVM_OK) {
          for (int i = 0; i < want; ++i) CHECK(ids[i] >= 0 && ids[i] < n && (i == 0 || ids[i] > ids[i - 1]));
          n_free -= want;
          held.push_back(ids);
        } else {
          CHECK(rc == KVM_ENOMEM && want > n_free);
          for (int32_t id : ids) CHECK(id == -7);   // nothing written
        }
      }
      CHECK(kvm_freelist_available(fl) == n_free);
    }
    int32_t bad[2] = {n, -1};
    CHECK(kvm_freelist_free(fl, 2, bad) == KVM_EINVAL);
    CHECK(kvm_freelist_reserve(fl, 2, bad) == KVM_EINVAL);
    kvm_freelist_destroy(fl);
  }
  CHECK(kvm_freelist_create(0, nullptr) == nullptr);
}

static void divider(std::mt19937& rng) {
  for (int trial = 0; trial < 300; ++trial) {
    const int n = rng() % 50, nl = 1 + rng() % 4, ni = 1 + rng() % 4;
    std::vector<kvm_move> mv(n);
    for (auto& m : mv) {
      m.link = rng() % nl;
      m.dst = rng() % ni;
      m.kv_bytes = (int64_t)(rng() % 1000) << 40;   // products of two such values need 128 bits
      m.tokens = (int64_t)(rng() % 100000) << 20;
    }
    std::vector<int64_t> comm(nl), comp(ni);
    for (auto& c : comm) c = (int64_t)(rng() % 3000) << 40;
    for (auto& c : comp) c = (int64_t)(rng() % 300000) << 20;
    std::vector<int32_t> cls(n, -1);
    for (int pol = 0; pol < 2; ++pol) {
      CHECK(kvm_divide_moves(mv.data(), n, comm.data(), nl, comp.data(), ni, pol, cls.data()) == KVM_OK);
      std::vector<int64_t> link(comm), inst(comp);
      for (int i = 0; i < n; ++i) {   // the division respects both boundaries
        CHECK(cls[i] >= KVM_CLASS_KV && cls[i] <= KVM_CLASS_DEFER);
        if (cls[i] == KVM_CLASS_KV) CHECK((link[mv[i].link] -= mv[i].kv_bytes) >= 0);
        if (cls[i] == KVM_CLASS_TOKENS) CHECK((inst[mv[i].dst] -= mv[i].tokens) >= 0);
      }
    }
    CHECK(kvm_divide_moves(mv.data(), n, comm.data(), nl, comp.data(), ni, 2, cls.data()) == KVM_EINVAL);
  }
}

static void validation(std::mt19937& rng) {
  kvm_layout lay;
  CHECK(kvm_layout_canonical(&lay, 32, 8, 32, 128, 16, KVM_BF16, 65536) == KVM_OK);
  CHECK(kvm_pool_span_bytes(&lay, 65536) == (int64_t)65536 * kvm_block_bytes(&lay));
  kvm_pool pool{(void*)0x7f0000000000, 65536, lay};
  for (int trial = 0; trial < 300; ++trial) {
    const int n_req = rng() % 6;
    std::vector<int32_t> off(n_req + 1, 0), k(n_req), st(n_req);
    for (int r = 0; r < n_req; ++r) off[r + 1] = off[r] + rng() % 5;
    std::vector<int32_t> blk(off[n_req]);
    for (auto& b : blk) b = rng() % 65536;
    int64_t tokens = 0, blocks = 0;
    for (int r = 0; r < n_req; ++r) {
      const int cap = (off[r + 1] - off[r]) * 16;
      k[r] = rng() % (cap + 1);
      st[r] = rng() % (k[r] + 1);
      tokens += k[r] - st[r];
      blocks += k[r] > st[r] ? (k[r] + 15) / 16 - st[r] / 16 : 0;
    }
    kvm_batch b{n_req, off.data(), (const int32_t*)0x7f1000000000, blk.data(), k.data(), st.data()};
    kvm::BatchView v;
    CHECK(kvm::validate_side("t", &pool, &b, false, &v) == KVM_OK);
    CHECK(v.total_tokens == tokens && v.total_blocks == blocks);
    CHECK(kvm_staging_bytes(&lay, &b) == tokens * kvm_bytes_per_token(&lay));
    if (n_req) {   // one bad value at a time is refused
      const int r = rng() % n_req;
      const int32_t keep = k[r];
      k[r] = (off[r + 1] - off[r]) * 16 + 1;
      CHECK(kvm::validate_side("t", &pool, &b, false, &v) == KVM_EINVAL);
      k[r] = keep;
      if (v.nb[r] > v.jb[r]) {
        int32_t& id = blk[off[r] + v.jb[r]];
        const int32_t keep_id = id;
        id = 65536;
        CHECK(kvm::validate_side("t", &pool, &b, false, &v) == KVM_EINVAL);
        id = keep_id;
      }
    }
  }
}

static void launch_splitting() {
  // grid of the staging-order kernels: every workgroup count below 2^31 fits two
  // dimensions whose extents in work-items stay below 2^32
  const int64_t cases[] = {1, 2, 65535, 65536, 65537, (1ll << 24) - 1, 1ll << 24, (1ll << 24) + 1, 26214400,
                           (1ll << 31) - 1};
  for (int64_t n : cases) {
    const kvm::StageGrid g = kvm::stage_grid(n);
    CHECK(g.x >= 1 && g.y >= 1 && g.y <= 65535);
    CHECK((uint64_t)g.x * 256 <= 0xffffffffull);
    CHECK((int64_t)g.x * g.y >= n && (int64_t)g.x * (g.y - 1) < n);
  }
}

int main() {
  std::mt19937 rng(20250106);
  free_list(rng);
  divider(rng);
  validation(rng);
  launch_splitting();
  CHECK(kvm_set_option("copy.order", 3) == KVM_EINVAL && kvm_set_option("reset", 0) == KVM_OK);
  CHECK(kvm_set_option(nullptr, 0) == KVM_EINVAL);
  printf("host driver ok\n");
  return 0;
}
