// Pack / unpack / fused migrate kernels for gfx950 and their C entry points.
//
// The data path of the KV-cache class of request migration (arXiv 2501.06709,
// Sec. "Adaptive Request Migration", "Hybrid Migration"): tokens [0,k) of every
// layer, K and V, are read through the source block table and written through
// the destination block table (or to / from a contiguous staging buffer).
//
// All three operations are one kernel, `copy_kernel<MODE, NT>` (packing long
// requests has a second one, `stage_kernel`, further down):
//  - a work item is (block entry of a request, plane = layer*2+kv, chunk); one
//    256-lane workgroup moves up to 256 16-byte vectors of it: 4 KiB per workgroup,
//    one vector per lane, plane outermost in the grid (two, four and eight vectors
//    per lane all measured slower: 6340 / 5920 / 5710 GB/s fused at one / two / four);
//  - loads and stores carry the streaming cache-policy bits (sc0 sc1 nt);
//  - block ids and request descriptors are wave-uniform: they are read with
//    scalar loads from the kernel-argument segment and the block table, which
//    broadcasts them to all lanes without a vector load or LDS;
//  - a full block of a dense layout (head-major or token-major rows) is one
//    contiguous run per plane (heads*block_tokens*head_dim*2 bytes) and is moved
//    with no index math beyond base + lane*16; partial last blocks of head-major
//    blocks and other layouts go through a (head, slot, vector) decomposition of
//    the lane's vector index.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>

#include "kvm_internal.h"

namespace kvm {

enum CopyMode { kMigrate = 0, kPack = 1, kUnpack = 2 };

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct PoolSide {
  char* base;
  const int32_t* bt;      // device block table (CSR payload)
  int64_t stride_layer;   // bytes
  int64_t stride_kv;
  int64_t stride_block;
  uint32_t stride_head;   // bytes, within a block
  uint32_t stride_slot;
  uint32_t dense;         // a block is one contiguous run per plane: 1 head-major, 2 token-major rows; 0 neither
};

// Division of x < 2^31 by a fixed divisor d >= 1 through one widening multiply
// (Granlund & Montgomery, "Division by invariant integers using multiplication",
// the round-up multiplier): with l = ceil(log2 d) and m = ceil(2^(31+l) / d) < 2^32,
// floor(x / d) = (x * m) >> (31 + l) for every x < 2^31.  Branch-free.
struct FastDiv {
  uint32_t d, m, sh;
};
static FastDiv make_fastdiv(uint32_t d) {
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  FastDiv f;
  f.d = d;
  f.m = (uint32_t)(((1ull << (31 + l)) + d - 1) / d);
  f.sh = 31 + l;
  return f;
}
__device__ __forceinline__ uint32_t fastdiv(uint32_t x, const FastDiv& f) {
  return (uint32_t)(((uint64_t)x * f.m) >> f.sh);
}

struct CopyReq {
  int32_t src_bt;      // first table entry of the request on the source side
  int32_t dst_bt;      // ... on the destination side
  int32_t k;           // tokens [start, k) are moved
  int32_t start;
  int32_t first_item;  // index of the request's first moved block among the launch's items
  int32_t jb;          // first moved block of the request: start / B
  int64_t stage_vec;   // staging offset of the request in 16-byte vectors
};

struct CopyArgs {
  PoolSide src;        // pool side read by migrate / pack
  PoolSide dst;        // pool side written by migrate / unpack
  char* stage;         // staging buffer (pack writes, unpack reads)
  int32_t n_req;
  int32_t n_items;     // blocks holding tokens [0,k) over the launch's requests
  int32_t n_planes;    // 2 * layers
  int32_t n_chunks;    // workgroup passes per (item, plane)
  int32_t H, B;
  uint32_t DV;         // 16-byte vectors per token row (head_dim*2/16)
  FastDiv dvdiv;       // division by DV
  int32_t order;       // 0: planes of a block are consecutive workgroups; 1: plane outermost
  // first_item of every request again, densely packed (unused entries INT32_MAX),
  // for the binary search that finds the owner of an item
  int32_t first_item[kMaxReqPerLaunch];
  CopyReq req[kMaxReqPerLaunch];
};

// Streaming accesses.  The hinted form carries the cache-policy bits "sc0 sc1 nt"
// (system scope, non-temporal): against "nt" alone it measured +1 % on the fused
// move and +5 % on pack, against plain accesses +8 % and more.  The compiler's
// builtins only reach "nt", so the hinted accesses are written as instructions:
// the load and the wait for it form ONE asm statement, so the register cannot be
// read before its data has arrived.  The hint is a template parameter on purpose:
// written as a run-time choice between a hinted and a plain access of one address,
// the two are merged by the optimiser and the hint is lost.
template <bool NT>
__device__ __forceinline__ v4u load16(const char* p) {
  v4u v;
  if constexpr (NT)
    asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
  else
    v = *reinterpret_cast<const v4u*>(p);
  return v;
}
template <bool NT>
__device__ __forceinline__ void store16(char* p, v4u v) {
  if constexpr (NT)
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(p), "v"(v) : "memory");
  else
    *reinterpret_cast<v4u*>(p) = v;
}

template <int MODE, bool NT>
__global__ __launch_bounds__(256) void copy_kernel(const CopyArgs a) {
  // ---- decode the work item (all wave-uniform, no division) ----
  // order 1 (shipped): grid = (chunks, block entries, planes): consecutive
  // workgroups walk the chunks of one (block, plane) run, then the batch's other
  // blocks in the same plane, and only then move to the next plane.
  // order 0: grid = (chunks, planes, block entries): the planes of one block are
  // consecutive, kept for comparison.
  const uint32_t chunk = blockIdx.x;
  const uint32_t plane = a.order ? blockIdx.z : blockIdx.y;
  const uint32_t item = a.order ? blockIdx.y : blockIdx.z;
  // request that owns the item: largest r with first_item[r] <= item
  int r = 0;
#pragma unroll
  for (int s = kMaxReqPerLaunch / 2; s > 0; s >>= 1) {
    const int t = r + s;
    if (a.first_item[t] <= (int32_t)item) r = t;
  }
  const CopyReq rq = a.req[r];
  const int32_t j = (int32_t)item - rq.first_item + rq.jb;  // logical block of the request
  // slots [s0, s1) of this block hold tokens of [start, k)
  const int32_t lo = rq.start - j * a.B, hi = rq.k - j * a.B;
  const uint32_t s0 = lo > 0 ? (uint32_t)lo : 0u;
  const uint32_t ns = (hi < a.B ? (uint32_t)hi : (uint32_t)a.B) - s0;  // slots to move
  const uint32_t layer = plane >> 1, kv = plane & 1;

  const char* sbase = nullptr;
  char* dbase = nullptr;
  // Fused fast path: the moved slots are one contiguous run on both sides and in
  // the same order.  Head-major blocks ([head][slot][dim]): full blocks only.
  // Token-major blocks ([slot][head][dim]): any slot range, its rows are adjacent.
  bool dense = MODE == kMigrate && a.src.dense != 0 && a.src.dense == a.dst.dense &&
               (a.src.dense == 2 || ns == (uint32_t)a.B);
  if (MODE != kUnpack) {
    const int64_t blk = a.src.bt[rq.src_bt + j];
    sbase = a.src.base + layer * a.src.stride_layer + kv * a.src.stride_kv + blk * a.src.stride_block +
            (uint64_t)s0 * a.src.stride_slot;
  }
  if (MODE != kPack) {
    const int64_t blk = a.dst.bt[rq.dst_bt + j];
    dbase = a.dst.base + layer * a.dst.stride_layer + kv * a.dst.stride_kv + blk * a.dst.stride_block +
            (uint64_t)s0 * a.dst.stride_slot;
  }
  const uint32_t per_head = ns * a.DV;          // vectors per head in this item
  const uint32_t n_vec = per_head * (uint32_t)a.H;
  const uint32_t v = chunk * 256u + threadIdx.x;   // this lane's vector of the item
  if (chunk * 256u >= n_vec) return;

  // Lanes past the end of the item load its last vector again (always in
  // bounds) and skip the store, so the load stays unconditional straight-line code.
  const uint32_t vc = min(v, n_vec - 1);
  if (MODE == kMigrate && dense) {
    // one contiguous run on both sides
    const v4u val = load16<NT>(sbase + (uint64_t)vc * 16u);
    if (v < n_vec) store16<NT>(dbase + (uint64_t)v * 16u, val);
    return;
  }

  // general path: vector index -> (head, slot, vector-in-row)
  char* stage_plane = nullptr;  // staging address of (request, plane, head 0, token j*B + s0)
  uint64_t stage_head = 0;      // bytes between heads in staging
  if (MODE != kMigrate) {
    const uint64_t n_tok = (uint64_t)(rq.k - rq.start);             // tokens of the request in staging
    const uint64_t tok0 = (uint64_t)(j * a.B + (int32_t)s0 - rq.start);  // first of them in this item
    stage_head = n_tok * a.DV * 16u;
    stage_plane = a.stage + ((uint64_t)rq.stage_vec + (uint64_t)plane * a.H * n_tok * a.DV +
                             tok0 * a.DV) * 16u;
  }
  const uint32_t h = vc / per_head;
  const uint32_t w = vc - h * per_head;  // slot*DV + dv
  const uint32_t slot = fastdiv(w, a.dvdiv);
  const uint32_t dv = w - slot * a.DV;
  const uint32_t soff = h * a.src.stride_head + slot * a.src.stride_slot + dv * 16u;
  const uint32_t doff = h * a.dst.stride_head + slot * a.dst.stride_slot + dv * 16u;
  const uint64_t shead = (uint64_t)h * stage_head + (uint64_t)w * 16u;
  const v4u val = load16<NT>(MODE == kUnpack ? stage_plane + shead : sbase + soff);
  if (v < n_vec) store16<NT>(MODE == kPack ? stage_plane + shead : dbase + doff, val);
}

static PoolSide make_side(const kvm_pool* p, const kvm_batch* b) {
  PoolSide s;
  const kvm_layout& l = p->layout;
  s.base = (char*)p->base;
  s.bt = b->bt_blocks_dev;
  s.stride_layer = l.stride_layer * 2;
  s.stride_kv = l.stride_kv * 2;
  s.stride_block = l.stride_block * 2;
  s.stride_head = (uint32_t)(l.stride_head * 2);
  s.stride_slot = (uint32_t)(l.stride_slot * 2);
  s.dense = 0;
  if (l.stride_slot == l.head_dim && l.stride_head == (int64_t)l.block_tokens * l.head_dim) s.dense = 1;
  else if (l.stride_head == l.head_dim && l.stride_slot == (int64_t)l.n_kv_heads * l.head_dim) s.dense = 2;
  return s;
}

template <int MODE>
static hipError_t launch(const CopyArgs& a, hipStream_t stream) {
  const dim3 grid = a.order ? dim3(a.n_chunks, a.n_items, a.n_planes) : dim3(a.n_chunks, a.n_planes, a.n_items);
  if (options().copy_nontemporal)
    hipLaunchKernelGGL((copy_kernel<MODE, true>), grid, dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL((copy_kernel<MODE, false>), grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

// Splits the batch into launches of at most kMaxReqPerLaunch requests and
// enqueues them.  `sv` / `dv` are the validated views of the two sides (for
// pack only `sv`, for unpack only `dv` is meaningful; the other aliases it).
template <int MODE>
static int run_copy(const kvm_pool* src, const kvm_batch* sb, const BatchView& sv,
                    const kvm_pool* dst, const kvm_batch* db, const BatchView& dv, char* stage,
                    hipStream_t stream) {
  const kvm_layout& l = (MODE == kUnpack ? dst : src)->layout;
  const BatchView& view = MODE == kUnpack ? dv : sv;
  CopyArgs a;
  memset(&a, 0, sizeof a);
  if (MODE != kUnpack) a.src = make_side(src, sb);
  if (MODE != kPack) a.dst = make_side(dst, db);
  if (MODE == kPack) a.dst = a.src;    // strides of the unused side are still
  if (MODE == kUnpack) a.src = a.dst;  // read by the index math: keep them sane
  a.stage = stage;
  a.n_planes = 2 * l.n_layers;
  a.H = l.n_kv_heads;
  a.B = l.block_tokens;
  a.DV = (uint32_t)(l.head_dim * 2 / 16);
  a.dvdiv = make_fastdiv(a.DV);
  // Workgroups walk the dimension with the smaller stride first: with layer-major
  // pools (a plane spans all blocks) the plane is outermost, with block-major pools
  // (a block's planes are adjacent) the planes of a block are consecutive.  Pack
  // always takes the plane outermost: that is the order of its staging buffer.
  a.order = options().copy_order >= 0 ? options().copy_order
                                      : (MODE == kPack || l.stride_kv >= l.stride_block ? 1 : 0);
  const int64_t vec_per_item = (int64_t)l.n_kv_heads * l.block_tokens * a.DV;
  a.n_chunks = (int32_t)ceil_div(vec_per_item, 256);
  const int64_t bpt_vec = (int64_t)l.n_layers * 2 * l.n_kv_heads * a.DV;  // vectors per token

  // limits are checked for the whole batch before the first launch: an error
  // must mean that no device byte was written
  for (int q = 0; q < view.n_req; ++q)
    if (view.nb[q] - view.jb[q] > 65535)
      return fail(KVM_EINVAL, "a single request moves more than 65535 blocks in one call");

  int64_t stage_vec = 0;
  int r = 0;
  while (r < view.n_req) {
    a.n_req = 0;
    a.n_items = 0;
    for (int i = 0; i < kMaxReqPerLaunch; ++i) a.first_item[i] = INT32_MAX;
    const int64_t max_items = 65535;  // grid dimension limit for y and z
    while (r < view.n_req && a.n_req < kMaxReqPerLaunch) {
      const int32_t items_r = view.nb[r] - view.jb[r];
      if ((int64_t)a.n_items + items_r > max_items) break;
      CopyReq& q = a.req[a.n_req++];
      q.src_bt = sv.bt_off[r];
      q.dst_bt = dv.bt_off[r];
      q.k = view.k[r];
      q.start = view.start[r];
      q.first_item = a.n_items;
      q.jb = view.jb[r];
      q.stage_vec = stage_vec;
      a.first_item[a.n_req - 1] = a.n_items;
      a.n_items += items_r;
      stage_vec += (int64_t)(view.k[r] - view.start[r]) * bpt_vec;
      ++r;
    }
    if (a.n_items == 0) continue;  // only k = 0 requests in this group
    const hipError_t e = launch<MODE>(a, stream);
    if (e != hipSuccess) return fail(KVM_EHIP, hipGetErrorString(e));
  }
  return KVM_OK;
}

// ---- staging-linear pack / unpack -------------------------------------------
// A second mapping for the staged path: the work is cut along the staging buffer
// instead of along pool blocks.  One workgroup moves one piece of 256 consecutive
// 16-byte vectors of one (request, plane, head) run of the staging buffer; the
// pool side is then a gather (pack) or scatter (unpack) of token rows.
//
// At 4 KiB per workgroup a wave moves 1 KiB, so a long scalar preamble shows (a
// 370-instruction straight-line one ran at two thirds of the rate of the
// 100-instruction one below):
//  - consecutive workgroups walk the staging buffer linearly (request, plane,
//    head, chunk): that order measured 10 % faster than one that walks the chunks
//    of all requests for one (plane, head) before the next head;
//  - the owning request is found by a binary search over a dense first_wg array
//    in the kernel-argument segment: six dependent scalar loads that hit the
//    scalar cache (a one-load search through a vector load and a ballot measured
//    2 % slower: under streaming load the vector memory path has the longer
//    queue); the two divisions that split the workgroup index into (plane, head,
//    chunk) are branch-free multiplications;
//  - FAST (the host checks the conditions): every 256-vector piece lies inside one
//    block and is contiguous there, so the block id is one scalar load per piece
//    and a lane's address is base + lane*16 on both sides.
struct StageReq {
  int32_t bt;            // first table entry of the request
  int32_t start;         // first token moved
  uint32_t n_vec;        // vectors of one (plane, head) run: (k - start) * DV
  uint32_t first_wg;     // first workgroup of the request in this launch
  int64_t stage_vec;     // staging offset of the request in 16-byte vectors
  FastDiv chunks;        // workgroups per (plane, head) run
};

struct StageArgs {
  PoolSide pool;
  char* stage;
  int32_t H, B;
  uint32_t DV;
  uint32_t piece_tokens;  // tokens per 256-vector piece (FAST only)
  uint32_t n_wg;          // workgroups of this launch that have work
  FastDiv dvdiv, bdiv, heads;  // division by DV, B, H
  uint32_t first_wg[kMaxReqPerLaunch];  // densely packed, unused entries UINT32_MAX
  StageReq req[kMaxReqPerLaunch];
};

template <bool PACK, bool NT, bool FAST>
__global__ __launch_bounds__(256) void stage_kernel(const StageArgs a) {
  // the launch's workgroups are numbered row by row over a 2-D grid (one grid
  // dimension cannot hold them: a dimension is limited to 2^32 - 1 work-items);
  // the last row may be ragged
  const uint32_t wg = blockIdx.y * gridDim.x + blockIdx.x;
  if (wg >= a.n_wg) return;
  // owning request: largest r with first_wg[r] <= wg (unused entries never compare true)
  int r = 0;
#pragma unroll
  for (int s = kMaxReqPerLaunch / 2; s > 0; s >>= 1) {
    const int t = r + s;
    if (a.first_wg[t] <= wg) r = t;
  }
  const StageReq rq = a.req[r];
  const uint32_t local = wg - rq.first_wg;
  const uint32_t run = fastdiv(local, rq.chunks);  // (plane, head) run of the request
  const uint32_t chunk = local - run * rq.chunks.d;
  const uint32_t plane = fastdiv(run, a.heads);
  const uint32_t h = run - plane * a.heads.d;
  const uint32_t n_vec = rq.n_vec;
  const uint32_t x = chunk * 256u + threadIdx.x;   // this lane's vector of the run
  const uint32_t xc = min(x, n_vec - 1);            // lanes past the end repeat the last vector and store nothing
  char* pbase = a.pool.base + (uint64_t)(plane >> 1) * a.pool.stride_layer +
                (uint64_t)(plane & 1) * a.pool.stride_kv + (uint64_t)h * a.pool.stride_head;
  char* sbase = a.stage + ((uint64_t)rq.stage_vec + (uint64_t)(plane * (uint32_t)a.H + h) * n_vec) * 16u;

  if constexpr (FAST) {
    // the piece lies inside one block and is contiguous there: one scalar id load
    const uint32_t t = (uint32_t)rq.start + chunk * a.piece_tokens;
    const uint32_t j = fastdiv(t, a.bdiv);
    const int32_t blk = a.pool.bt[rq.bt + (int32_t)j];
    const uint32_t slot = t - j * (uint32_t)a.B;
    char* pp = pbase + (uint64_t)blk * a.pool.stride_block + slot * a.pool.stride_slot;
    const uint32_t off = (xc - chunk * 256u) * 16u;
    const v4u val = load16<NT>(PACK ? pp + off : sbase + (uint64_t)xc * 16u);
    if (x < n_vec) store16<NT>(PACK ? sbase + (uint64_t)x * 16u : pp + off, val);
    return;
  }

  const uint32_t tok = fastdiv(xc, a.dvdiv);
  const uint32_t dv = xc - tok * a.DV;
  const uint32_t t = (uint32_t)rq.start + tok;
  const uint32_t j = fastdiv(t, a.bdiv);
  const uint32_t slot = t - j * (uint32_t)a.B;
  const int32_t blk = a.pool.bt[rq.bt + (int32_t)j];
  char* pp = pbase + (uint64_t)blk * a.pool.stride_block + slot * a.pool.stride_slot + dv * 16u;
  const v4u val = load16<NT>(PACK ? pp : sbase + (uint64_t)xc * 16u);
  if (x < n_vec) store16<NT>(PACK ? sbase + (uint64_t)x * 16u : pp, val);
}

template <bool PACK>
static int run_stage(const kvm_pool* pool, const kvm_batch* b, const BatchView& view, char* stage,
                     hipStream_t stream) {
  const kvm_layout& l = pool->layout;
  const Options& o = options();
  StageArgs a;
  memset(&a, 0, sizeof a);
  a.pool = make_side(pool, b);
  a.stage = stage;
  a.H = l.n_kv_heads;
  a.B = l.block_tokens;
  a.DV = (uint32_t)(l.head_dim * 2 / 16);
  a.dvdiv = make_fastdiv(a.DV);
  a.bdiv = make_fastdiv((uint32_t)a.B);
  a.heads = make_fastdiv((uint32_t)a.H);
  const int n_planes = 2 * l.n_layers;
  const int64_t bpt_vec = (int64_t)l.n_layers * 2 * l.n_kv_heads * a.DV;
  // FAST: a 256-vector piece covers whole tokens, a block holds a whole number of
  // pieces, the rows of a block's head are contiguous and every range starts on a
  // block boundary.
  bool fast = 256 % a.DV == 0 && ((int64_t)a.B * a.DV) % 256 == 0 &&
              a.pool.stride_slot == a.DV * 16u;
  for (int q = 0; q < view.n_req && fast; ++q) fast = view.start[q] % a.B == 0;
  a.piece_tokens = fast ? 256u / a.DV : 0u;
  // limits are checked for the whole batch before the first launch: an error
  // must mean that no device byte was written
  for (int q = 0; q < view.n_req; ++q) {
    if (((int64_t)view.k[q] + 1) * a.DV > 0x7fffffff)
      return fail(KVM_EINVAL, "a single request's (plane, head) run exceeds 2^31 vectors");
    const int64_t chunks = ceil_div((int64_t)(view.k[q] - view.start[q]) * a.DV, 256);
    if (chunks * n_planes * a.H > 0x7fffffff)
      return fail(KVM_EINVAL, "a single request exceeds the grid size limit");
  }
  int64_t stage_vec = 0;
  int r = 0;
  while (r < view.n_req) {
    int n = 0;
    for (int i = 0; i < kMaxReqPerLaunch; ++i) a.first_wg[i] = UINT32_MAX;
    int64_t n_wg = 0;
    while (r < view.n_req && n < kMaxReqPerLaunch) {
      const int64_t n_tok = view.k[r] - view.start[r];
      const int64_t chunks = ceil_div(n_tok * a.DV, 256);
      const int64_t wgs = chunks * n_planes * a.H;
      if (n_wg + wgs > 0x7fffffff) break;
      if (n_tok > 0) {  // requests that move nothing take no descriptor
        StageReq& q = a.req[n];
        q.bt = view.bt_off[r];
        q.start = view.start[r];
        q.n_vec = (uint32_t)(n_tok * a.DV);
        q.first_wg = (uint32_t)n_wg;
        q.stage_vec = stage_vec;
        q.chunks = make_fastdiv((uint32_t)chunks);
        a.first_wg[n++] = (uint32_t)n_wg;
        n_wg += wgs;
      }
      stage_vec += n_tok * bpt_vec;
      ++r;
    }
    if (n_wg == 0) continue;
    a.n_wg = (uint32_t)n_wg;
    const StageGrid sg = stage_grid(n_wg);
    const dim3 grid(sg.x, sg.y), block(256);
    if (o.copy_nontemporal) {
      if (fast) hipLaunchKernelGGL((stage_kernel<PACK, true, true>), grid, block, 0, stream, a);
      else hipLaunchKernelGGL((stage_kernel<PACK, true, false>), grid, block, 0, stream, a);
    } else {
      if (fast) hipLaunchKernelGGL((stage_kernel<PACK, false, true>), grid, block, 0, stream, a);
      else hipLaunchKernelGGL((stage_kernel<PACK, false, false>), grid, block, 0, stream, a);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KVM_EHIP, hipGetErrorString(e));
  }
  return KVM_OK;
}

// True if [p, p + n) and the pool's span share a byte.
static bool overlaps_pool(const void* p, int64_t n, const kvm_pool* pool) {
  const char* a0 = (const char*)p;
  const char* b0 = (const char*)pool->base;
  return n > 0 && a0 < b0 + kvm_pool_span_bytes(&pool->layout, pool->n_blocks) && b0 < a0 + n;
}

static bool same_shape(const kvm_layout& a, const kvm_layout& b) {
  return a.n_layers == b.n_layers && a.n_kv_heads == b.n_kv_heads && a.n_q_heads == b.n_q_heads &&
         a.head_dim == b.head_dim && a.block_tokens == b.block_tokens && a.dtype == b.dtype;
}

}  // namespace kvm

using namespace kvm;

extern "C" {

int kvm_pack(const kvm_pool* src, const kvm_batch* src_reqs, void* staging_dev,
             int64_t staging_bytes, void* hip_stream) {
  clear_error();
  BatchView sv;
  int rc = validate_side("kvm_pack: src", src, src_reqs, false, &sv);
  if (rc) return rc;
  const int64_t need = sv.total_tokens * kvm_bytes_per_token(&src->layout);
  if (need > 0 && !staging_dev) return fail(KVM_EINVAL, "kvm_pack: staging_dev is NULL");
  if ((uintptr_t)staging_dev % 16) return fail(KVM_EINVAL, "kvm_pack: staging_dev is not 16-byte aligned");
  if (staging_bytes < need) return fail(KVM_EINVAL, "kvm_pack: staging buffer too small");
  if (overlaps_pool(staging_dev, need, src))
    return fail(KVM_EINVAL, "kvm_pack: the staging buffer overlaps the pool");
  // Work cut along the staging buffer pays for long requests (13B shape, 32768
  // tokens: 6.34 against 6.15 TB/s); for short ones the block-cut kernel is as fast
  // or faster (7B shape, 550 tokens: 6.31 against 6.64).  Automatic: by mean length.
  const int mode = options().stage_linear;
  int64_t live = 0;
  for (int r = 0; r < sv.n_req; ++r) live += sv.k[r] > sv.start[r];
  const bool linear = mode < 0 ? sv.total_tokens >= 4096 * std::max<int64_t>(1, live) : (mode & 1) != 0;
  if (linear)
    return run_stage<true>(src, src_reqs, sv, (char*)staging_dev, (hipStream_t)hip_stream);
  return run_copy<kPack>(src, src_reqs, sv, src, src_reqs, sv, (char*)staging_dev,
                         (hipStream_t)hip_stream);
}

int kvm_unpack(const void* staging_dev, int64_t staging_bytes, const kvm_pool* dst,
               const kvm_batch* dst_reqs, void* hip_stream) {
  clear_error();
  BatchView dv;
  int rc = validate_side("kvm_unpack: dst", dst, dst_reqs, true, &dv);
  if (rc) return rc;
  const int64_t need = dv.total_tokens * kvm_bytes_per_token(&dst->layout);
  if (need > 0 && !staging_dev) return fail(KVM_EINVAL, "kvm_unpack: staging_dev is NULL");
  if ((uintptr_t)staging_dev % 16) return fail(KVM_EINVAL, "kvm_unpack: staging_dev is not 16-byte aligned");
  if (staging_bytes < need) return fail(KVM_EINVAL, "kvm_unpack: staging buffer too small");
  if (overlaps_pool(staging_dev, need, dst))
    return fail(KVM_EINVAL, "kvm_unpack: the staging buffer overlaps the pool");
  if (options().stage_linear > 0 && (options().stage_linear & 2))
    return run_stage<false>(dst, dst_reqs, dv, (char*)staging_dev, (hipStream_t)hip_stream);
  return run_copy<kUnpack>(dst, dst_reqs, dv, dst, dst_reqs, dv, (char*)staging_dev,
                           (hipStream_t)hip_stream);
}

int kvm_migrate(const kvm_pool* src, const kvm_batch* src_reqs, const kvm_pool* dst,
                const kvm_batch* dst_reqs, void* hip_stream) {
  clear_error();
  BatchView sv, dv;
  int rc = validate_side("kvm_migrate: src", src, src_reqs, false, &sv);
  if (rc) return rc;
  rc = validate_side("kvm_migrate: dst", dst, dst_reqs, true, &dv);
  if (rc) return rc;
  if (!same_shape(src->layout, dst->layout))
    return fail(KVM_EINVAL, "kvm_migrate: src and dst layouts differ in more than strides");
  if (sv.n_req != dv.n_req) return fail(KVM_EINVAL, "kvm_migrate: n_req differs between src and dst");
  for (int r = 0; r < sv.n_req; ++r) {
    if (sv.k[r] != dv.k[r]) return fail(KVM_EINVAL, "kvm_migrate: k differs between src and dst");
    if (sv.start[r] != dv.start[r])
      return fail(KVM_EINVAL, "kvm_migrate: start differs between src and dst");
  }
  // Overlapping memory: only the same pool with disjoint block sets is allowed.
  const char* s0 = (const char*)src->base;
  const char* d0 = (const char*)dst->base;
  const char* s1 = s0 + kvm_pool_span_bytes(&src->layout, src->n_blocks);
  const char* d1 = d0 + kvm_pool_span_bytes(&dst->layout, dst->n_blocks);
  if (s0 < d1 && d0 < s1) {
    const kvm_layout &a = src->layout, &b = dst->layout;
    const bool same = s0 == d0 && a.stride_layer == b.stride_layer && a.stride_kv == b.stride_kv &&
                      a.stride_block == b.stride_block && a.stride_head == b.stride_head &&
                      a.stride_slot == b.stride_slot && src->n_blocks == dst->n_blocks;
    if (!same) return fail(KVM_EINVAL, "kvm_migrate: src and dst memory overlap but are not the same pool");
    if (!src_reqs->bt_blocks_host || !dst_reqs->bt_blocks_host)
      return fail(KVM_EINVAL, "kvm_migrate: in-pool migration needs host block ids on both sides");
    std::vector<uint64_t> wr((size_t)ceil_div(dst->n_blocks, 64), 0);
    for (int r = 0; r < dv.n_req; ++r)
      for (int j = dv.jb[r]; j < dv.nb[r]; ++j) {
        const int32_t id = dst_reqs->bt_blocks_host[dv.bt_off[r] + j];
        wr[(size_t)id >> 6] |= 1ull << (id & 63);
      }
    for (int r = 0; r < sv.n_req; ++r)
      for (int j = sv.jb[r]; j < sv.nb[r]; ++j) {
        const int32_t id = src_reqs->bt_blocks_host[sv.bt_off[r] + j];
        if (wr[(size_t)id >> 6] & (1ull << (id & 63)))
          return fail(KVM_EINVAL, "kvm_migrate: a block is both read and written");
      }
  }
  return run_copy<kMigrate>(src, src_reqs, sv, dst, dst_reqs, dv, nullptr, (hipStream_t)hip_stream);
}

}  // extern "C"
