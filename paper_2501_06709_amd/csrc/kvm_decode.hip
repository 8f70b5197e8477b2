// Paged decode attention for gfx950 and its C entry point.
//
// The decoding phase reads the KV cache of all earlier tokens to produce the
// next one (arXiv 2501.06709, Sec. "Background & Related Work").  Running it
// over the destination pool after a migration shows that the moved cache is
// usable.  One query token per (request, layer, query head):
//   out = softmax(scale * q K^T) V  over tokens [0,k) read through the block table.
//
// The operation streams K and V once and does 1 (MHA) to 8 (grouped-query, group
// of eight) flops per byte, so it is bound by HBM and written around coalesced
// 16-byte loads:
//  - one 256-lane workgroup per (request, layer, KV head[, context split]); the
//    G query heads that share the KV head are served from the same loads;
//  - a token row of D*2 bytes is spread over D/8 adjacent lanes (16 bytes each), so
//    one load instruction covers 1 KiB of consecutive cache bytes; for head_dim 128
//    each of the 4 waves takes four token rows of EVERY block (other shapes: whole
//    blocks, every 4th one per wave);
//  - scores: dot instructions and DPP reductions on the vector unit, or, for groups
//    of four and eight query heads, the matrix cores; P.V on the vector unit;
//  - every (wave, lane row) keeps its own online-softmax state (running max, sum,
//    fp32 accumulator); rows are merged in registers, waves through LDS by the wave
//    that finishes last;
//  - block ids come through scalar loads, one step ahead of their use;
//  - long contexts can be split over several workgroups whose partial states are
//    merged by a second small kernel (log-sum-exp merge).
// The order of every reduction depends on logical token positions only, so the
// same logical cache in different physical blocks gives bit-identical output.
#include <hip/hip_runtime.h>

#include <cmath>
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <type_traits>

#include "kvm_internal.h"

namespace kvm {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

typedef const __attribute__((address_space(4))) int32_t* ConstTable;  // block table seen as constant memory

constexpr float kNegBig = -1.0e30f;  // finite stand-in for "no token seen yet"

struct DecReq {
  int32_t bt;   // first table entry of the request
  int32_t k;    // context length
  int32_t row;  // row of q and out that belongs to the request
  int32_t slot; // request index within the batch: its workspace entries
};

struct DecArgs {
  const char* base;
  const int32_t* bt;
  int64_t stride_layer;  // bytes
  int64_t stride_kv;
  int64_t stride_block;
  uint32_t stride_head;
  uint32_t stride_slot;
  const uint16_t* q;
  void* out;
  float* ws;
  int32_t L, H, Hq;
  int32_t passes;       // query-head groups per KV head handled by separate workgroups
  int32_t n_splits;
  int32_t out_f32;
  float scale_log2e;    // softmax scale * log2(e): scores live in the exp2 domain
  int32_t spread_log2;  // sliced kernels: log2 of the table-entry distance between the four blocks of a step
  DecReq req[kMaxReqPerLaunch];
};

__device__ __forceinline__ float dpp_xor1(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_xor2(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_half_mirror(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_mirror(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
}

// Sum over groups of LPT adjacent lanes (LPT = 8 or 16); every lane of a group
// ends with the group's total.  Steps: neighbours in a quad, then the other
// quad of an 8-lane half (half mirror), then the other half of the 16-lane row.
template <int LPT>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_xor1(v);
  v += dpp_xor2(v);
  v += dpp_half_mirror(v);
  if (LPT == 16) v += dpp_mirror(v);
  return v;
}

template <bool BF16>
__device__ __forceinline__ void widen8(v4u raw, float* f) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (BF16) {
      f[2 * i] = __builtin_bit_cast(float, raw[i] << 16);
      f[2 * i + 1] = __builtin_bit_cast(float, raw[i] & 0xffff0000u);
    } else {
      typedef _Float16 h2 __attribute__((ext_vector_type(2)));
      const unsigned int w = raw[i];  // bit_cast needs a scalar object, not a vector element
      const h2 h = __builtin_bit_cast(h2, w);
      f[2 * i] = (float)h[0];
      f[2 * i + 1] = (float)h[1];
    }
  }
}

// Dot product of eight 16-bit pairs-packed values with fp32 accumulation
// (v_dot2c_f32_f16 / v_dot2c_f32_bf16: two multiply-adds per instruction).
template <bool BF16>
__device__ __forceinline__ float dot8(const uint32_t* qv, v4u kv) {
  float acc = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t x = qv[c], y = kv[c];
    if (BF16) {
      typedef __bf16 b2 __attribute__((ext_vector_type(2)));
      acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2, x), __builtin_bit_cast(b2, y), acc, false);
    } else {
      typedef _Float16 h2 __attribute__((ext_vector_type(2)));
      acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, x), __builtin_bit_cast(h2, y), acc, false);
    }
  }
  return acc;
}

template <bool BF16>
__device__ __forceinline__ uint16_t narrow(float f) {
  if (BF16) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even
    return (uint16_t)(u >> 16);
  }
  return __builtin_bit_cast(uint16_t, (_Float16)f);
}

// Workspace entry of one (request slot, layer, query head, split): D unnormalised
// accumulator values, then the running max (exp2 domain) and the running sum.
__device__ __forceinline__ float* ws_entry(float* ws, const DecArgs& a, int row, int l, int hq,
                                           int split, int D) {
  return ws + ((((int64_t)row * a.L + l) * a.Hq + hq) * a.n_splits + split) * (D + 2);
}

// What one workgroup of the tuned kernels works on: grid = (KV heads x passes,
// layers, requests x splits); a split covers blocks [jb, je) of the context.
struct WorkItem {
  DecReq rq;
  int h, l, split;  // KV head, layer, split index
  int hq0;          // first query head served by this workgroup
  int jb, je;       // block range; jb >= je: nothing to do
};
template <int B, int G>
__device__ __forceinline__ WorkItem work_item(const DecArgs& a) {
  WorkItem w;
  const int pass = blockIdx.x % a.passes;
  w.h = blockIdx.x / a.passes;
  // Workgroups are handed to the chip's eight dies round-robin in dispatch order, so
  // with the head as the fastest grid dimension die i would always read the heads
  // congruent to i modulo 8, i.e. always the same 4 KiB-aligned pieces of a block's
  // run.  The decode reads faster when the pieces a die reads vary (measured on
  // MI355X, 32 KV heads, 32 blocks per workgroup: 6.64 against 6.27 TB/s; no
  // difference with 8 KV heads), so the low three bits of the head are rotated by
  // layer and request: a bijection within each group of 8.
  if ((a.H & 7) == 0) w.h = (w.h & ~7) | ((w.h + (int)blockIdx.y + (int)blockIdx.z) & 7);
  w.l = blockIdx.y;
  w.split = blockIdx.z % a.n_splits;
  w.rq = a.req[blockIdx.z / a.n_splits];
  w.hq0 = (w.h * a.passes + pass) * G;
  const int nb = (max(w.rq.k, 0) + B - 1) / B;
  const int per = (nb + a.n_splits - 1) / a.n_splits;
  w.jb = w.split * per;
  w.je = min(nb, w.jb + per);
  return w;
}

// Which four blocks a step of the sliced kernels reads.  Reading four blocks that are
// neighbours in memory with one burst of loads is the slowest way to read them: a
// stream of 4 KiB pieces fetched four at a time runs at 6.23 TB/s when the four lie
// 32 .. 160 KiB apart, at 6.50 when they lie 0.5 .. 1 MiB apart (or are one 16 KiB run),
// at 6.0 when 4 .. 8 MiB apart (measured on MI355X; consecutive block ids, which a
// lowest-id-first allocator hands out on a fresh pool, put the blocks of a request
// exactly one block run apart).  So the table entries of a range are taken in an
// interleaved order: while at least 4e entries remain, step o of such a group reads
// entries o, o + e, o + 2e, o + 3e of the group (e = 2^spread_log2 entries, about
// 1 MiB in consecutive ids); the remainder repeats this with e/2, e/4, ..., and the
// last entries (fewer than 8) go in table order, so that the block that may be partly
// context is still the very last position.  Returns the entry of instruction 0 of
// step `it` and the distance e_out to the entries of instructions 1..3.  Uniform
// over the wave, shifts and compares only: it runs on the scalar unit.
__device__ __forceinline__ int step_first_entry(int it, int nblk, int spread_log2, int& e_out) {
  const int pos0 = 4 * it;
  int base = 0, sh = spread_log2;
  while (sh > 0) {
    const int full = ((nblk - base) >> (sh + 2)) << (sh + 2);   // entries in whole groups of 4e
    if (pos0 - base < full) break;
    base += full;
    --sh;
  }
  const int rel = pos0 - base;
  e_out = 1 << sh;
  return base + ((rel >> (sh + 2)) << (sh + 2)) + ((rel & ((4 << sh) - 1)) >> 2);
}

// ---- end of a workgroup: from per-lane states to the output row ---------------
// After the block loop every lane holds, per query head g, the online-softmax state
// of its token row: running max m[g] (exp2 domain) and sum lsum[g], equal over the
// lanes of the row, and o[g][0..7], dims sub*8.. of the row's unnormalised output.
//  1. The 64/LPT token rows of a wave are merged in registers (xor shuffles over the
//     row bits of the lane index), so a wave leaves ONE state per head.
//  2. Lanes of row 0 write it to LDS and the wave counts itself done.  There is no
//     workgroup barrier at the end: a wave that is not the last one simply ends and
//     frees its slot, so waves that finish early (a wave can have one block less than
//     its neighbours) do not wait for the slowest one.
//  3. The wave that arrives last merges the four wave states in wave order and
//     writes the normalised output row, or, when the context is split, the workspace
//     entry of this split.
// The order of every combination depends on logical token positions only.
template <int D, int G>
struct WaveStates {
  float m[4][G];
  float l[4][G];
  __attribute__((aligned(16))) float o[4][G][D];
  unsigned int done;   // waves that have written their state; zeroed at workgroup start
};

// head_of[g]: the head (0 .. G-1) whose state this lane keeps in slot g; the same for
// lanes that differ only in the token row, so that rows merge slot by slot.
template <int D, int G, bool BF16>
__device__ __forceinline__ void finish_workgroup(const DecArgs& a, const DecReq& rq, int l, int hq0, int split,
                                                 int wave, int lane, float (&m)[G], float (&lsum)[G],
                                                 float (&o)[G][8], WaveStates<D, G>& ws, const int (&head_of)[G]) {
  constexpr int LPT = D / 8;
  const int sub = lane % LPT;
  // 1. merge the token rows of the wave: first the maximum over the rows, then every
  // row rescales its own state once and the rows are added up (all shuffles of a round
  // are independent, so a round costs one cross-lane latency, not one per value)
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mx = m[g];
#pragma unroll
    for (int x = LPT; x < 64; x <<= 1) mx = fmaxf(mx, __shfl_xor(mx, x));
    const float w = __builtin_amdgcn_exp2f(m[g] - mx);
    m[g] = mx;
    lsum[g] *= w;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[g][c] *= w;
  }
#pragma unroll
  for (int x = LPT; x < 64; x <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      lsum[g] += __shfl_xor(lsum[g], x);
#pragma unroll
      for (int c = 0; c < 8; ++c) o[g][c] += __shfl_xor(o[g][c], x);
    }
  }
  // 2. row 0 holds the wave's state
  if (lane < LPT) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (lane == 0) {
        ws.m[wave][head_of[g]] = m[g];
        ws.l[wave][head_of[g]] = lsum[g];
      }
      v4f* dst = reinterpret_cast<v4f*>(&ws.o[wave][head_of[g]][sub * 8]);
      dst[0] = v4f{o[g][0], o[g][1], o[g][2], o[g][3]};
      dst[1] = v4f{o[g][4], o[g][5], o[g][6], o[g][7]};
    }
  }
  unsigned int before = 0;
  if (lane == 0)  // release: this wave's LDS writes precede the count; acquire: the last wave sees all
    before = __hip_atomic_fetch_add(&ws.done, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
  if (__builtin_amdgcn_readfirstlane(before) != 3u) return;
  // 3. the last wave combines the four wave states, in wave order: a lane takes eight
  // consecutive dims of one head (G * D / 8 such pieces over the 64 lanes)
  for (int piece = lane; piece < G * LPT; piece += 64) {
    const int g = piece / LPT, d0 = (piece % LPT) * 8;
    float mw[4], mx = kNegBig;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      mw[w] = ws.m[w][g];
      mx = fmaxf(mx, mw[w]);
    }
    float acc[8], den = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(mw[w] - mx);
      den = fmaf(ws.l[w][g], wgt, den);
      const v4f* src = reinterpret_cast<const v4f*>(&ws.o[w][g][d0]);
      const v4f lo = src[0], hi = src[1];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        acc[c] = fmaf(lo[c], wgt, acc[c]);
        acc[4 + c] = fmaf(hi[c], wgt, acc[4 + c]);
      }
    }
    const int hq = hq0 + g;
    if (a.n_splits == 1) {
      const int64_t oi = (((int64_t)rq.row * a.L + l) * a.Hq + hq) * D + d0;
      // out is only required to be 4-byte aligned; a 16-byte aligned one (a row starts
      // at a multiple of 16 bytes from it) gets 16-byte stores: a quarter of the write
      // requests the workgroup has to see acknowledged before it can end
      const bool wide = (reinterpret_cast<uintptr_t>(a.out) & 15u) == 0;
      float r[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) r[c] = acc[c] / den;
      if (a.out_f32) {
        float* dst = reinterpret_cast<float*>(a.out) + oi;
        if (wide) {
          reinterpret_cast<v4f*>(dst)[0] = v4f{r[0], r[1], r[2], r[3]};
          reinterpret_cast<v4f*>(dst)[1] = v4f{r[4], r[5], r[6], r[7]};
        } else {
#pragma unroll
          for (int c = 0; c < 8; ++c) dst[c] = r[c];
        }
      } else {
        uint32_t* dst = reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(a.out) + oi);
        uint32_t pk[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
          pk[c] = (uint32_t)narrow<BF16>(r[2 * c]) | ((uint32_t)narrow<BF16>(r[2 * c + 1]) << 16);
        if (wide) {
          *reinterpret_cast<v4u*>(dst) = v4u{pk[0], pk[1], pk[2], pk[3]};
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) dst[c] = pk[c];
        }
      }
    } else {
      float* e = ws_entry(a.ws, a, rq.slot, l, hq, split, D);
#pragma unroll
      for (int c = 0; c < 8; ++c) e[d0 + c] = acc[c];
      if (d0 == 0) {
        e[D] = mx;
        e[D + 1] = den;
      }
    }
  }
}

template <int D, int G, bool BF16>
__device__ __forceinline__ void finish_workgroup(const DecArgs& a, const DecReq& rq, int l, int hq0, int split,
                                                 int wave, int lane, float (&m)[G], float (&lsum)[G],
                                                 float (&o)[G][8], WaveStates<D, G>& ws) {
  int head_of[G];
#pragma unroll
  for (int g = 0; g < G; ++g) head_of[g] = g;
  finish_workgroup<D, G, BF16>(a, rq, l, hq0, split, wave, lane, m, lsum, o, ws, head_of);
}

// WMAX caps the waves per SIMD.  The capped instance (two waves per SIMD, up to 256
// registers each) keeps two tiles in flight per wave and is the faster one from about
// a dozen blocks per workgroup on (measured on MI355X, one head per KV head, 32 blocks:
// 6.64 against 6.37 TB/s); below that the uncapped instance wins because set-up and
// merge of a workgroup are no longer hidden (8 blocks: 6.28 against 5.66).  The host
// picks by mean context.
template <int D, int B, int G, bool BF16, int WMAX>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, WMAX))) void decode_kernel(const DecArgs a) {
  constexpr int LPT = D / 8;       // lanes per token row
  constexpr int TPI = 64 / LPT;    // token rows per load instruction
  constexpr int NI = B / TPI;      // load instructions per block and per K / V
  // Tiles in flight per wave and per K / V: the capped instances (two waves per SIMD,
  // up to 256 registers each) keep two blocks ahead, the others one.
  constexpr int P = (WMAX == 2 && G < 8) ? 2 : 1;
  static_assert(LPT == 8 || LPT == 16, "head_dim must be 64 or 128");
  static_assert(B % TPI == 0, "block_tokens must be a multiple of the rows per load");

  __shared__ WaveStates<D, G> s_ws;   // 8 KiB for G = 4, D = 128

  const WorkItem wi = work_item<B, G>(a);
  if (wi.jb >= wi.je) return;  // empty context or an empty split: uniform over the workgroup
  const DecReq rq = wi.rq;
  const int h = wi.h, l = wi.l, split = wi.split, k = rq.k, jb = wi.jb, je = wi.je;

  const int lane = threadIdx.x & 63;
  // uniform over the wave; saying so keeps the block loop's control flow and the
  // block address arithmetic on the scalar unit
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane % LPT;
  const int row = lane / LPT;
  const int hq0 = wi.hq0;  // first query head served here
  // the only workgroup barrier: at the start, where the four waves arrive together
  if (threadIdx.x == 0) s_ws.done = 0u;
  __syncthreads();

  // query fragment: dims sub*8 .. sub*8+7 of each of the G heads, kept as four
  // packed 16-bit pairs per head; the softmax scale is applied to the reduced score
  uint32_t qp[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint16_t* qptr = a.q + (((int64_t)rq.row * a.L + l) * a.Hq + hq0 + g) * D + sub * 8;
    const v4u raw = *reinterpret_cast<const v4u*>(qptr);
#pragma unroll
    for (int c = 0; c < 4; ++c) qp[g][c] = raw[c];
  }
  const float sc = a.scale_log2e;

  float m[G], lsum[G], o[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNegBig;
    lsum[g] = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[g][c] = 0.f;
  }

  const char* kbase = a.base + (int64_t)l * a.stride_layer + (int64_t)h * a.stride_head;
  const char* vbase = kbase + a.stride_kv;

  // Which part of the context a wave takes.
  //  SLICED (head_dim 128, 16-token blocks: one load instruction covers four token
  //  rows): wave w takes token rows 4w .. 4w+3 of EVERY block, and one step of its loop
  //  covers four consecutive blocks, one load instruction each.  The four waves then
  //  read every 4 KiB piece together, advance in lockstep and do exactly the same
  //  amount of work, which is what lets a workgroup hand its slot on without one wave
  //  trailing the others (measured on MI355X against the whole-blocks form: 32 KV
  //  heads, mean context 550 tokens, 0.366 -> 0.347 ms).
  //  Otherwise wave w takes whole blocks jb + w, jb + w + 4, ...
  constexpr bool SLICED = (TPI * 4 == B);
  constexpr int NID = SLICED ? NI : 1;   // block ids per step
  const int nblk = je - jb;
  const int n_it = SLICED ? (nblk + 3) / 4 : (nblk - wave + 3) / 4;  // the latter may be <= 0
  v4u kcs[P][NI], vcs[P][NI];
  // Block ids are uniform over the wave: they are read with scalar loads, one step
  // ahead of their use, on the scalar cache's own path instead of queueing behind
  // the streamed tiles.  (The table does not change while the kernel runs; reading
  // it through the constant address space is what makes the compiler use scalar
  // loads inside the loop, where it otherwise falls back to a vector load and a
  // full wait.)  Indices past the range are clamped to its last entry.
  const ConstTable tab = (ConstTable)(a.bt + rq.bt + jb + (SLICED ? 0 : wave));
  struct Ids { int v[NID]; int first, dist; };   // ids; sliced: entry of instruction 0 and distance to the next
  auto block_ids = [&](int it) {
    Ids r;
    if constexpr (SLICED) {
      r.first = step_first_entry(min(it, n_it - 1), nblk, a.spread_log2, r.dist);
#pragma unroll
      for (int i = 0; i < NID; ++i) r.v[i] = tab[min(r.first + i * r.dist, nblk - 1)];
    } else {
      r.first = r.dist = 0;
      r.v[0] = tab[4 * min(it, n_it - 1)];
    }
    return r;
  };
  const uint32_t lane_off = (uint32_t)((SLICED ? 4 * wave : 0) + row) * a.stride_slot + (uint32_t)sub * 16u;
  const uint32_t inst_off = (uint32_t)TPI * a.stride_slot;

  // Software pipeline with P K and P V register tiles: K of step it + P is
  // requested as soon as the scores of step it are formed, V of step it + P as
  // soon as the V rows of step it are accumulated, so loads are always in flight
  // while a tile is being consumed.  Every step issues both tile loads
  // unconditionally; loads that have no block to read (after the last step, or
  // past the last block of a sliced step) go to the wave's own query row (valid,
  // aligned, cached), which keeps the loop free of the register copies a
  // conditional load would need.
  // s_waitcnt immediates (vmcnt in bits 3:0 and 15:14, the other counters left at
  // their maximum).  The explicit waits below keep the compiler from draining all
  // loads at the top of every iteration: without it it cannot prove that the query
  // registers (loaded before the loop) are ready, and inserts vmcnt(0) on the hot path.
  constexpr int kTileLoads = 2 * P * NI;                 // tile loads that may stay in flight (<= 63)
  constexpr int kWaitAllButTiles = 0x0F70 | (kTileLoads & 15) | ((kTileLoads >> 4) << 14);
  const char* dummy = reinterpret_cast<const char*>(
      a.q + (((int64_t)rq.row * a.L + l) * a.Hq + hq0) * D) + (uint32_t)sub * 16u;   // D*2 >= 128 bytes, 16-byte aligned
  // tile of step `it` (ids: its block ids); it >= n_it reads the dummy row
  auto load_tile = [&](int it, const char* base, const Ids& ids, v4u* td) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const bool real = it < n_it && (!SLICED || ids.first + i * ids.dist < nblk);
      const char* p = real ? base + (int64_t)ids.v[SLICED ? i : 0] * a.stride_block + lane_off + (SLICED ? 0u : i * inst_off)
                           : dummy;
      td[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
    }
  };
  // Context slots of the block that instruction i of step `it` reads, counted from
  // the instruction's first token row: only the request's last block can be partly
  // context.
  auto token_limit = [&](int it, int i) {
    if constexpr (SLICED) {
      int dist;
      const int bi = step_first_entry(it, nblk, a.spread_log2, dist) + i * dist;
      return bi < nblk ? min(B, k - (jb + bi) * B) - 4 * wave : 0;
    } else {
      return k - (jb + wave + 4 * it) * B - i * TPI;
    }
  };
  Ids id_next = {};   // ids of step it + P while step it is being consumed
  // One step.  MASKED handles a step that contains slots past the context; full
  // steps take the mask-free instance.
  auto step = [&](auto masked_tag, auto slot_tag, int it) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    constexpr int S = decltype(slot_tag)::value;   // register tile that holds step it
    v4u(&kc)[NI] = kcs[S];
    v4u(&vc)[NI] = vcs[S];
    int lim[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) lim[i] = MASKED ? token_limit(it, i) : TPI;
    float s[NI][G];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int g = 0; g < G; ++g) s[i][g] = group_sum<LPT>(dot8<BF16>(qp[g], kc[i]));
    __builtin_amdgcn_sched_barrier(0);
    const Ids id_after = block_ids(it + P + 1);
    load_tile(it + P, kbase, id_next, kc);
    __builtin_amdgcn_sched_barrier(0);

#pragma unroll
    for (int g = 0; g < G; ++g) {
      // raw scores; the softmax scale enters through the fused multiply-add in
      // front of each exponential (m[] holds scaled maxima)
      float mx = m[g];
#pragma unroll
      for (int i = 0; i < NI; ++i)
        if (!MASKED || row < lim[i]) mx = fmaxf(mx, s[i][g] * sc);
      const float alpha = __builtin_amdgcn_exp2f(m[g] - mx);
      m[g] = mx;
      float add = 0.f;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const float e = __builtin_amdgcn_exp2f(fmaf(s[i][g], sc, -mx));
        s[i][g] = (!MASKED || row < lim[i]) ? e : 0.f;
        add += s[i][g];
      }
      lsum[g] = lsum[g] * alpha + add;
#pragma unroll
      for (int c = 0; c < 8; ++c) o[g][c] *= alpha;
    }
    if (MASKED) {
      // Slots past the context may hold anything (NaN patterns included): clear
      // their V rows so that a zero weight cannot turn them into NaN.
#pragma unroll
      for (int i = 0; i < NI; ++i)
        if (row >= lim[i]) vc[i] = v4u{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float vf[8];
      widen8<BF16>(vc[i], vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) o[g][c] = fmaf(s[i][g], vf[c], o[g][c]);
    }
    __builtin_amdgcn_sched_barrier(0);
    load_tile(it + P, vbase, id_next, vc);
    id_next = id_after;
    __builtin_amdgcn_sched_barrier(0);
  };
  // Only the request's last block can be partly context, so at most the wave's last
  // step needs masks: all other steps run the mask-free instance in a loop of their own.
  if (n_it > 0) {
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, P - 1>;
#pragma unroll
    for (int j = 0; j < P; ++j) {
      const Ids idj = block_ids(j);
      load_tile(j, kbase, idj, kcs[j]);
      __builtin_amdgcn_sched_barrier(0);
      load_tile(j, vbase, idj, vcs[j]);
      __builtin_amdgcn_sched_barrier(0);
    }
    id_next = block_ids(P);
    __builtin_amdgcn_s_waitcnt(kWaitAllButTiles);       // queries have arrived
    // steps whose slots are all context
    int n_main;
    if constexpr (SLICED) {
      const int n_full = min(nblk, (k - jb * B) / B);   // full blocks of the range
      n_main = n_full / 4;
    } else {
      const int t_last = k - (jb + wave + 4 * (n_it - 1)) * B;  // context slots in this wave's last block
      n_main = t_last < B ? n_it - 1 : n_it;
    }
    if constexpr (P == 1) {
      for (int it = 0; it < n_main; ++it) step(std::false_type{}, S0{}, it);
      if (n_main < n_it) step(std::true_type{}, S0{}, n_main);
    } else {
      // steps alternate between the two register tiles: even ones in tile 0
      int it = 0;
      for (; it + 1 < n_main; it += 2) {
        step(std::false_type{}, S0{}, it);
        step(std::false_type{}, S1{}, it + 1);
      }
      if (it < n_main) step(std::false_type{}, S0{}, it);
      if (n_main < n_it) {
        if (n_main & 1) step(std::true_type{}, S1{}, n_main);
        else step(std::true_type{}, S0{}, n_main);
      }
    }
  }

  finish_workgroup<D, G, BF16>(a, rq, l, hq0, split, wave, lane, m, lsum, o, s_ws);
}

// Grouped-query decode with the scores on the matrix cores, whole blocks per wave
// (head_dim 128, 16-token blocks; launched for groups of eight query heads, groups
// of four have decode_mfma4_kernel below).  q.K^T of one block is a
// 16 x G x 128 contraction: four v_mfma_f32_16x16x32 with K as the A operand and
// the query heads as columns of the B operand replace 64 dot instructions and 64
// cross-lane additions of the vector version.
// Operand layouts of the instruction (checked on the device against a plain
// matrix product): A: lane x holds row x%16, k = 8*(x/16) .. +7; B: lane x holds
// column x%16, k = 8*(x/16) .. +7; D: lane x holds rows 4*(x/16) .. +3 of column x%16.
// Taking the sixteen rows as the block's sixteen tokens would make each load
// instruction read 64 bytes of every token, two instructions per 128-byte line,
// and a share of those lines is then fetched from HBM twice (measured: 3 % more
// bytes than the cache holds tokens).  Instead one instruction reads whole lines:
// rows 0..7 are eight tokens with the first half of a line as their k range, rows
// 8..15 the same eight tokens with the second half; the query heads occupy 2G
// columns, G with the dims of the first half and G with those of the second.  The
// result tile then holds the two partial scores of (token, head) in two lanes (and
// cross products nobody reads); one ds_bpermute per score adds them.  MFMA i
// covers tokens 8*(i/2) .. +7 and line i%2; for the second eight tokens the halves
// are swapped so that lane (head, lane row g) ends up owning the scores of tokens
// 4g .. 4g+3 of the block and keeps the online-softmax state of that pair.  The V
// tile is loaded so that lane row g holds tokens 4g .. 4g+3 as well, 16 bytes of
// each per lane; the four weights and the rescale factor of every head then travel
// from lane (head, g) to the sixteen lanes of the row with ds_bpermute (no LDS
// memory is touched) and P.V stays on the vector unit.
// WMAX as for decode_kernel.
template <int D, int B, int G, bool BF16, int WMAX>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, WMAX))) void decode_mfma_kernel(const DecArgs a) {
  static_assert(D == 128 && B == 16 && (G == 4 || G == 8), "shape of the matrix-core variant");
  constexpr int P = (WMAX == 2 && G < 8) ? 2 : 1;   // tiles in flight per wave and per K / V (as in decode_kernel)
  __shared__ WaveStates<D, G> s_ws;

  const WorkItem wi = work_item<B, G>(a);
  if (wi.jb >= wi.je) return;  // empty context or an empty split: uniform over the workgroup
  const DecReq rq = wi.rq;
  const int h = wi.h, l = wi.l, split = wi.split, k = rq.k, jb = wi.jb, je = wi.je;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane % 16;
  const int row = lane / 16;
  const int hq0 = wi.hq0;
  if (threadIdx.x == 0) s_ws.done = 0u;
  __syncthreads();

  // B operand of line ln (dims 64*ln .. 64*ln+63): column c < 2G holds head c % G,
  // dims 64*ln + 32*(c / G) + 8*row .. +7; columns >= 2G are zero
  const uint16_t* qrow = a.q + (((int64_t)rq.row * a.L + l) * a.Hq + hq0) * D;
  v4u qb[2];
#pragma unroll
  for (int ln = 0; ln < 2; ++ln) {
    qb[ln] = v4u{0u, 0u, 0u, 0u};
    if (sub < 2 * G) qb[ln] = *reinterpret_cast<const v4u*>(qrow + (sub % G) * D + 64 * ln + 32 * (sub / G) + 8 * row);
  }
  const float sc = a.scale_log2e;

  float m = kNegBig, lsum = 0.f;  // state of (head sub, lane row); meaningful for sub < G
  float o[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int c = 0; c < 8; ++c) o[g][c] = 0.f;

  const char* kbase = a.base + (int64_t)l * a.stride_layer + (int64_t)h * a.stride_head;
  const char* vbase = kbase + a.stride_kv;
  // A operand of MFMA i: tokens 8*(i/2) .. +7 of the block, line i%2 of their rows;
  // lane row-halves carry the two 64-byte halves of the line (swapped for i >= 2)
  const uint32_t k_off_a = (uint32_t)(sub % 8) * a.stride_slot + (uint32_t)(sub / 8) * 64u + (uint32_t)row * 16u;
  const uint32_t k_off_b = (uint32_t)(8 + sub % 8) * a.stride_slot + (uint32_t)(1 - sub / 8) * 64u + (uint32_t)row * 16u;
  const uint32_t v_off = (uint32_t)(4 * row) * a.stride_slot + (uint32_t)sub * 16u;  // + i*stride_slot
  const char* dummy = reinterpret_cast<const char*>(qrow) + (uint32_t)sub * 16u;     // 256 valid bytes
  const int bp_row = 16 * row * 4;  // ds_bpermute byte address of lane (head 0, this lane's row)
  const int bp_pair = ((lane ^ 32) + G) * 4;   // lane that holds the other half-line's partial scores
  const bool low_rows = row < 2;

  const int n_it = (je - jb - wave + 3) / 4;
  v4u kcs[P][4], vcs[P][4];
  // block ids through scalar loads, two blocks ahead (as in decode_kernel)
  const ConstTable tab = (ConstTable)(a.bt + rq.bt + jb + wave);
  auto block_id = [&](int it) { return tab[4 * min(it, n_it - 1)]; };
  int id_next = 0;
  auto load_k = [&](bool real, int blk_id, v4u* kc) {
    const char* pa = real ? kbase + (int64_t)blk_id * a.stride_block + k_off_a : dummy;
    const char* pb = real ? kbase + (int64_t)blk_id * a.stride_block + k_off_b : dummy;
    const uint32_t stp = real ? 128u : 0u;
    kc[0] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(pa));
    kc[1] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(pa + stp));
    kc[2] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(pb));
    kc[3] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(pb + stp));
  };
  auto load_v = [&](bool real, int blk_id, v4u* vc) {
    const char* p = real ? vbase + (int64_t)blk_id * a.stride_block + v_off : dummy;
    const uint32_t stp = real ? a.stride_slot : 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      vc[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p + i * stp));
  };
  constexpr int kTileLoads = 8 * P;
  constexpr int kWaitAllButTiles = 0x0F70 | (kTileLoads & 15) | ((kTileLoads >> 4) << 14);

  auto step = [&](auto masked_tag, auto slot_tag, int it, int t_limit) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    constexpr int S = decltype(slot_tag)::value;   // register tile that holds block it
    v4u(&kc)[4] = kcs[S];
    v4u(&vc)[4] = vcs[S];
    const bool more = it + P < n_it;
    v4f half[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};   // partial scores of tokens 0..7 and 8..15
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (BF16) {
        typedef __bf16 b8 __attribute__((ext_vector_type(8)));
        half[i / 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, kc[i]),
                                                              __builtin_bit_cast(b8, qb[i % 2]), half[i / 2], 0, 0, 0);
      } else {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        half[i / 2] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, kc[i]),
                                                             __builtin_bit_cast(h8, qb[i % 2]), half[i / 2], 0, 0, 0);
      }
    }
    // Lane (column c, row g) holds rows 4g .. 4g+3 of column c.  The products that
    // pair a half-line with the query dims of the same half sit, for tokens 0..7, in
    // (c < G, g < 2) and (G <= c < 2G, g >= 2), and for tokens 8..15 (halves swapped)
    // in (c < G, g >= 2) and (G <= c < 2G, g < 2): lane (head, g) adds its own part
    // and the part of lane (head + G, g ^ 2), which makes it the owner of tokens
    // 4g .. 4g+3 of the block.
    v4f acc;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float own = low_rows ? half[0][t] : half[1][t];
      const float give = low_rows ? half[1][t] : half[0][t];
      acc[t] = own + __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(bp_pair, __builtin_bit_cast(int, give)));
    }
    __builtin_amdgcn_sched_barrier(0);
    const int id_after = block_id(it + P + 1);
    load_k(more, id_next, kc);
    __builtin_amdgcn_sched_barrier(0);

    // online softmax of (head sub, lane row) over tokens 4*row .. 4*row+3 of the block
    float mx = m;
#pragma unroll
    for (int t = 0; t < 4; ++t)
      if (!MASKED || 4 * row + t < t_limit) mx = fmaxf(mx, acc[t] * sc);
    const float alpha = __builtin_amdgcn_exp2f(m - mx);
    m = mx;
    float p[4], add = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float e = __builtin_amdgcn_exp2f(fmaf(acc[t], sc, -mx));
      p[t] = (!MASKED || 4 * row + t < t_limit) ? e : 0.f;
      add += p[t];
    }
    lsum = lsum * alpha + add;
    // weights and rescale factor of head g: from lane (g, row) to the whole lane row
    float pw[G][4], al[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      al[g] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(bp_row + 4 * g, __builtin_bit_cast(int, alpha)));
#pragma unroll
      for (int t = 0; t < 4; ++t)
        pw[g][t] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(bp_row + 4 * g, __builtin_bit_cast(int, p[t])));
    }
    if (MASKED) {
      // rows past the context may hold anything: clear them so that a zero weight
      // cannot turn a NaN pattern into NaN
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (4 * row + i >= t_limit) vc[i] = v4u{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int c = 0; c < 8; ++c) o[g][c] *= al[g];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float vf[8];
      widen8<BF16>(vc[i], vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) o[g][c] = fmaf(pw[g][i], vf[c], o[g][c]);
    }
    __builtin_amdgcn_sched_barrier(0);
    load_v(more, id_next, vc);
    id_next = id_after;
    __builtin_amdgcn_sched_barrier(0);
  };
  if (n_it > 0) {
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, P - 1>;
#pragma unroll
    for (int j = 0; j < P; ++j) {   // a wave with fewer than P blocks loads its last one twice
      const int idj = block_id(j);
      load_k(true, idj, kcs[j]);
      __builtin_amdgcn_sched_barrier(0);
      load_v(true, idj, vcs[j]);
      __builtin_amdgcn_sched_barrier(0);
    }
    id_next = block_id(P);
    __builtin_amdgcn_s_waitcnt(kWaitAllButTiles);  // queries have arrived
    const int t_last = k - (jb + wave + 4 * (n_it - 1)) * B;
    const int n_main = t_last < B ? n_it - 1 : n_it;
    if constexpr (P == 1) {
      for (int it = 0; it < n_main; ++it) step(std::false_type{}, S0{}, it, B);
      if (n_main < n_it) step(std::true_type{}, S0{}, n_main, t_last);
    } else {
      int it = 0;
      for (; it + 1 < n_main; it += 2) {
        step(std::false_type{}, S0{}, it, B);
        step(std::false_type{}, S1{}, it + 1, B);
      }
      if (it < n_main) step(std::false_type{}, S0{}, it, B);
      if (n_main < n_it) {
        if (n_main & 1) step(std::true_type{}, S1{}, n_main, t_last);
        else step(std::true_type{}, S0{}, n_main, t_last);
      }
    }
  }

  // the state of head g sits in lane (g, row): hand it to all lanes of the row
  float mg[G], lg[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    mg[g] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(bp_row + 4 * g, __builtin_bit_cast(int, m)));
    lg[g] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(bp_row + 4 * g, __builtin_bit_cast(int, lsum)));
  }
  finish_workgroup<D, G, BF16>(a, rq, l, hq0, split, wave, lane, mg, lg, o, s_ws);
}

// Groups of four query heads, scores on the matrix cores, waves sliced by token row
// as in decode_kernel: wave w takes token rows 4w .. 4w+3 of every block and one step
// covers four consecutive blocks.  One v_mfma_f32_16x16x32 then handles the four token
// rows a wave owns in one block, over all 128 dims and all four heads, from ONE load
// instruction that reads the rows' 1 KiB as a contiguous run:
//   lane x = 16g + 4t + p loads the 16 bytes (8 dims) number 4g + p of token row t.
//   As the A operand (row x%16 = 4t + p, k = 8g .. 8g+7) this is a matrix whose row
//   (t, p) holds, of token t, the dims of chunk set p = {p, 4+p, 8+p, 12+p}.
//   The B operand holds in column 4h + p', k = 8g .. 8g+7, the dims of chunk 4g + p'
//   of head h's query: chunk set p' of head h.
//   Element ((t, p), (h, p')) of the product is the partial score of token t and head
//   h over chunk set p when p = p' (a cross product nobody reads otherwise); the
//   sixteen dims chunks are covered by p = 0..3, so the score is the sum of the four
//   diagonal elements.  Lane x of the result holds rows 4(x/16) .. +3 of column x%16,
//   i.e. token row x/16, chunk sets 0..3 in its four registers, for head (x%16)/4 and
//   p' = x%4: register x%4 is the useful one, and the four lanes of a quad add up
//   to the score (four quad-broadcast DPP operations).
// Every lane of quad (token row r, head h) then keeps the online-softmax state of
// that pair; the V rows are loaded one token row per lane row (1 KiB contiguous per
// instruction as well) and P.V stays on the vector unit.  A lane needs the weights
// of all four heads for its token row: they come from the other quads of its lane
// row by DPP row rotations (no LDS round trip), which makes output slot j of a lane
// belong to the head of the quad j places to its left; the end of the kernel sorts
// the slots back by head.
template <int D, int B, bool BF16, int WMAX>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WMAX <= 3 ? 1 : 4, WMAX))) void decode_mfma4_kernel(const DecArgs a) {
  static_assert(D == 128 && B == 16, "shape of the matrix-core variant");
  constexpr int G = 4;
  // Two instances: four waves per SIMD (at most 128 registers) with one tile in flight
  // per wave and per K / V, or three waves per SIMD with two.
  constexpr int P = WMAX <= 3 ? 2 : 1;
  __shared__ WaveStates<D, G> s_ws;

  const WorkItem wi = work_item<B, G>(a);
  if (wi.jb >= wi.je) return;  // empty context or an empty split: uniform over the workgroup
  const DecReq rq = wi.rq;
  const int h = wi.h, l = wi.l, split = wi.split, k = rq.k, jb = wi.jb, je = wi.je;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = lane % 16;
  const int row = lane / 16;
  const int hq0 = wi.hq0;
  if (threadIdx.x == 0) s_ws.done = 0u;
  __syncthreads();

  // B operand: column sub = 4h + p', k slice `row`: dims 8 * (4 * row + p') .. +7 of head h
  const uint16_t* qrow = a.q + (((int64_t)rq.row * a.L + l) * a.Hq + hq0) * D;
  const v4u qb = *reinterpret_cast<const v4u*>(qrow + (sub / 4) * D + 8 * (4 * row + sub % 4));
  const float sc = a.scale_log2e;

  float m = kNegBig, lsum = 0.f;  // state of (head sub / 4, token row `row`), equal over the quad
  float o[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int c = 0; c < 8; ++c) o[g][c] = 0.f;

  const char* kbase = a.base + (int64_t)l * a.stride_layer + (int64_t)h * a.stride_head;
  const char* vbase = kbase + a.stride_kv;
  const uint32_t k_off = (uint32_t)(4 * wave + sub / 4) * a.stride_slot + (uint32_t)(4 * row + sub % 4) * 16u;
  const uint32_t v_off = (uint32_t)(4 * wave + row) * a.stride_slot + (uint32_t)sub * 16u;
  const char* dummy = reinterpret_cast<const char*>(qrow) + (uint32_t)sub * 16u;     // 256 valid bytes
  // Slot j of this lane's output state belongs to the head of the quad j places to the
  // left in the lane row (cyclically): the weights of that head reach the lane through
  // a rotation of the row by 4j lanes (DPP, no LDS round trip), and so does the head's
  // number, which is what tells the end of the kernel where slot j goes.
  auto rot = [](float v, auto quads) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + 4 * decltype(quads)::value, 0xF, 0xF, true));
  };
  using Q1 = std::integral_constant<int, 1>;
  using Q2 = std::integral_constant<int, 2>;
  using Q3 = std::integral_constant<int, 3>;
  auto rot4 = [&](float v, float (&out)[4]) {
    out[0] = v;
    out[1] = rot(v, Q1{});
    out[2] = rot(v, Q2{});
    out[3] = rot(v, Q3{});
  };

  const int nblk = je - jb;
  const int n_it = (nblk + 3) / 4;
  v4u kcs[P][4], vcs[P][4];
  const ConstTable tab = (ConstTable)(a.bt + rq.bt + jb);
  struct Ids { int v[4]; int first, dist; };   // ids, entry of instruction 0, distance to the next (step_first_entry)
  auto block_ids = [&](int it) {
    Ids r;
    r.first = step_first_entry(min(it, n_it - 1), nblk, a.spread_log2, r.dist);
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = tab[min(r.first + i * r.dist, nblk - 1)];
    return r;
  };
  // tile of step `it`: instruction i reads the wave's rows of block 4*it + i, or the
  // query row (valid, cached) where the range has no such block
  auto load_tile = [&](int it, const char* base, uint32_t off, const Ids& ids, v4u* td) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const char* p = it < n_it && ids.first + i * ids.dist < nblk ? base + (int64_t)ids.v[i] * a.stride_block + off : dummy;
      td[i] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
    }
  };
  constexpr int kTileLoads = 8 * P;
  constexpr int kWaitAllButTiles = 0x0F70 | (kTileLoads & 15) | ((kTileLoads >> 4) << 14);
  Ids id_next = {};

  auto step = [&](auto masked_tag, auto slot_tag, int it) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    constexpr int S = decltype(slot_tag)::value;   // register tile that holds step it
    v4u(&kc)[4] = kcs[S];
    v4u(&vc)[4] = vcs[S];
    // context rows of block 4*it + i, counted from this wave's first row
    int lim[4];
    int e_dist = 1;
    const int e_first = MASKED ? step_first_entry(it, nblk, a.spread_log2, e_dist) : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int bi = e_first + i * e_dist;
      lim[i] = !MASKED ? 4 : (bi < nblk ? min(B, k - (jb + bi) * B) - 4 * wave : 0);
    }
    float s[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v4f d = {0.f, 0.f, 0.f, 0.f};
      if (BF16) {
        typedef __bf16 b8 __attribute__((ext_vector_type(8)));
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, kc[i]), __builtin_bit_cast(b8, qb), d, 0, 0, 0);
      } else {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        d = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, kc[i]), __builtin_bit_cast(h8, qb), d, 0, 0, 0);
      }
      // lane p' of the quad contributes its register p'
      auto bcast = [](float v, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value, 0xF, 0xF, true));
      };
      s[i] = bcast(d[0], std::integral_constant<int, 0x00>{}) + bcast(d[1], std::integral_constant<int, 0x55>{}) +
             bcast(d[2], std::integral_constant<int, 0xAA>{}) + bcast(d[3], std::integral_constant<int, 0xFF>{});
    }
    __builtin_amdgcn_sched_barrier(0);
    const Ids id_after = block_ids(it + P + 1);
    load_tile(it + P, kbase, k_off, id_next, kc);
    __builtin_amdgcn_sched_barrier(0);

    // online softmax of (head sub / 4, token row `row`) over the step's four blocks
    float mx = m;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (!MASKED || row < lim[i]) mx = fmaxf(mx, s[i] * sc);
    const float alpha = __builtin_amdgcn_exp2f(m - mx);
    m = mx;
    float p[4], add = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float e = __builtin_amdgcn_exp2f(fmaf(s[i], sc, -mx));
      p[i] = (!MASKED || row < lim[i]) ? e : 0.f;
      add += p[i];
    }
    lsum = lsum * alpha + add;
    // weights of the four heads for this lane's token row: slot j from the quad j to the left
    float pw[4][G];
#pragma unroll
    for (int i = 0; i < 4; ++i) rot4(p[i], pw[i]);
    // the accumulators only need rescaling when some running maximum of the wave moved
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
      float al[G];
      rot4(alpha, al);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) o[g][c] *= al[g];
    }
    if (MASKED) {
      // rows past the context may hold anything: clear them so that a zero weight
      // cannot turn a NaN pattern into NaN
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (row >= lim[i]) vc[i] = v4u{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float vf[8];
      widen8<BF16>(vc[i], vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < 8; ++c) o[g][c] = fmaf(pw[i][g], vf[c], o[g][c]);
    }
    __builtin_amdgcn_sched_barrier(0);
    load_tile(it + P, vbase, v_off, id_next, vc);
    id_next = id_after;
    __builtin_amdgcn_sched_barrier(0);
  };
  {
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, P - 1>;
#pragma unroll
    for (int j = 0; j < P; ++j) {
      const Ids idj = block_ids(j);
      load_tile(j, kbase, k_off, idj, kcs[j]);
      __builtin_amdgcn_sched_barrier(0);
      load_tile(j, vbase, v_off, idj, vcs[j]);
      __builtin_amdgcn_sched_barrier(0);
    }
    id_next = block_ids(P);
    __builtin_amdgcn_s_waitcnt(kWaitAllButTiles);  // queries have arrived
    const int n_full = min(nblk, (k - jb * B) / B);   // full blocks of the range
    const int n_main = n_full / 4;                    // steps whose rows are all context
    if constexpr (P == 1) {
      for (int it = 0; it < n_main; ++it) step(std::false_type{}, S0{}, it);
      if (n_main < n_it) step(std::true_type{}, S0{}, n_main);
    } else {
      int it = 0;
      for (; it + 1 < n_main; it += 2) {
        step(std::false_type{}, S0{}, it);
        step(std::false_type{}, S1{}, it + 1);
      }
      if (it < n_main) step(std::false_type{}, S0{}, it);
      if (n_main < n_it) {
        if (n_main & 1) step(std::true_type{}, S1{}, n_main);
        else step(std::true_type{}, S0{}, n_main);
      }
    }
  }

  // running maximum, sum and head number of every slot, by the same rotations
  float mg[G], lg[G], hf[G];
  rot4(m, mg);
  rot4(lsum, lg);
  rot4((float)(sub / 4), hf);
  int head_of[G];
#pragma unroll
  for (int g = 0; g < G; ++g) head_of[g] = (int)hf[g];
  finish_workgroup<D, G, BF16>(a, rq, l, hq0, split, wave, lane, mg, lg, o, s_ws, head_of);
}

// Log-sum-exp merge of the context splits, in split order.
template <int D, int B, bool BF16>
__global__ __launch_bounds__(D) void merge_kernel(const DecArgs a) {
  const int hq = blockIdx.x, l = blockIdx.y;
  const DecReq rq = a.req[blockIdx.z];
  if (rq.k <= 0) return;
  const int nb = (rq.k + B - 1) / B;
  const int per = (nb + a.n_splits - 1) / a.n_splits;
  const int n_eff = (nb + per - 1) / per;  // splits that saw at least one block
  const int d = threadIdx.x;
  float mx = kNegBig;
  for (int s = 0; s < n_eff; ++s) mx = fmaxf(mx, ws_entry(a.ws, a, rq.slot, l, hq, s, D)[D]);
  float acc = 0.f, den = 0.f;
  for (int s = 0; s < n_eff; ++s) {
    const float* e = ws_entry(a.ws, a, rq.slot, l, hq, s, D);
    const float wgt = __builtin_amdgcn_exp2f(e[D] - mx);
    acc = fmaf(e[d], wgt, acc);
    den = fmaf(e[D + 1], wgt, den);
  }
  const float res = acc / den;
  const int64_t oi = (((int64_t)rq.row * a.L + l) * a.Hq + hq) * D + d;
  if (a.out_f32)
    reinterpret_cast<float*>(a.out)[oi] = res;
  else
    reinterpret_cast<uint16_t*>(a.out)[oi] = narrow<BF16>(res);
}

// Fallback for shapes the tiled kernel is not instantiated for (any block size,
// head_dim a multiple of 8 up to 512): one wave per (request, layer, query head),
// one token per iteration, lane c owning dims 8c..8c+7 of the row.  Correct and
// in bounds for every layout the descriptor can express, not tuned.
template <bool BF16>
__global__ __launch_bounds__(64) void decode_generic_kernel(const DecArgs a, int D, int B) {
  const int hq = blockIdx.x, l = blockIdx.y;
  const DecReq rq = a.req[blockIdx.z];
  const int k = rq.k;
  if (k <= 0) return;
  const int lane = threadIdx.x;
  const bool active = lane < D / 8;
  const int h = hq / (a.Hq / a.H);
  uint32_t qv[4] = {0u, 0u, 0u, 0u};
  if (active) {
    const uint16_t* qptr = a.q + (((int64_t)rq.row * a.L + l) * a.Hq + hq) * D + lane * 8;
    const v4u raw = *reinterpret_cast<const v4u*>(qptr);
#pragma unroll
    for (int c = 0; c < 4; ++c) qv[c] = raw[c];
  }
  const char* kbase = a.base + (int64_t)l * a.stride_layer + (int64_t)h * a.stride_head + lane * 16;
  const char* vbase = kbase + a.stride_kv;
  float m = kNegBig, lsum = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int t = 0; t < k; ++t) {
    const int64_t blk = a.bt[rq.bt + t / B];
    const int64_t off = blk * a.stride_block + (int64_t)(t % B) * a.stride_slot;
    v4u kr = {0u, 0u, 0u, 0u}, vr = {0u, 0u, 0u, 0u};
    if (active) {
      kr = *reinterpret_cast<const v4u*>(kbase + off);
      vr = *reinterpret_cast<const v4u*>(vbase + off);
    }
    float s = dot8<BF16>(qv, kr);
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) s += __shfl_xor(s, d);
    s *= a.scale_log2e;
    const float mx = fmaxf(m, s);
    const float alpha = __builtin_amdgcn_exp2f(m - mx), p = __builtin_amdgcn_exp2f(s - mx);
    m = mx;
    lsum = lsum * alpha + p;
    float vf[8];
    widen8<BF16>(vr, vf);
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = fmaf(p, vf[c], o[c] * alpha);
  }
  if (active) {
    const int64_t oi = (((int64_t)rq.row * a.L + l) * a.Hq + hq) * D + lane * 8;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float res = o[c] / lsum;
      if (a.out_f32)
        reinterpret_cast<float*>(a.out)[oi + c] = res;
      else
        reinterpret_cast<uint16_t*>(a.out)[oi + c] = narrow<BF16>(res);
    }
  }
}

struct DecodePlan {
  int g_tile;    // query heads per workgroup (1, 2, 4 or 8)
  int passes;    // workgroups per KV head
  int n_splits;
  bool cap;      // at most two waves per SIMD
  bool mfma;     // scores on the matrix cores (groups of four and eight, head_dim 128, 16-token blocks)
};

static DecodePlan plan_decode(const kvm_layout& l, int n_req, int max_nb) {
  DecodePlan p;
  const int G = l.n_q_heads / l.n_kv_heads;
  // eight query heads per KV head are served from one pass over K and V (two
  // passes of four would read them twice)
  p.g_tile = G % 8 == 0 ? 8 : (G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1));
  p.passes = G / p.g_tile;
  const Options& o = options();
  int s = 1;
  if (o.decode_force_splits > 0) {
    s = o.decode_force_splits;
  } else {
    // Fill 256 CUs (x4 resident workgroups) when the batch alone cannot, but
    // keep at least 16 blocks (4 per wave) in every split.
    const int64_t base = (int64_t)n_req * l.n_layers * l.n_kv_heads * p.passes;
    const int64_t want = base > 0 ? ceil_div(o.decode_split_target, base) : 1;
    const int64_t room = max_nb / 16;
    s = (int)std::max<int64_t>(1, std::min<int64_t>(want, room));
    s = std::min(s, o.decode_max_splits);
  }
  p.n_splits = std::max(1, std::min(s, 64));
  p.cap = false;
  p.mfma = false;
  return p;
}

static int64_t ws_bytes_for(const kvm_layout& l, int n_req, int n_splits) {
  return (int64_t)n_req * l.n_layers * l.n_q_heads * n_splits * (l.head_dim + 2) * 4;
}

template <int D, int B, bool BF16, int WMAX>
static void launch_main(const DecArgs& a, const DecodePlan& p, const dim3 grid, hipStream_t st) {
  if constexpr (D == 128 && B == 16) {
    if (p.mfma && p.g_tile == 8) {
      hipLaunchKernelGGL((decode_mfma_kernel<D, B, 8, BF16, WMAX>), grid, dim3(256), 0, st, a);
      return;
    }
    if (p.mfma && p.g_tile == 4) {
      hipLaunchKernelGGL((decode_mfma4_kernel<D, B, BF16, (WMAX == 2 ? 3 : 8)>), grid, dim3(256), 0, st, a);
      return;
    }
  }
  switch (p.g_tile) {
    case 8: hipLaunchKernelGGL((decode_kernel<D, B, 8, BF16, WMAX>), grid, dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL((decode_kernel<D, B, 4, BF16, WMAX>), grid, dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL((decode_kernel<D, B, 2, BF16, WMAX>), grid, dim3(256), 0, st, a); break;
    default: hipLaunchKernelGGL((decode_kernel<D, B, 1, BF16, WMAX>), grid, dim3(256), 0, st, a); break;
  }
}

template <int D, int B, bool BF16>
static hipError_t launch_decode(const DecArgs& a, const DecodePlan& p, int n_req, hipStream_t st) {
  const dim3 grid(a.H * p.passes, a.L, n_req * p.n_splits);
  if (p.cap) launch_main<D, B, BF16, 2>(a, p, grid, st);
  else launch_main<D, B, BF16, 8>(a, p, grid, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.n_splits == 1) return e;
  hipLaunchKernelGGL((merge_kernel<D, B, BF16>), dim3(a.Hq, a.L, n_req), dim3(D), 0, st, a);
  return hipGetLastError();
}

}  // namespace kvm

using namespace kvm;

// ---- static scratch of kvm_paged_decode_static -------------------------------
// One file-scope device array per GPU (every device that loads the library holds
// its own copy until the process ends) stands in for the caller's context-split
// workspace.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the device address is looked up once per device, with that
// device current, and that pointer is what the kernels receive.
// The split kernels write every workspace entry the merge kernel reads (a split
// that sees no block is skipped by both), so nothing has to be cleared between
// calls; calls that overlap in time on one GPU would share the entries and race.
// No `used` attribute here: the compiler gives a static device variable that host
// code names an externally visible device symbol, which is what the runtime looks
// up; with the attribute the symbol stays local and the lookup cannot find it.
static __device__ __align__(256) unsigned char scratch[KVM_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch`, per device

static int static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(KVM_EHIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(KVM_EINVAL, "kvm_paged_decode_static: device index out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(KVM_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return KVM_OK;
}

// Body of kvm_paged_decode and kvm_paged_decode_static.  With `static_scratch`
// the context-split workspace is the library's own file-scope device array and
// nothing is allocated; a plan whose workspace would not fit it is an error.
static int decode_impl(const kvm_pool* pool, const kvm_batch* reqs, const int32_t* rows, const void* q_dev,
                       void* out_dev, int out_is_f32, float scale, void* workspace_dev,
                       int64_t workspace_bytes, bool static_scratch, void* hip_stream) {
  clear_error();
  BatchView v;
  int rc = validate_side(static_scratch ? "kvm_paged_decode_static" : "kvm_paged_decode", pool, reqs,
                         false, &v);
  if (rc) return rc;
  for (int r = 0; r < v.n_req; ++r)
    if (v.start[r] != 0) return fail(KVM_EINVAL, "kvm_paged_decode: reqs->start must be NULL or zero");
  if (v.n_req == 0 || v.total_blocks == 0) return KVM_OK;
  if (rows) {
    // rows of requests that produce output must be non-negative and distinct
    std::vector<int32_t> used;
    for (int r = 0; r < v.n_req; ++r)
      if (v.k[r] > 0) {
        if (rows[r] < 0) return fail(KVM_EINVAL, "kvm_paged_decode_rows: negative row");
        used.push_back(rows[r]);
      }
    std::sort(used.begin(), used.end());
    if (std::adjacent_find(used.begin(), used.end()) != used.end())
      return fail(KVM_EINVAL, "kvm_paged_decode_rows: two requests share an output row");
  }
  if (!q_dev || !out_dev) return fail(KVM_EINVAL, "kvm_paged_decode: q_dev or out_dev is NULL");
  if ((uintptr_t)q_dev % 16 || (uintptr_t)out_dev % 4)
    return fail(KVM_EINVAL, "kvm_paged_decode: q_dev must be 16-byte and out_dev 4-byte aligned");
  if (!(scale >= 0.f) || !std::isfinite(scale))
    return fail(KVM_EINVAL, "kvm_paged_decode: scale must be finite and >= 0");
  const kvm_layout& l = pool->layout;
  const bool tiled = l.block_tokens == 16 && (l.head_dim == 64 || l.head_dim == 128);
  if (l.head_dim > 512)
    return fail(KVM_EINVAL, "kvm_paged_decode: supported shapes have head_dim <= 512");
  int max_nb = 0;
  for (int r = 0; r < v.n_req; ++r) max_nb = std::max(max_nb, v.nb[r]);
  DecodePlan p = plan_decode(l, v.n_req, max_nb);
  if (!tiled) p.n_splits = 1;  // the fallback kernel does not split contexts
  if (static_scratch && p.n_splits > 1) {
    // the plan the automatic split count asks for must fit the static array
    const int64_t need = ws_bytes_for(l, v.n_req, p.n_splits);
    if (need > (int64_t)KVM_STATIC_SCRATCH_BYTES) {
      char buf[160];
      snprintf(buf, sizeof buf,
               "kvm_paged_decode_static: the batch needs %lld bytes of split workspace, the static "
               "scratch holds %lld",
               (long long)need, (long long)KVM_STATIC_SCRATCH_BYTES);
      return fail(KVM_EINVAL, buf);
    }
    rc = static_scratch_ptr(&workspace_dev);
    if (rc) return rc;
    workspace_bytes = KVM_STATIC_SCRATCH_BYTES;
  }
  if (p.n_splits > 1) {
    // an absent or short workspace only limits how far the context is split
    const int64_t per_split = ws_bytes_for(l, v.n_req, 1);
    int64_t fit = (workspace_dev && (uintptr_t)workspace_dev % 16 == 0) ? workspace_bytes / per_split : 0;
    if (fit < 2) fit = 1;
    p.n_splits = (int)std::min<int64_t>(p.n_splits, fit);
  }

  {
    // Which instance runs, by group width and mean context per workgroup (measured
    // on MI355X with equal-length batches, GB/s of KV read; "capped" = at most two
    // waves per SIMD, which also leaves the registers for two tiles in flight):
    //  - vector kernel, one head per KV head: capped wins from 16 blocks per workgroup
    //    on (32 blocks: 6640 against 6370, 128: 6600 against 6470), uncapped below
    //    (8 blocks: 6280 against 5660, 4 blocks: 5970 against 4110);
    //  - groups of four and of eight run with the scores on the matrix cores at every
    //    length (groups of four, 60 blocks: 6220 against 5370 for the vector kernel,
    //    2048 blocks: 6280 against 6150); the kernel for groups of four is never capped
    //    (16 blocks: 5920 against 5730, 128 blocks: 6320 against 6260).
    // "decode.cap_waves" (0 never, 1 always) and "decode.mfma" (0 never, 1 always)
    // override.
    int64_t live = 0;
    for (int r = 0; r < v.n_req; ++r) live += v.nb[r] > 0;
    const int64_t mean_blocks = v.total_blocks / std::max<int64_t>(1, live * p.n_splits);
    const int cap_mode = options().decode_cap_waves, mfma_mode = options().decode_mfma;
    p.mfma = l.head_dim == 128 && l.block_tokens == 16 && (p.g_tile == 8 || p.g_tile == 4) && mfma_mode != 0;
    p.cap = cap_mode < 0 ? (mean_blocks >= 12 && !(p.mfma && p.g_tile == 4)) : cap_mode != 0;
  }

  DecArgs a;
  memset(&a, 0, sizeof a);
  a.base = (const char*)pool->base;
  a.bt = reqs->bt_blocks_dev;
  a.stride_layer = l.stride_layer * 2;
  a.stride_kv = l.stride_kv * 2;
  a.stride_block = l.stride_block * 2;
  a.stride_head = (uint32_t)(l.stride_head * 2);
  a.stride_slot = (uint32_t)(l.stride_slot * 2);
  a.q = (const uint16_t*)q_dev;
  a.out = out_dev;
  a.ws = (float*)workspace_dev;
  a.L = l.n_layers;
  a.H = l.n_kv_heads;
  a.Hq = l.n_q_heads;
  a.passes = p.passes;
  {
    // the four blocks of a step about 1 MiB apart when block ids are consecutive
    // (step_first_entry); option "decode.spread" overrides (log2 of the entry distance)
    int lg = 0;
    while (lg < 6 && (a.stride_block << (lg + 1)) <= (1 << 20)) ++lg;
    if (a.stride_block <= 0 || a.stride_block > (1 << 20)) lg = 0;
    a.spread_log2 = options().decode_spread >= 0 ? options().decode_spread : lg;
  }
  a.n_splits = p.n_splits;
  a.out_f32 = out_is_f32 ? 1 : 0;
  const float sc = scale == 0.f ? 1.0f / std::sqrt((float)l.head_dim) : scale;
  a.scale_log2e = sc * 1.4426950408889634f;

  // Longest context first: workgroups are dispatched in grid order, so the long
  // requests start early and the short ones fill the tail of the launch.  Every
  // request keeps its own reduction order, so results do not depend on this.
  std::vector<int> order(v.n_req);
  for (int r = 0; r < v.n_req; ++r) order[r] = r;
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return v.k[x] > v.k[y]; });

  for (int r0 = 0; r0 < v.n_req; r0 += kMaxReqPerLaunch) {
    const int n = std::min(kMaxReqPerLaunch, v.n_req - r0);
    for (int i = 0; i < n; ++i) {
      const int r = order[r0 + i];
      a.req[i].bt = v.bt_off[r];
      a.req[i].k = v.k[r];
      a.req[i].row = rows ? rows[r] : r;
      a.req[i].slot = r;
    }
    hipError_t e;
    const hipStream_t st = (hipStream_t)hip_stream;
    const bool bf = l.dtype == KVM_BF16;
    if (!tiled) {
      const dim3 grid(a.Hq, a.L, n);
      if (bf)
        hipLaunchKernelGGL(decode_generic_kernel<true>, grid, dim3(64), 0, st, a, l.head_dim, l.block_tokens);
      else
        hipLaunchKernelGGL(decode_generic_kernel<false>, grid, dim3(64), 0, st, a, l.head_dim, l.block_tokens);
      e = hipGetLastError();
    } else if (l.head_dim == 128) {
      e = bf ? launch_decode<128, 16, true>(a, p, n, st) : launch_decode<128, 16, false>(a, p, n, st);
    } else {
      e = bf ? launch_decode<64, 16, true>(a, p, n, st) : launch_decode<64, 16, false>(a, p, n, st);
    }
    if (e != hipSuccess) return fail(KVM_EHIP, hipGetErrorString(e));
  }
  return KVM_OK;
}

extern "C" {

int64_t kvm_decode_workspace_bytes(const kvm_layout* layout, const kvm_batch* reqs) {
  if (!layout_ok(layout, nullptr) || !reqs || reqs->n_req < 0 || (reqs->n_req > 0 && !reqs->k))
    return -1;
  int max_nb = 0;
  for (int r = 0; r < reqs->n_req; ++r)
    max_nb = std::max<int64_t>(max_nb, ceil_div(std::max(reqs->k[r], 0), layout->block_tokens));
  const DecodePlan p = plan_decode(*layout, reqs->n_req, max_nb);
  const bool tiled = layout->block_tokens == 16 && (layout->head_dim == 64 || layout->head_dim == 128);
  return tiled && p.n_splits > 1 ? ws_bytes_for(*layout, reqs->n_req, p.n_splits) : 0;
}

int kvm_paged_decode(const kvm_pool* pool, const kvm_batch* reqs, const void* q_dev, void* out_dev,
                     int out_is_f32, float scale, void* workspace_dev, int64_t workspace_bytes,
                     void* hip_stream) {
  return decode_impl(pool, reqs, nullptr, q_dev, out_dev, out_is_f32, scale, workspace_dev, workspace_bytes,
                     /*static_scratch=*/false, hip_stream);
}

int kvm_paged_decode_rows(const kvm_pool* pool, const kvm_batch* reqs, const int32_t* rows,
                          const void* q_dev, void* out_dev, int out_is_f32, float scale,
                          void* workspace_dev, int64_t workspace_bytes, void* hip_stream) {
  return decode_impl(pool, reqs, rows, q_dev, out_dev, out_is_f32, scale, workspace_dev, workspace_bytes,
                     /*static_scratch=*/false, hip_stream);
}

int kvm_paged_decode_static(const kvm_pool* pool, const kvm_batch* reqs, const void* q_dev, void* out_dev,
                            int out_is_f32, float scale, void* hip_stream) {
  return decode_impl(pool, reqs, nullptr, q_dev, out_dev, out_is_f32, scale, nullptr, 0,
                     /*static_scratch=*/true, hip_stream);
}

}  // extern "C"
