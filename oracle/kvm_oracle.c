/*
 * kvm_oracle.c - TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow CPU statement of what paged-KV migration and paged decode
 * attention compute, written from arXiv 2501.06709 and used only by the test
 * suite, the smoke check and the benchmark's cpu_baseline leg.  It shares no
 * code, header or table with the HIP library and is never called by it.
 *
 * What the paper fixes (own words):
 *  - Sec. "Background & Related Work": the KV cache holds keys and values of
 *    all earlier tokens of a request for every layer and may be stored in
 *    non-contiguous fixed-size pages reached through a block table.
 *  - Sec. "Motivation", Finding 4 and Sec. "Adaptive Request Migration",
 *    "Hybrid Migration": a request can be migrated by copying its KV cache to
 *    the other GPU; the cache is append-only so an already copied prefix stays
 *    valid; the remaining tokens may instead be sent as ids and re-prefilled.
 *  - Sec. "Adaptive Request Migration", "Boundary Profiling": the source copy
 *    stays allocated until the transfer has finished, i.e. migration reads the
 *    source and never modifies it.
 *  - Sec. "System Model": KV bytes of a request are linear in its token count.
 *
 * Migration is therefore a definition, not an approximation; every function
 * below is that definition walked one 16-bit element at a time.  Attention is
 * the textbook scaled-dot-product form in double precision (the paper gives no
 * formula of its own for the decode step).
 *
 * Pool addressing used here: element (layer l, kv, block b, head h, slot s,
 * dim d) is pool[l*st[0] + kv*st[1] + b*st[2] + h*st[3] + s*st[4] + d] with
 * `pool` a uint16_t array and st[] strides in elements.
 * Block tables are CSR: request r owns blocks[off[r] .. off[r+1]).
 *
 * Parity pins for every function are in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

static int64_t pool_index(const int64_t* st, int l, int kv, int64_t b, int h, int s, int d) {
  return (int64_t)l * st[0] + (int64_t)kv * st[1] + b * st[2] + (int64_t)h * st[3] +
         (int64_t)s * st[4] + d;
}

/* Bytes of KV per token: layers x {K,V} x heads x dim x 2-byte elements
 * (Sec. "System Model": size linear in tokens; Sec. "Motivation" worked value
 * for a 4096-token request). */
int64_t orc_bytes_per_token(int L, int H, int D) { return (int64_t)L * 2 * H * D * 2; }

/* Fused migration: logical token t of request r keeps its logical index and
 * changes only its physical block.  Tokens [start[r], k[r]) are moved: start = 0
 * is a whole prefix; start > 0 is one round of a live migration in which an
 * earlier round moved [0,start) (the cache is append-only, so that part is still
 * valid: Sec. "Background & Related Work" on live migration, Sec. "Motivation",
 * Finding 4).  Layers [l_begin, l_end) are processed so that a caller may hand
 * disjoint layer ranges to several threads. */
void orc_migrate(const uint16_t* src, const int64_t* src_st, uint16_t* dst, const int64_t* dst_st,
                 int L, int H, int D, int B, int n_req, const int32_t* src_off,
                 const int32_t* src_blocks, const int32_t* dst_off, const int32_t* dst_blocks,
                 const int32_t* k, const int32_t* start, int l_begin, int l_end) {
  (void)L;
  for (int r = 0; r < n_req; ++r)
    for (int l = l_begin; l < l_end; ++l)
      for (int kv = 0; kv < 2; ++kv)
        for (int t = start[r]; t < k[r]; ++t) {
          int64_t bs = src_blocks[src_off[r] + t / B];
          int64_t bd = dst_blocks[dst_off[r] + t / B];
          for (int h = 0; h < H; ++h)
            for (int d = 0; d < D; ++d)
              dst[pool_index(dst_st, l, kv, bd, h, t % B, d)] =
                  src[pool_index(src_st, l, kv, bs, h, t % B, d)];
        }
}

/* Staging index of (request r, layer l, kv, head h, moved token number u, dim
 * d): requests concatenated in batch order, each [layer][kv][head][token][dim]
 * over exactly its n = k[r] - start[r] moved tokens, u = t - start[r]. */
static int64_t stage_index(int64_t req_base, int H, int D, int n, int l, int kv, int h, int u,
                           int d) {
  return req_base + ((((int64_t)l * 2 + kv) * H + h) * n + u) * D + d;
}

void orc_pack(const uint16_t* src, const int64_t* src_st, uint16_t* stage, int L, int H, int D,
              int B, int n_req, const int32_t* off, const int32_t* blocks, const int32_t* k,
              const int32_t* start, int l_begin, int l_end) {
  int64_t req_base = 0;
  for (int r = 0; r < n_req; ++r) {
    int n = k[r] - start[r];
    for (int l = l_begin; l < l_end; ++l)
      for (int kv = 0; kv < 2; ++kv)
        for (int h = 0; h < H; ++h)
          for (int t = start[r]; t < k[r]; ++t) {
            int64_t b = blocks[off[r] + t / B];
            for (int d = 0; d < D; ++d)
              stage[stage_index(req_base, H, D, n, l, kv, h, t - start[r], d)] =
                  src[pool_index(src_st, l, kv, b, h, t % B, d)];
          }
    req_base += (int64_t)n * L * 2 * H * D;
  }
}

void orc_unpack(const uint16_t* stage, uint16_t* dst, const int64_t* dst_st, int L, int H, int D,
                int B, int n_req, const int32_t* off, const int32_t* blocks, const int32_t* k,
                const int32_t* start, int l_begin, int l_end) {
  int64_t req_base = 0;
  for (int r = 0; r < n_req; ++r) {
    int n = k[r] - start[r];
    for (int l = l_begin; l < l_end; ++l)
      for (int kv = 0; kv < 2; ++kv)
        for (int h = 0; h < H; ++h)
          for (int t = start[r]; t < k[r]; ++t) {
            int64_t b = blocks[off[r] + t / B];
            for (int d = 0; d < D; ++d)
              dst[pool_index(dst_st, l, kv, b, h, t % B, d)] =
                  stage[stage_index(req_base, H, D, n, l, kv, h, t - start[r], d)];
          }
    req_base += (int64_t)n * L * 2 * H * D;
  }
}

/* Exact widening of a 16-bit float pattern to double.
 * dtype 0: IEEE binary16 (1 sign, 5 exponent, 10 fraction bits).
 * dtype 1: bfloat16 (the upper half of an IEEE binary32). */
double orc_widen(uint16_t bits, int dtype) {
  int sign = bits >> 15;
  int ebits = dtype == 0 ? 5 : 8, fbits = dtype == 0 ? 10 : 7;
  int bias = (1 << (ebits - 1)) - 1;
  int e = (bits >> fbits) & ((1 << ebits) - 1);
  int f = bits & ((1 << fbits) - 1);
  double v;
  if (e == (1 << ebits) - 1)
    v = f ? NAN : INFINITY;
  else if (e == 0)
    v = ldexp((double)f, 1 - bias - fbits); /* subnormal or zero */
  else
    v = ldexp((double)((1 << fbits) | f), e - bias - fbits);
  return sign ? -v : v;
}

/* Paged decode attention in double precision.
 * q:   [n_req][L][Hq][D] 16-bit patterns of `dtype`.
 * out: [n_req][L][Hq][D] doubles.  Rows of a request with k[r] = 0 are left
 * untouched.  Query head hq reads KV head hq / (Hq/H).  scale multiplies the
 * dot products (callers pass 1/sqrt(D)). */
void orc_paged_decode(const uint16_t* pool, const int64_t* st, int L, int H, int Hq, int D, int B,
                      int dtype, int n_req, const int32_t* off, const int32_t* blocks,
                      const int32_t* k, const uint16_t* q, double* out, double scale) {
  int group = Hq / H;
  for (int r = 0; r < n_req; ++r) {
    int n = k[r];
    if (n <= 0) continue;
    double* s = (double*)malloc(sizeof(double) * (size_t)n);
    for (int l = 0; l < L; ++l)
      for (int hq = 0; hq < Hq; ++hq) {
        int g = hq / group;
        const uint16_t* qrow = q + (((int64_t)r * L + l) * Hq + hq) * D;
        double* orow = out + (((int64_t)r * L + l) * Hq + hq) * D;
        double m = -INFINITY;
        for (int t = 0; t < n; ++t) {
          int64_t b = blocks[off[r] + t / B];
          double acc = 0.0;
          for (int d = 0; d < D; ++d)
            acc += orc_widen(qrow[d], dtype) *
                   orc_widen(pool[pool_index(st, l, 0, b, g, t % B, d)], dtype);
          s[t] = acc * scale;
          if (s[t] > m) m = s[t];
        }
        double z = 0.0;
        for (int t = 0; t < n; ++t) {
          s[t] = exp(s[t] - m);
          z += s[t];
        }
        for (int d = 0; d < D; ++d) orow[d] = 0.0;
        for (int t = 0; t < n; ++t) {
          int64_t b = blocks[off[r] + t / B];
          double p = s[t] / z;
          for (int d = 0; d < D; ++d)
            orow[d] += p * orc_widen(pool[pool_index(st, l, 1, b, g, t % B, d)], dtype);
        }
      }
    free(s);
  }
}
