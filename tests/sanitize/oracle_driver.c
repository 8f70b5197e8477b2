/* Seeded random driver over the C oracle (copy and decode functions) with buffers of
 * exactly the size the calls need, built by tests/test_sanitizers.py with
 * -fsanitize=address,undefined: an access outside them ends the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void orc_migrate(const uint16_t*, const int64_t*, uint16_t*, const int64_t*, int, int, int, int, int,
                 const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*,
                 const int32_t*, int, int);
void orc_pack(const uint16_t*, const int64_t*, uint16_t*, int, int, int, int, int, const int32_t*,
              const int32_t*, const int32_t*, const int32_t*, int, int);
void orc_unpack(const uint16_t*, uint16_t*, const int64_t*, int, int, int, int, int, const int32_t*,
                const int32_t*, const int32_t*, const int32_t*, int, int);
void orc_paged_decode(const uint16_t*, const int64_t*, int, int, int, int, int, int, int, const int32_t*,
                      const int32_t*, const int32_t*, const uint16_t*, double*, double);
double orc_widen(uint16_t, int);

int main(void) {
  srand(20250106);
  for (int trial = 0; trial < 300; ++trial) {
    int L = 1 + rand() % 3, H = 1 + rand() % 3, G = 1 + rand() % 3, D = 8, B = 4;
    int nblk = 8 + rand() % 8, nreq = 1 + rand() % 3, dtype = rand() % 2;
    int64_t st[5] = {2LL * nblk * H * B * D, (int64_t)nblk * H * B * D, (int64_t)H * B * D, B * D, D};
    size_t n = (size_t)L * 2 * nblk * H * B * D;
    uint16_t* src = malloc(n * 2);
    uint16_t* dst = malloc(n * 2);
    for (size_t i = 0; i < n; ++i) {
      src[i] = (uint16_t)(0x3800 + rand() % 0x400);
      dst[i] = (uint16_t)rand();
    }
    int32_t off[4] = {0}, blocks[16], k[3], start[3], perm[16];
    for (int i = 0; i < nblk; ++i) perm[i] = i;
    for (int i = nblk - 1; i > 0; --i) {
      int j = rand() % (i + 1), t = perm[i];
      perm[i] = perm[j];
      perm[j] = t;
    }
    int used = 0;
    long tokens = 0;
    for (int r = 0; r < nreq; ++r) {
      int nb = 1 + rand() % 2;
      if (used + nb > nblk) nb = 0;
      for (int j = 0; j < nb; ++j) blocks[used + j] = perm[used + j];
      used += nb;
      off[r + 1] = used;
      k[r] = nb ? rand() % (nb * B + 1) : 0;
      start[r] = k[r] ? rand() % (k[r] + 1) : 0;
      tokens += k[r] - start[r];
    }
    size_t ns = (size_t)tokens * L * 2 * H * D;
    uint16_t* stage = malloc(ns * 2 + 2);
    orc_migrate(src, st, dst, st, L, H, D, B, nreq, off, blocks, off, blocks, k, start, 0, L);
    orc_pack(src, st, stage, L, H, D, B, nreq, off, blocks, k, start, 0, L);
    orc_unpack(stage, dst, st, L, H, D, B, nreq, off, blocks, k, start, 0, L);
    size_t nq = (size_t)nreq * L * H * G * D;
    uint16_t* q = malloc(nq * 2);
    double* out = malloc(nq * 8);
    for (size_t i = 0; i < nq; ++i) q[i] = (uint16_t)(0x3800 + rand() % 0x400);
    orc_paged_decode(src, st, L, H, H * G, D, B, dtype, nreq, off, blocks, k, q, out, 0.35);
    free(src);
    free(dst);
    free(stage);
    free(q);
    free(out);
  }
  double acc = 0;
  for (int bits = 0; bits < 65536; ++bits) {   /* every pattern of both types widens without a fault */
    double a = orc_widen((uint16_t)bits, 0), b = orc_widen((uint16_t)bits, 1);
    if (a == a) acc += a > 0 ? 1 : 0;
    if (b == b) acc += b > 0 ? 1 : 0;
  }
  printf("oracle driver ok (%g)\n", acc);
  return 0;
}
