// Device side of the synthetic input generator: fills a block pool (or part of
// it) with the same counter-based values the numpy generator produces, so the
// host can regenerate any block of a 100+ GiB pool without downloading it.
// Input generation only: nothing of the migration path lives here.
//
// Element (plane p = layer*2+kv, block b, w = (head*B + slot)*D + dim):
//   key = mix32(seed ^ mix32(stream * 0x9E3779B9 + p + 1))      (host, per plane)
//   kb  = mix32(key + b * 0x85EBCA6B)
//   x   = mix32(kb + w);  y = mix32(x ^ 0x68E31DA4)
//   n   = (sum of the 8 bytes of x and y) - 1020
//   val = round_to_nearest_even_16bit(float(n) * 0x1.398896p-8f)
#include <hip/hip_runtime.h>
#include <stdint.h>

static __host__ __device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

__device__ inline uint32_t byte_sum(uint32_t v) {
  return (v & 0xff) + ((v >> 8) & 0xff) + ((v >> 16) & 0xff) + (v >> 24);
}

__device__ inline uint16_t gen16(uint32_t kb, uint32_t w, int bf16) {
  const uint32_t x = mix32(kb + w);
  const uint32_t y = mix32(x ^ 0x68E31DA4u);
  const float f = (float)((int)(byte_sum(x) + byte_sum(y)) - 1020) * 0x1.398896p-8f /* float32(1/209.0239) */;
  if (bf16) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
  return __builtin_bit_cast(uint16_t, (_Float16)f);
}

struct FillArgs {
  char* base;
  int64_t stride_layer, stride_kv, stride_block;  // bytes
  uint32_t stride_head, stride_slot;              // bytes
  int32_t H, B, D;
  int32_t b0;      // first block to fill
  int32_t bf16;
  uint32_t seed, stream;
};

// grid: x = 8-element vectors of one (plane, block) / 256, y = block - b0, z = plane
__global__ __launch_bounds__(256) void fill_kernel(const FillArgs a) {
  const uint32_t plane = blockIdx.z;
  const uint32_t b = a.b0 + blockIdx.y;
  const uint32_t dv = a.D / 8;
  const uint32_t vec = blockIdx.x * 256u + threadIdx.x;
  if (vec >= (uint32_t)a.H * a.B * dv) return;
  const uint32_t key = mix32(a.seed ^ mix32(a.stream * 0x9E3779B9u + plane + 1u));
  const uint32_t kb = mix32(key + b * 0x85EBCA6Bu);
  const uint32_t w0 = vec * 8u;
  const uint32_t h = vec / (a.B * dv), rem = vec % (a.B * dv);
  const uint32_t s = rem / dv, c = rem % dv;
  uint32_t out[4];
  for (int i = 0; i < 4; ++i)
    out[i] = (uint32_t)gen16(kb, w0 + 2 * i, a.bf16) | ((uint32_t)gen16(kb, w0 + 2 * i + 1, a.bf16) << 16);
  char* p = a.base + (int64_t)(plane >> 1) * a.stride_layer + (int64_t)(plane & 1) * a.stride_kv +
            (int64_t)b * a.stride_block + (uint64_t)h * a.stride_head + (uint64_t)s * a.stride_slot +
            c * 16u;
  *reinterpret_cast<uint4*>(p) = make_uint4(out[0], out[1], out[2], out[3]);
}

// Fills blocks [b0, b1) of every (layer, kv) plane.  strides_bytes: layer, kv,
// block, head, slot.  Returns the hipError_t of the launch as an int.
extern "C" int kvmw_fill_pool(void* base_dev, const int64_t* strides_bytes, int L, int H, int D,
                              int B, int bf16, int64_t b0, int64_t b1, uint32_t seed,
                              uint32_t stream_id, void* hip_stream) {
  if (!base_dev || !strides_bytes || D % 8 || b1 <= b0) return -1;
  FillArgs a;
  a.base = (char*)base_dev;
  a.stride_layer = strides_bytes[0];
  a.stride_kv = strides_bytes[1];
  a.stride_block = strides_bytes[2];
  a.stride_head = (uint32_t)strides_bytes[3];
  a.stride_slot = (uint32_t)strides_bytes[4];
  a.H = H; a.B = B; a.D = D;
  a.bf16 = bf16;
  a.seed = seed;
  a.stream = stream_id;
  const uint32_t vecs = (uint32_t)H * B * (D / 8);
  for (int64_t b = b0; b < b1; b += 32768) {
    const int64_t n = b1 - b < 32768 ? b1 - b : 32768;
    a.b0 = (int32_t)b;
    hipLaunchKernelGGL(fill_kernel, dim3((vecs + 255) / 256, (uint32_t)n, 2 * L), dim3(256), 0,
                       (hipStream_t)hip_stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

// Regenerates chosen blocks of one plane into a dense buffer out[i][head][slot][dim]
// (block i = generator content of block id ids[i]): what a pool block must hold if
// it was filled by kvmw_fill_pool, without touching the pool.  Test support: lets a
// check compare every block of a 100+ GiB pool against the generator on the device.
struct GenArgs {
  char* out;
  const int32_t* ids;
  int32_t H, B, D;
  int32_t bf16;
  uint32_t seed, stream, plane;
};

// grid: x = 8-element vectors of one block / 256, y = index into ids
__global__ __launch_bounds__(256) void gen_blocks_kernel(const GenArgs a) {
  const uint32_t dv = a.D / 8;
  const uint32_t n_vec = (uint32_t)a.H * a.B * dv;
  const uint32_t vec = blockIdx.x * 256u + threadIdx.x;
  if (vec >= n_vec) return;
  const uint32_t b = (uint32_t)a.ids[blockIdx.y];
  const uint32_t key = mix32(a.seed ^ mix32(a.stream * 0x9E3779B9u + a.plane + 1u));
  const uint32_t kb = mix32(key + b * 0x85EBCA6Bu);
  const uint32_t w0 = vec * 8u;
  uint32_t out[4];
  for (int i = 0; i < 4; ++i)
    out[i] = (uint32_t)gen16(kb, w0 + 2 * i, a.bf16) | ((uint32_t)gen16(kb, w0 + 2 * i + 1, a.bf16) << 16);
  char* p = a.out + ((uint64_t)blockIdx.y * n_vec + vec) * 16u;
  *reinterpret_cast<uint4*>(p) = make_uint4(out[0], out[1], out[2], out[3]);
}

extern "C" int kvmw_gen_blocks(void* out_dev, const int32_t* ids_dev, int64_t n_ids, int H, int B, int D,
                               int bf16, uint32_t seed, uint32_t stream_id, uint32_t plane,
                               void* hip_stream) {
  if (!out_dev || !ids_dev || D % 8 || n_ids <= 0) return -1;
  GenArgs a;
  a.H = H; a.B = B; a.D = D;
  a.bf16 = bf16;
  a.seed = seed;
  a.stream = stream_id;
  a.plane = plane;
  const uint32_t vecs = (uint32_t)H * B * (D / 8);
  for (int64_t i = 0; i < n_ids; i += 32768) {
    const int64_t n = n_ids - i < 32768 ? n_ids - i : 32768;
    a.out = (char*)out_dev + (uint64_t)i * vecs * 16u;
    a.ids = ids_dev + i;
    hipLaunchKernelGGL(gen_blocks_kernel, dim3((vecs + 255) / 256, (uint32_t)n), dim3(256), 0,
                       (hipStream_t)hip_stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

// Position-sensitive 64-bit hash of every (plane, block) of a pool whose blocks are
// dense runs of `words` 8-byte words per plane:
//   hash = sum_i mix64(word_i + (i + 1) * 0x9E3779B97F4A7C15)   (mod 2^64)
// with mix64 the public splitmix64 finaliser.  Moving, swapping or changing words
// inside a block changes the hash (a plain sum of the words would not see a
// permutation).  Test support: "this block was left untouched" for pools too large
// to compare on the host.
static __host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// grid: x = block - b0, y = plane; out[plane][block]
__global__ __launch_bounds__(256) void block_hash_kernel(const char* base, int64_t stride_layer,
                                                         int64_t stride_kv, int64_t stride_block,
                                                         uint32_t words, int64_t b0, int64_t n_blocks,
                                                         unsigned long long* out) {
  const uint32_t plane = blockIdx.y;
  const int64_t b = b0 + blockIdx.x;
  const uint64_t* p = reinterpret_cast<const uint64_t*>(
      base + (int64_t)(plane >> 1) * stride_layer + (int64_t)(plane & 1) * stride_kv +
      b * stride_block);
  uint64_t acc = 0;
  for (uint32_t i = threadIdx.x; i < words; i += 256)
    acc += mix64(p[i] + (uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull);
  // workgroup sum through LDS (addition mod 2^64 is order-independent)
  __shared__ unsigned long long part[256];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[(int64_t)plane * n_blocks + b] = part[0];
}

// Hashes blocks [0, n_blocks) of all 2*L planes into out_dev[2L][n_blocks] (uint64).
// strides_bytes: layer, kv, block; words = 8-byte words of one block's run in a plane.
extern "C" int kvmw_block_hashes(const void* base_dev, const int64_t* strides_bytes, int L,
                                 int64_t n_blocks, int64_t words, void* out_dev, void* hip_stream) {
  if (!base_dev || !strides_bytes || !out_dev || n_blocks <= 0 || words <= 0 || words > 0x7fffffff) return -1;
  for (int64_t b = 0; b < n_blocks; b += 1 << 20) {
    const int64_t n = n_blocks - b < (1 << 20) ? n_blocks - b : (1 << 20);
    hipLaunchKernelGGL(block_hash_kernel, dim3((uint32_t)n, 2 * L), dim3(256), 0, (hipStream_t)hip_stream,
                       (const char*)base_dev, strides_bytes[0], strides_bytes[1], strides_bytes[2],
                       (uint32_t)words, b, n_blocks, (unsigned long long*)out_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

// Plain contiguous device-to-device copy of `bytes` (multiple of 16) with 16-byte
// vectors, 4 KiB per workgroup: the reference the benchmark reports beside the
// gather/scatter kernels, and a kernel of known size for scaling HBM counters.
typedef unsigned int kvmw_v4u __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void plain_copy_kernel(const char* src, char* dst, uint64_t n_vec) {
  const uint64_t v = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (v < n_vec) {
    // same cache-policy bits as the library's copy kernels, so that the reference
    // is not handicapped
    const kvmw_v4u* s = reinterpret_cast<const kvmw_v4u*>(src) + v;
    kvmw_v4u* d = reinterpret_cast<kvmw_v4u*>(dst) + v;
    kvmw_v4u x;
    asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_waitcnt vmcnt(0)" : "=&v"(x) : "v"(s) : "memory");
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(d), "v"(x) : "memory");
  }
}

extern "C" int kvmw_plain_copy(void* dst_dev, const void* src_dev, int64_t bytes, void* hip_stream) {
  if (!dst_dev || !src_dev || bytes <= 0 || bytes % 16) return -1;
  const uint64_t n_vec = (uint64_t)bytes / 16;
  const uint64_t grid = (n_vec + 255) / 256;
  if (grid > 0xffffffffull / 256) return -1;  // a grid dimension holds at most 2^32 - 1 work-items
  hipLaunchKernelGGL(plain_copy_kernel, dim3((uint32_t)grid), dim3(256), 0, (hipStream_t)hip_stream,
                     (const char*)src_dev, (char*)dst_dev, n_vec);
  return (int)hipGetLastError();
}


// Reference access patterns for the benchmark (no tables, no requests): what the
// memory system gives a kernel of the same shape as the library's copy kernels
// (256 lanes, one 16-byte vector per lane, 4 KiB per workgroup, the same
// cache-policy bits) when the addresses come from arithmetic alone.
//   mode 0: copy   mode 1: read only   mode 2: write only
// The buffer on each side is cut into runs of `run_vecs` vectors; workgroup w works
// on chunk (w % chunks) of run (w / chunks); run r sits at run slot r of its side
// (bits = 0: sequential) or at slot perm(r), a fixed pseudo-random permutation of
// the side's first 2^bits slots (ref_perm below).
struct RefArgs {
  const char* src;
  char* dst;
  uint32_t run_vecs, chunks;     // vectors per run, workgroups per run
  uint64_t n_runs;
  uint32_t src_bits, dst_bits;
  uint32_t src_rot, dst_rot;     // workgroup c of run r takes chunk (c + (rot & 7) + (rot >> 3) * r) % chunks on that side
  int32_t mode;
  uint32_t* sink;                // read-only mode: never written unless a loaded word equals the magic
};

// A bijection on `bits`-bit values: add a key, then multiply by odd constants, fold the
// upper half into the lower and rotate by half the width (a product's low bits depend
// on low bits only; the rotation hands them to the next product's upper bits).  The two
// sides of a copy use different keys, so their run slots are unrelated.
__device__ inline uint64_t ref_perm(uint64_t r, uint32_t bits, uint64_t key) {
  if (bits == 0) return r;
  const uint64_t mask = (1ull << bits) - 1;
  const uint32_t h = (bits + 1) / 2;
  r = (r + key) & mask;
  r = (r * 0x9E3779B97F4A7C15ull) & mask;
  r ^= r >> h;
  r = ((r << h) | (r >> (bits - h))) & mask;
  r = (r * 0xBF58476D1CE4E5B9ull) & mask;
  r ^= r >> h;
  r = (r * 0x94D049BB133111EBull) & mask;
  r ^= r >> h;
  return r;
}
constexpr uint64_t kRefKeySrc = 0, kRefKeyDst = 0x5851F42D4C957F2Dull;

__global__ __launch_bounds__(256) void ref_stream_kernel(const RefArgs a) {
  const uint64_t w = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
  const uint64_t r = w / a.chunks;
  if (r >= a.n_runs) return;
  const uint32_t c = (uint32_t)(w - r * a.chunks);
  const uint32_t v = c * 256u + threadIdx.x;
  if (v >= a.run_vecs) return;
  // rotated sides are only offered for runs of whole chunks (checked on the host)
  uint32_t sv = v, dv = v;
  if (a.src_rot | a.dst_rot) {   // uniform; chunks is a power of two here (checked on the host): masks, no division
    const uint32_t mask = a.chunks - 1u, rr = (uint32_t)r;
    sv = ((c + (a.src_rot & 7u) + (a.src_rot >> 3) * rr) & mask) * 256u + threadIdx.x;
    dv = ((c + (a.dst_rot & 7u) + (a.dst_rot >> 3) * rr) & mask) * 256u + threadIdx.x;
  }
  const uint64_t s_slot = ref_perm(r, a.src_bits, kRefKeySrc), d_slot = ref_perm(r, a.dst_bits, kRefKeyDst);
  const kvmw_v4u* sp = reinterpret_cast<const kvmw_v4u*>(a.src) + s_slot * a.run_vecs + sv;
  kvmw_v4u* dp = reinterpret_cast<kvmw_v4u*>(a.dst) + d_slot * a.run_vecs + dv;
  kvmw_v4u x = {v, v, v, v};
  if (a.mode != 2)
    asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_waitcnt vmcnt(0)" : "=&v"(x) : "v"(sp) : "memory");
  if (a.mode != 1)
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(dp), "v"(x) : "memory");
  else if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x5EEDF00Du && x[0] == 0x0BADC0DEu)
    *a.sink = x[2];   // keeps the loaded value observable; practically never taken
}

// bytes = n_runs * run_bytes are moved.  *_bits = 0: runs at consecutive slots; else
// permuted over the side's first 2^bits slots (the buffer must hold them, and
// n_runs <= 2^bits).  Returns 0, -1 on a bad argument, or the hipError_t of the launch.
// *_rot: workgroup c of run r works on chunk (c + (rot & 7) + (rot >> 3) * r) % chunks of
// that side instead of chunk c.  Workgroups go to the eight dies round-robin, so with
// eight chunks per run rot = 0 lets every die touch one residue class of 4 KiB pieces
// (its own number), rot = 1..7 another fixed class, and rot = 8 a class that changes
// from run to run.  Needs runs of a power-of-two number of whole 4 KiB chunks.
extern "C" int kvmw_ref_stream(int mode, const void* src_dev, void* dst_dev, int64_t run_bytes,
                               int64_t n_runs, int src_bits, int dst_bits, int src_rot, int dst_rot,
                               void* sink_dev, void* hip_stream) {
  if (mode < 0 || mode > 2 || run_bytes <= 0 || run_bytes % 16 || n_runs <= 0 || src_bits < 0 ||
      src_bits > 40 || dst_bits < 0 || dst_bits > 40 || src_rot < 0 || src_rot > 63 || dst_rot < 0 || dst_rot > 63)
    return -1;
  if ((src_rot || dst_rot) && (run_bytes % 4096 || ((run_bytes / 4096) & (run_bytes / 4096 - 1)))) return -1;
  if ((src_bits && n_runs > (1ll << src_bits)) || (dst_bits && n_runs > (1ll << dst_bits))) return -1;
  if ((mode != 2 && !src_dev) || (mode != 1 && !dst_dev) || (mode == 1 && !sink_dev)) return -1;
  RefArgs a;
  a.src = (const char*)src_dev;
  a.dst = (char*)dst_dev;
  a.run_vecs = (uint32_t)(run_bytes / 16);
  a.chunks = (a.run_vecs + 255) / 256;
  a.n_runs = (uint64_t)n_runs;
  a.src_bits = (uint32_t)src_bits;
  a.dst_bits = (uint32_t)dst_bits;
  a.src_rot = (uint32_t)src_rot;
  a.dst_rot = (uint32_t)dst_rot;
  a.mode = mode;
  a.sink = (uint32_t*)sink_dev;
  const uint64_t n_wg = a.n_runs * a.chunks;
  if (n_wg > 0x7fffffffull) return -1;
  const uint32_t gx = n_wg < 65536 ? (uint32_t)n_wg : 65536u;
  const uint32_t gy = (uint32_t)((n_wg + 65535) / 65536);
  hipLaunchKernelGGL(ref_stream_kernel, dim3(gx, gy), dim3(256), 0, (hipStream_t)hip_stream, a);
  return (int)hipGetLastError();
}

// ---- reference: waves that walk sequences of 4 KiB pieces -----------------------
// The read shape of a paged decode without its arithmetic: a workgroup of four waves
// makes n_steps steps; a step reads four 4 KiB pieces of a K-like stream (the lower half
// of the buffer) and the four pieces at the same offsets of a V-like stream (the upper
// half), two steps in flight.  The four pieces of a step lie stride_pieces * 4 KiB apart,
// the first at a pseudo-random place.
//   sliced = 0: wave w reads piece w of the step whole (four loads of 1 KiB)
//   sliced = 1: every wave reads quarter w of all four pieces (four loads of 1 KiB)
// Same bytes, same addresses, same number of loads: only who reads what differs.
struct WalkArgs {
  const char* src;
  uint64_t half_pieces;    // pieces per stream
  uint32_t stride_pieces;
  int32_t n_steps;
  int32_t sliced;
  uint64_t n_wg;
  uint32_t* sink;
};

__device__ inline uint64_t walk_mix(uint64_t r) {
  r *= 0x9E3779B97F4A7C15ull;
  r ^= r >> 29;
  r *= 0xBF58476D1CE4E5B9ull;
  r ^= r >> 32;
  return r;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void ref_walk_kernel(const WalkArgs a) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t wg = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
  if (wg >= a.n_wg) return;
  const uint64_t span = a.half_pieces - 3ull * a.stride_pieces;   // first pieces that keep the step in bounds
  kvmw_v4u t[2][2][4];
  auto issue = [&](int step, int slot) {
    const uint64_t base = walk_mix(wg * (uint64_t)a.n_steps + (uint64_t)step) % span;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // sliced: piece j, quarter `wave`; else: piece `wave`, quarter j
        const uint64_t piece = base + (uint64_t)(a.sliced ? j : wave) * a.stride_pieces;
        const uint32_t quarter = a.sliced ? (uint32_t)wave : (uint32_t)j;
        t[slot][s][j] = __builtin_nontemporal_load(reinterpret_cast<const kvmw_v4u*>(
            a.src + ((uint64_t)s * a.half_pieces + piece) * 4096 + quarter * 1024u + (uint32_t)lane * 16u));
      }
  };
  uint32_t x = 0;
  auto consume = [&](int slot) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int j = 0; j < 4; ++j) x ^= t[slot][s][j][0] ^ t[slot][s][j][1] ^ t[slot][s][j][2] ^ t[slot][s][j][3];
  };
  issue(0, 0);
  issue(a.n_steps > 1 ? 1 : 0, 1);
  for (int it = 0; it + 2 <= a.n_steps; it += 2) {   // past the end: the last step again
    consume(0);
    __builtin_amdgcn_sched_barrier(0);
    issue(it + 2 < a.n_steps ? it + 2 : a.n_steps - 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    consume(1);
    __builtin_amdgcn_sched_barrier(0);
    issue(it + 3 < a.n_steps ? it + 3 : a.n_steps - 1, 1);
    __builtin_amdgcn_sched_barrier(0);
  }
  consume(0);
  consume(1);
  if (x == 0x5EEDF00Du && a.sink) *a.sink = x;   // keeps the loads observable; practically never taken
}

// Reads n_wg * n_steps * 8 pieces (32 KiB per workgroup and step) of a buffer of
// 2 * half_pieces pieces.  Returns 0, -1 on a bad argument, or the hipError_t of the launch.
extern "C" int kvmw_ref_walk(const void* src_dev, int64_t half_pieces, int stride_pieces, int n_steps,
                             int64_t n_wg, int sliced, void* sink_dev, void* hip_stream) {
  if (!src_dev || !sink_dev || half_pieces <= 0 || stride_pieces < 1 || n_steps < 1 || n_wg < 1 ||
      n_wg > 0x7fffffffll || 3ll * stride_pieces >= half_pieces)
    return -1;
  WalkArgs a;
  a.src = (const char*)src_dev;
  a.half_pieces = (uint64_t)half_pieces;
  a.stride_pieces = (uint32_t)stride_pieces;
  a.n_steps = n_steps;
  a.sliced = sliced ? 1 : 0;
  a.n_wg = (uint64_t)n_wg;
  a.sink = (uint32_t*)sink_dev;
  const uint32_t gx = n_wg < 65536 ? (uint32_t)n_wg : 65536u;
  const uint32_t gy = (uint32_t)((n_wg + 65535) / 65536);
  hipLaunchKernelGGL(ref_walk_kernel, dim3(gx, gy), dim3(256), 0, (hipStream_t)hip_stream, a);
  return (int)hipGetLastError();
}
