// Internal declarations shared by the host and device translation units of libkvm.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "kvm.h"

namespace kvm {

// Requests carried by one kernel launch.  Their descriptors travel in the kernel
// argument segment, so the library needs no device-side metadata buffer.
constexpr int kMaxReqPerLaunch = 64;

// Records the failure detail for kvm_last_error() and returns `status`.
int fail(int status, const std::string& msg);
void clear_error();

bool layout_ok(const kvm_layout* l, std::string* why);
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// One side of a transfer after validation: for every request the table offset,
// k and the number of blocks that hold tokens [0,k).
struct BatchView {
  int n_req = 0;
  std::vector<int32_t> bt_off;  // first table entry of request r
  std::vector<int32_t> k;
  std::vector<int32_t> start;   // first token moved (0 without a range)
  std::vector<int32_t> jb;      // first block that holds a moved token: start / B
  std::vector<int32_t> nb;      // one past the last such block: ceil(k / B), or jb if k == start
  int64_t total_tokens = 0;     // sum of k - start
  int64_t total_blocks = 0;     // sum of nb - jb
};

// Checks pool + batch (pointers, alignment, layout, offsets, k range, id range).
// `writing`: also reject an id that appears twice among the entries that will be
// written.  On success fills `out`.
int validate_side(const char* what, const kvm_pool* pool, const kvm_batch* batch, bool writing,
                  BatchView* out);

// Grid of a launch whose n_wg 256-lane workgroups are numbered linearly (the
// staging-order kernels): HIP holds each grid dimension in work-items as a 32-bit
// value, so one dimension carries at most (2^32 - 1) / 256 workgroups (64 GiB of
// staging at 4 KiB per workgroup).  Rows of 65536 workgroups, as many rows as
// needed: x * y >= n_wg, x * 256 < 2^32, y <= 65535 for every n_wg < 2^31.
struct StageGrid {
  uint32_t x, y;
};
constexpr int64_t kStageGridRow = 65536;
inline StageGrid stage_grid(int64_t n_wg) {
  StageGrid g;
  g.x = (uint32_t)(n_wg < kStageGridRow ? n_wg : kStageGridRow);
  g.y = (uint32_t)ceil_div(n_wg, kStageGridRow);
  return g;
}

struct Options {
  int copy_nontemporal = 1;   // streaming (no-reuse) cache hints
  int copy_order = -1;        // -1: by layout (plane outermost for layer-major pools); 1: plane outermost; 0: planes of a block consecutive
  int stage_linear = -1;      // -1: automatic (pack of long requests only); else bit 0: pack, bit 1: unpack cut along the staging buffer
  int decode_cap_waves = -1;    // -1: by group width and mean context length; 0 / 1: never / always cap at two waves per SIMD
  int decode_mfma = -1;         // scores on the matrix cores (head_dim 128, 16-token blocks, groups of 4 and 8): -1 and 1 yes, 0 never
  int decode_spread = -1;       // -1: about 1 MiB between the four blocks of a decode step in consecutive ids; else log2 of the entry distance (0..6)
  int decode_split_target = 2048;  // workgroups a decode launch should reach by splitting contexts
  int decode_max_splits = 16;
  int decode_force_splits = 0;  // > 0: use exactly this many context splits
};
Options& options();

}  // namespace kvm
