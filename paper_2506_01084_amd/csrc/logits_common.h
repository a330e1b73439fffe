// Shared pieces of the extended_logits kernels (HIP, gfx950).
//
// Joint softmax over the base and hyper vocabularies (zip2zip paper, section 2.3, steps 7-9) reduced on
// the fly: every kernel folds the logits it produces into per-row triples (max, sum of exp(x - max),
// column of the max) and leaves one triple per (part, row); a small kernel merges the parts.
#pragma once

#include "z2z_internal.h"

#include <math.h>

namespace z2z_logits {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr float kNegInf = -INFINITY;
constexpr int kNoColumn = 0x7FFFFFFF;

struct Triple {
  float m;   // running maximum
  float s;   // sum of exp(x - m)
  int i;     // column of the maximum
};

__device__ __forceinline__ Triple empty_triple() {
  Triple t;
  t.m = kNegInf;
  t.s = 0.f;
  t.i = kNoColumn;
  return t;
}

// Merge b into a; equal maxima keep the lower column.
__device__ __forceinline__ void merge_triple(Triple& a, const Triple& b) {
  const bool b_wins = (b.m > a.m) || (b.m == a.m && b.i < a.i);
  const float hi = b_wins ? b.m : a.m;
  const float lo = b_wins ? a.m : b.m;
  const float s_hi = b_wins ? b.s : a.s;
  const float s_lo = b_wins ? a.s : b.s;
  const float scale = (lo == kNegInf) ? 0.f : __expf(lo - hi);
  a.s = s_hi + s_lo * scale;
  a.m = hi;
  a.i = b_wins ? b.i : a.i;
}

// Arguments of one tile-kernel launch (base part or hyper part).
struct LogitsArgs {
  const void* H;          // [rows, d]
  const void* W;          // base: [V, d]; hyper: [B, cap, d]
  const int32_t* size;    // hyper: [B] C_b; base: nullptr
  int32_t rows, rows_per_seq, d;
  int32_t w_rows;         // rows of one W matrix: V (base) or cap (hyper)
  int32_t col0;           // column of this part's first entry in a logits row: 0 or V
  int32_t n_vtiles;       // vocabulary tiles of one W matrix
  int32_t strip;          // vocabulary tiles per workgroup
  int32_t n_strips;       // strips of one W matrix
  int32_t part0;          // index of this launch's first partial
  int32_t row_tiles;      // base: tiles over all rows; hyper: tiles per sequence
  int32_t n_work;         // workgroups with work: row tiles (x sequences) x strips
  // workgroup -> (row tile, strip) mapping of the base part: workgroup ids go round-robin over the 8
  // XCDs; each XCD walks blocks of map_lr x map_ls (row tiles x strips), and the 8 XCDs' blocks sit
  // side by side as map_xr x map_xs inside one super block, so that what runs at the same time shares
  // W strips and hidden-row tiles through the XCD's L2 and the memory-side cache.
  int32_t map_lr, map_ls, map_xr, map_xs, map_sb_r;
  float* part_m;          // [parts, rows]
  float* part_s;
  int32_t* part_i;
  float* logits;          // nullptr or [rows, ld]
  int32_t ld;
};

}  // namespace z2z_logits

// kernel launchers, one per translation unit
int z2z_launch_logits_general(bool bf16, bool hyper, const z2z_logits::LogitsArgs& a, unsigned grid, hipStream_t s);
int z2z_launch_logits_fast(bool hyper, const z2z_logits::LogitsArgs& a, unsigned grid, hipStream_t s);
int z2z_logits_fast_prepare(z2z_ctx* c);
