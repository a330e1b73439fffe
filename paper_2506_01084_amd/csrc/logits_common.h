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

// The running best of a Gumbel-max draw.
struct Draw {
  float v;   // largest perturbed value so far
  float l;   // logit / T at that column
  int i;     // that column
};

__device__ __forceinline__ Draw empty_draw() {
  Draw d;
  d.v = kNegInf;
  d.l = 0.f;
  d.i = kNoColumn;
  return d;
}

__device__ __forceinline__ void merge_draw(Draw& a, const Draw& b) {
  if (b.v > a.v || (b.v == a.v && b.i < a.i)) a = b;
}

// One accumulator element, AGPR -> VGPR.  Spelled as an instruction so that the accumulators stay in
// the accumulation registers and are fetched block by block: left to itself the compiler copies the whole
// accumulator tile into VGPRs at the end of the K loop, and what that displaces is spilled inside the loop.
__device__ __forceinline__ float read_acc(float in_agpr) {
  float x;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(in_agpr));
  return x;
}

// Largest of three in one instruction.  (Spelled as an instruction: on values that come out of read_acc the
// compiler knows nothing about, fmaxf costs a quieting instruction per operand.)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Fold one finished accumulator tile into the running triples.  acc[i][j] is a 32x32 MFMA result block:
// register v of this lane is the logit of hidden row (j, lane & 31) and vocabulary column
// col_base + i * 32 + (v >> 2) * 8 + (v & 3), where col_base already holds the tile origin, the wave's
// offset and (lane >> 5) * 4.  Columns at and beyond n_valid do not exist (read as -inf; TAIL = false is the
// instance for tiles that lie wholly below n_valid, which is all but the last tile of a matrix: it carries no
// column tests at all).  The fold goes block by block (16 values live at a time, the accumulators are only
// read), in increasing column order per lane, so strict comparisons keep the lowest column among equal
// maxima.  The running sum is kept against the running maximum in base-2 units: exp(x - m) is one
// multiply-add and one hardware exponential per logit.
template <int NI, int NJ, bool TAIL>
__device__ __forceinline__ void fold_tile_impl(const f32x16 (&acc)[NI][NJ], Triple (&run)[NJ], int col_base, int col0,
                                               int n_valid) {
  constexpr float kLog2e = 1.4426950408889634f;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float x[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        x[v] = read_acc(acc[i][j][v]);
        if (TAIL && col_base + i * 32 + (v >> 2) * 8 + (v & 3) >= n_valid) x[v] = kNegInf;
      }
      float gmax = max3(x[0], x[1], x[2]);
#pragma unroll
      for (int v = 3; v < 15; v += 2) gmax = max3(gmax, x[v], x[v + 1]);
      gmax = max3(gmax, x[15], x[15]);
      if (gmax > run[j].m) {
        int targ = 15;
#pragma unroll
        for (int v = 14; v >= 0; --v) targ = (x[v] == gmax) ? v : targ;
        run[j].s = (run[j].m == kNegInf) ? 0.f : run[j].s * __expf(run[j].m - gmax);
        run[j].m = gmax;
        run[j].i = col0 + col_base + i * 32 + (targ >> 2) * 8 + (targ & 3);
      }
      if (!TAIL || run[j].m != kNegInf) {
        // (without a tail every logit is finite, so the running maximum is finite from the first block on)
        const float m2 = -run[j].m * kLog2e;
        float add0 = 0.f, add1 = 0.f;
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
          add0 += __builtin_amdgcn_exp2f(fmaf(x[v], kLog2e, m2));
          add1 += __builtin_amdgcn_exp2f(fmaf(x[v + 1], kLog2e, m2));
        }
        run[j].s += add0 + add1;
      }
    }
  }
}

template <int NI, int NJ>
__device__ __forceinline__ void fold_tile(const f32x16 (&acc)[NI][NJ], Triple (&run)[NJ], int col_base, int col0,
                                          int n_valid, bool tail) {
  if (tail)
    fold_tile_impl<NI, NJ, true>(acc, run, col_base, col0, n_valid);
  else
    fold_tile_impl<NI, NJ, false>(acc, run, col_base, col0, n_valid);
}

__device__ __forceinline__ uint32_t bf16_bits_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// GELU(x) = x * Phi(x) with the exact (erf) Phi.  erf by the rational approximation 7.1.26 of Abramowitz and
// Stegun, erf(z) = 1 - (a1 t + ... + a5 t^5) exp(-z^2), t = 1 / (1 + p z), z >= 0: absolute error below
// 1.5e-7, far inside the bf16 rounding of the result, at a third of the instructions of the library erff (the
// epilogue of a dense layer evaluates it 65536 times per tile with the matrix cores waiting).
__device__ __forceinline__ float gelu_erf(float x) {
  const float z = fabsf(x) * 0.70710678f;
  const float t = __frcp_rn(fmaf(0.3275911f, z, 1.0f));
  const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f),
                              0.254829592f);
  const float erf_abs = 1.0f - poly * __expf(-z * z);
  const float phi = 0.5f * (1.0f + copysignf(erf_abs, x));
  return x * phi;
}

// ---- the counter-based generator of the sampling kernels: Philox4x32-10 (Salmon et al., SC'11) -------
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
    c = uint4{hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0};
  }
  return c;
}

// The Gumbel value -ln(-ln u) of one generator word, u = ((w >> 9) + 0.5) * 2^-23.  u and 1 - u are both
// exact in float.  e = -ln u has to be accurate relative to itself where it is small (u next to 1: the
// largest perturbations, the ones that win): there it is the series of -ln(1 - x); elsewhere the hardware
// logarithm's absolute error of ~1e-7 is relative 1e-5 at worst.  The outer logarithm only needs absolute
// accuracy.
__device__ __forceinline__ float gumbel_from_word(uint32_t w) {
  const float x = ((float)(0x7FFFFFu - (w >> 9)) + 0.5f) * 0x1p-23f;        // 1 - u
  const float e = x < 0.015625f ? x * (1.f + x * (0.5f + x * (0.33333334f + 0.25f * x))) : -__logf(1.f - x);
  return -__logf(e);
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
  int32_t n_parts;        // partials per hidden row (row stride of the part arrays)
  int32_t row_tiles;      // base: tiles over all rows; hyper: tiles per sequence
  int32_t n_work;         // workgroups with work: row tiles (x sequences) x strips
  // workgroup -> (row tile, strip) mapping of the base part: workgroup ids go round-robin over the 8
  // XCDs; each XCD walks blocks of map_lr x map_ls (row tiles x strips), and the 8 XCDs' blocks sit
  // side by side as map_xr x map_xs inside one super block, so that what runs at the same time shares
  // W strips and hidden-row tiles through the XCD's L2 and the memory-side cache.
  int32_t map_lr, map_ls, map_xr, map_xs, map_sb_r;
  float* part_m;          // [rows, n_parts]
  float* part_s;
  int32_t* part_i;
  float* logits;          // nullptr or [rows, ld]
  int32_t ld;
  // linear mode of the bf16 MFMA kernel (a dense layer instead of a softmax fold):
  // out[r, n] = act(H[r, :] . W[n, :] + bias[n]) + residual[r, n], bf16, row stride ldo
  void* out;
  const float* bias;      // [w_rows] or nullptr
  const void* residual;   // [rows, ldo] bf16 or nullptr
  int32_t act;            // 0 none, 1 GELU (erf)
  int32_t ldo;
  int32_t stream_f32;     // 1: residual and out are fp32 (a residual stream kept unrounded between layers)
  // probability mode (the backward pass of the loss): out[r, c] = g[r] * (exp(logit - lse[r]) - [col0 + c == target[r]])
  // for the existing columns c < n_valid, 0 for the other columns below ldo; bf16, row stride ldo
  const float* lse;       // [rows]
  const float* row_grad;  // [rows] g: the upstream gradient, 0 for rows without a usable target
  const int32_t* targets; // [rows]
  const int32_t* rows_dev;  // nullptr, or the number of rows that exist (<= rows), known on the device only
  int32_t strip_blocks;     // > 0: linear mode with the XCD-per-row-tile mapping, = ceil(n_strips / map_ls)
  // linear mode with K split over ksplit workgroups per tile (few rows: too few tiles to fill the machine):
  // part ks covers K slabs [ks * slabs_per_part, ...) and leaves its fp32 tile in partial[ks][row][col]
  int32_t ksplit, slabs_per_part;
  float* partial;           // [ksplit][rows][ldo]
  // sampling fold (base part of a sampled decode step with many rows): the triples are taken over
  // logit * inv_temperature, and next to them the largest perturbed value (part_v), the scaled logit there
  // (part_l) and its column (part_i, instead of the maximum's); generator key and counter words as in the
  // decode kernel: word col & 3 of Philox4x32-10 at counter (col >> 2, row, ctr2, ctr3)
  int32_t sample;         // 1: fold the draw (part_v, part_l); 2: store logit * inv_temperature in `logits` and fold
  float inv_temperature;
  uint32_t key0, key1, ctr2, ctr3;
  float* part_v;
  float* part_l;
  // dense layer whose contraction length is only known on the device (a product over the rows of a pass):
  // K beyond *k_dev, up to the next multiple of 64, holds zeros and the slabs after that are not read
  const int32_t* k_dev;
};

// fold_tile for a filtered sampled pick: x = logit * inv_temperature enters the running triple and is stored,
// fp32, at logits[row, col0 + column] (the selection kernels read the rows back); 16-byte stores where the four
// columns of a group all exist.
template <int NI, int NJ>
__device__ __forceinline__ void fold_tile_store(const f32x16 (&acc)[NI][NJ], Triple (&run)[NJ], const LogitsArgs& a,
                                                int row_base, int r_end, int col_base, int n_valid) {
  const int lane31 = threadIdx.x & 31;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = row_base + j * 32 + lane31;
    float* out = a.logits + (size_t)min(row, r_end - 1) * a.ld + a.col0;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float x[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int col = col_base + i * 32 + (v >> 2) * 8 + (v & 3);
        x[v] = col < n_valid ? read_acc(acc[i][j][v]) * a.inv_temperature : kNegInf;
      }
      float gmax = x[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) gmax = fmaxf(gmax, x[v]);
      if (gmax > run[j].m) {
        int targ = 15;
#pragma unroll
        for (int v = 14; v >= 0; --v) targ = (x[v] == gmax) ? v : targ;
        run[j].s = (run[j].m == kNegInf) ? 0.f : run[j].s * __expf(run[j].m - gmax);
        run[j].m = gmax;
        run[j].i = a.col0 + col_base + i * 32 + (targ >> 2) * 8 + (targ & 3);
      }
      if (run[j].m != kNegInf) {
        const float m = run[j].m;
        float add = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) add += __expf(x[v] - m);
        run[j].s += add;
      }
      if (row < r_end) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = col_base + i * 32 + q * 8;
          // (a row of the logits starts 4-byte aligned only: ld = V + cap is any number)
          if (col + 3 < n_valid && ((((size_t)row * a.ld + a.col0 + col) & 3) == 0)) {
            *reinterpret_cast<float4*>(out + col) = float4{x[q * 4], x[q * 4 + 1], x[q * 4 + 2], x[q * 4 + 3]};
          } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
              if (col + k < n_valid) out[col + k] = x[q * 4 + k];
          }
        }
      }
    }
  }
}

// fold_tile for a sampled pick: the same register layout; x = logit * inv_temperature enters the running triple,
// and x + Gumbel(u[row, col]) the running draw.  A lane's columns come in aligned fours (one generator call
// each) and in increasing order, so a strict comparison keeps the lowest column among equal values.  The four
// groups of a 32 x 32 block are a real loop (the generator is long: unrolled 256 times per tile it would not fit
// the register file next to the accumulators).
template <int NI, int NJ>
__device__ __forceinline__ void fold_tile_sample(const f32x16 (&acc)[NI][NJ], Triple (&run)[NJ], Draw (&draw)[NJ],
                                                 const LogitsArgs& a, int row_base, int col_base, int n_valid) {
  const int lane31 = threadIdx.x & 31;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const uint32_t row = (uint32_t)(row_base + j * 32 + lane31);
    Triple t = run[j];
    Draw dr = draw[j];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float x[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) x[v] = read_acc(acc[i][j][v]);
#pragma unroll 1
      for (int q = 0; q < 4; ++q) {
        const int c0 = a.col0 + col_base + i * 32 + q * 8;
        const uint4 w = philox4x32_10(uint4{(uint32_t)(c0 >> 2), row, a.ctr2, a.ctr3}, a.key0, a.key1);
        const uint32_t word[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float xv = q == 0 ? x[k] : (q == 1 ? x[4 + k] : (q == 2 ? x[8 + k] : x[12 + k]));
          // (columns past the last valid one: -inf never enters the triple or wins the draw)
          const bool ok = c0 - a.col0 + k < n_valid;
          const float z = ok ? xv * a.inv_temperature : kNegInf;
          if (z > t.m) {
            t.s = (t.m == kNegInf) ? 1.f : t.s * __expf(t.m - z) + 1.f;
            t.m = z;
            t.i = c0 + k;
          } else if (ok) {
            t.s += __expf(z - t.m);
          }
          const float pv = z + gumbel_from_word(word[k]);
          if (pv > dr.v) {
            dr.v = pv;
            dr.l = z;
            dr.i = c0 + k;
          }
        }
      }
    }
    run[j] = t;
    draw[j] = dr;
  }
}

// Store one finished accumulator tile as a dense layer's output (same register layout as fold_tile):
// out[row, col] = act(acc + bias[col]) + residual[row, col], rounded once to bf16.  A lane holds runs of 4
// consecutive columns of one row: 8-byte stores.  Columns come in fours, so n_valid must be a multiple of 4.
// The loads the epilogue needs are issued in batches ahead of their use (the bias of all the lane's columns
// once, the residual of a whole 32-row block at a time): one memory round trip per batch instead of one per
// run, during which the matrix cores have nothing to do.
template <int NI, int NJ>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[NI][NJ], const LogitsArgs& a, int row_base, int r_end,
                                           int col_base, int n_valid) {
  const int lane31 = threadIdx.x & 31;
  float4 bias[NI][4];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int col = col_base + i * 32 + g * 8;
      bias[i][g] = (a.bias && col < n_valid) ? *reinterpret_cast<const float4*>(a.bias + col) : float4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = row_base + j * 32 + lane31;
    const bool row_ok = row < r_end;
    uint2 res[NI][4];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = col_base + i * 32 + g * 8;
        res[i][g] = (a.residual && row_ok && col < n_valid)
                        ? *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.residual) +
                                                          (size_t)row * a.ldo + col)
                        : uint2{0u, 0u};
      }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = col_base + i * 32 + g * 8;
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = read_acc(acc[i][j][g * 4 + e]);
        x[0] += bias[i][g].x;
        x[1] += bias[i][g].y;
        x[2] += bias[i][g].z;
        x[3] += bias[i][g].w;
        if (a.act == 1) {
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = gelu_erf(x[e]);
        }
        x[0] += __uint_as_float(res[i][g].x << 16);
        x[1] += __uint_as_float(res[i][g].x & 0xFFFF0000u);
        x[2] += __uint_as_float(res[i][g].y << 16);
        x[3] += __uint_as_float(res[i][g].y & 0xFFFF0000u);
        if (row_ok && col < n_valid) {
          uint2 o;
          o.x = bf16_bits_rne(x[0]) | (bf16_bits_rne(x[1]) << 16);
          o.y = bf16_bits_rne(x[2]) | (bf16_bits_rne(x[3]) << 16);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + (size_t)row * a.ldo + col) = o;
        }
      }
    }
  }
}

// The same with the residual and the output in fp32 (no rounding): 16-byte loads and stores.
template <int NI, int NJ>
__device__ __forceinline__ void store_tile_f32(const f32x16 (&acc)[NI][NJ], const LogitsArgs& a, int row_base, int r_end,
                                               int col_base, int n_valid) {
  const int lane31 = threadIdx.x & 31;
  const float* res = reinterpret_cast<const float*>(a.residual);
  float* out = reinterpret_cast<float*>(a.out);
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = row_base + j * 32 + lane31;
    if (row >= r_end) continue;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float4 rv[4], bv[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = col_base + i * 32 + g * 8;
        const bool ok = col < n_valid;
        rv[g] = (res && ok) ? *reinterpret_cast<const float4*>(res + (size_t)row * a.ldo + col) : float4{0.f, 0.f, 0.f, 0.f};
        bv[g] = (a.bias && ok) ? *reinterpret_cast<const float4*>(a.bias + col) : float4{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = col_base + i * 32 + g * 8;
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = read_acc(acc[i][j][g * 4 + e]);
        x[0] += bv[g].x;
        x[1] += bv[g].y;
        x[2] += bv[g].z;
        x[3] += bv[g].w;
        if (a.act == 1) {
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = gelu_erf(x[e]);
        }
        if (col < n_valid)
          *reinterpret_cast<float4*>(out + (size_t)row * a.ldo + col) =
              float4{x[0] + rv[g].x, x[1] + rv[g].y, x[2] + rv[g].z, x[3] + rv[g].w};
      }
    }
  }
}

// Store one finished accumulator tile as it is (fp32), for a dense layer whose K range is split over several
// workgroups: 16-byte stores.
template <int NI, int NJ>
__device__ __forceinline__ void store_partial_tile(const f32x16 (&acc)[NI][NJ], float* part, int ld, int row_base,
                                                   int r_end, int col_base, int n_valid) {
  const int lane31 = threadIdx.x & 31;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = row_base + j * 32 + lane31;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = col_base + i * 32 + q * 8;
        float4 x;
        x.x = read_acc(acc[i][j][q * 4 + 0]);
        x.y = read_acc(acc[i][j][q * 4 + 1]);
        x.z = read_acc(acc[i][j][q * 4 + 2]);
        x.w = read_acc(acc[i][j][q * 4 + 3]);
        if (row < r_end && col < n_valid) *reinterpret_cast<float4*>(part + (size_t)row * ld + col) = x;
      }
    }
  }
}

// Store one finished accumulator tile as the gradient of the loss with respect to the logits (same register
// layout as fold_tile; see LogitsArgs, probability mode).  Columns come in fours; ldo is a multiple of 4.
template <int NI, int NJ>
__device__ __forceinline__ void store_prob_tile(const f32x16 (&acc)[NI][NJ], const LogitsArgs& a, int row_base, int r_end,
                                                int col_base, int n_valid) {
  const int lane31 = threadIdx.x & 31;
  float lse[NJ], g[NJ];
  int tgt[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = row_base + j * 32 + lane31;
    const bool ok = row < r_end;
    lse[j] = ok ? a.lse[row] : 0.f;
    g[j] = ok ? a.row_grad[row] : 0.f;
    tgt[j] = ok ? a.targets[row] - a.col0 : -1;
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int row = row_base + j * 32 + lane31;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = col_base + i * 32 + q * 8;
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float z = read_acc(acc[i][j][q * 4 + e]);
          const float p = __expf(z - lse[j]) - (col + e == tgt[j] ? 1.f : 0.f);
          x[e] = col + e < n_valid ? g[j] * p : 0.f;
        }
        if (row < r_end && col < a.ldo) {
          uint2 o;
          o.x = bf16_bits_rne(x[0]) | (bf16_bits_rne(x[1]) << 16);
          o.y = bf16_bits_rne(x[2]) | (bf16_bits_rne(x[3]) << 16);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) + (size_t)row * a.ldo + col) = o;
        }
      }
    }
  }
}

}  // namespace z2z_logits

// kernel launchers, one per translation unit
int z2z_launch_logits_general(bool bf16, bool hyper, const z2z_logits::LogitsArgs& a, unsigned grid, hipStream_t s);
// mode: 0 base part, 1 hyper part (both fold the joint softmax), 2 dense layer (stores the tile),
// 3 base part, 4 hyper part storing the gradient with respect to the logits, 5 dense layer with K split
// (fp32 partial tiles)
int z2z_launch_logits_fast(int mode, const z2z_logits::LogitsArgs& a, unsigned grid, hipStream_t s);
// out[R, N] = act(A[R, K] . W[N, K]^T + bias) + residual, all matrices bf16 (bias float), on the bf16 MFMA kernel
// (R rows are laid out; with rows_dev only the first *rows_dev of them exist: the others are neither read nor
// written).  stream_f32: residual and out are fp32 instead (a residual stream that is not rounded between layers).
// bf16 transpose with zero padding of the output rows (see dense.hip)
int z2z_launch_transpose(const void* in, void* out, int R, const int32_t* rows_dev, int C, int ld_in, int ld_out,
                         int batch, size_t in_batch, size_t out_batch, hipStream_t s);
int z2z_launch_linear(z2z_ctx* c, const void* A, const void* W, const float* bias, const void* residual, int act,
                      void* out, int R, const int32_t* rows_dev, int N, int K, hipStream_t s, const int32_t* k_dev = nullptr,
                      bool stream_f32 = false);
int z2z_logits_fast_prepare(z2z_ctx* c);
int z2z_launch_logits_part(z2z_ctx* c, bool hyper, bool fast, z2z_logits::LogitsArgs a, const void* W, int w_rows, int col0,
                           int part0, int strip, int rows, int rows_per_seq, int* n_strips_out, bool timed,
                           hipStream_t s, bool prob = false, int seq0 = 0, int n_seq = 0);
// temperature sampling (one-row-per-sequence kernel only): softmax(logit / temperature), generator key and
// counter words from seed and step
struct z2z_sample_params {
  float temperature;
  uint64_t seed, step;
};
// hyper_only_base_parts >= 0: only the per-sequence hyper units run, and they leave their partials behind that
// many parts per row, which another launch (the tile kernel over the base vocabulary) fills
// parts: where the partial triples go (nullptr: the context's buffers)
int z2z_launch_logits_decode(z2z_ctx* c, const void* H, const void* W_base, const void* W_hyper, int* n_parts,
                             bool timed, const z2z_sample_params* sample, float* logits, hipStream_t s,
                             int hyper_only_base_parts = -1, const z2z_parts* parts = nullptr, int rows_per_seq = 1);
// rows_per_seq in 2..64 (with hyper_only_base_parts >= 0): the hyper part on the matrix-core units, one workgroup
// per sequence and 256 rows of its W_hyper; parts per row then: base parts + z2z_logits_decode_seq_units
int z2z_logits_decode_seq_units(const z2z_ctx* c);
// `logits` hold logit / temperature as the decode kernel stored them, `row_stat` the rows' maxima, then their
// log-sum-exps, of those values; `work` is scratch of z2z_sample_truncated_work_floats(rows) floats.
// z2z_sample_truncated_merges_parts: true when the selection's first kernel merges the parts into `row_stat` itself
// (the caller then launches no merge); otherwise `row_stat` must hold them when the call is made.
bool z2z_sample_truncated_merges_parts(const z2z_ctx* c, int n_parts, int32_t top_k, int base_columns);
int z2z_launch_sample_truncated(z2z_ctx* c, const float* logits, float* row_stat, int32_t rows, int n_parts,
                                float* work, const z2z_sample_params* sp, int32_t top_k, float top_p,
                                int32_t* token, float* logprob, hipStream_t s, int base_columns = 0);
size_t z2z_sample_truncated_work_floats(int32_t rows);
// the same layer on the bandwidth-bound kernel of the decode step (few rows: every weight byte is read once per
// 64 rows); K a multiple of 128, N even
int z2z_launch_linear_skinny(z2z_ctx* c, const void* A, const void* W, const float* bias, const void* residual,
                             int act, void* out, int R, const int32_t* rows_dev, int N, int K, hipStream_t s,
                             bool stream_f32 = false);
int z2z_logits_decode_parts(const z2z_ctx* c);
void z2z_logits_decode_units(int* base_columns, int* hyper_columns);
bool z2z_logits_decode_ok(const z2z_ctx* c);
int z2z_logits_decode_prepare(z2z_ctx* c);
