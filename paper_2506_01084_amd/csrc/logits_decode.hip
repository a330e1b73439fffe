// extended_logits for a decode step (one hidden row per sequence), bf16, gfx950: bound by HBM bandwidth.
//
// Per step the path reads W_base once for all sequences and every sequence's own W_hyper once (zip2zip
// paper, section 2.3 steps 7-9 with the hyper-embedding cache of the same section): the bytes are
// d * 2 * (V + sum_b C_b) and there are only about 20 flops per byte, so everything is arranged around
// keeping many wide loads in flight and touching every weight byte exactly once.
//
// One launch, two kinds of workgroup (8 waves each), so both streams share the machine:
//  * base units: 256 rows of W_base against up to 64 hidden rows.  A weight row has to meet 64 hidden
//    rows, which is matrix-core work (v_mfma_f32_16x16x32_bf16: weight rows are operand A, hidden rows
//    operand B).  The hidden rows cannot be kept whole near the MFMAs (64 x d x 2 bytes), so K is cut in
//    slices of 128: a wave holds the 64 x 128 slice of H in 64 registers and streams that slice of the
//    unit's weight rows through it, 16 rows at a time.  The eight waves work on eight adjacent slices of
//    the same 16 rows (2 KiB contiguous per weight row), drop their 16 x 64 partial products into LDS
//    slots, meet at a barrier, and each wave then sums the slots for two of the 16 rows into the unit's
//    [256][64] fp32 logit tile in LDS (rows it alone owns: no atomics -- LDS float atomics measured an
//    order of magnitude too slow for this).  After d / 1024 such phases the tile is folded into one
//    (max, sum-exp, argmax) triple per hidden row.
//  * hyper units: 512 rows of one sequence's W_hyper against that sequence's single hidden row: plain
//    dot products (v_dot2c_f32_bf16), one weight row per wave at a time, 1 KiB per load instruction,
//    the hidden row held in registers; rows at and beyond C_b are never touched.
// Each unit leaves one triple per hidden row in the same [row][part] scratch the prefill kernels use.
//
// Where at most four hidden rows meet a weight row -- a decode step of up to four sequences, or the per-sequence
// part of a call with two to four hidden rows per sequence (a verification step over drafted codes) -- those rows
// fit in registers, and the dot-product units take that work too (dot_unit below): whole weight rows streamed
// once, nothing handed over through LDS.
#include "logits_common.h"

#include <string.h>

namespace {

using namespace z2z_logits;

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

constexpr int D_UNIT = 512;            // weight rows per hyper unit
constexpr int D_BASE_UNIT = 256;       // weight rows per base unit
constexpr int D_LINEAR_UNIT = 64;      // output features per unit of a dense layer (MODE 3)
constexpr int D_THREADS = 512;
constexpr int D_KSLICE = 128;          // K elements a wave keeps of H
constexpr int D_QB = D_KSLICE / 32;    // MFMA k-blocks per slice
constexpr int D_TILE_BYTES = D_BASE_UNIT * 64 * 4;       // [256][64] fp32 logits of a base unit
constexpr int D_SLOT_STRIDE = 20;                         // floats per hidden-row column of a slot (16 + pad)
constexpr int D_SLOT_FLOATS = 64 * D_SLOT_STRIDE;         // one wave's 16 x 64 partial block, column-major
constexpr int D_SLOTS_BYTES = 2 * 8 * D_SLOT_FLOATS * 4;  // two buffers x eight waves
constexpr int D_LDS = D_TILE_BYTES + D_SLOTS_BYTES;       // 144 KiB (the triple exchange reuses the slots)
constexpr int D_MAXQ = 8;              // hyper units: d <= 512 * D_MAXQ
#ifndef D_DOT_ROWS
#define D_DOT_ROWS 4                   // hidden rows per sequence up to which the per-sequence part runs on dot-product units
#endif
#ifndef D_DOT_BATCH
#define D_DOT_BATCH 4                  // sequences per decode step up to which the base vocabulary does too
#endif

struct DecodeArgs {
  const uint4* H;         // [B, d] bf16
  const uint4* W_base;    // [V, d]
  const uint4* W_hyper;   // [B, cap, d]
  const int32_t* size;    // [B]
  int32_t B, V, cap, d;
  int32_t n_base_units;   // ceil(V / 256)
  int32_t n_groups;       // ceil(B / 64) groups of hidden rows for the base part
  int32_t units_per_seq;  // ceil(cap / 512)
  int32_t n_parts;        // partials per hidden row
  float* part_m;          // [B, n_parts]
  float* part_s;
  int32_t* part_i;
  // sampling variant: the triples are taken over logit / temperature, and next to them the kernel keeps
  // the largest perturbed value (part_v), the scaled logit there (part_l) and its column (part_i)
  float* part_v;
  float* part_l;
  float inv_temperature;
  float* logits;          // MODE 2: [B, ld] logits * inv_temperature out (columns at and beyond V + C_b are not written)
  int32_t ld;
  uint32_t key0, key1;    // generator key: the seed
  uint32_t ctr2, ctr3;    // generator counter words 2, 3: the step
  // MODE 3, a dense layer on a few rows: out[h, v] = act(H[h, :] . W_base[v, :] + bias[v]) + residual[h, v],
  // bf16, row stride ldo; no triples are kept
  void* out;
  const float* bias;
  const void* residual;
  int32_t act;            // 0 none, 1 GELU (erf)
  int32_t ldo;
  int32_t stream_f32;     // 1: residual and out are fp32 (a residual stream kept unrounded between layers)
  const int32_t* rows_dev;  // MODE 3: nullptr, or the number of hidden rows that exist (<= B), on the device
  // MODE 3, K split over ksplit workgroups per unit (layers with few units would leave most CUs idle): each
  // leaves its partial tile in `partial`; linear_reduce_kernel adds them up and runs the epilogue
  int32_t ksplit;
  float* partial;           // [n_groups * n_base_units][ksplit][unit rows * 64]
  // MODE 4, the hyper part of a call with 2..64 hidden rows per sequence: workgroup (b, u) takes rows
  // [256 u, 256 u + 256) of W_hyper[b] against the sequence's rows_per_seq hidden rows
  int32_t rows_per_seq;
  int32_t seq_units;        // ceil(cap / 256)
};

__device__ __forceinline__ void fold_value(Triple& t, float x, int col) {
  if (x > t.m) {
    t.s = (t.m == kNegInf) ? 1.f : t.s * __expf(t.m - x) + 1.f;
    t.m = x;
    t.i = col;
  } else if (x != kNegInf) {
    t.s += __expf(x - t.m);
  }
}

// ---- sampling (section 2.3 of the zip2zip paper, step 9: the next token is a draw from the joint
//      softmax).  Gumbel-max: the column that maximises logit / T - ln(-ln u) is distributed as
//      softmax(logit / T); u comes from Philox4x32-10 (Salmon et al., SC'11) with counter
//      (column >> 2, hidden row, step) and key = seed, so a draw is a pure function of its coordinates.
// Generator words for the columns 4 * group .. 4 * group + 3 of one hidden row are produced together;
// a thread that walks consecutive columns keeps them until it leaves the group.
struct Noise {
  uint4 words;
  int group;
};

__device__ __forceinline__ float gumbel_at(const DecodeArgs& a, Noise& n, int hrow, int col) {
  const int group = col >> 2;
  if (group != n.group) {
    n.words = philox4x32_10(uint4{(uint32_t)group, (uint32_t)hrow, a.ctr2, a.ctr3}, a.key0, a.key1);
    n.group = group;
  }
  const int k = col & 3;
  const uint32_t w = k == 0 ? n.words.x : (k == 1 ? n.words.y : (k == 2 ? n.words.z : n.words.w));
  return gumbel_from_word(w);
}

template <int MODE>
__device__ __forceinline__ void fold_logit(const DecodeArgs& a, Triple& t, Draw& dr, Noise& n, float x, int hrow,
                                           int col) {
  if (MODE == 1) {
    const float z = x * a.inv_temperature;
    fold_value(t, z, col);
    const float p = z + gumbel_at(a, n, hrow, col);
    if (p > dr.v) {                 // columns arrive in increasing order: strict comparison keeps the lowest
      dr.v = p;
      dr.l = z;
      dr.i = col;
    }
  } else if (MODE == 2) {
    fold_value(t, x * a.inv_temperature, col);       // what is stored is folded: logit / T (T = 1 for plain logits)
  } else {
    fold_value(t, x, col);
  }
}

// The epilogue of a dense layer on one unit: tile [D_LINEAR_UNIT][64] (output feature, row of the group) is
// transposed through `stage` [64][D_LINEAR_UNIT + 1] so that LDS accesses and global stores both run along
// consecutive addresses; then bias, activation, residual and one rounding per element.  All threads call it.
__device__ __forceinline__ void linear_epilogue(const DecodeArgs& a, const float* tile, float* stage, int v0, int h0,
                                                int n_h) {
  constexpr int UNIT = D_LINEAR_UNIT;
  constexpr int ST = UNIT + 1;
  const int tid = threadIdx.x;
  for (int i = tid; i < UNIT * 64; i += D_THREADS) stage[(i & 63) * ST + (i >> 6)] = tile[i];
  __syncthreads();
  for (int i = tid; i < 64 * (UNIT / 2); i += D_THREADS) {
    const int jj = i / (UNIT / 2), r = 2 * (i - jj * (UNIT / 2));     // a pair of columns
    if (jj < n_h && v0 + r < a.V) {                                   // V is even
      float x0 = stage[jj * ST + r], x1 = stage[jj * ST + r + 1];
      if (a.bias) {
        x0 += a.bias[v0 + r];
        x1 += a.bias[v0 + r + 1];
      }
      if (a.act == 1) {
        x0 = gelu_erf(x0);
        x1 = gelu_erf(x1);
      }
      const size_t at = (size_t)(h0 + jj) * a.ldo + v0 + r;
      if (a.stream_f32) {
        if (a.residual) {
          const float2 rv = *reinterpret_cast<const float2*>(reinterpret_cast<const float*>(a.residual) + at);
          x0 += rv.x;
          x1 += rv.y;
        }
        *reinterpret_cast<float2*>(reinterpret_cast<float*>(a.out) + at) = float2{x0, x1};
        continue;
      }
      if (a.residual) {
        const uint32_t rv = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint16_t*>(a.residual) + at);
        x0 += __uint_as_float(rv << 16);
        x1 += __uint_as_float(rv & 0xFFFF0000u);
      }
      *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(a.out) + at) = bf16_bits_rne(x0) | (bf16_bits_rne(x1) << 16);
    }
  }
}

template <int MODE>
__device__ __forceinline__ void base_unit(const DecodeArgs& a, int unit, int group, int ks, unsigned char* lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // weight rows per unit: 256 for the vocabulary; a dense layer has few output rows and needs many
  // workgroups to fill the machine, so its units are 64 rows
  constexpr int UNIT = MODE == 3 ? D_LINEAR_UNIT : D_BASE_UNIT;
  // MODE 4 (a sequence's own weights against its few hidden rows): `group` is the sequence, `unit` the block of
  // 256 rows of its W_hyper, of which only the first C_b exist
  constexpr bool SEQ = MODE == 4;
  float* tile = reinterpret_cast<float*>(lds);                      // [UNIT][64]
  float* slots = reinterpret_cast<float*>(lds + D_TILE_BYTES);       // [2][8][64][D_SLOT_STRIDE]
  const int chunks_per_row = a.d >> 3;             // 16-byte chunks per row
  const int v0 = unit * UNIT;
  const int h0 = SEQ ? group * a.rows_per_seq : group * 64;
  const int n_rows = SEQ ? h0 + a.rows_per_seq : ((MODE == 3 && a.rows_dev) ? min(a.B, *a.rows_dev) : a.B);
  if (h0 >= n_rows) return;                        // (the whole workgroup: nothing is shared yet)
  const int n_h = min(64, n_rows - h0);            // hidden rows of this group
  const uint4* Wsrc = SEQ ? a.W_hyper + (size_t)group * a.cap * chunks_per_row : a.W_base;
  const int w_valid = SEQ ? min(max(a.size[group], 0), a.cap) : a.V;      // weight rows that exist
  const int col0 = SEQ ? a.V : 0;                  // column of weight row 0 in a logits row
  const int part = SEQ ? a.n_base_units + unit : unit;
  if (SEQ && v0 >= w_valid) {
    // none of this block's rows exist: the part is empty for every hidden row of the sequence
    if (threadIdx.x < n_h) {
      const size_t p = (size_t)(h0 + threadIdx.x) * a.n_parts + part;
      a.part_m[p] = kNegInf;
      a.part_s[p] = 0.f;
      a.part_i[p] = kNoColumn;
    }
    return;
  }
  // 16-row blocks to stream: all of the unit, or (MODE 4) those that hold existing rows, in fours
  const int n_blk = SEQ ? min(UNIT / 16, (((min(UNIT, w_valid - v0) + 15) >> 4) + 3) & ~3) : UNIT / 16;
  const int g_eff = SEQ ? (n_h + 15) >> 4 : 4;     // groups of 16 hidden rows that hold a valid row
  const int n_slices = a.d / D_KSLICE;
  const int n_phases_all = (n_slices + 7) >> 3;
  // this workgroup's share of K: phases [phase0, phase0 + n_phases) (all of them unless MODE 3 splits K)
  const int per_part = (MODE == 3 && a.ksplit > 1) ? (n_phases_all + a.ksplit - 1) / a.ksplit : n_phases_all;
  const int phase0 = ks * per_part;
  const int n_phases = min(per_part, n_phases_all - phase0);
  constexpr int N_BLK = UNIT / 16;

  for (int i = tid; i < UNIT * 64; i += D_THREADS) tile[i] = 0.f;

  const int m16 = lane & 15;     // MFMA row (A) / column (B) index of this lane
  const int kg = lane >> 4;      // which 8 of the 32 k of an MFMA this lane feeds
  // One step = one 16-row block of one phase.  Weight blocks are requested three steps ahead into four
  // register buffers (the loop is unrolled by four so that each buffer has a fixed name); requests past
  // the end of the unit re-read its last block.
  const int n_steps = n_phases * n_blk;
  // step -> (phase, block): n_blk is 4, 8, 12 or 16 and there are at most a few hundred steps, for which the
  // multiplication below divides exactly
  const uint32_t inv_blk = (65536u + (uint32_t)n_blk - 1) / (uint32_t)n_blk;
  auto phase_of = [&](int step) { return SEQ ? (int)(((uint32_t)step * inv_blk) >> 16) : step / N_BLK; };
  auto chunk0 = [&](int phase) {
    const int slice = min((phase0 + phase) * 8 + wave, n_slices - 1);
    return slice * (D_KSLICE / 8) + kg;            // first 16-byte chunk of this lane in the slice
  };
  auto load_block = [&](uint4 (&w)[D_QB], int step) {
    step = min(step, n_steps - 1);
    const int phase = phase_of(step), blk = step - phase * n_blk;
    const int wrow = min(v0 + blk * 16 + m16, w_valid - 1);
    const uint4* p = Wsrc + (size_t)wrow * chunks_per_row + chunk0(phase);
#pragma unroll
    for (int q = 0; q < D_QB; ++q) w[q] = p[q * 4];
  };
  uint4 hreg[4][D_QB];                             // the wave's slice of H: 4 x 16 hidden rows x D_QB k-blocks
  auto load_h = [&](int phase) {
    const int c0 = chunk0(phase);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int hrow = min(h0 + g * 16 + m16, n_rows - 1);
      if (!SEQ || g < g_eff) {
#pragma unroll
        for (int q = 0; q < D_QB; ++q) hreg[g][q] = a.H[(size_t)hrow * chunks_per_row + c0 + q * 4];
      }
    }
  };
  auto compute = [&](const uint4 (&w)[D_QB], int step) {
    const int phase = phase_of(step), blk = step - phase * n_blk;
    const bool valid = (phase0 + phase) * 8 + wave < n_slices;   // wave-uniform
    f32x4 acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (valid) {
#pragma unroll
      for (int q = 0; q < D_QB; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          if (!SEQ || g < g_eff)                               // (wave-uniform)
            acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[q]),
                                                             __builtin_bit_cast(bf16x8, hreg[g][q]), acc[g], 0, 0, 0);
    }
    // slot layout: hidden-row column c at c * D_SLOT_STRIDE, its 16 weight rows contiguous; this lane
    // holds rows 4 * kg .. + 3 of column g * 16 + m16: one 16-byte store per group
    float* slot = slots + ((step & 1) * 8 + wave) * D_SLOT_FLOATS;
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<f32x4*>(slot + (g * 16 + m16) * D_SLOT_STRIDE + 4 * kg) = acc[g];
    __syncthreads();
    // this wave owns rows 2 * wave, 2 * wave + 1 of the block; lane = hidden-row column.  The slot
    // buffer written at step + 2 is this one again: the barrier of step + 1 lies in between.
    const float* rd = slots + (step & 1) * 8 * D_SLOT_FLOATS + lane * D_SLOT_STRIDE + 2 * wave;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const float2 p = *reinterpret_cast<const float2*>(rd + s * D_SLOT_FLOATS);
      s0 += p.x;
      s1 += p.y;
    }
    float* trow = tile + (blk * 16 + 2 * wave) * 64 + lane;
    trow[0] += s0;
    trow[64] += s1;
    if (blk == n_blk - 1 && phase + 1 < n_phases) load_h(phase + 1);   // next phase: next slice of H
  };
  uint4 w0[D_QB], w1[D_QB], w2[D_QB], w3[D_QB];
  load_h(0);
  load_block(w0, 0);
  load_block(w1, 1);
  load_block(w2, 2);
  for (int step = 0; step < n_steps; step += 4) {   // n_blk is a multiple of 4, so is n_steps
    load_block(w3, step + 3);
    compute(w0, step);
    load_block(w0, step + 4);
    compute(w1, step + 1);
    load_block(w1, step + 5);
    compute(w2, step + 2);
    load_block(w2, step + 6);
    compute(w3, step + 3);
  }
  __syncthreads();

  if (MODE == 2) {
    // the unit's logits go out row-major per hidden row: transposed through the (now idle) slot area so
    // that both the LDS accesses and the global stores run along consecutive addresses
    constexpr int ST = D_BASE_UNIT + 1;
    float* stage = slots;                                            // [64][257]
    for (int i = tid; i < D_BASE_UNIT * 64; i += D_THREADS) stage[(i & 63) * ST + (i >> 6)] = tile[i];
    __syncthreads();
    for (int i = tid; i < 64 * D_BASE_UNIT; i += D_THREADS) {
      const int jj = i / D_BASE_UNIT, r = i - jj * D_BASE_UNIT;
      if (jj < n_h && v0 + r < a.V)
        a.logits[(size_t)(h0 + jj) * a.ld + v0 + r] = stage[jj * ST + r] * a.inv_temperature;
    }
    __syncthreads();
  }
  if (MODE == 3 && a.ksplit > 1) {
    // K is split over several workgroups: leave the partial tile; linear_reduce_kernel adds them up (in a
    // launch of its own: making them visible to one another inside this launch takes device-wide fences,
    // which cost more than the launch)
    const size_t slot = (size_t)group * a.n_base_units + unit;
    float* mine = a.partial + (slot * a.ksplit + ks) * (size_t)(UNIT * 64);
    for (int i = tid; i < UNIT * 64; i += D_THREADS) mine[i] = tile[i];
    return;
  }
  if (MODE == 3) {
    linear_epilogue(a, tile, slots, v0, h0, n_h);
    return;
  }
  // fold: thread t takes hidden row t & 63 and weight rows (t >> 6) * 32 .. + 32, in increasing order
  Triple* xch = reinterpret_cast<Triple*>(lds + D_TILE_BYTES);       // the slots are idle now
  Draw* xdr = reinterpret_cast<Draw*>(xch + D_THREADS);
  const int j = tid & 63;
  const int seg = tid >> 6;
  Triple t = empty_triple();
  Draw dr = empty_draw();
  Noise noise;
  noise.group = -1;
  const int r_hi = min(D_BASE_UNIT, w_valid - v0);
  for (int r = seg * 32; r < min(seg * 32 + 32, r_hi); ++r)
    fold_logit<MODE>(a, t, dr, noise, tile[r * 64 + j], h0 + j, col0 + v0 + r);
  xch[tid] = t;
  if (MODE == 1) xdr[tid] = dr;
  __syncthreads();
  if (tid < 64 && j < n_h) {
    Triple r = xch[j];
#pragma unroll
    for (int s = 1; s < 8; ++s) merge_triple(r, xch[s * 64 + j]);
    const size_t p = (size_t)(h0 + j) * a.n_parts + part;
    a.part_m[p] = r.m;
    a.part_s[p] = r.s;
    if (MODE == 1) {
      Draw d0 = xdr[j];
#pragma unroll
      for (int s = 1; s < 8; ++s) merge_draw(d0, xdr[s * 64 + j]);
      a.part_v[p] = d0.v;
      a.part_l[p] = d0.l;
      a.part_i[p] = d0.i;
    } else {
      a.part_i[p] = r.i;
    }
  }
}

template <int NQ, int MODE>
__device__ __forceinline__ void hyper_rows(const DecodeArgs& a, int b, int r0, int r1, int lane, int wave, Triple& t,
                                           Draw& dr) {
  Noise noise;
  noise.group = -1;
  const int chunks_per_row = a.d >> 3;
  // this lane's part of the hidden row: chunk q * 64 + lane, q < NQ (chunks past the row end are zero)
  uint4 h[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int c = q * 64 + lane;
    h[q] = c < chunks_per_row ? a.H[(size_t)b * chunks_per_row + c] : uint4{0u, 0u, 0u, 0u};
  }
  const uint4* W = a.W_hyper + (size_t)b * a.cap * chunks_per_row;
  for (int r = r0 + wave; r < r1; r += 16) {
    // two rows per trip (r and r + 8) keep 2 * NQ KiB of loads in flight per wave
    const int rb = r + 8;
    const bool has_b = rb < r1;
    uint4 wa[NQ], wb[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int c = q * 64 + lane;
      const bool in = c < chunks_per_row;
      wa[q] = in ? W[(size_t)r * chunks_per_row + c] : uint4{0u, 0u, 0u, 0u};
      wb[q] = (in && has_b) ? W[(size_t)rb * chunks_per_row + c] : uint4{0u, 0u, 0u, 0u};
    }
    float sa = 0.f, sb = 0.f;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const uint32_t hw[4] = {h[q].x, h[q].y, h[q].z, h[q].w};
      const uint32_t xa[4] = {wa[q].x, wa[q].y, wa[q].z, wa[q].w};
      const uint32_t xb[4] = {wb[q].x, wb[q].y, wb[q].z, wb[q].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sa = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, xa[e]), __builtin_bit_cast(bf16x2, hw[e]), sa,
                                             false);
        sb = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, xb[e]), __builtin_bit_cast(bf16x2, hw[e]), sb,
                                             false);
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      sa += __shfl_xor(sa, o);
      sb += __shfl_xor(sb, o);
    }
    fold_logit<MODE>(a, t, dr, noise, sa, b, a.V + r);
    if (has_b) fold_logit<MODE>(a, t, dr, noise, sb, b, a.V + rb);
    if (MODE == 2 && lane == 0) {
      a.logits[(size_t)b * a.ld + a.V + r] = sa * a.inv_temperature;
      if (has_b) a.logits[(size_t)b * a.ld + a.V + rb] = sb * a.inv_temperature;
    }
  }
}

template <int MODE>
__device__ __forceinline__ void hyper_unit(const DecodeArgs& a, int b, int u, unsigned char* lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  Triple* xch = reinterpret_cast<Triple*>(lds);
  Draw* xdr = reinterpret_cast<Draw*>(xch + 8);
  const int C = min(max(a.size[b], 0), a.cap);
  const int r0 = u * D_UNIT;
  const int r1 = min(C, r0 + D_UNIT);
  Triple t = empty_triple();
  Draw dr = empty_draw();
  if (r0 < r1) {
    const int nq = (a.d + 511) >> 9;
    if (nq <= 4)
      hyper_rows<4, MODE>(a, b, r0, r1, lane, wave, t, dr);
    else
      hyper_rows<D_MAXQ, MODE>(a, b, r0, r1, lane, wave, t, dr);
  }
  // every lane of a wave holds the same triple; waves took rows w, w + 8, ...: merging by value and
  // column restores the lowest-column rule
  if (lane == 0) {
    xch[wave] = t;
    if (MODE == 1) xdr[wave] = dr;
  }
  __syncthreads();
  if (tid == 0) {
    Triple r = xch[0];
#pragma unroll
    for (int s = 1; s < 8; ++s) merge_triple(r, xch[s]);
    const size_t p = (size_t)b * a.n_parts + a.n_base_units + u;
    a.part_m[p] = r.m;
    a.part_s[p] = r.s;
    if (MODE == 1) {
      Draw d0 = xdr[0];
#pragma unroll
      for (int s = 1; s < 8; ++s) merge_draw(d0, xdr[s]);
      a.part_v[p] = d0.v;
      a.part_l[p] = d0.l;
      a.part_i[p] = d0.i;
    } else {
      a.part_i[p] = r.i;
    }
  }
}

// Dot-product units for R = 1..4 hidden rows: as hyper_rows, with all R rows in registers (R x NQ x 4 of them), so
// that every weight row streams past once, whole and contiguous -- the access pattern HBM serves best (6.3 TB/s
// for the per-sequence part of a call with 2 rows per sequence, against 5.2 on the matrix-core units).  Rows
// [r0, r1) of the matrix W against the hidden rows hrow0 .. hrow0 + R - 1; weight row r is column col0 + r.
template <int NQ, int R, int MODE>
__device__ __forceinline__ void dot_rows(const DecodeArgs& a, const uint4* W, int hrow0, int col0, int r0, int r1,
                                         int lane, int wave, Triple (&t)[R], Draw (&dr)[R]) {
  const int chunks_per_row = a.d >> 3;
  Noise noise[R];
  uint4 h[R][NQ];
#pragma unroll
  for (int i = 0; i < R; ++i) {
    noise[i].group = -1;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int c = q * 64 + lane;
      h[i][q] = c < chunks_per_row ? a.H[(size_t)(hrow0 + i) * chunks_per_row + c] : uint4{0u, 0u, 0u, 0u};
    }
  }
  for (int r = r0 + wave; r < r1; r += 16) {
    // two rows per trip (r and r + 8) keep 2 * NQ KiB of loads in flight per wave
    const int rb = r + 8;
    const bool has_b = rb < r1;
    uint4 wa[NQ], wb[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int c = q * 64 + lane;
      const bool in = c < chunks_per_row;
      wa[q] = in ? W[(size_t)r * chunks_per_row + c] : uint4{0u, 0u, 0u, 0u};
      wb[q] = (in && has_b) ? W[(size_t)rb * chunks_per_row + c] : uint4{0u, 0u, 0u, 0u};
    }
    float sa[R], sb[R];
#pragma unroll
    for (int i = 0; i < R; ++i) sa[i] = sb[i] = 0.f;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const uint32_t xa[4] = {wa[q].x, wa[q].y, wa[q].z, wa[q].w};
      const uint32_t xb[4] = {wb[q].x, wb[q].y, wb[q].z, wb[q].w};
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const uint32_t hw[4] = {h[i][q].x, h[i][q].y, h[i][q].z, h[i][q].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          sa[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, xa[e]), __builtin_bit_cast(bf16x2, hw[e]),
                                                  sa[i], false);
          sb[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, xb[e]), __builtin_bit_cast(bf16x2, hw[e]),
                                                  sb[i], false);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < R; ++i) {
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        sa[i] += __shfl_xor(sa[i], o);
        sb[i] += __shfl_xor(sb[i], o);
      }
      fold_logit<MODE>(a, t[i], dr[i], noise[i], sa[i], hrow0 + i, col0 + r);
      if (has_b) fold_logit<MODE>(a, t[i], dr[i], noise[i], sb[i], hrow0 + i, col0 + rb);
      if (MODE == 2 && lane == 0) {
        a.logits[(size_t)(hrow0 + i) * a.ld + col0 + r] = sa[i] * a.inv_temperature;
        if (has_b) a.logits[(size_t)(hrow0 + i) * a.ld + col0 + rb] = sb[i] * a.inv_temperature;
      }
    }
  }
}

// One unit: rows [r0, r1) (r1 <= r0 may be: an empty part) -> part `part` of the hidden rows hrow0 .. hrow0 + R - 1.
template <int R, int MODE>
__device__ __forceinline__ void dot_unit(const DecodeArgs& a, const uint4* W, int hrow0, int col0, int r0, int r1,
                                         int part, unsigned char* lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  Triple* xch = reinterpret_cast<Triple*>(lds);                 // [8 waves][R]
  Draw* xdr = reinterpret_cast<Draw*>(xch + 8 * R);
  Triple t[R];
  Draw dr[R];
#pragma unroll
  for (int i = 0; i < R; ++i) {
    t[i] = empty_triple();
    dr[i] = empty_draw();
  }
  if (r0 < r1) {
    const int nq = (a.d + 511) >> 9;
    if (nq <= 4)
      dot_rows<4, R, MODE>(a, W, hrow0, col0, r0, r1, lane, wave, t, dr);
    else
      dot_rows<D_MAXQ, R, MODE>(a, W, hrow0, col0, r0, r1, lane, wave, t, dr);
  }
  // every lane of a wave holds the same triples; the waves took rows w, w + 8, ...: merging by value and column
  // restores the lowest-column rule
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < R; ++i) {
      xch[wave * R + i] = t[i];
      if (MODE == 1) xdr[wave * R + i] = dr[i];
    }
  }
  __syncthreads();
  if (tid < R) {
    Triple r = xch[tid];
#pragma unroll
    for (int s = 1; s < 8; ++s) merge_triple(r, xch[s * R + tid]);
    const size_t p = (size_t)(hrow0 + tid) * a.n_parts + part;
    a.part_m[p] = r.m;
    a.part_s[p] = r.s;
    if (MODE == 1) {
      Draw d0 = xdr[tid];
#pragma unroll
      for (int s = 1; s < 8; ++s) merge_draw(d0, xdr[s * R + tid]);
      a.part_v[p] = d0.v;
      a.part_l[p] = d0.l;
      a.part_i[p] = d0.i;
    } else {
      a.part_i[p] = r.i;
    }
  }
}

constexpr size_t D_DOT_LDS = 8 * 4 * (sizeof(Triple) + sizeof(Draw));

template <int MODE>
__global__ void __launch_bounds__(D_THREADS) logits_decode_kernel(DecodeArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  // the hyper units come first: they read twice as many weight rows as a base unit, and the workgroups
  // that finish last should be the short ones
  const int n_hyper = a.B * a.units_per_seq;
  const int bid = blockIdx.x;
  if (MODE == 4) {
    base_unit<MODE>(a, bid % a.seq_units, bid / a.seq_units, 0, lds);
  } else if (bid < n_hyper) {
    hyper_unit<MODE>(a, bid / a.units_per_seq, bid % a.units_per_seq, lds);
  } else {
    const int bu = bid - n_hyper;
    // workgroup ids go round-robin over the 8 XCDs: the row groups of one unit get ids 8 apart, so they run
    // on one XCD at about the same time and its L2 serves the unit's weights to all but the first of them
    // (one group, i.e. up to 64 rows: unit = bu)
    const int units8 = (a.n_base_units + 7) >> 3;
    const int q = bu >> 3;
    const int group = q % a.n_groups;
    const int rest = q / a.n_groups;
    const int unit = (rest % units8) * 8 + (bu & 7);
    if (unit >= a.n_base_units) return;
    base_unit<MODE>(a, unit, group, MODE == 3 ? rest / units8 : 0, lds);
  }
}

// The per-sequence part of a call with R = 2..4 hidden rows per sequence (R = a.rows_per_seq) on dot-product units:
// workgroup (b, u) takes rows [256 u, 256 u + 256) of W_hyper[b], one part each (the layout of the matrix-core
// units that take more rows per sequence); plain logits only.
template <int R>
__global__ void __launch_bounds__(D_THREADS) logits_decode_rows_kernel(DecodeArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int b = blockIdx.x / a.seq_units, u = blockIdx.x % a.seq_units;
  const int C = min(max(a.size[b], 0), a.cap);
  dot_unit<R, 0>(a, a.W_hyper + (size_t)b * a.cap * (a.d >> 3), b * R, a.V, u * D_BASE_UNIT, min(C, (u + 1) * D_BASE_UNIT),
                 a.n_base_units + u, lds);
}

// A decode step of R = B <= 4 sequences: the base vocabulary on dot-product units as well (256 rows of W_base
// against all R hidden rows, part = unit as for the matrix-core units), behind the hyper units of
// logits_decode_kernel.
template <int R, int MODE>
__global__ void __launch_bounds__(D_THREADS) logits_decode_small_kernel(DecodeArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int n_hyper = a.B * a.units_per_seq;
  const int bid = blockIdx.x;
  if (bid < n_hyper) {
    hyper_unit<MODE>(a, bid / a.units_per_seq, bid % a.units_per_seq, lds);
  } else {
    const int unit = bid - n_hyper;
    if (unit >= a.n_base_units) return;
    dot_unit<R, MODE>(a, a.W_base, 0, 0, unit * D_BASE_UNIT, min(a.V, (unit + 1) * D_BASE_UNIT), unit, lds);
  }
}

template <int R>
void launch_small(int mode, unsigned grid, hipStream_t s, const DecodeArgs& a) {
  if (mode == 2)
    hipLaunchKernelGGL((logits_decode_small_kernel<R, 2>), dim3(grid), dim3(D_THREADS), D_DOT_LDS, s, a);
  else if (mode == 1)
    hipLaunchKernelGGL((logits_decode_small_kernel<R, 1>), dim3(grid), dim3(D_THREADS), D_DOT_LDS, s, a);
  else
    hipLaunchKernelGGL((logits_decode_small_kernel<R, 0>), dim3(grid), dim3(D_THREADS), D_DOT_LDS, s, a);
}

// Dense layer with K split: one workgroup per (unit, group) adds the ksplit partial tiles in a fixed order and
// runs the layer's epilogue.
__global__ void __launch_bounds__(D_THREADS) linear_reduce_kernel(DecodeArgs a) {
  __shared__ float tile[D_LINEAR_UNIT * 64];
  __shared__ float stage[64 * (D_LINEAR_UNIT + 1)];
  const int tid = threadIdx.x;
  const int unit = blockIdx.x % a.n_base_units, group = blockIdx.x / a.n_base_units;
  const int h0 = group * 64;
  const int n_rows = a.rows_dev ? min(a.B, *a.rows_dev) : a.B;
  if (h0 >= n_rows) return;
  const float* all = a.partial + (size_t)blockIdx.x * a.ksplit * (D_LINEAR_UNIT * 64);
  constexpr int PER_THREAD = D_LINEAR_UNIT * 64 / D_THREADS;
  float sum[PER_THREAD];
#pragma unroll
  for (int e = 0; e < PER_THREAD; ++e) sum[e] = 0.f;
  for (int k = 0; k < a.ksplit; ++k) {
#pragma unroll
    for (int e = 0; e < PER_THREAD; ++e) sum[e] += all[(size_t)k * (D_LINEAR_UNIT * 64) + e * D_THREADS + tid];
  }
#pragma unroll
  for (int e = 0; e < PER_THREAD; ++e) tile[e * D_THREADS + tid] = sum[e];
  __syncthreads();
  linear_epilogue(a, tile, stage, unit * D_LINEAR_UNIT, h0, min(64, n_rows - h0));
}

}  // namespace

// Parts written: n_base_units + units_per_seq per hidden row.  With `sample` the kernel works on
// logit / temperature and also leaves the best perturbed value per part (part_v, part_l, part_i); with
// `logits` it stores every logit it computes, row-major [B, V + cap] (divided by the temperature when `sample`
// is given as well: the partials are then those of the scaled logits, and nothing is drawn).
int z2z_launch_logits_decode(z2z_ctx* c, const void* H, const void* W_base, const void* W_hyper, int* n_parts,
                             bool timed, const z2z_sample_params* sample, float* logits, hipStream_t s,
                             int hyper_only_base_parts, const z2z_parts* parts, int rows_per_seq) {
  c->n_launch[Z2Z_KERNEL_DECODE]++;
  DecodeArgs a;
  memset(&a, 0, sizeof(a));
  a.H = reinterpret_cast<const uint4*>(H);
  a.W_base = reinterpret_cast<const uint4*>(W_base);
  a.W_hyper = reinterpret_cast<const uint4*>(W_hyper);
  a.size = c->st.size;
  a.B = c->cfg.B;
  a.V = c->cfg.V;
  a.cap = c->cfg.cap;
  a.d = c->cfg.d;
  a.n_base_units = (a.V + D_BASE_UNIT - 1) / D_BASE_UNIT;
  a.n_groups = (a.B + 63) / 64;
  a.units_per_seq = (a.cap + D_UNIT - 1) / D_UNIT;
  a.part_m = parts ? parts->m : c->part_m;
  a.part_s = parts ? parts->s : c->part_s;
  a.part_i = parts ? parts->i : c->part_i;
  a.part_v = c->part_v;
  a.part_l = c->part_l;
  a.logits = logits;
  a.ld = a.V + a.cap;
  a.inv_temperature = sample ? 1.0f / sample->temperature : 1.0f;
  a.key0 = sample ? (uint32_t)sample->seed : 0u;
  a.key1 = sample ? (uint32_t)(sample->seed >> 32) : 0u;
  a.ctr2 = sample ? (uint32_t)sample->step : 0u;
  a.ctr3 = sample ? (uint32_t)(sample->step >> 32) : 0u;
  *n_parts = a.n_base_units + a.units_per_seq;
  a.n_parts = *n_parts;
  unsigned grid = (unsigned)(8 * ((a.n_base_units + 7) / 8) * a.n_groups + a.B * a.units_per_seq);
  if (hyper_only_base_parts >= 0) {
    // the hyper units alone: workgroup ids below B * units_per_seq; their parts start behind the base parts
    a.n_base_units = hyper_only_base_parts;
    *n_parts = a.n_base_units + a.units_per_seq;
    a.n_parts = *n_parts;
    grid = (unsigned)(a.B * a.units_per_seq);
    if (grid == 0) return Z2Z_OK;
  }
  if (rows_per_seq > 1) {
    // the hyper part of a call with 2..64 hidden rows per sequence (the base vocabulary is another launch's):
    // one workgroup per (sequence, 256 rows of its W_hyper), the matrix-core units
    if (hyper_only_base_parts < 0 || rows_per_seq > 64 || sample || logits) return Z2Z_EUNSUPPORTED;
    a.rows_per_seq = rows_per_seq;
    a.seq_units = (a.cap + D_BASE_UNIT - 1) / D_BASE_UNIT;
    *n_parts = a.n_base_units + a.seq_units;
    a.n_parts = *n_parts;
    grid = (unsigned)(a.B * a.seq_units);
    if (grid == 0) return Z2Z_OK;
    if (timed) Z2Z_HIP_TRY(hipEventRecord(c->ev_start[c->n_timed], s));
    constexpr size_t rows_lds = D_DOT_LDS;
    if (rows_per_seq == 2 && D_DOT_ROWS >= 2)       // few enough to keep in registers: whole weight rows streamed
      hipLaunchKernelGGL(logits_decode_rows_kernel<2>, dim3(grid), dim3(D_THREADS), rows_lds, s, a);
    else if (rows_per_seq == 3 && D_DOT_ROWS >= 3)
      hipLaunchKernelGGL(logits_decode_rows_kernel<3>, dim3(grid), dim3(D_THREADS), rows_lds, s, a);
    else if (rows_per_seq == 4 && D_DOT_ROWS >= 4)
      hipLaunchKernelGGL(logits_decode_rows_kernel<4>, dim3(grid), dim3(D_THREADS), rows_lds, s, a);
    else
      hipLaunchKernelGGL(logits_decode_kernel<4>, dim3(grid), dim3(D_THREADS), D_LDS, s, a);
    if (timed) {
      Z2Z_HIP_TRY(hipEventRecord(c->ev_stop[c->n_timed], s));
      c->n_timed++;
    }
    Z2Z_HIP_TRY(hipGetLastError());
    return Z2Z_OK;
  }
  if (timed) Z2Z_HIP_TRY(hipEventRecord(c->ev_start[c->n_timed], s));
  if (hyper_only_base_parts < 0 && a.B <= D_DOT_BATCH) {
    // up to 4 sequences: their hidden rows fit in registers, so the base vocabulary streams through dot-product
    // units too (whole rows, no hand-over through LDS)
    const int mode = logits ? 2 : (sample ? 1 : 0);
    grid = (unsigned)(a.B * a.units_per_seq + a.n_base_units);
    if (a.B == 1)
      launch_small<1>(mode, grid, s, a);
    else if (a.B == 2)
      launch_small<2>(mode, grid, s, a);
    else if (a.B == 3)
      launch_small<3>(mode, grid, s, a);
    else
      launch_small<4>(mode, grid, s, a);
  } else if (logits)                                  // with `sample`: stored and folded as logit / temperature
    hipLaunchKernelGGL(logits_decode_kernel<2>, dim3(grid), dim3(D_THREADS), D_LDS, s, a);
  else if (sample)
    hipLaunchKernelGGL(logits_decode_kernel<1>, dim3(grid), dim3(D_THREADS), D_LDS, s, a);
  else
    hipLaunchKernelGGL(logits_decode_kernel<0>, dim3(grid), dim3(D_THREADS), D_LDS, s, a);
  if (timed) {
    Z2Z_HIP_TRY(hipEventRecord(c->ev_stop[c->n_timed], s));
    c->n_timed++;
  }
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// A dense layer on few rows (R up to a few hundred) is bound by the weight bytes like the decode step: the
// base-unit workgroups of the kernel above, with the layer's epilogue instead of the softmax fold.
int z2z_launch_linear_skinny(z2z_ctx* c, const void* A, const void* W, const float* bias, const void* residual,
                             int act, void* out, int R, const int32_t* rows_dev, int N, int K, hipStream_t s,
                             bool stream_f32) {
  if (c->lds_limit < D_LDS || K % D_KSLICE != 0 || N % 2 != 0 || R < 1) return Z2Z_EUNSUPPORTED;
  DecodeArgs a;
  memset(&a, 0, sizeof(a));
  a.H = reinterpret_cast<const uint4*>(A);
  a.W_base = reinterpret_cast<const uint4*>(W);
  a.B = R;
  a.V = N;
  a.cap = 0;
  a.d = K;
  a.n_base_units = (N + D_LINEAR_UNIT - 1) / D_LINEAR_UNIT;
  a.n_groups = (R + 63) / 64;
  a.units_per_seq = 0;
  a.out = out;
  a.bias = bias;
  a.residual = residual;
  a.act = act;
  a.ldo = N;
  a.stream_f32 = stream_f32 ? 1 : 0;
  a.rows_dev = rows_dev;
  // enough workgroups for every CU: split K (in phases of 1024) where the units alone are too few
  const int n_phases_all = (K / D_KSLICE + 7) / 8;
  int ksplit = 1;
  while (a.n_base_units * a.n_groups * ksplit <= 128 && ksplit * 2 <= n_phases_all) ksplit *= 2;
  const int per_part = (n_phases_all + ksplit - 1) / ksplit;
  ksplit = (n_phases_all + per_part - 1) / per_part;          // no empty parts
  a.ksplit = ksplit;
  if (ksplit > 1) {
    const size_t slots = (size_t)a.n_base_units * a.n_groups;
    const size_t need = slots * ksplit * D_LINEAR_UNIT * 64 * sizeof(float);
    if (need > c->skinny_partial_bytes) {
      Z2Z_TRY_GROW(s);
      if (c->skinny_partial) (void)hipFree(c->skinny_partial);
      c->skinny_partial = nullptr;
      c->skinny_partial_bytes = 0;
      const size_t want_bytes = need > ((size_t)16 << 20) ? need : ((size_t)16 << 20);
      if (hipMalloc(&c->skinny_partial, want_bytes) != hipSuccess) return Z2Z_ENOMEM;
      c->skinny_partial_bytes = want_bytes;
    }
    a.partial = reinterpret_cast<float*>(c->skinny_partial);
  }
  const unsigned grid = 8u * (unsigned)((a.n_base_units + 7) / 8) * (unsigned)(a.n_groups * ksplit);
  hipLaunchKernelGGL(logits_decode_kernel<3>, dim3(grid), dim3(D_THREADS), D_LDS, s, a);
  if (ksplit > 1)
    hipLaunchKernelGGL(linear_reduce_kernel, dim3((unsigned)(a.n_base_units * a.n_groups)), dim3(D_THREADS), 0, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_logits_decode_parts(const z2z_ctx* c) {
  return (c->cfg.V + D_BASE_UNIT - 1) / D_BASE_UNIT + (c->cfg.cap + D_UNIT - 1) / D_UNIT;
}

int z2z_logits_decode_seq_units(const z2z_ctx* c) { return (c->cfg.cap + D_BASE_UNIT - 1) / D_BASE_UNIT; }

void z2z_logits_decode_units(int* base_columns, int* hyper_columns) {
  *base_columns = D_BASE_UNIT;
  *hyper_columns = D_UNIT;
}

bool z2z_logits_decode_ok(const z2z_ctx* c) {
  return c->cfg.dtype == Z2Z_BF16 && c->cfg.d % D_KSLICE == 0 && c->cfg.d <= 512 * D_MAXQ && c->lds_limit >= D_LDS;
}

int z2z_logits_decode_prepare(z2z_ctx* c) {
  if (c->lds_limit < D_LDS) return Z2Z_EUNSUPPORTED;
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_decode_kernel<0>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_decode_kernel<1>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_decode_kernel<2>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_decode_kernel<3>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_decode_kernel<4>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS));
  return Z2Z_OK;
}
