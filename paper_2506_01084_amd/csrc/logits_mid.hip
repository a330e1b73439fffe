// extended_logits, base-vocabulary part for up to 192 hidden rows in all (gfx950, bf16, d a multiple of 64): a
// decode step of 65..192 sequences, a few rows per sequence at a small batch, a short chunk.  (zip2zip paper,
// section 2.3, steps 7-9.)
//
// With so few rows the part is bound by the bytes of W_base, like the one-row-per-sequence step.  That kernel's
// base units hold 64 hidden rows in registers (one pass over W_base per 64 rows); the 256 x 256 tile kernel stages
// both operands through two LDS stages and waits for memory once per slab (3.4-3.5 TB/s of weights at these row
// counts).  Here the weights never touch LDS:
//
//   workgroup = 8 waves = one tile of 256 weight rows x all hidden rows; wave w owns weight rows 32 w .. 32 w + 31:
//   2, 4 or 6 blocks of v_mfma_f32_32x32x16_bf16 (the kernel is built for up to 64, 128 and 192 rows).
//   K advances in slabs of 64.  A wave loads its own weight fragments straight from global memory in MFMA operand
//   layout (lane = row, 16 bytes of each 32-byte k-step; the four k-steps of a slab use up whole 128-byte lines),
//   two slabs at a time (256 contiguous bytes per row: +5 % over single slabs), four to five slabs ahead of their
//   use in six register buffers (two to three ahead in four with 6 blocks of accumulators).  The hidden rows of a
//   slab (up to 192 x 128 bytes, shared by the 8 waves, served by
//   L2) go straight from global memory into one of three LDS stages, two slabs ahead, in the tile kernel's
//   swizzled layout (conflict-free operand reads); one barrier per slab.
//   The tiles start their walk over K at different slabs (+5-7 %: see below).
//
// Measured at V = 128256, d = 4096: 4.1-4.9 TB/s of W_base (the tile kernel: 3.4-3.5; the decode kernel's base
// units in a launch of their own: 4.5 at up to 64 rows).  The fold of the finished tile into (max, sum-exp,
// argmax) triples is the tile kernel's; the 8 waves' triples of a hidden row are merged through LDS and leave one
// part per (row, weight tile).
#include "logits_mid.h"

#include <string.h>

namespace {

using namespace z2z_logits;

constexpr int M_WAVES = 8;
constexpr int M_THREADS = 64 * M_WAVES;
constexpr int M_WT = 32 * M_WAVES;        // weight rows of a workgroup's tile
constexpr int M_HT = 192;                 // hidden rows of a call at most (the builds below: 2, 4 or 6 blocks of 32)
constexpr int M_MAX_ROWS = M_HT;
constexpr int M_SLAB = 128;               // bytes per row per K slab (64 bf16)
constexpr int M_STAGE = M_HT * M_SLAB;    // the hidden rows of one slab: 24 KiB
constexpr int M_NSTAGE = 3;
constexpr int M_LDS = M_NSTAGE * M_STAGE;
// weight register buffers per instance (what fits beside 16 NJV accumulators without spilling inside the K loop)
#ifndef M_NBUF
#define M_NBUF 6                          // up to 128 hidden rows
#endif
#ifndef M_NBUF_6
#define M_NBUF_6 4                        // up to 192 (96 accumulator registers)
#endif
// 1: the weights of two consecutive slabs are requested together, every other step: 256 contiguous bytes per row
#ifndef M_PAIR
#define M_PAIR 1
#endif
static_assert(M_WAVES * M_HT * (int)(sizeof(Triple) + sizeof(Draw)) <= M_LDS, "the waves' triples are merged in the idle stages");

// 16 bytes per lane, global -> LDS without passing through registers (as in the tile kernel): address = 64-bit
// scalar base + 32-bit per-lane offset; the LDS address is the wave-uniform byte offset in M0 plus 16 * lane.
// Inline assembly, so the compiler does not count these loads: every wait for them is written out below.
__device__ __forceinline__ void load16_to_lds(const unsigned char* base, uint32_t lane_offset, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_offset), "s"(base), "s"(lds_dst)
               : "memory");
}

// Wait until at most N of this wave's loads are in flight.  Inline assembly with a memory clobber: the compiler
// moves no load across it, so the number of requests that follow a given one is the number written below.
template <int N>
__device__ __forceinline__ void wait_loads() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

__device__ __forceinline__ uint32_t lds_offset_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// NJV: blocks of 32 hidden rows the instance is built for (rows of the tile <= 32 NJV); NBUF: weight register
// buffers (slabs in flight + the one in use); SMODE: 0 = fold the logits, 1 = fold logit / T and the Gumbel-max
// draw (a.sample = 1: part_v, part_l, and the drawn column in part_i), 2 = store logit / T and fold it
// (a.sample = 2) -- the tile kernel's epilogues for its modes 0, 6 and 7; 3 = a dense layer with K split over
// gridDim.y workgroups per tile: the fp32 partial tile goes to a.partial[ks][row][col] (the tile kernel's mode 5).
template <int NJV, int NBUF, int SMODE>
__global__ void __launch_bounds__(M_THREADS) logits_mid_kernel(LogitsArgs a) {
  extern __shared__ __align__(1024) unsigned char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5;
  const int vt = blockIdx.x;                               // weight tile
  const int r0 = 0;                                        // (one row tile: the call has at most M_HT rows)
  // SMODE 3 (a dense layer's partial sums): the rows that exist may be known on the device only, and blockIdx.y is
  // the part of K this workgroup takes (slabs [ks * slabs_per_part, ...))
  const int r_end = (SMODE == 3 && a.rows_dev) ? min(a.rows, *a.rows_dev) : a.rows;
  if (r_end <= r0) return;                                 // (the whole workgroup)
  const int nr = min(32 * NJV, r_end - r0);                // valid hidden rows
  const int n_valid = a.w_rows;
  const int v0 = vt * M_WT;
  const size_t row_bytes = (size_t)a.d * 2;
  const int ks = SMODE == 3 ? (int)blockIdx.y : 0;
  const int slab0 = SMODE == 3 ? ks * a.slabs_per_part : 0;
  const int n_slabs = SMODE == 3 ? min(a.slabs_per_part, (int)(row_bytes / M_SLAB) - slab0) : (int)(row_bytes / M_SLAB);

  // The tiles walk K in the same order but start at different slabs (tile t at slab t mod n_slabs, wrapping round):
  // at any moment the workgroups in flight ask for different 128-byte columns of their weight rows, not all for
  // the same one, which would keep landing on the same few memory channels (rows are a power of two apart).
#ifndef M_ROTATE
#define M_ROTATE 1
#endif
  const int rot = M_ROTATE ? vt % n_slabs : 0;
  auto slab_at = [&](int s) {                              // step -> slab (steps past the end repeat the last one)
    const int x = min(s, n_slabs - 1) + rot;
    return slab0 + (x >= n_slabs ? x - n_slabs : x);
  };
  // weights: this lane's row, clamped onto the last one that exists; 16 bytes at (2 q + half) * 16 of a slab
  const int wrow = min(v0 + wave * 32 + (lane & 31), n_valid - 1);
  const unsigned char* wp = reinterpret_cast<const unsigned char*>(a.W) + (size_t)wrow * row_bytes + half * 16;
  auto load_w = [&](uint4 (&w)[4], int slab) {
    const unsigned char* p = wp + (size_t)slab_at(slab) * M_SLAB;
#pragma unroll
    for (int q = 0; q < 4; ++q) w[q] = *reinterpret_cast<const uint4*>(p + q * 32);
  };
  // hidden rows: the 4 NJV groups of 8 rows of a slab are dealt to the waves, group g = i * 8 + wave for the
  // wave's i-th request; lane l moves, for row g * 8 + (l >> 3), the chunk that lands at position l & 7 of the row's
  // 128 LDS bytes: chunk (l & 7) ^ ((row >> 1) & 7).  Rows past the last valid one read the last valid one.
  constexpr int HL = (4 * NJV) / M_WAVES;                  // requests per wave and slab
  static_assert(HL * M_WAVES == 4 * NJV, "whole groups per wave");
  const unsigned char* Ht = reinterpret_cast<const unsigned char*>(a.H) + (size_t)r0 * row_bytes;
  const uint32_t lds_base = lds_offset_of(lds);
  uint32_t hsrc[HL];
#pragma unroll
  for (int i = 0; i < HL; ++i) {
    const int row = (i * M_WAVES + wave) * 8 + (lane >> 3);
    hsrc[i] = (uint32_t)(min(row, nr - 1) * (int)row_bytes + (((lane & 7) ^ ((row >> 1) & 7)) << 4));
  }
  auto issue_h = [&](int slab, int stage) {
    const unsigned char* p = Ht + (size_t)slab_at(slab) * M_SLAB;
#pragma unroll
    for (int i = 0; i < HL; ++i)
      load16_to_lds(p, hsrc[i], lds_base + (uint32_t)(stage * M_STAGE + (i * M_WAVES + wave) * 1024));
  };
  // operand reads: block j, row lane & 31, logical chunk 2 q + half
  const int sw = (lane >> 1) & 7;
  const int offB = (lane & 31) * M_SLAB;

  f32x16 acc[1][NJV];
#pragma unroll
  for (int j = 0; j < NJV; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][j][v] = 0.f;

  auto compute = [&](const uint4 (&w)[4], int stage) {
    const unsigned char* Bs = lds + stage * M_STAGE + offB;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int pos = ((2 * q + half) ^ sw) << 4;
#pragma unroll
      for (int j = 0; j < NJV; ++j) {
        const uint4 b = *reinterpret_cast<const uint4*>(Bs + j * 32 * M_SLAB + pos);
        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w[q]),
                                                            __builtin_bit_cast(bf16x8, b), acc[0][j], 0, 0, 0);
      }
    }
  };

  // One step = one slab.  On entry to step s: stage s % 3 holds the hidden rows of slab s, visible to all; those of
  // slab s + 1 are on their way into stage (s + 1) % 3; buffer s % NBUF holds the weights of slab s, the weights of
  // the next slabs are on their way.  Loads complete in the order of their requests.  Requested during step s, in
  // this order: the hidden rows of slab s + 2 (HL requests; the stage's last readers, those of slab s - 1, passed
  // the barrier of step s - 1), then weights: of slab s + NBUF - 1 (4 requests), or with M_PAIR of the slabs
  // s + NBUF - 2 and s + NBUF - 1 before every other step (8 requests).  Before the barrier of step s the hidden
  // rows of slab s + 1 must have landed: after them came the weight requests of step s - 1 and the HL + weight
  // requests of step s, HL + 8 in all either way, which may stay in flight.
  int stage = 0;                                           // s % 3
  uint4 w[NBUF][4];
  static_assert(!M_PAIR || NBUF % 2 == 0, "pairs of slabs");
  auto requests = [&](int u, int s) {                      // u = s % NBUF, a constant where this is expanded
    issue_h(s + 2, stage == 0 ? 2 : stage - 1);            // stage (s + 2) % 3
    if (M_PAIR) {
      if ((u & 1) == 0) {                                  // the two buffers used last
        load_w(w[(u + NBUF - 2) % NBUF], s + NBUF - 2);
        load_w(w[(u + NBUF - 1) % NBUF], s + NBUF - 1);
      }
    } else {
      load_w(w[(u + NBUF - 1) % NBUF], s + NBUF - 1);
    }
  };
  // (in_loop: the count above holds inside the loop, where every weight request feeds a later iteration.  In the
  // steps after the loop the compiler drops the requests whose buffers no step reads any more, so there
  // everything in flight is awaited: a handful of steps per tile.)
  auto finish = [&](int u, bool in_loop) {
    compute(w[u], stage);
    if (in_loop)
      wait_loads<HL + 8>();
    else
      wait_loads<0>();
    __syncthreads();
    stage = stage == 2 ? 0 : stage + 1;
  };

  issue_h(0, 0);
  issue_h(1, 1);
  constexpr int PRE = M_PAIR ? NBUF - 2 : NBUF - 1;        // slabs whose weights are requested ahead of the loop
#pragma unroll
  for (int u = 0; u < PRE; ++u) load_w(w[u], u);
  wait_loads<HL + 4 * PRE>();                              // slab 0's hidden rows; what followed may be in flight
  __syncthreads();
  // whole rounds of the buffers without a test inside (a loop the register allocator keeps the buffers fixed in),
  // then the rest
  int s0 = 0;
  for (; s0 + NBUF <= n_slabs; s0 += NBUF) {
#pragma unroll
    for (int u = 0; u < NBUF; ++u) {
      requests(u, s0 + u);
      finish(u, true);
    }
  }
#pragma unroll
  for (int u = 0; u < NBUF - 1; ++u)
    if (s0 + u < n_slabs) {                                // (uniform)
      requests(u, s0 + u);
      finish(u, false);
    }
  // the requests past the end of the stream (slabs clamped onto the last one) must land before the stages are reused
  wait_loads<0>();
  __syncthreads();

  // ---- fold the tile, then one triple (and draw) per hidden row --------------------------------------------
  Triple run[NJV];
  Draw draw[NJV];
#pragma unroll
  for (int j = 0; j < NJV; ++j) {
    run[j] = empty_triple();
    draw[j] = empty_draw();
  }
  const int col_base = v0 + wave * 32 + half * 4;
  if (SMODE == 3) {
    // a dense layer's K part: the fp32 tile as it is; linear_sum_kernel adds the parts and runs the layer's epilogue
    store_partial_tile<1, NJV>(acc, a.partial + (size_t)ks * a.rows * a.ldo, a.ldo, r0, r_end, col_base, n_valid);
    return;
  }
  if (SMODE == 1)
    fold_tile_sample<1, NJV>(acc, run, draw, a, r0, col_base, n_valid);
  else if (SMODE == 2)
    fold_tile_store<1, NJV>(acc, run, a, r0, r_end, col_base, n_valid);
  else
    fold_tile<1, NJV>(acc, run, col_base, a.col0, n_valid, v0 + M_WT > n_valid);
#pragma unroll
  for (int j = 0; j < NJV; ++j) {                          // lanes l and l + 32 hold the same hidden row
    Triple o;
    o.m = __shfl_xor(run[j].m, 32);
    o.s = __shfl_xor(run[j].s, 32);
    o.i = __shfl_xor(run[j].i, 32);
    merge_triple(run[j], o);
    if (SMODE == 1) {
      Draw od;
      od.v = __shfl_xor(draw[j].v, 32);
      od.l = __shfl_xor(draw[j].l, 32);
      od.i = __shfl_xor(draw[j].i, 32);
      merge_draw(draw[j], od);
    }
  }
  Triple* xch = reinterpret_cast<Triple*>(lds);            // [wave][hidden row of the tile]
  Draw* xdr = reinterpret_cast<Draw*>(xch + M_WAVES * M_HT);
  if (lane < 32) {
#pragma unroll
    for (int j = 0; j < NJV; ++j) {
      xch[wave * M_HT + j * 32 + lane] = run[j];
      if (SMODE == 1) xdr[wave * M_HT + j * 32 + lane] = draw[j];
    }
  }
  __syncthreads();
  if (tid < nr) {
    Triple t = xch[tid];
#pragma unroll
    for (int w = 1; w < M_WAVES; ++w) merge_triple(t, xch[w * M_HT + tid]);
    const size_t p = (size_t)(r0 + tid) * a.n_parts + a.part0 + vt;
    a.part_m[p] = t.m;
    a.part_s[p] = t.s;
    if (SMODE == 1) {
      Draw dw = xdr[tid];
#pragma unroll
      for (int w = 1; w < M_WAVES; ++w) merge_draw(dw, xdr[w * M_HT + tid]);
      a.part_v[p] = dw.v;
      a.part_l[p] = dw.l;
      a.part_i[p] = dw.i;
    } else {
      a.part_i[p] = t.i;
    }
  }
}

}  // namespace

bool z2z_logits_mid_ok(const z2z_ctx* c, int rows) {
  return c->mid_ready && c->cfg.dtype == Z2Z_BF16 && c->cfg.d % 64 == 0 && rows >= 1 && rows <= M_MAX_ROWS;
}

// The base part of a call: one part per tile of 256 weight rows.  a: H, rows, d, the part arrays, n_parts, part0
// filled by the caller; with a.sample = 1 or 2 also the generator words, inv_temperature and part_v / part_l or
// logits / ld, as for the tile kernel's sampling modes.
int z2z_launch_logits_mid(z2z_ctx* c, LogitsArgs a, const void* W, int w_rows, int col0, hipStream_t s) {
  if (!z2z_logits_mid_ok(c, a.rows) || w_rows < 1) return Z2Z_EUNSUPPORTED;
  a.W = W;
  a.w_rows = w_rows;
  a.col0 = col0;
  a.n_vtiles = (w_rows + M_WT - 1) / M_WT;
  c->n_launch[Z2Z_KERNEL_MID]++;
  // (two workgroups of the 64-row build per weight tile for 65..128 rows, sharing the tile's weights through an
  // XCD's L2, measured slower than one of the 128-row build: 383 against 293 us at config 2's shape)
  const dim3 grid((unsigned)a.n_vtiles), block(M_THREADS);
  // builds: 2, 4 or 6 blocks of 32 hidden rows; the sampling calls come with one row per sequence and more than 64
  // of them.  (8 blocks, up to 256 rows, leave the registers for four buffers at most and measured level with the
  // tile kernel: 650 against 645 us for a decode step of 256 sequences.)
  const int blocks = a.rows <= 64 ? 2 : (a.rows <= 128 ? 4 : 6);
  if (a.sample == 1) {
    if (blocks <= 4)
      hipLaunchKernelGGL((logits_mid_kernel<4, M_NBUF, 1>), grid, block, M_LDS, s, a);
    else
      hipLaunchKernelGGL((logits_mid_kernel<6, M_NBUF_6, 1>), grid, block, M_LDS, s, a);
  } else if (a.sample == 2) {
    if (blocks <= 4)
      hipLaunchKernelGGL((logits_mid_kernel<4, M_NBUF, 2>), grid, block, M_LDS, s, a);
    else
      hipLaunchKernelGGL((logits_mid_kernel<6, M_NBUF_6, 2>), grid, block, M_LDS, s, a);
  } else {
    if (blocks == 2)
      hipLaunchKernelGGL((logits_mid_kernel<2, M_NBUF, 0>), grid, block, M_LDS, s, a);
    else if (blocks == 4)
      hipLaunchKernelGGL((logits_mid_kernel<4, M_NBUF, 0>), grid, block, M_LDS, s, a);
    else
      hipLaunchKernelGGL((logits_mid_kernel<6, M_NBUF_6, 0>), grid, block, M_LDS, s, a);
  }
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// Parts of K per weight tile: the split (parts of at least four slabs, at most 16 parts) with the fewest slab steps
// on the busiest CU -- rounds of 256 workgroups x (slabs per part + 3 for filling and draining the pipeline); a
// split that puts a few workgroups into a second round costs a whole round.
int z2z_linear_mid_ksplit(int N, int K) {
  const int n_vt = (N + M_WT - 1) / M_WT, n_slabs = K / 64;
  int best = 1;
  long long best_cost = -1;
  for (int ks = 1; ks <= 16 && (ks == 1 || n_slabs / ks >= 4); ++ks) {
    const int per = (n_slabs + ks - 1) / ks;
    const int parts = (n_slabs + per - 1) / per;           // no empty parts
    const long long cost = (long long)((n_vt * parts + 255) / 256) * (per + 3);
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best = parts;
    }
  }
  return best;
}

// Dense layer out = act(A W^T + bias) + residual on R <= 128 rows (or fewer, *rows_dev): the weight-streaming kernel
// leaves ksplit fp32 partial tiles per weight tile in `partial` ([ksplit][R][N]); the caller sums them
// (linear_sum_kernel in dense.hip).  Returns the ksplit chosen through *ksplit_out.
int z2z_launch_linear_mid(z2z_ctx* c, const void* A, const void* W, int R, const int32_t* rows_dev, int N, int K,
                          float* partial, size_t partial_floats, int* ksplit_out, hipStream_t s) {
  if (!z2z_logits_mid_ok(c, R) || R > 128 || K % 64 != 0 || N < 1) return Z2Z_EUNSUPPORTED;
  const int n_vt = (N + M_WT - 1) / M_WT, n_slabs = K / 64;
  const int ksplit = z2z_linear_mid_ksplit(N, K);
  const int per = (n_slabs + ksplit - 1) / ksplit;
  if ((size_t)ksplit * R * N > partial_floats) return Z2Z_ELIMIT;
  LogitsArgs a;
  memset(&a, 0, sizeof(a));
  a.H = A;
  a.W = W;
  a.rows = R;
  a.d = K;
  a.w_rows = N;
  a.n_vtiles = n_vt;
  a.ldo = N;
  a.rows_dev = rows_dev;
  a.ksplit = ksplit;
  a.slabs_per_part = per;
  a.partial = partial;
  *ksplit_out = ksplit;
  c->n_launch[Z2Z_KERNEL_MID]++;
  const dim3 grid((unsigned)n_vt, (unsigned)ksplit), block(M_THREADS);
  if (R <= 64)
    hipLaunchKernelGGL((logits_mid_kernel<2, M_NBUF, 3>), grid, block, M_LDS, s, a);
  else
    hipLaunchKernelGGL((logits_mid_kernel<4, M_NBUF, 3>), grid, block, M_LDS, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_logits_mid_tiles(int w_rows) { return (w_rows + M_WT - 1) / M_WT; }

int z2z_logits_mid_prepare(z2z_ctx* c) {
  if (c->lds_limit < M_LDS) return Z2Z_EUNSUPPORTED;
  const void* kernels[9] = {reinterpret_cast<const void*>(logits_mid_kernel<2, M_NBUF, 3>),
                            reinterpret_cast<const void*>(logits_mid_kernel<4, M_NBUF, 3>),
                            reinterpret_cast<const void*>(logits_mid_kernel<2, M_NBUF, 0>),
                            reinterpret_cast<const void*>(logits_mid_kernel<4, M_NBUF, 0>),
                            reinterpret_cast<const void*>(logits_mid_kernel<4, M_NBUF, 1>),
                            reinterpret_cast<const void*>(logits_mid_kernel<4, M_NBUF, 2>),
                            reinterpret_cast<const void*>(logits_mid_kernel<6, M_NBUF_6, 0>),
                            reinterpret_cast<const void*>(logits_mid_kernel<6, M_NBUF_6, 1>),
                            reinterpret_cast<const void*>(logits_mid_kernel<6, M_NBUF_6, 2>)};
  for (int k = 0; k < 9; ++k)
    Z2Z_HIP_TRY(hipFuncSetAttribute(kernels[k], hipFuncAttributeMaxDynamicSharedMemorySize, M_LDS));
  return Z2Z_OK;
}
