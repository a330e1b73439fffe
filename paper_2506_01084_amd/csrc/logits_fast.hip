// extended_logits, bf16 MFMA kernel for gfx950 (d a multiple of 64).
//
// Workgroup tile 256 (vocabulary rows, MFMA "A") x 256 (hidden rows, MFMA "B"), 8 waves in a 2 x 4 grid,
// each wave 128 x 64 = 4 x 2 blocks of v_mfma_f32_32x32x16_bf16 (128 accumulator registers per lane).
// K advances in slabs of 64 elements (128 bytes per row).  Both operand tiles of a slab (2 x 32 KiB) are
// written straight from global memory into LDS by 16-byte global_load ... lds instructions, double
// buffered: slab s+1 streams in while slab s is multiplied, one barrier per slab.  The stream runs on
// across the vocabulary tiles of a strip, so the first slab of the next tile is in flight during the
// softmax fold of the current one.  Two waves per SIMD: one wave's LDS reads and its softmax arithmetic
// overlap the other's MFMAs.
//
// LDS layout of an operand tile: row r = 128 bytes = 8 chunks of 16 B; chunk c is stored at position
// c ^ (r & 7).  A wave's direct load writes 1 KiB = 8 rows in lane order, so lane l fetches global chunk
// (l & 7) ^ (l >> 3) of row l >> 3; the MFMA operand reads (32 rows x one chunk per half-wave) then
// touch every bank once.
//
// In the 32x32 result block a lane holds 16 vocabulary entries of one hidden row, so the running
// (max, sum-exp, argmax) of the joint softmax (zip2zip paper, section 2.3, step 8) lives in registers
// and crosses lanes once per strip.
#include "logits_common.h"

namespace {

using namespace z2z_logits;

constexpr int FT = 256;                   // tile edge, vocabulary and hidden rows
constexpr int F_SLAB = 128;               // bytes per row per K slab
constexpr int F_OPER = FT * F_SLAB;       // one operand tile of one slab: 32 KiB
constexpr int F_STAGE = 2 * F_OPER;       // A + B
constexpr int F_LDS = 2 * F_STAGE;        // two stages: 128 KiB
constexpr int F_THREADS = 512;

// 16 bytes per lane, global -> LDS without passing through registers.  The LDS address is the
// wave-uniform byte offset in M0 plus 16 * lane.  Written as inline assembly on purpose: the compiler
// cannot tell the two LDS stages apart and would make every LDS read wait for all outstanding direct
// loads, which serialises the pipeline.  Completion is awaited explicitly (s_waitcnt vmcnt(0)) before
// the barrier that publishes a stage.  One wait state is required between the write of M0 and its use.
__device__ __forceinline__ void load16_to_lds(const unsigned char* g, uint32_t lds_byte_offset) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(g), "s"(lds_byte_offset)
               : "memory");   // M0 is reserved: the compiler keeps nothing in it across statements
}

__device__ __forceinline__ uint32_t lds_offset_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// Workgroup id -> (row tile, strip) for the base part; returns false when the id maps to no work.
__device__ __forceinline__ bool map_base(const LogitsArgs& a, int bid, int* rt, int* st) {
  const int xcd = bid & 7;
  const int j = bid >> 3;
  const int per = a.map_lr * a.map_ls;
  const int g = j / per;
  const int within = j - g * per;
  const int lr = within % a.map_lr;
  const int ls = within / a.map_lr;
  const int xr = xcd % a.map_xr;
  const int xs = xcd / a.map_xr;
  const int sb_r = g % a.map_sb_r;
  const int sb_s = g / a.map_sb_r;
  *rt = (sb_r * a.map_xr + xr) * a.map_lr + lr;
  *st = (sb_s * a.map_xs + xs) * a.map_ls + ls;
  return *rt < a.row_tiles && *st < a.n_strips;
}

template <int HYPER>
__global__ void __launch_bounds__(F_THREADS) logits_fast_kernel(LogitsArgs a) {
  extern __shared__ __align__(1024) unsigned char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wv = wave & 1;    // which 128 vocabulary rows of the tile
  const int wr = wave >> 1;   // which 64 hidden rows of the tile

  int rt, st;
  int r0, r_end, n_valid;
  const unsigned char* Wp = reinterpret_cast<const unsigned char*>(a.W);
  const size_t row_bytes = (size_t)a.d * 2;
  if (HYPER) {
    if ((int)blockIdx.x >= a.n_work) return;
    st = blockIdx.x % a.n_strips;
    rt = blockIdx.x / a.n_strips;
    const int b = rt / a.row_tiles;
    r0 = b * a.rows_per_seq + (rt % a.row_tiles) * FT;
    r_end = (b + 1) * a.rows_per_seq;
    n_valid = min(max(a.size[b], 0), a.w_rows);
    Wp += (size_t)b * a.w_rows * row_bytes;
  } else {
    if (!map_base(a, blockIdx.x, &rt, &st)) return;
    r0 = rt * FT;
    r_end = a.rows;
    n_valid = a.w_rows;
  }
  const unsigned char* Hp = reinterpret_cast<const unsigned char*>(a.H);
  const int vt0 = st * a.strip;
  const int vt_end = min(min(vt0 + a.strip, a.n_vtiles), (n_valid + FT - 1) / FT);
  const int n_tiles = vt_end - vt0;          // vocabulary tiles this workgroup sweeps (may be <= 0)
  const int n_slabs = (int)(row_bytes / F_SLAB);

  Triple run[2];
  run[0] = empty_triple();
  run[1] = empty_triple();

  // ---- loader: lane l of wave w, instruction i moves the chunk that lands at LDS byte
  //      ((w * 4 + i) * 8 + (l >> 3)) * 128 + (l & 7) * 16 of the operand tile --------------------------
  const uint32_t lds_base = lds_offset_of(lds);
  const int ld_row = lane >> 3;
  const int ld_chunk = (lane & 7) ^ ld_row;
  const unsigned char* gB[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (wave * 4 + i) * 8 + ld_row;
    gB[i] = Hp + (size_t)min(r0 + row, r_end - 1) * row_bytes + ld_chunk * 16;
  }
  const unsigned char* gA[4];
  auto set_tile = [&](int vt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (wave * 4 + i) * 8 + ld_row;
      gA[i] = Wp + (size_t)min(vt * FT + row, n_valid - 1) * row_bytes + ld_chunk * 16;
    }
  };
  auto issue = [&](int slab, int stage) {
    const uint32_t A = lds_base + stage * F_STAGE + wave * 4096;
    const uint32_t Bt = A + F_OPER;
    const size_t kb = (size_t)slab * F_SLAB;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      load16_to_lds(gA[i] + kb, A + i * 1024);
      load16_to_lds(gB[i] + kb, Bt + i * 1024);
    }
  };

  // ---- MFMA operand addresses (bytes inside an operand tile), swizzle folded in ---------------------
  const int sw = lane & 7;
  const int half = lane >> 5;
  int offA[4], offB[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) offA[i] = (wv * 128 + i * 32 + (lane & 31)) * F_SLAB;
#pragma unroll
  for (int j = 0; j < 2; ++j) offB[j] = (wr * 64 + j * 32 + (lane & 31)) * F_SLAB;

  f32x16 acc[4][2];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  };

  if (n_tiles > 0) {
    zero_acc();
    set_tile(vt0);
    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wave's direct loads have landed
    __syncthreads();
    const int total = n_tiles * n_slabs;
    int slab = 0, vt = vt0;
    for (int g = 0; g < total; ++g) {
      const int stage = g & 1;
      // stream in the next slab (possibly the first slab of the next vocabulary tile)
      if (g + 1 < total) {
        if (slab + 1 == n_slabs) {
          set_tile(vt + 1);
          issue(0, stage ^ 1);
        } else {
          issue(slab + 1, stage ^ 1);
        }
      }
      const unsigned char* A = lds + stage * F_STAGE;
      const unsigned char* Bt = A + F_OPER;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int pos = ((2 * q + half) ^ sw) << 4;
        uint4 fa[4], fb[2];
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const uint4*>(A + offA[i] + pos);
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const uint4*>(Bt + offB[j] + pos);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),
                                                                __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
      }

      if (slab + 1 == n_slabs) {
        // ---- this vocabulary tile is complete: fold its 128 x 64 logits into the running triples -----
        const int v0 = vt * FT;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int hrow = r0 + wr * 64 + j * 32 + (lane & 31);
          float tmax = kNegInf;
          int targ = kNoColumn;
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int col = v0 + wv * 128 + i * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
              float x = acc[i][j][v];
              if (col >= n_valid) x = kNegInf;
              acc[i][j][v] = x;
              if (x > tmax) {
                tmax = x;
                targ = col;
              }
              if (a.logits != nullptr && col < n_valid && hrow < r_end)
                a.logits[(size_t)hrow * a.ld + a.col0 + col] = x;
            }
          if (tmax > run[j].m) {
            run[j].s = (run[j].m == kNegInf) ? 0.f : run[j].s * __expf(run[j].m - tmax);
            run[j].m = tmax;
            run[j].i = a.col0 + targ;
          }
          if (run[j].m != kNegInf) {
            float add = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int v = 0; v < 16; ++v) add += __expf(acc[i][j][v] - run[j].m);
            run[j].s += add;
          }
        }
        zero_acc();
        slab = 0;
        ++vt;
      } else {
        ++slab;
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);   // the next slab is in LDS ...
      __syncthreads();                      // ... for every wave, and everyone is done with this one
    }
  }

  // ---- end of strip: lanes l and l+32 hold the same hidden row; then the two vocabulary halves ------
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    Triple o;
    o.m = __shfl_xor(run[j].m, 32);
    o.s = __shfl_xor(run[j].s, 32);
    o.i = __shfl_xor(run[j].i, 32);
    merge_triple(run[j], o);
  }
  Triple* xch = reinterpret_cast<Triple*>(lds);   // [4 row quarters][64 rows]; operand tiles are idle now
  if (wv == 1 && lane < 32) {
    xch[wr * 64 + lane] = run[0];
    xch[wr * 64 + 32 + lane] = run[1];
  }
  __syncthreads();
  if (wv == 0 && lane < 32) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      merge_triple(run[j], xch[wr * 64 + j * 32 + lane]);
      const int hrow = r0 + wr * 64 + j * 32 + lane;
      if (hrow < r_end) {
        const size_t p = (size_t)(a.part0 + st) * a.rows + hrow;
        a.part_m[p] = run[j].m;
        a.part_s[p] = run[j].s;
        a.part_i[p] = run[j].i;
      }
    }
  }
}

}  // namespace

int z2z_launch_logits_fast(bool hyper, const LogitsArgs& a, unsigned grid, hipStream_t s) {
  if (hyper)
    hipLaunchKernelGGL(logits_fast_kernel<1>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else
    hipLaunchKernelGGL(logits_fast_kernel<0>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_logits_fast_prepare(z2z_ctx* c) {
  if (c->lds_limit < F_LDS) return Z2Z_EUNSUPPORTED;
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<0>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<1>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  return Z2Z_OK;
}
