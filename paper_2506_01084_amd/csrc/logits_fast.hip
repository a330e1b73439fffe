// extended_logits, bf16 MFMA kernel for gfx950 (d a multiple of 64), one wave per SIMD.
//
// Workgroup tile 256 (vocabulary rows, MFMA "A") x 256 (hidden rows, MFMA "B"), 4 waves in a 2 x 2 grid,
// each wave 128 x 128 = 4 x 4 blocks of v_mfma_f32_32x32x16_bf16 (256 accumulator registers per lane):
// per 16-deep k-step a wave reads 8 operand fragments from LDS for 16 MFMAs, which keeps the LDS read
// port at about half of its 128 B/clk (a 128 x 64 wave tile needs three quarters of it and starves the
// matrix cores).  With one wave per SIMD all overlap is inside the instruction stream: the fragments of
// k-step t+1 are read while the MFMAs of k-step t run, and the global->LDS requests of slab s+2 are issued
// as soon as slab s has been read.
//
// K advances in slabs of 64 elements (128 bytes per row, four k-steps): the global -> LDS stream moves
// whole 128-byte lines, which it does markedly faster than half lines (measured on a bare streaming
// kernel: 14-22 TB/s against 12-15 TB/s out of L2).  Both operand tiles of a slab (2 x 32 KiB) go straight
// from global memory into LDS (16-byte global_load ... lds), two stages.  Once per slab, in the middle of
// its last k-step, the waves meet at a barrier: at that point everybody has read the slab completely (its
// stage is refilled with slab s+2) and slab s+1 has landed (its first fragments are read next).  The stream
// runs on across the vocabulary tiles of a strip.
//
// LDS layout of an operand tile: row r = 128 bytes = 8 chunks of 16 B; chunk c is stored at position
// c ^ ((r >> 1) & 7).  The LDS has 64 four-byte banks and serves a 16-byte-per-lane read 16 lanes at a
// time; an MFMA operand read has 16 consecutive lanes on 16 consecutive rows at one logical chunk, whose
// bank group is (r & 1) * 8 + position -- all 16 distinct with this swizzle.
//
// In the 32x32 result block a lane holds 16 vocabulary entries of one hidden row, so the running
// (max, sum-exp, argmax) of the joint softmax (zip2zip paper, section 2.3, step 8) lives in registers
// and crosses lanes once per strip.
#include "logits_common.h"

namespace {

using namespace z2z_logits;

constexpr int FT = 256;                   // tile edge, vocabulary and hidden rows
constexpr int F_SLAB = 128;               // bytes per row per K slab (64 bf16)
constexpr int F_OPER = FT * F_SLAB;       // one operand tile of one slab: 32 KiB
constexpr int F_STAGE = 2 * F_OPER;       // A + B
constexpr int F_NSTAGE = 2;
constexpr int F_LDS = F_NSTAGE * F_STAGE; // 128 KiB
constexpr int F_THREADS = 256;

// 16 bytes per lane, global -> LDS without passing through registers: address = 64-bit scalar base +
// 32-bit per-lane offset; the LDS address is the wave-uniform byte offset in M0 plus 16 * lane.  Inline
// assembly on purpose: the compiler cannot tell the LDS stages apart and would make every LDS read wait
// for all outstanding direct loads.  Completion is awaited explicitly (s_waitcnt vmcnt) before the
// barrier that publishes a stage.  One wait state is required between the write of M0 and its use.
__device__ __forceinline__ void load16_to_lds(const unsigned char* base, uint32_t lane_offset, uint32_t lds_byte_offset) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_offset), "s"(base), "s"(lds_byte_offset)
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

struct Frags {
  uint4 a[4];
  uint4 b[4];
};

template <int HYPER>
__global__ void __launch_bounds__(F_THREADS) logits_fast_kernel(LogitsArgs a) {
  extern __shared__ __align__(1024) unsigned char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wv = wave & 1;    // which 128 vocabulary rows of the tile
  const int wr = wave >> 1;   // which 128 hidden rows of the tile

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
  const unsigned char* Hp = reinterpret_cast<const unsigned char*>(a.H) + (size_t)r0 * row_bytes;
  const int vt0 = st * a.strip;
  const int vt_end = min(min(vt0 + a.strip, a.n_vtiles), (n_valid + FT - 1) / FT);
  const int n_tiles = vt_end - vt0;          // vocabulary tiles this workgroup sweeps (may be <= 0)
  const int n_slabs = (int)(row_bytes / F_SLAB);

  Triple run[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) run[j] = empty_triple();

  // ---- loader: lane l of wave w, instruction i moves the chunk that lands at LDS byte
  //      ((w * 8 + i) * 8 + (l >> 3)) * 128 + (l & 7) * 16 of the operand tile; offsets are relative to
  //      the first row of the tile, rows past the last valid one are clamped onto it ------------------
  const uint32_t lds_base = lds_offset_of(lds);
  const int ld_row = lane >> 3;                                  // row inside the 8-row group
  const int limB = r_end - 1 - r0;                               // last valid hidden row of the tile
  const unsigned char* Wtile = Wp;
  int limA = 0;                                                  // last valid vocabulary row of the tile
  auto set_tile = [&](int vt) {
    Wtile = Wp + (size_t)vt * FT * row_bytes;
    limA = n_valid - 1 - vt * FT;
  };
  // request the slab that follows (lslab, lvt) in the stream, if any, and advance the cursor; the
  // per-lane offsets are recomputed each time (a few VALU operations) rather than kept in registers.
  // A request is 16 instructions per wave; issue_rows(i) issues the pair for row group i so that the
  // caller can place the pairs between MFMAs.
  int lslab = 0, lvt = vt0;
  uint32_t isA = 0, isB = 0;                 // LDS destinations of the slab being requested
  const unsigned char* is_ga = Wp;
  const unsigned char* is_gb = Hp;
  bool is_on = false;
  auto issue_begin = [&](int stage) {
    is_on = lvt < vt_end;
    isA = lds_base + stage * F_STAGE + wave * 8192;
    isB = isA + F_OPER;
    is_ga = Wtile + (size_t)lslab * F_SLAB;
    is_gb = Hp + (size_t)lslab * F_SLAB;
  };
  auto issue_rows = [&](int i) {
    if (is_on) {
      const int row = (wave * 8 + i) * 8 + ld_row;
      const int chunk16 = ((lane & 7) ^ ((row >> 1) & 7)) * 16;
      load16_to_lds(is_ga, (uint32_t)(min(row, limA) * (int)row_bytes + chunk16), isA + i * 1024);
      load16_to_lds(is_gb, (uint32_t)(min(row, limB) * (int)row_bytes + chunk16), isB + i * 1024);
    }
  };
  auto issue_end = [&]() {
    if (is_on && ++lslab == n_slabs) {
      lslab = 0;
      ++lvt;
      if (lvt < vt_end) set_tile(lvt);
    }
  };
  auto issue_next = [&](int stage) {
    issue_begin(stage);
#pragma unroll
    for (int i = 0; i < 8; ++i) issue_rows(i);
    issue_end();
  };

  // ---- MFMA operand addresses (bytes inside an operand tile), swizzle folded in ---------------------
  const int sw = (lane >> 1) & 7;   // ((row >> 1) & 7) of every row this lane reads
  const int half = lane >> 5;
  const int offA0 = (wv * 128 + (lane & 31)) * F_SLAB;
  const int offB0 = (wr * 128 + (lane & 31)) * F_SLAB;
  auto read_frags = [&](Frags& f, int stage, int q) {
    const unsigned char* A = lds + stage * F_STAGE + offA0 + (((2 * q + half) ^ sw) << 4);
    const unsigned char* Bt = lds + stage * F_STAGE + F_OPER + offB0 + (((2 * q + half) ^ sw) << 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) f.a[i] = *reinterpret_cast<const uint4*>(A + i * 32 * F_SLAB);
#pragma unroll
    for (int j = 0; j < 4; ++j) f.b[j] = *reinterpret_cast<const uint4*>(Bt + j * 32 * F_SLAB);
  };

  f32x16 acc[4][4];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  };
  auto mfma_rows = [&](const Frags& f, int i_lo, int i_hi) {
#pragma unroll
    for (int i = i_lo; i < i_hi; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i]),
                                                            __builtin_bit_cast(bf16x8, f.b[j]), acc[i][j], 0, 0, 0);
  };

  if (n_tiles > 0) {
    zero_acc();
    set_tile(vt0);
    const int total = n_tiles * n_slabs;
    // prologue: slabs 0 and 1 requested, slab 0 landed and visible, its first fragments on the way
    issue_next(0);
    issue_next(1);
    if (total >= 2)
      __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16): all but the youngest slab (16 requests per wave)
    else
      __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    Frags f0, f1;
    read_frags(f0, 0, 0);
    int g = 0;
    for (int vt = vt0; vt < vt_end; ++vt) {
      for (int slab = 0; slab < n_slabs; ++slab, ++g) {
        const int stage = g & 1;
        read_frags(f1, stage, 1);
        mfma_rows(f0, 0, 4);
        read_frags(f0, stage, 2);
        mfma_rows(f1, 0, 4);
        read_frags(f1, stage, 3);
        mfma_rows(f0, 0, 4);
        // last k-step: a quarter of its MFMAs, then the slab hand-over; the 16 requests for slab g+2
        // are then issued between the remaining MFMAs (a burst of them would leave the matrix cores
        // idle for as long as it takes to issue)
        mfma_rows(f1, 0, 1);
        const bool more = g + 1 < total;
        if (more) {
          __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): slab g+1 (the only one in flight) has landed
          __syncthreads();                      // slab g+1 visible to all; everyone has read slab g
          read_frags(f0, stage ^ 1, 0);
          issue_begin(stage);                   // refill this stage with slab g+2
        } else {
          is_on = false;
        }
#pragma unroll
        for (int i = 1; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f1.a[i]),
                                                                __builtin_bit_cast(bf16x8, f1.b[j]), acc[i][j], 0, 0, 0);
            if (((i - 1) * 4 + j) % 3 == 2 || (i == 3 && j == 3)) {
              __builtin_amdgcn_sched_barrier(0);
              const int grp = ((i - 1) * 4 + j) / 3;          // 0..3 -> row groups 2*grp, 2*grp+1
              issue_rows(2 * grp);
              issue_rows(2 * grp + 1);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        if (more) issue_end();
      }
      // ---- this vocabulary tile is complete: fold its 128 x 128 logits into the running triples ------
      const int v0 = vt * FT;
      fold_tile<4, 4>(acc, run, v0 + wv * 128 + half * 4, a.col0, n_valid, v0 + FT > n_valid);
      zero_acc();
    }
  }

  // ---- end of strip: lanes l and l+32 hold the same hidden row; then the two vocabulary halves ------
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    Triple o;
    o.m = __shfl_xor(run[j].m, 32);
    o.s = __shfl_xor(run[j].s, 32);
    o.i = __shfl_xor(run[j].i, 32);
    merge_triple(run[j], o);
  }
  __syncthreads();                                 // every wave is done with the operand stages
  Triple* xch = reinterpret_cast<Triple*>(lds);    // [2 row halves][128 rows]
  if (wv == 1 && lane < 32) {
#pragma unroll
    for (int j = 0; j < 4; ++j) xch[wr * 128 + j * 32 + lane] = run[j];
  }
  __syncthreads();
  if (wv == 0 && lane < 32) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      merge_triple(run[j], xch[wr * 128 + j * 32 + lane]);
      const int hrow = r0 + wr * 128 + j * 32 + lane;
      if (hrow < r_end) {
        const size_t p = (size_t)hrow * a.n_parts + a.part0 + st;
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
