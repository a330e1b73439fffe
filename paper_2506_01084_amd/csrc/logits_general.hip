// extended_logits, general tile kernel (any d that is a multiple of the 16-byte chunk, bf16 or fp32).
//
// Both operands are stored with the contraction index k contiguous, so a lane fetches 16 bytes of a row
// for each MFMA operand.  The vocabulary rows are the MFMA "A" operand and the hidden rows the "B"
// operand: in the 32x32 result block a lane then holds 16 vocabulary entries of ONE hidden row, so the
// running (max, sum-exp, argmax) of a row is kept in that lane's registers and crosses lanes only once
// per strip.  A workgroup owns one tile of hidden rows and sweeps a strip of vocabulary tiles.
// This is the fallback for shapes the fast bf16 kernel does not take, and the fp32 path.
#include "logits_common.h"

namespace {

using namespace z2z_logits;

// ------------------------------------------------------------------------------------------------
// Tile kernel, 128 (vocabulary) x 128 (hidden rows) per workgroup, 4 waves of 64 x 64, K slabs of
// 128 bytes per row.  LDS holds two buffers of (128 + 128) rows x 128 B; the 16-byte chunk c of row
// r sits at chunk (c ^ ((r >> 1) & 7)) so that the 16 rows a quarter-wave reads hit all 64 banks.
// T = bf16 bits (uint16_t) or float.
// ------------------------------------------------------------------------------------------------
constexpr int TV = 128;
constexpr int TR = 128;
constexpr int SLAB_BYTES = 128;
constexpr int TILE_BYTES = TV * SLAB_BYTES;   // one operand tile in LDS (16 KiB)

template <typename T>
__device__ __forceinline__ void mfma_chunk(const uint4& a, const uint4& b, f32x16& acc);

template <>
__device__ __forceinline__ void mfma_chunk<uint16_t>(const uint4& a, const uint4& b, f32x16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0,
                                                0, 0);
}

template <>
__device__ __forceinline__ void mfma_chunk<float>(const uint4& a, const uint4& b, f32x16& acc) {
  // a 16-byte chunk holds 4 consecutive k; lanes 0-31 and 32-63 hold different chunks, and the
  // pairing of k between the two operands is the same, so any order of the 4 steps is a valid sum
  const f32x4 af = __builtin_bit_cast(f32x4, a);
  const f32x4 bf = __builtin_bit_cast(f32x4, b);
#pragma unroll
  for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[e], bf[e], acc, 0, 0, 0);
}

template <typename T, int HYPER>
__global__ void __launch_bounds__(256) logits_general_kernel(LogitsArgs a) {
  __shared__ __align__(16) unsigned char lds[4 * TILE_BYTES];   // [buf][A|B][TILE_BYTES]
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wv = wave & 1;    // which 64 vocabulary rows of the tile
  const int wr = wave >> 1;   // which 64 hidden rows of the tile

  // ---- which rows, which W, which strip ---------------------------------------------------------
  const int st = blockIdx.x % a.n_strips;
  const int rt = blockIdx.x / a.n_strips;
  int r0, r_end, n_valid;
  const unsigned char* Wp = reinterpret_cast<const unsigned char*>(a.W);
  const size_t row_bytes = (size_t)a.d * sizeof(T);
  if (HYPER) {
    const int b = rt / a.row_tiles;
    r0 = b * a.rows_per_seq + (rt % a.row_tiles) * TR;
    r_end = (b + 1) * a.rows_per_seq;
    n_valid = min(max(a.size[b], 0), a.w_rows);
    Wp += (size_t)b * a.w_rows * row_bytes;
  } else {
    r0 = rt * TR;
    r_end = a.rows;
    n_valid = a.w_rows;
  }
  const unsigned char* Hp = reinterpret_cast<const unsigned char*>(a.H);
  const int vt0 = st * a.strip;
  const int vt1 = min(vt0 + a.strip, a.n_vtiles);

  Triple run[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    run[j] = empty_triple();
  }

  // global -> LDS staging: thread t moves chunks t, t+256, t+512, t+768 of each operand tile
  const int n_slabs = (int)((row_bytes + SLAB_BYTES - 1) / SLAB_BYTES);

  for (int vt = vt0; vt < vt1; ++vt) {
    const int v0 = vt * TV;
    if (v0 >= n_valid) break;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 stage_a[4], stage_b[4];
    auto fetch = [&](int slab) {
      const size_t kb = (size_t)slab * SLAB_BYTES;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int id = tid + 256 * i;
        const int row = id >> 3;
        const int c = id & 7;
        const size_t off = kb + (size_t)c * 16;
        const bool in_k = off < row_bytes;
        const int wrow = min(v0 + row, n_valid - 1);
        const int hrow = min(r0 + row, r_end - 1);
        const uint4 z = {0u, 0u, 0u, 0u};
        stage_a[i] = in_k ? *reinterpret_cast<const uint4*>(Wp + (size_t)wrow * row_bytes + off) : z;
        stage_b[i] = in_k ? *reinterpret_cast<const uint4*>(Hp + (size_t)hrow * row_bytes + off) : z;
      }
    };
    auto stash = [&](int buf) {
      unsigned char* A = lds + (size_t)buf * 2 * TILE_BYTES;
      unsigned char* Bt = A + TILE_BYTES;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int id = tid + 256 * i;
        const int row = id >> 3;
        const int c = id & 7;
        const int o = row * SLAB_BYTES + ((c ^ ((row >> 1) & 7)) << 4);
        *reinterpret_cast<uint4*>(A + o) = stage_a[i];
        *reinterpret_cast<uint4*>(Bt + o) = stage_b[i];
      }
    };

    fetch(0);
    __syncthreads();          // the previous tile's readers are done with buffer 0
    stash(0);
    __syncthreads();
    for (int slab = 0; slab < n_slabs; ++slab) {
      const int buf = slab & 1;
      if (slab + 1 < n_slabs) fetch(slab + 1);
      const unsigned char* A = lds + (size_t)buf * 2 * TILE_BYTES;
      const unsigned char* Bt = A + TILE_BYTES;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int chunk = 2 * q + (lane >> 5);
        uint4 fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int row = wv * 64 + i * 32 + (lane & 31);
          fa[i] = *reinterpret_cast<const uint4*>(A + row * SLAB_BYTES + ((chunk ^ ((row >> 1) & 7)) << 4));
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int row = wr * 64 + j * 32 + (lane & 31);
          fb[j] = *reinterpret_cast<const uint4*>(Bt + row * SLAB_BYTES + ((chunk ^ ((row >> 1) & 7)) << 4));
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) mfma_chunk<T>(fa[i], fb[j], acc[i][j]);
      }
      if (slab + 1 < n_slabs) {
        stash(buf ^ 1);       // buffer buf^1 was last read two slabs ago, behind the barrier below
        __syncthreads();
      }
    }

    // ---- epilogue of this tile: fold the 128 x 128 logits into the running triples -------------
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int hrow = r0 + wr * 64 + j * 32 + (lane & 31);
      float tmax = kNegInf;
      int targ = kNoColumn;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int col = v0 + wv * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          float x = acc[i][j][v];
          if (col >= n_valid) x = kNegInf;
          acc[i][j][v] = x;
          if (x > tmax) {
            tmax = x;
            targ = col;
          }
          if (a.logits != nullptr && col < n_valid && hrow < r_end) a.logits[(size_t)hrow * a.ld + a.col0 + col] = x;
        }
      if (tmax > run[j].m) {
        run[j].s = (run[j].m == kNegInf) ? 0.f : run[j].s * __expf(run[j].m - tmax);
        run[j].m = tmax;
        run[j].i = a.col0 + targ;
      }
      if (run[j].m != kNegInf) {
        float add = 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) add += __expf(acc[i][j][v] - run[j].m);
        run[j].s += add;
      }
    }
  }

  // ---- end of strip: lanes l and l+32 hold the same hidden row; then the two vocabulary halves ---
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    Triple o;
    o.m = __shfl_xor(run[j].m, 32);
    o.s = __shfl_xor(run[j].s, 32);
    o.i = __shfl_xor(run[j].i, 32);
    merge_triple(run[j], o);
  }
  __syncthreads();            // all waves are done reading the operand tiles
  Triple* xch = reinterpret_cast<Triple*>(lds);   // [2 row halves][64 rows]
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
        const size_t p = (size_t)hrow * a.n_parts + a.part0 + st;
        a.part_m[p] = run[j].m;
        a.part_s[p] = run[j].s;
        a.part_i[p] = run[j].i;
      }
    }
  }
}

}  // namespace

int z2z_launch_logits_general(bool bf16, bool hyper, const LogitsArgs& a, unsigned grid, hipStream_t s) {
  if (bf16) {
    if (hyper)
      hipLaunchKernelGGL((logits_general_kernel<uint16_t, 1>), dim3(grid), dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((logits_general_kernel<uint16_t, 0>), dim3(grid), dim3(256), 0, s, a);
  } else {
    if (hyper)
      hipLaunchKernelGGL((logits_general_kernel<float, 1>), dim3(grid), dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((logits_general_kernel<float, 0>), dim3(grid), dim3(256), 0, s, a);
  }
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}
