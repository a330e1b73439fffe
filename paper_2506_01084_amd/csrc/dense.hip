// Dense layers out = act(A W^T + bias) + residual on the logits kernels (bf16): which kernel serves which row
// count, the workgroup -> tile mapping of the tile kernel, and the sum of K-split partial tiles.  Used by the
// learned hyper-encoder (zip2zip paper, section 2.2) and by the backward pass of the loss (section 2.4).
#include "logits_common.h"
#include "logits_mid.h"

#include <string.h>

#include <algorithm>

using namespace z2z_logits;

namespace {

// Dense layer with K split over workgroups of the tile kernel: out = act(sum_ks partial[ks] + bias) + residual,
// the parts added in a fixed order; one thread per run of 4 columns.
__global__ void __launch_bounds__(256) linear_sum_kernel(const float* partial, int ksplit, int rows, const int32_t* rows_dev,
                                                         int N, const float* bias, int act, const void* residual,
                                                         void* out, int stream_f32) {
  const int n4 = N >> 2;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  const int r_end = rows_dev ? min(rows, *rows_dev) : rows;
  if (i >= (long long)r_end * n4) return;
  const int row = (int)(i / n4), col = (int)(i % n4) * 4;
  const size_t at = (size_t)row * N + col;
  float4 x = *reinterpret_cast<const float4*>(partial + at);
  for (int k = 1; k < ksplit; ++k) {
    const float4 y = *reinterpret_cast<const float4*>(partial + (size_t)k * rows * N + at);
    x.x += y.x;
    x.y += y.y;
    x.z += y.z;
    x.w += y.w;
  }
  if (bias) {
    const float4 b = *reinterpret_cast<const float4*>(bias + col);
    x.x += b.x;
    x.y += b.y;
    x.z += b.z;
    x.w += b.w;
  }
  if (act == 1) {
    x.x = gelu_erf(x.x);
    x.y = gelu_erf(x.y);
    x.z = gelu_erf(x.z);
    x.w = gelu_erf(x.w);
  }
  if (stream_f32) {                                  // fp32 residual and output: no rounding
    if (residual) {
      const float4 rv = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(residual) + at);
      x.x += rv.x;
      x.y += rv.y;
      x.z += rv.z;
      x.w += rv.w;
    }
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + at) = x;
    return;
  }
  if (residual) {
    const uint2 rv = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(residual) + at);
    x.x += __uint_as_float(rv.x << 16);
    x.y += __uint_as_float(rv.x & 0xFFFF0000u);
    x.z += __uint_as_float(rv.y << 16);
    x.w += __uint_as_float(rv.y & 0xFFFF0000u);
  }
  uint2 o;
  o.x = bf16_bits_rne(x.x) | (bf16_bits_rne(x.y) << 16);
  o.y = bf16_bits_rne(x.z) | (bf16_bits_rne(x.w) << 16);
  *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + at) = o;
}

// out[b][c][r] = in[b][r][c] (bf16) for r < R (and r < *rows_dev when given), c < C; columns up to ld_out of out
// beyond that are zero (they pad the contraction of a product over rows).  64 x 64 tiles through LDS, 256
// threads, 16 bytes per lane on both sides (ld_in and ld_out are multiples of 8, the bases 16-byte aligned); grid
// (ceil(ld_out / 64), ceil(C / 64), batch).
__global__ void __launch_bounds__(256) transpose_bf16_kernel(const uint16_t* in, uint16_t* out, int R, const int32_t* rows_dev,
                                                             int C, int ld_in, int ld_out, size_t in_batch,
                                                             size_t out_batch) {
  __shared__ uint16_t t[64][72];                     // [column of the tile][row of the tile], rows padded
  if (rows_dev) R = min(R, *rows_dev);
  const uint16_t* src = in + (size_t)blockIdx.z * in_batch;
  uint16_t* dst = out + (size_t)blockIdx.z * out_batch;
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int chunk = threadIdx.x & 7, line = threadIdx.x >> 3;       // 8 chunks of 8 elements per line, 32 lines
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int i = line + 32 * h;                     // row of the tile
    const int r = r0 + i, c = c0 + chunk * 8;
    uint4 v = {0u, 0u, 0u, 0u};
    if (r < R && c < ld_in) v = *reinterpret_cast<const uint4*>(src + (size_t)r * ld_in + c);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      t[chunk * 8 + 2 * e][i] = (uint16_t)(w[e] & 0xFFFFu);
      t[chunk * 8 + 2 * e + 1][i] = (uint16_t)(w[e] >> 16);
    }
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int i = line + 32 * h;                     // column of the tile = row of the output
    const int c = c0 + i, r = r0 + chunk * 8;
    if (c < C && r < ld_out)
      *reinterpret_cast<uint4*>(dst + (size_t)c * ld_out + r) = *reinterpret_cast<const uint4*>(&t[i][chunk * 8]);
  }
}

}  // namespace

int z2z_launch_transpose(const void* in, void* out, int R, const int32_t* rows_dev, int C, int ld_in, int ld_out,
                         int batch, size_t in_batch, size_t out_batch, hipStream_t s) {
  if (R < 1 || C < 1 || batch < 1) return Z2Z_OK;
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3((ld_out + 63) / 64, (C + 63) / 64, batch), dim3(256), 0, s,
                     reinterpret_cast<const uint16_t*>(in), reinterpret_cast<uint16_t*>(out), R, rows_dev, C, ld_in,
                     ld_out, in_batch, out_batch);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_linear(z2z_ctx* c, const void* A, const void* W, const float* bias, const void* residual, int act,
                      void* out, int R, const int32_t* rows_dev, int N, int K, hipStream_t s, const int32_t* k_dev,
                      bool stream_f32) {
  // up to 128 rows (a decode step's new entries through the learned encoder at a small batch): bound by the weight
  // bytes; the weight-streaming kernel with K split over workgroups, its fp32 partial tiles summed with the layer's
  // epilogue.  (The encoder's newest-entry pass at d = 4096, d_ff = 4 d: 347 -> 302 us for 8 sequences, 401 -> 374
  // for 40; with the 192-row build for 129..192 rows laid out the tile kernel's K split below is faster, 432
  // against 459 us for 64 sequences.)
  if (R <= 128 && !k_dev && K % 64 == 0 && N % 4 == 0 && c->opt_logits_kernel == 0 && z2z_logits_mid_ok(c, R)) {
    const int ksplit = z2z_linear_mid_ksplit(N, K);
    const size_t need = (size_t)ksplit * R * N * sizeof(float);
    if (need > c->skinny_partial_bytes) {
      Z2Z_TRY_GROW(s);
      if (c->skinny_partial) (void)hipFree(c->skinny_partial);
      c->skinny_partial = nullptr;
      c->skinny_partial_bytes = 0;
      const size_t want = need > ((size_t)64 << 20) ? need : ((size_t)64 << 20);
      if (hipMalloc(&c->skinny_partial, want) != hipSuccess) return Z2Z_ENOMEM;
      c->skinny_partial_bytes = want;
    }
    int ks = 0;
    int rc = z2z_launch_linear_mid(c, A, W, R, rows_dev, N, K, reinterpret_cast<float*>(c->skinny_partial),
                                   c->skinny_partial_bytes / sizeof(float), &ks, s);
    if (rc != Z2Z_OK) return rc;
    const long long n_threads = (long long)R * (N / 4);
    hipLaunchKernelGGL(linear_sum_kernel, dim3((unsigned)((n_threads + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<const float*>(c->skinny_partial), ks, R, rows_dev, N, bias, act, residual, out,
                       stream_f32 ? 1 : 0);
    Z2Z_HIP_TRY(hipGetLastError());
    return Z2Z_OK;
  }
  // more rows than the 64 the decode-step kernel serves per pass over the weights, but fewer 256 x 256 output
  // tiles than would give every CU one (a few hundred rows, or up to a few thousand with a narrow layer): the
  // tile kernel with K split over workgroups, so that the weights stream once for all rows and every CU has a
  // part (without it a layer of 144 tiles ran on 144 of the 256 CUs: 1.5 ms against 0.8 ms for 422 rows)
  if (R > 64 && c->fast_ready && K % 64 == 0 && N % 8 == 0 && c->opt_logits_kernel != 1) {
    const int row_tiles = (R + 255) / 256, n_vt = (N + 255) / 256, tiles = row_tiles * n_vt;
    const int n_slabs = K / 64;
    int ksplit = 1;
    while (tiles * ksplit < 192 && n_slabs / (ksplit * 2) >= 8) ksplit *= 2;
    if (ksplit > 1) {
      const int per = (n_slabs + ksplit - 1) / ksplit;
      ksplit = (n_slabs + per - 1) / per;
      const size_t need = (size_t)ksplit * R * N * sizeof(float);
      if (need > c->skinny_partial_bytes) {
        Z2Z_TRY_GROW(s);
        if (c->skinny_partial) (void)hipFree(c->skinny_partial);
        c->skinny_partial = nullptr;
        c->skinny_partial_bytes = 0;
        const size_t want = need > ((size_t)64 << 20) ? need : ((size_t)64 << 20);
        if (hipMalloc(&c->skinny_partial, want) != hipSuccess) return Z2Z_ENOMEM;
        c->skinny_partial_bytes = want;
      }
      LogitsArgs a;
      memset(&a, 0, sizeof(a));
      a.H = A;
      a.W = W;
      a.rows = R;
      a.rows_per_seq = R;
      a.d = K;
      a.w_rows = N;
      a.n_vtiles = n_vt;
      a.row_tiles = row_tiles;
      a.strip = 1;
      a.n_strips = n_vt;
      a.ldo = N;
      a.rows_dev = rows_dev;
      a.ksplit = ksplit;
      a.slabs_per_part = per;
      a.partial = reinterpret_cast<float*>(c->skinny_partial);
      int rc = z2z_launch_logits_fast(5, a, (unsigned)(tiles * ksplit), s);
      if (rc != Z2Z_OK) return rc;
      const long long n_threads = (long long)R * (N / 4);
      hipLaunchKernelGGL(linear_sum_kernel, dim3((unsigned)((n_threads + 255) / 256)), dim3(256), 0, s,
                         reinterpret_cast<const float*>(c->skinny_partial), ksplit, R, rows_dev, N, bias, act, residual,
                         out, stream_f32 ? 1 : 0);
      Z2Z_HIP_TRY(hipGetLastError());
      return Z2Z_OK;
    }
  }
  // few rows: bound by the weight bytes, which the decode-step kernel streams at HBM rate (it re-reads them
  // once per 64 rows, so it loses to the tile kernel beyond a few hundred rows)
  if (R <= 512 && c->skinny_ready && K % 128 == 0 && N % 2 == 0 && c->opt_logits_kernel != 2)
    return z2z_launch_linear_skinny(c, A, W, bias, residual, act, out, R, rows_dev, N, K, s, stream_f32);
  if (!c->fast_ready || K % 64 != 0 || N % 8 != 0 || R < 1) return Z2Z_EUNSUPPORTED;
  LogitsArgs a;
  memset(&a, 0, sizeof(a));
  a.H = A;
  a.W = W;
  a.rows = R;
  a.rows_per_seq = R;
  a.d = K;
  a.w_rows = N;
  a.n_vtiles = (N + 255) / 256;
  a.row_tiles = (R + 255) / 256;
  // one tile per workgroup when the row count is only known on the device: the launch cannot be shaped to
  // it, and the finer the grain, the less of the last round of workgroups is wasted
  a.strip = (!rows_dev && (long long)a.row_tiles * a.n_vtiles >= 2048) ? 4 : 1;
  a.n_strips = (a.n_vtiles + a.strip - 1) / a.strip;
  a.n_work = a.row_tiles * a.n_strips;
  a.out = out;
  a.bias = bias;
  a.residual = residual;
  a.act = act;
  a.ldo = N;
  a.stream_f32 = stream_f32 ? 1 : 0;
  a.rows_dev = nullptr;
  a.k_dev = k_dev;
  if (rows_dev && a.row_tiles >= 16) {
    // the real row count is on the device: what an XCD owns is settled there (see map_rows_dev)
    a.rows_dev = rows_dev;
    a.map_lr = 4;
    unsigned grid;
    if (a.n_strips % 8 == 0) {
      // every XCD takes an eighth of the weight tiles and all row tiles
      const int strips_per_xcd = a.n_strips / 8;
      a.map_xs = 8;
      a.map_xr = 1;
      a.map_ls = strips_per_xcd >= 8 ? 8 : (strips_per_xcd >= 4 ? 4 : (strips_per_xcd >= 2 ? 2 : 1));
      a.strip_blocks = (strips_per_xcd + a.map_ls - 1) / a.map_ls;
      const int row_blocks = (a.row_tiles + a.map_lr - 1) / a.map_lr;
      grid = 8u * (unsigned)(a.map_lr * a.map_ls) * (unsigned)row_blocks * (unsigned)a.strip_blocks;
    } else {
      a.map_xs = 1;
      a.map_xr = 8;
      a.map_ls = a.n_strips >= 8 ? 8 : (a.n_strips >= 4 ? 4 : (a.n_strips >= 2 ? 2 : 1));
      a.strip_blocks = (a.n_strips + a.map_ls - 1) / a.map_ls;
      const int tiles_per_xcd = (a.row_tiles + 7) / 8;
      const int row_blocks = (tiles_per_xcd + a.map_lr - 1) / a.map_lr;
      grid = 8u * (unsigned)(a.map_lr * a.map_ls) * (unsigned)row_blocks * (unsigned)a.strip_blocks;
    }
    return z2z_launch_logits_fast(2, a, grid, s);
  }
  // (fewer row tiles than that: the tiles beyond the real rows only exit early)
  // Workgroup ids go round-robin over the 8 XCDs and the mapping gives XCD (xr_i, xs_i) the row tiles whose
  // block index is xr_i mod map_xr and the strips whose block index is xs_i mod map_xs: an XCD's share is the
  // product of the two counts.  Take the mapping with the smallest largest share (nobody waits for one XCD),
  // and among equals the one with the largest blocks (what runs together shares operand tiles through L2).
  {
    long long best_load = -1;
    int best_area = 0;
    const int xrs[4] = {8, 4, 2, 1};
    for (int xi = 0; xi < 4; ++xi)
      for (int lr = 4; lr >= 1; lr >>= 1)
        for (int ls = 8; ls >= 1; ls >>= 1) {
          const int xr = xrs[xi], xs = 8 / xr;
          long long worst = 0;
          for (int i = 0; i < xr; ++i) {
            long long rows_i = 0;
            for (int blk = i; blk * lr < a.row_tiles; blk += xr) rows_i += (blk + 1) * lr <= a.row_tiles ? lr : a.row_tiles - blk * lr;
            for (int j = 0; j < xs; ++j) {
              long long strips_j = 0;
              for (int blk = j; blk * ls < a.n_strips; blk += xs) strips_j += (blk + 1) * ls <= a.n_strips ? ls : a.n_strips - blk * ls;
              if (rows_i * strips_j > worst) worst = rows_i * strips_j;
            }
          }
          const int area = lr * ls;
          if (best_load < 0 || worst < best_load || (worst == best_load && area > best_area)) {
            best_load = worst;
            best_area = area;
            a.map_lr = lr;
            a.map_ls = ls;
            a.map_xr = xr;
            a.map_xs = xs;
          }
        }
  }
  const int sb_rows = a.map_xr * a.map_lr, sb_strips = a.map_xs * a.map_ls;
  a.map_sb_r = (a.row_tiles + sb_rows - 1) / sb_rows;
  const int sb_s = (a.n_strips + sb_strips - 1) / sb_strips;
  const unsigned grid = 8u * (unsigned)(a.map_lr * a.map_ls) * (unsigned)a.map_sb_r * (unsigned)sb_s;
  a.rows_dev = rows_dev;
  return z2z_launch_logits_fast(2, a, grid, s);
}

