// extended_logits: launch planning (which tile kernel, strips, workgroup mapping), the merge of the
// per-strip partial triples, and the scratch buffer that holds them.
//
// The base part (columns < V, shared W_base) and the hyper part (columns V.., one W_hyper per sequence,
// only the first C_b rows exist: section 2.3 of the zip2zip paper, "Consistent Vocabulary Updates") are
// two launches; both leave (max, sum-exp, argmax) triples per (strip, row), merged in column order.
#include "logits_common.h"

#include <string.h>

#include <algorithm>

namespace {

using namespace z2z_logits;

// ROW_THREADS (64 or 256) threads per hidden row: they take the row's partial triples round-robin
// (contiguous in memory), merge across lanes, then across the waves of the row; merge_triple keeps the
// lowest column among equal maxima, so the order of the merges does not matter.  A block is 256 threads:
// four rows with a wave each (few parts per row: prefill), or one row (a thousand parts: decode steps).
template <int ROW_THREADS>
__global__ void __launch_bounds__(256) logits_combine_kernel(const float* part_m, const float* part_s,
                                                             const int32_t* part_i, int n_parts, int rows,
                                                             int32_t* argmax, float* mx, float* lse) {
  constexpr int ROWS_PER_BLOCK = 256 / ROW_THREADS;
  const int lane = threadIdx.x & 63;
  const int t = threadIdx.x % ROW_THREADS;
  const int r = blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / ROW_THREADS;
  Triple tr = empty_triple();
  if (r < rows) {
    const size_t base = (size_t)r * n_parts;
    for (int p = t; p < n_parts; p += ROW_THREADS) {
      Triple o;
      o.m = part_m[base + p];
      o.s = part_s[base + p];
      o.i = part_i[base + p];
      merge_triple(tr, o);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Triple o;
    o.m = __shfl_xor(tr.m, off);
    o.s = __shfl_xor(tr.s, off);
    o.i = __shfl_xor(tr.i, off);
    merge_triple(tr, o);
  }
  if (ROW_THREADS > 64) {
    __shared__ Triple xch[4];
    if (lane == 0) xch[threadIdx.x >> 6] = tr;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
      for (int w = 1; w < 4; ++w) merge_triple(tr, xch[w]);
    }
  }
  if (t == 0 && r < rows) {
    if (argmax) argmax[r] = tr.i;
    if (mx) mx[r] = tr.m;
    if (lse) lse[r] = tr.m + logf(tr.s);
  }
}

int launch_combine(const z2z_ctx* c, int n_parts, int rows, int32_t* argmax, float* mx, float* lse, hipStream_t s) {
  if (n_parts > 256)
    hipLaunchKernelGGL(logits_combine_kernel<256>, dim3(rows), dim3(256), 0, s, c->part_m, c->part_s, c->part_i,
                       n_parts, rows, argmax, mx, lse);
  else
    hipLaunchKernelGGL(logits_combine_kernel<64>, dim3((rows + 3) / 4), dim3(256), 0, s, c->part_m, c->part_s,
                       c->part_i, n_parts, rows, argmax, mx, lse);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// Full-logits output only: unused hyper slots read -inf.
__global__ void __launch_bounds__(256) logits_mask_kernel(float* logits, int rows, int rows_per_seq, int V, int cap,
                                                          const int32_t* size) {
  const int r = blockIdx.x;
  if (r >= rows) return;
  const int b = r / rows_per_seq;
  const int C = min(max(size[b], 0), cap);
  float* row = logits + (size_t)r * (V + cap) + V;
  for (int c = C + threadIdx.x; c < cap; c += blockDim.x) row[c] = kNegInf;
}

// Sampling: merge the parts of a hidden row into the drawn column (largest perturbed value, lowest column
// among equals) and its log-probability, scaled logit there minus the log-sum-exp of the scaled logits.
// One block of 256 threads per row.
__global__ void __launch_bounds__(256) sample_combine_kernel(const float* part_m, const float* part_s,
                                                             const float* part_v, const float* part_l,
                                                             const int32_t* part_i, int n_parts, int rows,
                                                             int32_t* token, float* logprob) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x;
  Triple tr = empty_triple();        // .i unused here
  float bv = kNegInf, bl = 0.f;
  int bi = kNoColumn;
  const size_t base = (size_t)r * n_parts;
  for (int p = threadIdx.x; p < n_parts; p += 256) {
    Triple o;
    o.m = part_m[base + p];
    o.s = part_s[base + p];
    o.i = kNoColumn;
    merge_triple(tr, o);
    const float v = part_v[base + p];
    const int i = part_i[base + p];
    if (v > bv || (v == bv && i < bi)) {
      bv = v;
      bl = part_l[base + p];
      bi = i;
    }
  }
  __shared__ Triple xt[4];
  __shared__ float xv[4], xl[4];
  __shared__ int xi[4];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Triple o;
    o.m = __shfl_xor(tr.m, off);
    o.s = __shfl_xor(tr.s, off);
    o.i = kNoColumn;
    merge_triple(tr, o);
    const float v = __shfl_xor(bv, off), l = __shfl_xor(bl, off);
    const int i = __shfl_xor(bi, off);
    if (v > bv || (v == bv && i < bi)) {
      bv = v;
      bl = l;
      bi = i;
    }
  }
  if (lane == 0) {
    const int w = threadIdx.x >> 6;
    xt[w] = tr;
    xv[w] = bv;
    xl[w] = bl;
    xi[w] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      merge_triple(tr, xt[w]);
      if (xv[w] > bv || (xv[w] == bv && xi[w] < bi)) {
        bv = xv[w];
        bl = xl[w];
        bi = xi[w];
      }
    }
    token[r] = bi;
    if (logprob) logprob[r] = bl - (tr.m + logf(tr.s));
  }
}

// nll[r] = lse[r] - H[r] . W[target[r]] (section 2.4 of the zip2zip paper: the next-token objective taken
// over the compressed sequence; the target is a base token or a hypertoken of the row's sequence).  One
// wave per hidden row, 16-byte chunks, fp32 accumulation of the products of the stored values (what the
// tile kernels compute for that column).  target < 0: no target, 0; a column that does not exist: +inf.
template <bool BF16>
__global__ void __launch_bounds__(256) target_nll_kernel(const uint4* H, const uint4* W_base, const uint4* W_hyper,
                                                         const int32_t* size, const int32_t* targets,
                                                         const float* lse, float* nll, int rows, int rows_per_seq,
                                                         int V, int cap, int d) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int b = r / rows_per_seq;
  const int t = targets[r];
  const int C = min(max(size[b], 0), cap);
  if (t < 0 || t >= V + C) {
    if (lane == 0) nll[r] = t < 0 ? 0.f : INFINITY;
    return;
  }
  constexpr int EPC = BF16 ? 8 : 4;
  const int n_chunks = d / EPC;
  const uint4* w = t < V ? W_base + (size_t)t * n_chunks : W_hyper + ((size_t)b * cap + (t - V)) * n_chunks;
  const uint4* h = H + (size_t)r * n_chunks;
  float acc = 0.f;
  for (int c = lane; c < n_chunks; c += 64) {
    const uint4 x = h[c], y = w[c];
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (BF16) {
        acc = fmaf(__uint_as_float(xs[e] << 16), __uint_as_float(ys[e] << 16), acc);
        acc = fmaf(__uint_as_float(xs[e] & 0xFFFF0000u), __uint_as_float(ys[e] & 0xFFFF0000u), acc);
      } else {
        acc = fmaf(__uint_as_float(xs[e]), __uint_as_float(ys[e]), acc);
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if (lane == 0) nll[r] = lse[r] - acc;
}

int ensure_sample_scratch(z2z_ctx* c, size_t need) {
  if (need <= c->part_vl_capacity) return Z2Z_OK;
  if (c->part_v) (void)hipFree(c->part_v);
  if (c->part_l) (void)hipFree(c->part_l);
  c->part_v = nullptr;
  c->part_l = nullptr;
  c->part_vl_capacity = 0;
  if (hipMalloc(&c->part_v, need * sizeof(float)) != hipSuccess) return Z2Z_ENOMEM;
  if (hipMalloc(&c->part_l, need * sizeof(float)) != hipSuccess) return Z2Z_ENOMEM;
  c->part_vl_capacity = need;
  return Z2Z_OK;
}

int ensure_scratch(z2z_ctx* c, size_t need) {
  if (need <= c->part_capacity) return Z2Z_OK;
  if (c->part_m) (void)hipFree(c->part_m);
  if (c->part_s) (void)hipFree(c->part_s);
  if (c->part_i) (void)hipFree(c->part_i);
  c->part_m = nullptr;
  c->part_s = nullptr;
  c->part_i = nullptr;
  c->part_capacity = 0;
  if (hipMalloc(&c->part_m, need * sizeof(float)) != hipSuccess) return Z2Z_ENOMEM;
  if (hipMalloc(&c->part_s, need * sizeof(float)) != hipSuccess) return Z2Z_ENOMEM;
  if (hipMalloc(&c->part_i, need * sizeof(int32_t)) != hipSuccess) return Z2Z_ENOMEM;
  c->part_capacity = need;
  return Z2Z_OK;
}


int launch_part(z2z_ctx* c, bool hyper, bool fast, LogitsArgs a, const void* W, int w_rows, int col0, int part0,
                int strip, int rows, int rows_per_seq, int* n_strips_out, bool timed, hipStream_t s,
                bool prob = false) {
  const int tile = fast ? 256 : 128;
  const int B = c->cfg.B;
  a.W = W;
  a.size = hyper ? c->st.size : nullptr;
  a.w_rows = w_rows;
  a.col0 = col0;
  a.n_vtiles = (w_rows + tile - 1) / tile;
  a.strip = strip;
  a.n_strips = (a.n_vtiles + strip - 1) / strip;
  a.part0 = part0;
  a.row_tiles = hyper ? (rows_per_seq + tile - 1) / tile : (rows + tile - 1) / tile;
  a.n_work = (hyper ? B : 1) * a.row_tiles * a.n_strips;
  *n_strips_out = a.n_strips;
  unsigned grid = (unsigned)a.n_work;
  if (fast && !hyper) {
    const int m = c->opt_logits_map;
    a.map_lr = m ? (m & 0xFF) : 4;
    a.map_ls = m ? ((m >> 8) & 0xFF) : 8;
    a.map_xr = m ? ((m >> 16) & 0xFF) : 4;
    a.map_xs = m ? ((m >> 24) & 0xFF) : 2;
    const int sb_rows = a.map_xr * a.map_lr, sb_strips = a.map_xs * a.map_ls;
    a.map_sb_r = (a.row_tiles + sb_rows - 1) / sb_rows;
    const int sb_s = (a.n_strips + sb_strips - 1) / sb_strips;
    grid = 8u * (unsigned)(a.map_lr * a.map_ls) * (unsigned)a.map_sb_r * (unsigned)sb_s;
  }
  if (timed) Z2Z_HIP_TRY(hipEventRecord(c->ev_start[c->n_timed], s));
  int rc = fast ? z2z_launch_logits_fast(prob ? (hyper ? 4 : 3) : (hyper ? 1 : 0), a, grid, s)
                : z2z_launch_logits_general(c->cfg.dtype == Z2Z_BF16, hyper, a, grid, s);
  if (timed) {
    Z2Z_HIP_TRY(hipEventRecord(c->ev_stop[c->n_timed], s));
    c->n_timed++;
  }
  return rc;
}

}  // namespace

namespace {

// Dense layer with K split over workgroups of the tile kernel: out = act(sum_ks partial[ks] + bias) + residual,
// the parts added in a fixed order; one thread per run of 4 columns.
__global__ void __launch_bounds__(256) linear_sum_kernel(const float* partial, int ksplit, int rows, const int32_t* rows_dev,
                                                         int N, const float* bias, int act, const uint16_t* residual,
                                                         uint16_t* out) {
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
  if (residual) {
    const uint2 rv = *reinterpret_cast<const uint2*>(residual + at);
    x.x += __uint_as_float(rv.x << 16);
    x.y += __uint_as_float(rv.x & 0xFFFF0000u);
    x.z += __uint_as_float(rv.y << 16);
    x.w += __uint_as_float(rv.y & 0xFFFF0000u);
  }
  uint2 o;
  o.x = bf16_bits_rne(x.x) | (bf16_bits_rne(x.y) << 16);
  o.y = bf16_bits_rne(x.z) | (bf16_bits_rne(x.w) << 16);
  *reinterpret_cast<uint2*>(out + at) = o;
}

}  // namespace

int z2z_launch_linear(z2z_ctx* c, const void* A, const void* W, const float* bias, const void* residual, int act,
                      void* out, int R, const int32_t* rows_dev, int N, int K, hipStream_t s) {
  // between one and a few hundred rows (more than the 64 the decode-step kernel serves per pass over the
  // weights, too few for the tile kernel to have a tile per CU): the tile kernel with K split over workgroups,
  // so that the weights stream once for all rows and every CU has a part
  if (R > 64 && R <= 512 && c->fast_ready && K % 64 == 0 && N % 8 == 0 && c->opt_logits_kernel != 1) {
    const int row_tiles = (R + 255) / 256, n_vt = (N + 255) / 256, tiles = row_tiles * n_vt;
    const int n_slabs = K / 64;
    int ksplit = 1;
    while (tiles * ksplit < 192 && n_slabs / (ksplit * 2) >= 8) ksplit *= 2;
    if (ksplit > 1) {
      const int per = (n_slabs + ksplit - 1) / ksplit;
      ksplit = (n_slabs + per - 1) / per;
      const size_t need = (size_t)ksplit * R * N * sizeof(float);
      if (need > c->skinny_partial_bytes) {
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
                         reinterpret_cast<const float*>(c->skinny_partial), ksplit, R, rows_dev, N, bias, act,
                         reinterpret_cast<const uint16_t*>(residual), reinterpret_cast<uint16_t*>(out));
      Z2Z_HIP_TRY(hipGetLastError());
      return Z2Z_OK;
    }
  }
  // few rows: bound by the weight bytes, which the decode-step kernel streams at HBM rate (it re-reads them
  // once per 64 rows, so it loses to the tile kernel beyond a few hundred rows)
  if (R <= 512 && c->skinny_ready && K % 128 == 0 && N % 2 == 0 && c->opt_logits_kernel != 2)
    return z2z_launch_linear_skinny(c, A, W, bias, residual, act, out, R, rows_dev, N, K, s);
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
  a.rows_dev = nullptr;
  if (rows_dev && a.row_tiles >= 16) {
    // the real row count is on the device: row tiles are dealt to the XCDs one by one (see map_rows_dev)
    a.rows_dev = rows_dev;
    a.map_lr = 4;
    a.map_ls = a.n_strips >= 8 ? 8 : (a.n_strips >= 4 ? 4 : (a.n_strips >= 2 ? 2 : 1));
    a.strip_blocks = (a.n_strips + a.map_ls - 1) / a.map_ls;
    const int tiles_per_xcd = (a.row_tiles + 7) / 8;
    const int row_blocks = (tiles_per_xcd + a.map_lr - 1) / a.map_lr;
    const unsigned grid = 8u * (unsigned)(a.map_lr * a.map_ls) * (unsigned)row_blocks * (unsigned)a.strip_blocks;
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

int z2z_launch_extended_logits(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                               const void* W_hyper, int32_t* argmax, float* mx, float* lse, float* logits,
                               hipStream_t s) {
  const int V = c->cfg.V, cap = c->cfg.cap;
  const bool timed = c->opt_timing && c->n_timed < Z2Z_MAX_TIMED && c->ev_created;

  // decode step: one hidden row per sequence -> the bandwidth-bound kernel (it can store the logits too)
  if (rows_per_seq == 1 && c->decode_ready && c->opt_decode_kernel != 1) {
    int n_parts = z2z_logits_decode_parts(c);
    int rc = ensure_scratch(c, (size_t)n_parts * rows);
    if (rc != Z2Z_OK) return rc;
    rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &n_parts, timed, nullptr, logits, s);
    if (rc != Z2Z_OK) return rc;
    if (logits && cap > 0) {
      hipLaunchKernelGGL(logits_mask_kernel, dim3(rows), dim3(256), 0, s, logits, rows, rows_per_seq, V, cap,
                         c->st.size);
      Z2Z_HIP_TRY(hipGetLastError());
    }
    return launch_combine(c, n_parts, rows, argmax, mx, lse, s);
  }

  // the fast kernels never store logits: the full-logits output (small shapes) takes the general kernel
  const bool fast_ok = c->cfg.dtype == Z2Z_BF16 && c->cfg.d % 64 == 0 && c->fast_ready && logits == nullptr;
  bool fast_base = fast_ok && rows > 128;
  bool fast_hyper = fast_ok && rows_per_seq > 128;
  if (c->opt_logits_kernel == 1) fast_base = fast_hyper = false;
  if (c->opt_logits_kernel >= 2) fast_base = fast_hyper = fast_ok;
  const int strip = c->opt_logits_strip > 0 ? c->opt_logits_strip : 4;

  // number of parts (strips of both launches), then the scratch for them
  const int base_tile = fast_base ? 256 : 128, hyp_tile = fast_hyper ? 256 : 128;
  const int base_strips = (((V + base_tile - 1) / base_tile) + strip - 1) / strip;
  const int hyp_strips = cap > 0 ? (((cap + hyp_tile - 1) / hyp_tile) + strip - 1) / strip : 0;
  const int n_parts = base_strips + hyp_strips;
  int rc = ensure_scratch(c, (size_t)n_parts * rows);
  if (rc != Z2Z_OK) return rc;

  LogitsArgs a;
  a.H = H;
  a.rows = rows;
  a.rows_per_seq = rows_per_seq;
  a.d = c->cfg.d;
  a.part_m = c->part_m;
  a.part_s = c->part_s;
  a.part_i = c->part_i;
  a.logits = logits;
  a.ld = V + cap;
  a.n_parts = n_parts;
  a.map_lr = a.map_ls = a.map_xr = a.map_xs = a.map_sb_r = 1;

  int ns = 0;
  rc = launch_part(c, false, fast_base, a, W_base, V, 0, 0, strip, rows, rows_per_seq, &ns, timed, s);
  if (rc != Z2Z_OK) return rc;
  if (cap > 0) {
    rc = launch_part(c, true, fast_hyper, a, W_hyper, cap, V, base_strips, strip, rows, rows_per_seq, &ns, false, s);
    if (rc != Z2Z_OK) return rc;
    if (logits) {
      hipLaunchKernelGGL(logits_mask_kernel, dim3(rows), dim3(256), 0, s, logits, rows, rows_per_seq, V, cap,
                         c->st.size);
      Z2Z_HIP_TRY(hipGetLastError());
    }
  }
  return launch_combine(c, n_parts, rows, argmax, mx, lse, s);
}

int z2z_launch_extended_sample(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                               const void* W_hyper, float temperature, int32_t top_k, float top_p, uint64_t seed,
                               uint64_t step, int32_t* token, float* logprob, hipStream_t s) {
  // built for the generation step: one hidden row per sequence, the bandwidth-bound kernel
  if (rows_per_seq != 1 || !c->decode_ready) return Z2Z_EUNSUPPORTED;
  int n_parts = z2z_logits_decode_parts(c);
  int rc = ensure_scratch(c, (size_t)n_parts * rows);
  if (rc != Z2Z_OK) return rc;
  z2z_sample_params sp;
  sp.temperature = temperature;
  sp.seed = seed;
  sp.step = step;
  const bool timed = c->opt_timing && c->n_timed < Z2Z_MAX_TIMED && c->ev_created;
  if (top_k <= 0 && top_p >= 1.0f) {
    // no filter: the draw is folded into the kernel that computes the logits, which are never stored
    rc = ensure_sample_scratch(c, (size_t)n_parts * rows);
    if (rc != Z2Z_OK) return rc;
    rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &n_parts, timed, &sp, nullptr, s);
    if (rc != Z2Z_OK) return rc;
    hipLaunchKernelGGL(sample_combine_kernel, dim3(rows), dim3(256), 0, s, c->part_m, c->part_s, c->part_v,
                       c->part_l, c->part_i, n_parts, rows, token, logprob);
    Z2Z_HIP_TRY(hipGetLastError());
    return Z2Z_OK;
  }
  // filters: the kernel stores the rows' logits / T (rows x (V + cap) floats of library scratch), the merge
  // gives the row maxima and log-sum-exps, and one workgroup per row selects the kept prefix and draws
  if (!c->trunc_ready) return Z2Z_EUNSUPPORTED;
  const size_t need = (size_t)rows * (size_t)(c->cfg.V + c->cfg.cap);
  if (need > c->sample_logits_capacity) {
    if (c->sample_logits) (void)hipFree(c->sample_logits);
    if (c->row_max) (void)hipFree(c->row_max);
    c->sample_logits = nullptr;
    c->row_max = nullptr;
    c->sample_logits_capacity = 0;
    if (hipMalloc(&c->sample_logits, need * sizeof(float)) != hipSuccess) return Z2Z_ENOMEM;
    // the row maxima and log-sum-exps, followed by the selection kernels' scratch
    if (hipMalloc(&c->row_max, (2 * (size_t)rows + z2z_sample_truncated_work_floats(rows)) * sizeof(float)) != hipSuccess)
      return Z2Z_ENOMEM;
    c->sample_logits_capacity = need;
  }
  rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &n_parts, timed, &sp, c->sample_logits, s);
  if (rc != Z2Z_OK) return rc;
  rc = launch_combine(c, n_parts, rows, nullptr, c->row_max, c->row_max + rows, s);
  if (rc != Z2Z_OK) return rc;
  return z2z_launch_sample_truncated(c, c->sample_logits, c->row_max, rows, n_parts, c->row_max + 2 * (size_t)rows, &sp,
                                     top_k, top_p, token, logprob, s);
}

int z2z_launch_extended_nll(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                            const void* W_hyper, const int32_t* targets, float* nll, float* lse, hipStream_t s) {
  int rc = z2z_launch_extended_logits(c, H, rows, rows_per_seq, W_base, W_hyper, nullptr, nullptr, lse, nullptr, s);
  if (rc != Z2Z_OK) return rc;
  const dim3 grid((rows + 3) / 4), block(256);
  if (c->cfg.dtype == Z2Z_BF16)
    hipLaunchKernelGGL(target_nll_kernel<true>, grid, block, 0, s, reinterpret_cast<const uint4*>(H),
                       reinterpret_cast<const uint4*>(W_base), reinterpret_cast<const uint4*>(W_hyper), c->st.size,
                       targets, lse, nll, rows, rows_per_seq, c->cfg.V, c->cfg.cap, c->cfg.d);
  else
    hipLaunchKernelGGL(target_nll_kernel<false>, grid, block, 0, s, reinterpret_cast<const uint4*>(H),
                       reinterpret_cast<const uint4*>(W_base), reinterpret_cast<const uint4*>(W_hyper), c->st.size,
                       targets, lse, nll, rows, rows_per_seq, c->cfg.V, c->cfg.cap, c->cfg.d);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// ---- backward pass of the loss ----------------------------------------------------------------------------
namespace {

// g[r]: the upstream gradient of row r (1 without one), 0 for rows without a target or whose target names no
// existing column.
__global__ void __launch_bounds__(256) row_grad_kernel(const int32_t* targets, const float* grad_nll, const int32_t* size,
                                                       int rows, int rows_per_seq, int V, int cap, float* g) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  const int t = targets[r];
  const int C = min(max(size[r / rows_per_seq], 0), cap);
  g[r] = (t >= 0 && t < V + C) ? (grad_nll ? grad_nll[r] : 1.0f) : 0.f;
}

__global__ void __launch_bounds__(256) fill_zero_kernel(uint4* p, size_t n16) {
  const uint4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = z;
}

// out[b][c][r] = in[b][r][c] (bf16) for r < R, c < C; columns R .. ld_out - 1 of out are zero.  64 x 64 tiles
// through LDS, 256 threads, 16 bytes per lane on both sides (ld_in and ld_out are multiples of 8, the bases
// 16-byte aligned); grid (ceil(ld_out / 64), ceil(C / 64), batch).
__global__ void __launch_bounds__(256) transpose_bf16_kernel(const uint16_t* in, uint16_t* out, int R, int C, int ld_in,
                                                             int ld_out, size_t in_batch, size_t out_batch) {
  __shared__ uint16_t t[64][72];                     // [column of the tile][row of the tile], rows padded
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
    if (c < C && r < ld_out) *reinterpret_cast<uint4*>(dst + (size_t)c * ld_out + r) = *reinterpret_cast<const uint4*>(&t[i][chunk * 8]);
  }
}

int launch_transpose(const void* in, void* out, int R, int C, int ld_in, int ld_out, int batch, size_t in_batch,
                     size_t out_batch, hipStream_t s) {
  if (R < 1 || C < 1 || batch < 1) return Z2Z_OK;
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3((ld_out + 63) / 64, (C + 63) / 64, batch), dim3(256), 0, s,
                     reinterpret_cast<const uint16_t*>(in), reinterpret_cast<uint16_t*>(out), R, C, ld_in, ld_out,
                     in_batch, out_batch);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// dE[t_j] += a_j * dW_hyper[b, e] for the tokens of every existing entry: one wave per entry, float atomics
// (tokens recur across entries and sequences).
__global__ void __launch_bounds__(256) pool_backward_kernel(const uint16_t* dW, float* dE, const int32_t* size,
                                                            const int32_t* ent_tokens, const int32_t* ent_len, int B,
                                                            int V, int M, int cap, int d, int mean,
                                                            const float* coef /* [Z2Z_MAX_M + 1][Z2Z_MAX_M] */) {
  const int lane = threadIdx.x & 63;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= (long long)B * cap) return;
  const int b = (int)(row / cap), e = (int)(row % cap);
  if (e >= min(max(size[b], 0), cap)) return;
  const int L = min(max(ent_len[row], 1), M);
  for (int j = 0; j < L; ++j) {
    const int tok = min(max(ent_tokens[row * M + j], 0), V - 1);
    const float a = mean ? 1.0f / (float)L : coef[L * Z2Z_MAX_M + j];
    for (int c = lane; c < d; c += 64)
      atomicAdd(dE + (size_t)tok * d + c, a * __uint_as_float((uint32_t)dW[row * d + c] << 16));
  }
}

size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

}  // namespace

int z2z_launch_hyper_embed_backward(z2z_ctx* c, const void* dW_hyper, float* dE, hipStream_t s) {
  const int B = c->cfg.B, cap = c->cfg.cap;
  if (cap == 0) return Z2Z_OK;
  if (!c->coef_dev) {
    if (hipMalloc(&c->coef_dev, sizeof(c->coef)) != hipSuccess) return Z2Z_ENOMEM;
    Z2Z_HIP_TRY(hipMemcpyAsync(c->coef_dev, c->coef, sizeof(c->coef), hipMemcpyHostToDevice, s));
  }
  const long long rows = (long long)B * cap;
  hipLaunchKernelGGL(pool_backward_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                     reinterpret_cast<const uint16_t*>(dW_hyper), dE, c->st.size, c->st.ent_tokens, c->st.ent_len, B,
                     c->cfg.V, c->cfg.M, cap, c->cfg.d, c->cfg.pool == Z2Z_POOL_MEAN ? 1 : 0,
                     reinterpret_cast<const float*>(c->coef_dev));
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// Gradient of sum_r grad_nll[r] * nll[r] with respect to H, W_base and W_hyper.  The gradient with respect to
// the logits, dZ = g * (softmax - onehot), is written out once in bf16 (the logits are recomputed by the
// forward kernel with another epilogue, using the forward pass's lse), then
//   dH = dZ_base W_base + dZ_hyper[b] W_hyper[b],   dW_base = dZ_base^T H,   dW_hyper[b] = dZ_hyper[b]^T H[b]
// are four dense products on the same MFMA kernel, which wants both operands contiguous along the contraction:
// hence one transposed copy of each operand (weights, hidden rows, dZ), made by a bandwidth-bound kernel.
int z2z_launch_extended_nll_backward(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                                     const void* W_hyper, const int32_t* targets, const float* lse,
                                     const float* grad_nll, void* dH, void* dW_base, void* dW_hyper, hipStream_t s) {
  const int B = c->cfg.B, V = c->cfg.V, cap = c->cfg.cap, d = c->cfg.d;
  if (c->cfg.dtype != Z2Z_BF16 || d % 64 != 0 || !c->fast_ready) return Z2Z_EUNSUPPORTED;
  const size_t Vp = round_up(V, 64), capp = round_up(cap, 64), rows_p = round_up(rows, 64), Np = round_up(rows_per_seq, 64);
  // work space (bf16 unless noted), 256-byte aligned pieces
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += round_up(bytes, 256); return at; };
  const size_t o_g = take((size_t)rows * 4);                       // float g[rows]
  const size_t o_Pb = take((size_t)rows * Vp * 2);                 // dZ, base columns      [rows, Vp]
  const size_t o_PbT = take((size_t)V * rows_p * 2);               // its transpose         [V, rows_p]
  const size_t o_Ph = take((size_t)rows * capp * 2);               // dZ, hyper columns     [rows, capp]
  const size_t o_PhT = take((size_t)B * cap * Np * 2);             // per sequence          [B][cap, Np]
  const size_t o_WbT = take((size_t)d * Vp * 2);                   // W_base^T              [d, Vp]
  const size_t o_WhT = take((size_t)B * d * capp * 2);             // W_hyper[b]^T          [B][d, capp]
  const size_t o_HT = take((size_t)d * rows_p * 2);                // H^T                   [d, rows_p]
  const size_t o_HTs = take((size_t)B * d * Np * 2);               // H[b]^T                [B][d, Np]
  if (off > ((size_t)200 << 30)) return Z2Z_ENOMEM;
  if (off > c->bwd_ws_bytes) {
    if (c->bwd_ws) (void)hipFree(c->bwd_ws);
    c->bwd_ws = nullptr;
    c->bwd_ws_bytes = 0;
    if (hipMalloc(&c->bwd_ws, off) != hipSuccess) return Z2Z_ENOMEM;
    c->bwd_ws_bytes = off;
  }
  unsigned char* ws = reinterpret_cast<unsigned char*>(c->bwd_ws);
  float* g = reinterpret_cast<float*>(ws + o_g);
  void *Pb = ws + o_Pb, *PbT = ws + o_PbT, *Ph = ws + o_Ph, *PhT = ws + o_PhT, *WbT = ws + o_WbT, *WhT = ws + o_WhT,
       *HT = ws + o_HT, *HTs = ws + o_HTs;

  hipLaunchKernelGGL(row_grad_kernel, dim3((rows + 255) / 256), dim3(256), 0, s, targets, grad_nll, c->st.size, rows,
                     rows_per_seq, V, cap, g);
  // ---- dZ: the forward kernel with the probability epilogue ---------------------------------------------
  LogitsArgs a;
  memset(&a, 0, sizeof(a));
  a.H = H;
  a.rows = rows;
  a.rows_per_seq = rows_per_seq;
  a.d = d;
  a.map_lr = a.map_ls = a.map_xr = a.map_xs = a.map_sb_r = 1;
  a.lse = lse;
  a.row_grad = g;
  a.targets = targets;
  const int strip = c->opt_logits_strip > 0 ? c->opt_logits_strip : 4;
  int ns = 0;
  a.out = Pb;
  a.ldo = (int)Vp;
  int rc = launch_part(c, false, true, a, W_base, V, 0, 0, strip, rows, rows_per_seq, &ns, false, s, true);
  if (rc != Z2Z_OK) return rc;
  if (cap > 0) {
    const size_t n16 = (size_t)rows * capp * 2 / 16;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)std::min<size_t>((n16 + 255) / 256, 4096)), dim3(256), 0, s,
                       reinterpret_cast<uint4*>(Ph), n16);
    a.out = Ph;
    a.ldo = (int)capp;
    rc = launch_part(c, true, true, a, W_hyper, cap, V, 0, strip, rows, rows_per_seq, &ns, false, s, true);
    if (rc != Z2Z_OK) return rc;
  }
  // ---- transposed copies -------------------------------------------------------------------------------------
  if ((rc = launch_transpose(W_base, WbT, V, d, d, (int)Vp, 1, 0, 0, s)) != Z2Z_OK) return rc;
  if ((rc = launch_transpose(H, HT, rows, d, d, (int)rows_p, 1, 0, 0, s)) != Z2Z_OK) return rc;
  if ((rc = launch_transpose(Pb, PbT, rows, V, (int)Vp, (int)rows_p, 1, 0, 0, s)) != Z2Z_OK) return rc;
  if (cap > 0) {
    if ((rc = launch_transpose(W_hyper, WhT, cap, d, d, (int)capp, B, (size_t)cap * d, (size_t)d * capp, s)) != Z2Z_OK) return rc;
    if ((rc = launch_transpose(H, HTs, rows_per_seq, d, d, (int)Np, B, (size_t)rows_per_seq * d, (size_t)d * Np, s)) != Z2Z_OK) return rc;
    if ((rc = launch_transpose(Ph, PhT, rows_per_seq, cap, (int)capp, (int)Np, B, (size_t)rows_per_seq * capp, (size_t)cap * Np, s)) != Z2Z_OK) return rc;
  }
  // ---- the products --------------------------------------------------------------------------------------------
  if ((rc = z2z_launch_linear(c, Pb, WbT, nullptr, nullptr, 0, dH, rows, nullptr, d, (int)Vp, s)) != Z2Z_OK) return rc;
  if ((rc = z2z_launch_linear(c, PbT, HT, nullptr, nullptr, 0, dW_base, V, nullptr, d, (int)rows_p, s)) != Z2Z_OK) return rc;
  for (int b = 0; b < B && cap > 0; ++b) {
    uint16_t* dH_b = reinterpret_cast<uint16_t*>(dH) + (size_t)b * rows_per_seq * d;
    const uint16_t* Ph_b = reinterpret_cast<const uint16_t*>(Ph) + (size_t)b * rows_per_seq * capp;
    const uint16_t* WhT_b = reinterpret_cast<const uint16_t*>(WhT) + (size_t)b * d * capp;
    if ((rc = z2z_launch_linear(c, Ph_b, WhT_b, nullptr, dH_b, 0, dH_b, rows_per_seq, nullptr, d, (int)capp, s)) != Z2Z_OK) return rc;
    const uint16_t* PhT_b = reinterpret_cast<const uint16_t*>(PhT) + (size_t)b * cap * Np;
    const uint16_t* HTs_b = reinterpret_cast<const uint16_t*>(HTs) + (size_t)b * d * Np;
    uint16_t* dWh_b = reinterpret_cast<uint16_t*>(dW_hyper) + (size_t)b * cap * d;
    if ((rc = z2z_launch_linear(c, PhT_b, HTs_b, nullptr, nullptr, 0, dWh_b, cap, nullptr, d, (int)Np, s)) != Z2Z_OK) return rc;
  }
  return Z2Z_OK;
}
