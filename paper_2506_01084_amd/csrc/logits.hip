// extended_logits: launch planning (which tile kernel, strips, workgroup mapping), the merge of the
// per-strip partial triples, and the scratch buffer that holds them.
//
// The base part (columns < V, shared W_base) and the hyper part (columns V.., one W_hyper per sequence,
// only the first C_b rows exist: section 2.3 of the zip2zip paper, "Consistent Vocabulary Updates") are
// two launches; both leave (max, sum-exp, argmax) triples per (strip, row), merged in column order.
#include "logits_common.h"
#include "logits_mid.h"

#include <string.h>

#include <algorithm>
#include <mutex>

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

int launch_combine(const z2z_parts& p, int n_parts, int rows, int32_t* argmax, float* mx, float* lse, hipStream_t s) {
  if (n_parts > 256)
    hipLaunchKernelGGL(logits_combine_kernel<256>, dim3(rows), dim3(256), 0, s, p.m, p.s, p.i, n_parts, rows, argmax,
                       mx, lse);
  else
    hipLaunchKernelGGL(logits_combine_kernel<64>, dim3((rows + 3) / 4), dim3(256), 0, s, p.m, p.s, p.i, n_parts, rows,
                       argmax, mx, lse);
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

int ensure_sample_scratch(z2z_ctx* c, size_t need, hipStream_t s) {
  if (need <= c->part_vl_capacity) return Z2Z_OK;
  Z2Z_TRY_GROW(s);
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

int ensure_scratch(z2z_ctx* c, size_t need, hipStream_t s) {
  if (need <= c->part_capacity) return Z2Z_OK;
  Z2Z_TRY_GROW(s);
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

z2z_parts ctx_parts(const z2z_ctx* c) { return z2z_parts{c->part_m, c->part_s, c->part_i, c->part_capacity}; }

}  // namespace

// ---- the allocation-free entry point's scratch ------------------------------------------------------------
// One array per device (every GPU that loads the library holds its own copy, at its own address, until the
// process ends): three runs of Z2Z_STATIC_PARTS four-byte elements, the (max, sum-exp, argmax) partials.  In
// host code the array's name is a stand-in, not a device address: its address on a device is asked for once
// per device (with that device current) and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[3 * (size_t)Z2Z_STATIC_PARTS * 4];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // nullptr: not looked up yet on that device
static std::mutex g_scratch_mutex;

int z2z_static_scratch_prepare(z2z_ctx* c) {
  if (c->device < 0 || c->device >= kMaxDevices) return Z2Z_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[c->device]) return Z2Z_OK;
  int cur = -1;
  Z2Z_HIP_TRY(hipGetDevice(&cur));
  if (cur != c->device) return Z2Z_EHIP;   // the symbol's address is that of the current device's copy
  void* ptr = nullptr;
  Z2Z_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
  if (!ptr) return Z2Z_EHIP;
  g_scratch_ptr[c->device] = ptr;
  return Z2Z_OK;
}

namespace {

// The static array of the context's device as three part arrays; false if its address is not known.
bool static_parts(const z2z_ctx* c, z2z_parts* out) {
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (c->device >= 0 && c->device < kMaxDevices) ptr = g_scratch_ptr[c->device];
  }
  if (!ptr) return false;
  float* f = reinterpret_cast<float*>(ptr);
  out->m = f;
  out->s = f + Z2Z_STATIC_PARTS;
  out->i = reinterpret_cast<int32_t*>(f + 2 * (size_t)Z2Z_STATIC_PARTS);
  out->capacity = Z2Z_STATIC_PARTS;
  return true;
}

}  // namespace

// One launch of a tile kernel over the base part (hyper = false) or the per-sequence hyper part: fills in the
// shape-dependent fields of `a` (tiles, strips, workgroup mapping) and launches; prob = true selects the
// epilogue that stores the gradient with respect to the logits (the backward pass of the loss).
int z2z_launch_logits_part(z2z_ctx* c, bool hyper, bool fast, LogitsArgs a, const void* W, int w_rows, int col0,
                           int part0, int strip, int rows, int rows_per_seq, int* n_strips_out, bool timed,
                           hipStream_t s, bool prob, int seq0, int n_seq) {
  // (seq0, n_seq: the hyper part of a sub-range of the sequences -- the caller passes that range's rows and
  // its W_hyper; n_seq = 0 means all of them)
  const int tile = fast ? 256 : 128;
  const int B = n_seq > 0 ? n_seq : c->cfg.B;
  a.W = W;
  a.size = hyper ? c->st.size + seq0 : nullptr;
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
    if (!m && a.row_tiles < 16) {
      // few row tiles: the XCDs share out the strips alone (split over row tiles, most of them would idle)
      a.map_xr = 1;
      a.map_xs = 8;
      a.map_lr = a.row_tiles >= 4 ? 4 : (a.row_tiles >= 2 ? 2 : 1);
    }
    const int sb_rows = a.map_xr * a.map_lr, sb_strips = a.map_xs * a.map_ls;
    a.map_sb_r = (a.row_tiles + sb_rows - 1) / sb_rows;
    const int sb_s = (a.n_strips + sb_strips - 1) / sb_strips;
    grid = 8u * (unsigned)(a.map_lr * a.map_ls) * (unsigned)a.map_sb_r * (unsigned)sb_s;
  }
  c->n_launch[fast ? (hyper ? Z2Z_KERNEL_TILE_HYPER : Z2Z_KERNEL_TILE_BASE) : Z2Z_KERNEL_GENERAL]++;
  if (timed) Z2Z_HIP_TRY(hipEventRecord(c->ev_start[c->n_timed], s));
  // (measurement probes of the base part: see logits_fast_kernel, modes 8 and 9)
  const int plain_base = c->opt_logits_kernel == 2 ? 8 : (c->opt_logits_kernel == 3 ? 9 : 0);
  int rc = fast ? z2z_launch_logits_fast(prob ? (hyper ? 4 : 3) : (a.sample && !hyper ? (a.sample == 2 ? 7 : 6) : (hyper ? 1 : plain_base)), a, grid, s)
                : z2z_launch_logits_general(c->cfg.dtype == Z2Z_BF16, hyper, a, grid, s);
  if (timed) {
    Z2Z_HIP_TRY(hipEventRecord(c->ev_stop[c->n_timed], s));
    c->n_timed++;
  }
  return rc;
}



// A workgroup sweeps a strip of 4 weight tiles with its rows' tile resident; with few row tiles that leaves CUs
// idle, so the strips shorten until there are two workgroups per CU (or one tile per workgroup).
static int pick_strip_for(const z2z_ctx* c, long long row_tiles, int n_vt) {
  if (c->opt_logits_strip > 0) return c->opt_logits_strip;
  int st = 4;
  while (st > 1 && row_tiles * ((n_vt + st - 1) / st) < 512) st >>= 1;
  return st;
}


int z2z_launch_extended_logits(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                               const void* W_hyper, int32_t* argmax, float* mx, float* lse, float* logits,
                               hipStream_t s, bool use_static) {
  const int V = c->cfg.V, cap = c->cfg.cap;
  const bool timed = c->opt_timing && c->n_timed < Z2Z_MAX_TIMED && c->ev_created;
  z2z_parts parts;
  if (use_static && !static_parts(c, &parts)) return Z2Z_EHIP;
  // the partial triples of this call: the device's static array must hold them as it is, the context's
  // buffers grow to hold them
  auto reserve = [&](size_t need) -> int {
    if (use_static) return need <= parts.capacity ? Z2Z_OK : Z2Z_ELIMIT;
    const int rc = ensure_scratch(c, need, s);
    parts = ctx_parts(c);
    return rc;
  };

  // the fast kernels never store logits: the full-logits output (small shapes) takes the general kernel
  const bool fast_ok = c->cfg.dtype == Z2Z_BF16 && c->cfg.d % 64 == 0 && c->fast_ready && logits == nullptr;
  // decode step: one hidden row per sequence -> the bandwidth-bound kernel (it can store the logits too).
  // Its base units serve 64 rows per pass over W_base, each pass at about the cost of the first; from the second
  // pass on the tile kernel takes the base vocabulary (all rows at once) and only the hyper units run here
  const bool decode_step = rows_per_seq == 1 && c->decode_ready && c->opt_decode_kernel != 1;
  const bool decode_split = decode_step && fast_ok && rows > 64 && c->opt_logits_kernel != 1;
  // a few rows per sequence (2..64: a verification step over drafted codes, a short chunk): every sequence's
  // W_hyper meets only its own rows, so the hyper part is bandwidth-bound like the decode step's; it goes to
  // that kernel's matrix-core units (one pass over each W_hyper), the base vocabulary to the tile kernel
  const bool seq_split = !decode_step && fast_ok && rows_per_seq >= 2 && rows_per_seq <= 64 && cap > 0 &&
                         c->decode_ready && c->opt_decode_kernel != 1 && c->opt_logits_kernel != 1;
  if (decode_step && !decode_split) {
    int n_parts = z2z_logits_decode_parts(c);
    int rc = reserve((size_t)n_parts * rows);
    if (rc != Z2Z_OK) return rc;
    rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &n_parts, timed, nullptr, logits, s, -1, &parts);
    if (rc != Z2Z_OK) return rc;
    if (logits && cap > 0) {
      hipLaunchKernelGGL(logits_mask_kernel, dim3(rows), dim3(256), 0, s, logits, rows, rows_per_seq, V, cap,
                         c->st.size);
      Z2Z_HIP_TRY(hipGetLastError());
    }
    return launch_combine(parts, n_parts, rows, argmax, mx, lse, s);
  }

  // (the general kernel is many times slower per tile: even a tile with a few valid rows goes to the tile kernel)
  bool fast_base = fast_ok, fast_hyper = fast_ok;
  if (c->opt_logits_kernel == 1) fast_base = fast_hyper = false;

  // number of parts (strips of both launches), then the scratch for them.  A workgroup sweeps a strip of 4
  // weight tiles with its rows' tile resident; with few row tiles that leaves CUs idle, so the strips shorten
  // until there are two workgroups per CU (or one tile per workgroup)
  const int base_tile = fast_base ? 256 : 128, hyp_tile = fast_hyper ? 256 : 128;
  const int base_vt = (V + base_tile - 1) / base_tile, hyp_vt = (cap + hyp_tile - 1) / hyp_tile;
  auto pick_strip = [&](long long row_tiles, int n_vt) { return pick_strip_for(c, row_tiles, n_vt); };
  // few hidden rows in all (several per sequence, or 65..192 sequences): the base part is bound by the bytes of
  // W_base and goes to the kernel that streams the weights past all rows at once, one part per 256 weight rows
  // (measured against the decode kernel's base units in a launch of their own at up to 64 rows: 260 against 305 us
  // for the call at config 2's shape; two or three passes of those units for more rows cost more still)
  const bool mid_base = fast_base && c->opt_logits_kernel == 0 && z2z_logits_mid_ok(c, rows);
  const int strip_b = mid_base ? 1 : pick_strip((rows + base_tile - 1) / base_tile, base_vt);
  const int strip_h = pick_strip((long long)c->cfg.B * ((rows_per_seq + hyp_tile - 1) / hyp_tile), hyp_vt);
  const int base_strips = (base_vt + strip_b - 1) / strip_b;
  int hyp_strips = cap > 0 ? (hyp_vt + strip_h - 1) / strip_h : 0;
  if (decode_split) {
    int base_columns, hyper_columns;
    z2z_logits_decode_units(&base_columns, &hyper_columns);
    hyp_strips = (cap + hyper_columns - 1) / hyper_columns;
  }
  if (seq_split) hyp_strips = z2z_logits_decode_seq_units(c);
  const int n_parts = base_strips + hyp_strips;
  int rc = reserve((size_t)n_parts * rows);
  if (rc != Z2Z_OK) return rc;

  LogitsArgs a;
  memset(&a, 0, sizeof(a));
  a.H = H;
  a.rows = rows;
  a.rows_per_seq = rows_per_seq;
  a.d = c->cfg.d;
  a.part_m = parts.m;
  a.part_s = parts.s;
  a.part_i = parts.i;
  a.logits = logits;
  a.ld = V + cap;
  a.n_parts = n_parts;
  a.map_lr = a.map_ls = a.map_xr = a.map_xs = a.map_sb_r = 1;

  int ns = 0;
  if (mid_base) {
    if (timed) Z2Z_HIP_TRY(hipEventRecord(c->ev_start[c->n_timed], s));
    rc = z2z_launch_logits_mid(c, a, W_base, V, 0, s);
    if (timed) {
      Z2Z_HIP_TRY(hipEventRecord(c->ev_stop[c->n_timed], s));
      c->n_timed++;
    }
  } else {
    rc = z2z_launch_logits_part(c, false, fast_base, a, W_base, V, 0, 0, strip_b, rows, rows_per_seq, &ns, timed, s);
  }
  if (rc != Z2Z_OK) return rc;
  if (cap > 0 && (decode_split || seq_split)) {
    int np = 0;
    rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &np, false, nullptr, nullptr, s, base_strips, &parts,
                                  seq_split ? rows_per_seq : 1);
    if (rc != Z2Z_OK) return rc;
  } else if (cap > 0) {
    rc = z2z_launch_logits_part(c, true, fast_hyper, a, W_hyper, cap, V, base_strips, strip_h, rows, rows_per_seq, &ns, false, s);
    if (rc != Z2Z_OK) return rc;
    if (logits) {
      hipLaunchKernelGGL(logits_mask_kernel, dim3(rows), dim3(256), 0, s, logits, rows, rows_per_seq, V, cap,
                         c->st.size);
      Z2Z_HIP_TRY(hipGetLastError());
    }
  }
  return launch_combine(parts, n_parts, rows, argmax, mx, lse, s);
}

int z2z_launch_extended_sample(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                               const void* W_hyper, float temperature, int32_t top_k, float top_p, uint64_t seed,
                               uint64_t step, int32_t* token, float* logprob, hipStream_t s) {
  // built for the generation step: one hidden row per sequence, the bandwidth-bound kernel
  if (rows_per_seq != 1 || !c->decode_ready) return Z2Z_EUNSUPPORTED;
  int n_parts = z2z_logits_decode_parts(c);
  int rc = ensure_scratch(c, (size_t)n_parts * rows, s);
  if (rc != Z2Z_OK) return rc;
  z2z_sample_params sp;
  sp.temperature = temperature;
  sp.seed = seed;
  sp.step = step;
  const bool timed = c->opt_timing && c->n_timed < Z2Z_MAX_TIMED && c->ev_created;
  // 65..192 rows: the base vocabulary goes to the weight-streaming kernel (with the tile kernel's sampling epilogues)
  const bool mid_base = rows > 64 && c->opt_logits_kernel == 0 && z2z_logits_mid_ok(c, rows);
  if (top_k <= 0 && top_p >= 1.0f && (rows > 128 || mid_base) && c->cfg.d % 64 == 0 && c->fast_ready &&
      c->opt_logits_kernel != 1) {
    // no filter, more than two passes of the decode kernel's base units (the generator in the tile kernel's
    // epilogue costs more than the second pass): as for the argmax, the tile kernel takes the base vocabulary
    // (with the draw folded into its epilogue) and the hyper units run alone
    const int base_vt = (c->cfg.V + 255) / 256;
    const int strip_b = mid_base ? 1 : pick_strip_for(c, (rows + 255) / 256, base_vt);
    const int base_strips = (base_vt + strip_b - 1) / strip_b;
    int base_columns, hyper_columns;
    z2z_logits_decode_units(&base_columns, &hyper_columns);
    n_parts = base_strips + (c->cfg.cap + hyper_columns - 1) / hyper_columns;
    rc = ensure_scratch(c, (size_t)n_parts * rows, s);
    if (rc != Z2Z_OK) return rc;
    rc = ensure_sample_scratch(c, (size_t)n_parts * rows, s);
    if (rc != Z2Z_OK) return rc;
    LogitsArgs a;
    memset(&a, 0, sizeof(a));
    a.H = H;
    a.rows = rows;
    a.rows_per_seq = 1;
    a.d = c->cfg.d;
    a.part_m = c->part_m;
    a.part_s = c->part_s;
    a.part_i = c->part_i;
    a.part_v = c->part_v;
    a.part_l = c->part_l;
    a.n_parts = n_parts;
    a.map_lr = a.map_ls = a.map_xr = a.map_xs = a.map_sb_r = 1;
    a.sample = 1;
    a.inv_temperature = 1.0f / temperature;
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.ctr2 = (uint32_t)step;
    a.ctr3 = (uint32_t)(step >> 32);
    int ns = 0;
    if (mid_base)
      rc = z2z_launch_logits_mid(c, a, W_base, c->cfg.V, 0, s);
    else
      rc = z2z_launch_logits_part(c, false, true, a, W_base, c->cfg.V, 0, 0, strip_b, rows, 1, &ns, timed, s);
    if (rc != Z2Z_OK) return rc;
    if (c->cfg.cap > 0) {
      int np = 0;
      rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &np, false, &sp, nullptr, s, base_strips);
      if (rc != Z2Z_OK) return rc;
    }
    hipLaunchKernelGGL(sample_combine_kernel, dim3(rows), dim3(256), 0, s, c->part_m, c->part_s, c->part_v,
                       c->part_l, c->part_i, n_parts, rows, token, logprob);
    Z2Z_HIP_TRY(hipGetLastError());
    return Z2Z_OK;
  }
  if (top_k <= 0 && top_p >= 1.0f) {
    // no filter: the draw is folded into the kernel that computes the logits, which are never stored
    rc = ensure_sample_scratch(c, (size_t)n_parts * rows, s);
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
    Z2Z_TRY_GROW(s);
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
  int base_columns = 0;                              // of a base part: the decode kernel's unit unless set
  if (rows > 64 && c->cfg.d % 64 == 0 && c->fast_ready && c->opt_logits_kernel != 1) {
    // more than one pass of the decode kernel's base units: the tile kernel stores and folds the base
    // vocabulary's scaled logits, the hyper units run alone (strips of at most 2 tiles: the selection kernels'
    // short-list pass takes parts of up to 512 columns)
    const int base_vt = (c->cfg.V + 255) / 256;
    int strip_b = mid_base ? 1 : pick_strip_for(c, (rows + 255) / 256, base_vt);
    if (strip_b > 2) strip_b = 2;
    const int base_strips = (base_vt + strip_b - 1) / strip_b;
    int unit_base, unit_hyper;
    z2z_logits_decode_units(&unit_base, &unit_hyper);
    n_parts = base_strips + (c->cfg.cap + unit_hyper - 1) / unit_hyper;
    base_columns = strip_b * 256;
    LogitsArgs a;
    memset(&a, 0, sizeof(a));
    a.H = H;
    a.rows = rows;
    a.rows_per_seq = 1;
    a.d = c->cfg.d;
    a.part_m = c->part_m;
    a.part_s = c->part_s;
    a.part_i = c->part_i;
    a.n_parts = n_parts;
    a.map_lr = a.map_ls = a.map_xr = a.map_xs = a.map_sb_r = 1;
    a.sample = 2;
    a.inv_temperature = 1.0f / temperature;
    a.logits = c->sample_logits;
    a.ld = c->cfg.V + c->cfg.cap;
    int ns = 0;
    if (mid_base)
      rc = z2z_launch_logits_mid(c, a, W_base, c->cfg.V, 0, s);
    else
      rc = z2z_launch_logits_part(c, false, true, a, W_base, c->cfg.V, 0, 0, strip_b, rows, 1, &ns, timed, s);
    if (rc != Z2Z_OK) return rc;
    if (c->cfg.cap > 0) {
      int np = 0;
      rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &np, false, &sp, c->sample_logits, s, base_strips);
      if (rc != Z2Z_OK) return rc;
    }
  } else {
    rc = z2z_launch_logits_decode(c, H, W_base, W_hyper, &n_parts, timed, &sp, c->sample_logits, s);
    if (rc != Z2Z_OK) return rc;
  }
  if (!z2z_sample_truncated_merges_parts(c, n_parts, top_k, base_columns)) {
    rc = launch_combine(ctx_parts(c), n_parts, rows, nullptr, c->row_max, c->row_max + rows, s);
    if (rc != Z2Z_OK) return rc;
  }
  return z2z_launch_sample_truncated(c, c->sample_logits, c->row_max, rows, n_parts, c->row_max + 2 * (size_t)rows, &sp,
                                     top_k, top_p, token, logprob, s, base_columns);
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
