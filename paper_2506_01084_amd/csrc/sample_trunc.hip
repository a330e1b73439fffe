// Truncated sampling for the generation step (gfx950): top-k / nucleus filters on the joint softmax, then
// the Gumbel-max draw among the kept columns.
//
// Section 2.3 of the zip2zip paper, step 9, draws the next token from the joint distribution over base
// tokens and hypertokens; the filters are the usual ones and not the paper's.  Order the columns by logit
// (largest first, equal logits by lower column).  With q = softmax(logit / T) over all existing columns,
// the kept set is the first n columns of that order, n = min(k, n_p), n_p the smallest prefix whose q sums
// to at least p.  The draw is argmax over the kept columns of logit / T - ln(-ln u) with the same
// generator coordinates as the untruncated draw.
//
// Input: the row's logits / T as the decode kernel stored them, the row's maximum and log-sum-exp, and the
// maxima of the row's parts.  Rows with a short prefix (k up to 256, or a nucleus that closes within a few
// hundred columns) are settled by sample_list_kernel from the parts with the largest maxima alone (see
// there).  For the others one workgroup per hidden row finds the last kept element of the order, the "cut",
// without sorting the row:
//   1. histogram passes over the row.  The cut lies in a half-open value interval [lo, hi) (at first
//      everything); the interval is split into 32 bins by value, every lane counts elements and sums
//      exp((x - max) / T) per bin in its own LDS column (no two lanes share an address, so the LDS adds
//      never conflict), the columns are added up, and a walk over the 32 bins from the top finds the bin
//      in which the count reaches k or the mass reaches p * total: that bin is the next interval, what lies
//      above it is kept for certain.  The first pass uses bins of half a unit of logit / T below the
//      maximum, which also yields the total mass.
//   2. once the interval holds at most 4096 elements they are collected into LDS, sorted (bitonic, by value
//      then column), their masses scanned in that order, and the cut is the first position where count or
//      mass reaches its target.
//   3. an interval that cannot shrink (one float value, more than 4096 equal logits) is cut by column: one
//      ordered pass counts the equal elements up to the number still wanted.
//   4. the draw: one more pass, Gumbel-max over the elements at or before the cut.
#include "logits_common.h"

#include <string.h>

namespace {

using namespace z2z_logits;

constexpr int T_THREADS = 512;
constexpr int T_WAVES = T_THREADS / 64;
constexpr int T_BINS = 32;
constexpr int T_CAND = 4096;
constexpr int L_PARTS = 2048;                                  // list kernel: most parts per row it takes
constexpr int L_DEPTH = 256;                                   // list kernel: largest k, and the depth tried for a nucleus alone
static_assert(2 * L_PARTS <= T_CAND, "the list kernel keeps two runs per part in one candidate array");
constexpr int T_SPLIT = 4;                                     // workgroups per row in the first pass
constexpr int T_CHUNK = T_THREADS * 4;                         // columns per step: 4 consecutive ones per thread
constexpr int T_HIST_BYTES = T_WAVES * T_BINS * 64 * 4;        // one histogram (counts or masses): 64 KiB
constexpr int T_LDS = 2 * T_HIST_BYTES + 1024;                 // + edges, bin totals, state

struct TruncArgs {
  const float* logits;     // [rows, ld]: logit / T as the decode kernel stored them
  const int32_t* size;     // [B]
  const float* row_max;    // [rows] largest stored value of the row
  const float* row_lse;    // [rows] log-sum-exp of the row's stored values
  const float* part_m;     // [rows, n_parts] largest stored value per part of the row (the decode kernel's units)
  const float* part_s;     // list kernel, stats_out given: [rows, n_parts] the parts' sums of exp(value - part_m)
  const int32_t* part_i;   //                               [rows, n_parts] the columns of the parts' maxima
  float* stats_out;        // list kernel: nullptr (row_max / row_lse are given), or [2 rows]: it merges the row's parts
                           // itself and leaves the row maxima, then the log-sum-exps, here (= row_max, row_lse)
  int32_t n_parts, n_base_parts, base_columns, hyper_columns;
  int32_t list_depth;      // list kernel: how many of the row's largest parts bound the list
  int32_t* redo;           // [rows] list kernel out: 1 = this row is left to the passes over the whole row;
                           // the other kernels skip rows with 0 (nullptr: they take every row)
  int32_t V, cap, ld;
  float inv_temperature;   // applied to the stored values (1: they are scaled already)
  int32_t top_k;           // <= 0: off
  float top_p;             // >= 1: off
  uint32_t key0, key1, ctr2, ctr3;
  int32_t* token;          // [rows]
  float* logprob;          // [rows] or nullptr
};

struct State {              // written by thread 0, read by all after a barrier
  float lo, hi;             // the cut lies among the elements with lo <= x < hi
  uint32_t cnt_above;       // elements with x >= hi: kept for certain
  float mass_above;
  float total_mass;
  uint32_t pop;             // elements inside [lo, hi)
  int next;                 // 0 another histogram pass, 1 collect and sort, 2 cut by column, 3 everything is kept,
                            // 4 find the interval's smallest and largest element first
  float cut_x;
  int cut_c;
  float kept_mass;
};

__device__ __forceinline__ bool before(float xa, int ca, float xb, int cb) {   // a precedes b in the order
  return xa > xb || (xa == xb && ca < cb);
}

// The candidate list (cnt <= T_CAND entries: value, column) is sorted into the order of the rule (bitonic, in
// LDS), the masses exp((x - m) * inv_t) are scanned in that order (cand_w: inclusive prefix sums), and misc[1]
// receives the first position at which the count (cnt_above + position + 1) reaches k_eff or the mass
// (mass_above + prefix) reaches target, 0x7FFFFFFF if none does.  All threads call it; misc[8..16) is scratch.
__device__ __forceinline__ void sort_and_scan(float* cand_x, int* cand_c, float* cand_w, int cnt, float m, float inv_t,
                                              uint32_t cnt_above, float mass_above, uint32_t k_eff, float target,
                                              uint32_t* misc) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int n2 = 2;
  while (n2 < cnt) n2 <<= 1;
  if (cnt <= T_THREADS) {
    // a short list: every element's position is the number of elements that precede it (the order is strict:
    // columns differ).  The cnt^2 comparisons are dealt to all threads: thread (g, i) compares element i with
    // elements g, g + G, ...; a wave's lanes share g, so every LDS read of element j is a broadcast.
    int P = 64;
    while (P < cnt) P <<= 1;
    const int G = T_THREADS / P;
    uint32_t* rank = reinterpret_cast<uint32_t*>(cand_w);
    for (int i = tid; i < P; i += T_THREADS) rank[i] = 0u;
    __syncthreads();
    const int i = tid & (P - 1), g = tid / P;
    float xi = 0.f;
    int ci = 0;
    if (i < cnt) {
      xi = cand_x[i];
      ci = cand_c[i];
      uint32_t ahead = 0;
      for (int j = g; j < cnt; j += G) ahead += before(cand_x[j], cand_c[j], xi, ci) ? 1u : 0u;
      atomicAdd(&rank[i], ahead);
    }
    __syncthreads();
    const uint32_t rk = i < cnt ? rank[i] : 0u;
    __syncthreads();
    if (g == 0 && i < cnt) {
      cand_x[rk] = xi;
      cand_c[rk] = ci;
    }
    __syncthreads();
  } else {
  for (int i = cnt + tid; i < n2; i += T_THREADS) {
    cand_x[i] = -INFINITY;
    cand_c[i] = 0x7FFFFFFF;
  }
  __syncthreads();
  for (int k = 2; k <= n2; k <<= 1) {
    for (int j = k >> 1; j >= 1; j >>= 1) {
      for (int i = tid; i < n2; i += T_THREADS) {
        const int p = i ^ j;
        if (p > i) {
          const float xa = cand_x[i], xb = cand_x[p];
          const int ca = cand_c[i], cb = cand_c[p];
          const bool in_order = ((i & k) == 0) ? !before(xb, cb, xa, ca) : !before(xa, ca, xb, cb);
          if (!in_order) {
            cand_x[i] = xb;
            cand_c[i] = cb;
            cand_x[p] = xa;
            cand_c[p] = ca;
          }
        }
      }
      __syncthreads();
    }
  }
  }
  // masses in sorted order and their inclusive prefix sums: each thread owns a contiguous run
  const int per = (n2 + T_THREADS - 1) / T_THREADS;
  const int i0 = tid * per;
  float run = 0.f;
  for (int i = i0; i < min(i0 + per, n2); ++i) {
    run += i < cnt ? __expf((cand_x[i] - m) * inv_t) : 0.f;
    cand_w[i] = run;
  }
  // exclusive prefix of the run totals over the block
  float incl = run;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const float o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  float* wave_tot = reinterpret_cast<float*>(misc + 8);
  if (lane == 63) wave_tot[wave] = incl;
  if (tid == 0) misc[1] = 0x7FFFFFFFu;
  __syncthreads();
  float base = incl - run;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  for (int i = i0; i < min(i0 + per, cnt); ++i) {
    const float cum = mass_above + base + cand_w[i];
    if (cnt_above + (uint32_t)i + 1u >= k_eff || cum >= target) {
      atomicMin(&misc[1], (uint32_t)i);
      break;
    }
  }
  __syncthreads();
  for (int i = i0; i < min(i0 + per, n2); ++i) cand_w[i] += base;     // now inclusive over the whole list
  __syncthreads();
}

struct Best {               // the largest perturbed value so far: value, scaled logit and column
  float v, z;
  int i;
};

// Gumbel-max over the sorted list's positions 0 .. last (this thread's share).
__device__ __forceinline__ Best draw_from_list(const float* cand_x, const int* cand_c, int last, float inv_t, int r,
                                               uint32_t key0, uint32_t key1, uint32_t ctr2, uint32_t ctr3) {
  Best b{kNegInf, 0.f, kNoColumn};
  for (int i = threadIdx.x; i <= last; i += T_THREADS) {
    const float v = cand_x[i];
    const int c = cand_c[i];
    const uint4 words = philox4x32_10(uint4{(uint32_t)(c >> 2), (uint32_t)r, ctr2, ctr3}, key0, key1);
    const int j = c & 3;
    const uint32_t w = j == 0 ? words.x : (j == 1 ? words.y : (j == 2 ? words.z : words.w));
    const float z = v * inv_t;
    const float p = z + gumbel_from_word(w);
    if (p > b.v || (p == b.v && c < b.i)) {          // the list is not in column order
      b.v = p;
      b.z = z;
      b.i = c;
    }
  }
  return b;
}

// The block's best draw (lowest column among equal perturbed values), valid in thread 0.  All threads call
// it; `red` is scratch for 3 * T_WAVES words.
__device__ __forceinline__ Best block_best(Best b, uint32_t* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float v = __shfl_xor(b.v, off), z = __shfl_xor(b.z, off);
    const int i = __shfl_xor(b.i, off);
    if (v > b.v || (v == b.v && i < b.i)) {
      b.v = v;
      b.z = z;
      b.i = i;
    }
  }
  __syncthreads();
  float* xv = reinterpret_cast<float*>(red);
  float* xz = xv + T_WAVES;
  int* xi = reinterpret_cast<int*>(xz + T_WAVES);
  if (lane == 0) {
    xv[wave] = b.v;
    xz[wave] = b.z;
    xi[wave] = b.i;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < T_WAVES; ++w) {
      if (xv[w] > b.v || (xv[w] == b.v && xi[w] < b.i)) {
        b.v = xv[w];
        b.z = xz[w];
        b.i = xi[w];
      }
    }
  }
  return b;
}

// One histogram pass over the columns [c_begin, c_end) of a row (c_begin a multiple of 4): elements with
// lo <= x < hi are counted, and their masses summed, per bin of `edges` (edges[0] = hi >= ... >= edges[T_BINS]
// = lo; edges[T_BINS + 1], edges[T_BINS + 2]: start and density of the inner edges, for a first guess).
// Ends with the bin totals in bin_c / bin_m (all threads must call it; contains barriers).
__device__ __forceinline__ void histogram_pass(const float* x, int c_begin, int c_end, float lo, float hi, float m,
                                               float inv_t, const float* edges, uint32_t* hc, float* hm,
                                               uint32_t* bin_c, float* bin_m) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < T_WAVES * T_BINS * 64; i += T_THREADS) {
    hc[i] = 0u;
    hm[i] = 0.f;
  }
  __syncthreads();
  const float top = edges[T_BINS + 1], inv_w = edges[T_BINS + 2];
  uint32_t* my_c = hc + wave * T_BINS * 64 + lane;
  float* my_m = hm + wave * T_BINS * 64 + lane;
  for (int c0 = c_begin + tid * 4; c0 < c_end; c0 += T_CHUNK) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = c0 + j;
      if (c < c_end) {
        const float v = x[c];
        if (v >= lo && v < hi) {
          // bin b holds edges[b + 1] <= v < edges[b]: a guess from the spacing, settled by comparing
          // with the edges themselves (what decides is the same stored values in every pass)
          int b = (int)fminf(fmaxf((top - v) * inv_w, 0.f), (float)(T_BINS - 1));
          while (b < T_BINS - 1 && v < edges[b + 1]) ++b;
          while (b > 0 && v >= edges[b]) --b;
          atomicAdd(&my_c[b * 64], 1u);            // this lane's own column: never contended
          atomicAdd(&my_m[b * 64], __expf((v - m) * inv_t));
        }
      }
    }
  }
  __syncthreads();
  // bin totals: 16 threads per bin, each adds 32 of the 512 columns
  {
    const int b = tid >> 4, part = tid & 15;
    uint32_t sc = 0;
    float sm = 0.f;
    for (int i = part; i < T_WAVES * 64; i += 16) {
      const int w = i >> 6, l = i & 63;
      sc += hc[(w * T_BINS + b) * 64 + l];
      sm += hm[(w * T_BINS + b) * 64 + l];
    }
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
      sc += __shfl_xor(sc, off);
      sm += __shfl_xor(sm, off);
    }
    if (part == 0) {
      bin_c[b] = sc;
      bin_m[b] = sm;
    }
  }
  __syncthreads();
}

// The edges of the first pass: bins of half a unit of logit / T below the maximum, the last bin takes all
// the rest; the upper end is a finite value no element reaches.  Both kernels below compute them alike.
__device__ __forceinline__ void first_pass_edges(float m, float inv_t, float* edges) {
  const float w0 = 0.5f / inv_t;
  edges[0] = m + fmaxf(fabsf(m), 1.f) * 0x1p-10f;
  for (int i = 1; i < T_BINS; ++i) edges[i] = m - (float)i * w0;
  edges[T_BINS] = -INFINITY;
  edges[T_BINS + 1] = m;
  edges[T_BINS + 2] = 1.0f / w0;
}

// First pass, the one that classifies every element, spread over T_SPLIT workgroups per row: each takes a
// slice of the columns and leaves its bin totals in `partial` [rows][T_SPLIT][2][T_BINS].
__global__ void __launch_bounds__(T_THREADS) sample_first_pass_kernel(TruncArgs a, float* partial) {
  extern __shared__ __align__(16) unsigned char lds[];
  uint32_t* hc = reinterpret_cast<uint32_t*>(lds);
  float* hm = reinterpret_cast<float*>(lds + T_HIST_BYTES);
  float* edges = reinterpret_cast<float*>(lds + 2 * T_HIST_BYTES);
  uint32_t* bin_c = reinterpret_cast<uint32_t*>(edges + 40);
  float* bin_m = reinterpret_cast<float*>(bin_c + T_BINS);
  const int r = blockIdx.x / T_SPLIT, part = blockIdx.x % T_SPLIT;
  if (a.redo && a.redo[r] == 0) return;             // drawn by the list kernel
  const int C = min(max(a.size[r], 0), a.cap);
  const int n = a.V + C;
  const float m = a.row_max[r];
  if (threadIdx.x == 0) first_pass_edges(m, a.inv_temperature, edges);
  __syncthreads();
  const int per = ((n + T_SPLIT - 1) / T_SPLIT + 3) & ~3;
  const int c_begin = min(part * per, n), c_end = min(c_begin + per, n);
  histogram_pass(a.logits + (size_t)r * a.ld, c_begin, c_end, -INFINITY, edges[0], m, a.inv_temperature, edges, hc,
                 hm, bin_c, bin_m);
  float* out = partial + ((size_t)r * T_SPLIT + part) * 2 * T_BINS;
  if (threadIdx.x < T_BINS) {
    out[threadIdx.x] = __uint_as_float(bin_c[threadIdx.x]);
    out[T_BINS + threadIdx.x] = bin_m[threadIdx.x];
  }
}

// The passes over the whole row (steps 1-4 of the header) for row r, by all threads of a workgroup.  partial: the
// bin totals sample_first_pass_kernel left, or nullptr (the first pass is made here).  lds: T_LDS bytes.
__device__ __forceinline__ void truncated_row(const TruncArgs& a, const float* partial, int r, unsigned char* lds) {
  uint32_t* hc = reinterpret_cast<uint32_t*>(lds);                         // [wave][bin][lane]
  float* hm = reinterpret_cast<float*>(lds + T_HIST_BYTES);                // [wave][bin][lane]
  float* edges = reinterpret_cast<float*>(lds + 2 * T_HIST_BYTES);         // [T_BINS + 1]
  uint32_t* bin_c = reinterpret_cast<uint32_t*>(edges + 40);               // [T_BINS]
  float* bin_m = reinterpret_cast<float*>(bin_c + T_BINS);                 // [T_BINS]
  State* st = reinterpret_cast<State*>(bin_m + T_BINS);
  uint32_t* misc = reinterpret_cast<uint32_t*>(st + 1);                    // counters, wave totals (>= 32 words)
  // the candidate arrays reuse the histograms
  float* cand_x = reinterpret_cast<float*>(lds);                           // [T_CAND]
  int* cand_c = reinterpret_cast<int*>(lds + T_CAND * 4);                  // [T_CAND]
  float* cand_w = reinterpret_cast<float*>(lds + T_CAND * 8);              // [T_CAND] masses, then their prefix sums

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int C = min(max(a.size[r], 0), a.cap);
  const int n = a.V + C;
  const float* x = a.logits + (size_t)r * a.ld;
  const float m = a.row_max[r];
  const float inv_t = a.inv_temperature;
  const uint32_t k_eff = a.top_k > 0 ? (uint32_t)min(a.top_k, n) : (uint32_t)n;
  const bool use_p = a.top_p < 1.0f;

  if (tid == 0) {
    first_pass_edges(m, inv_t, edges);
    st->lo = -INFINITY;
    st->hi = edges[0];
    st->cnt_above = 0;
    st->mass_above = 0.f;
    st->total_mass = 0.f;
    st->pop = (uint32_t)n;
    st->next = 0;
  }
  __syncthreads();

  // ---- 1. histogram passes ---------------------------------------------------------------------------
  for (int pass = 0; pass < 40; ++pass) {
    if (st->next == 4) {
      // A pass that put the whole interval into one bin: the elements may be a tight cluster or all equal.
      // Their smallest and largest value give the next interval, or show that one value is all there is.
      const float blo = st->lo, bhi = st->hi;
      float vmin = INFINITY, vmax = -INFINITY;
      for (int c = tid; c < n; c += T_THREADS) {
        const float v = x[c];
        if (v >= blo && v < bhi) {
          vmin = fminf(vmin, v);
          vmax = fmaxf(vmax, v);
        }
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        vmin = fminf(vmin, __shfl_xor(vmin, off));
        vmax = fmaxf(vmax, __shfl_xor(vmax, off));
      }
      float* red = reinterpret_cast<float*>(misc + 8);
      if (lane == 0) {
        red[wave] = vmin;
        red[T_WAVES + wave] = vmax;
      }
      __syncthreads();
      if (tid == 0) {
        for (int w = 1; w < T_WAVES; ++w) {
          vmin = fminf(vmin, red[w]);
          vmax = fmaxf(vmax, red[T_WAVES + w]);
        }
        if (vmin == vmax) {
          st->lo = vmin;                             // every element of the interval equals this value
          st->next = 2;
        } else {
          const float nhi = vmax + fmaxf(fabsf(vmax), 1.f) * 0x1p-20f;    // just above the largest element
          const float w = (nhi - vmin) / (float)T_BINS;
          st->lo = vmin;
          st->hi = nhi;
          edges[0] = nhi;
          for (int i = 1; i < T_BINS; ++i) edges[i] = fmaxf(nhi - (float)i * w, vmin);
          edges[T_BINS] = vmin;
          edges[T_BINS + 1] = nhi;
          edges[T_BINS + 2] = w > 0.f ? 1.0f / w : 0.f;
          st->next = 0;
        }
      }
      __syncthreads();
      continue;
    }
    if (st->next != 0) break;                       // uniform: read after a barrier
    const float lo = st->lo, hi = st->hi;
    if (pass == 0 && partial) {
      // the first pass was done by sample_first_pass_kernel: add up its slices (fixed order)
      if (tid < T_BINS) {
        uint32_t sc = 0;
        float sm = 0.f;
        for (int p = 0; p < T_SPLIT; ++p) {
          const float* in = partial + ((size_t)r * T_SPLIT + p) * 2 * T_BINS;
          sc += __float_as_uint(in[tid]);
          sm += in[T_BINS + tid];
        }
        bin_c[tid] = sc;
        bin_m[tid] = sm;
      }
      __syncthreads();
    } else {
      histogram_pass(x, 0, n, lo, hi, m, inv_t, edges, hc, hm, bin_c, bin_m);
    }
    if (tid == 0) {
      if (pass == 0) {
        float tot = 0.f;
        for (int b = 0; b < T_BINS; ++b) tot += bin_m[b];
        st->total_mass = tot;
      }
      const float target = use_p ? a.top_p * st->total_mass : INFINITY;
      uint32_t cnt = st->cnt_above;
      float mass = st->mass_above;
      int hit = -1;
      for (int b = 0; b < T_BINS; ++b) {
        if (bin_c[b] == 0) continue;
        if (cnt + bin_c[b] >= k_eff || mass + bin_m[b] >= target) {
          hit = b;
          break;
        }
        cnt += bin_c[b];
        mass += bin_m[b];
      }
      if (hit < 0) {
        // neither target is reached inside the interval (k covers it, and rounding kept the mass below
        // p * total): everything down to the interval's lower end is kept
        st->next = 3;
        st->cnt_above = cnt;
        st->mass_above = mass;
      } else {
        const float nhi = edges[hit];
        const float nlo = edges[hit + 1];
        const bool no_progress = bin_c[hit] == st->pop;
        st->cnt_above = cnt;
        st->mass_above = mass;
        st->pop = bin_c[hit];
        st->hi = nhi;
        st->lo = nlo;
        if (bin_c[hit] <= (uint32_t)T_CAND) {
          st->next = 1;
        } else if (no_progress && !isinf(nlo)) {
          st->next = 4;
        } else {
          // split [nlo, nhi) again; an open lower end (the far tail) is given a span that grows with every
          // pass.
          const float bot = isinf(nlo) ? nhi - 64.f / inv_t * exp2f((float)(2 * pass)) : nlo;
          const float w = (nhi - bot) / (float)T_BINS;
          bool shrinks = false;
          edges[0] = nhi;
          for (int i = 1; i < T_BINS; ++i) {
            edges[i] = fmaxf(nhi - (float)i * w, bot);
            if (edges[i] < nhi && edges[i] > bot) shrinks = true;
          }
          edges[T_BINS] = nlo;
          edges[T_BINS + 1] = nhi;
          edges[T_BINS + 2] = w > 0.f ? 1.0f / w : 0.f;
          if (!isinf(nlo) && !shrinks) st->next = 4;   // nothing left to split by value: look at the elements
        }
      }
    }
    __syncthreads();
  }
  if (st->next == 0) {                               // pass limit: cannot happen for finite logits; keep the prefix found
    if (tid == 0) st->next = st->pop <= (uint32_t)T_CAND ? 1 : 2;
    __syncthreads();
  }

  const int mode = st->next;
  const float lo = st->lo, hi = st->hi;
  const float target = use_p ? a.top_p * st->total_mass : INFINITY;

  bool all_in = false;
  if (mode == 1) {
    // ---- 2. collect, sort, scan ------------------------------------------------------------------------
    // if what lies above the interval fits into the list as well, it is collected too: the sorted list then
    // holds every kept element and the draw needs no further pass over the row
    all_in = st->cnt_above + st->pop <= (uint32_t)T_CAND;
    __syncthreads();
    if (tid == 0) misc[0] = 0u;
    __syncthreads();
    for (int c0 = tid * 4; c0 < n; c0 += T_CHUNK) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + j;
        if (c < n) {
          const float v = x[c];
          if (v >= lo && (all_in || v < hi)) {
            const uint32_t slot = atomicAdd(&misc[0], 1u);
            if (slot < (uint32_t)T_CAND) {
              cand_x[slot] = v;
              cand_c[slot] = c;
            }
          }
        }
      }
    }
    __syncthreads();
    const int cnt = (int)min(misc[0], (uint32_t)T_CAND);
    const uint32_t cnt_above = all_in ? 0u : st->cnt_above;
    const float mass_above = all_in ? 0.f : st->mass_above;
    sort_and_scan(cand_x, cand_c, cand_w, cnt, m, inv_t, cnt_above, mass_above, k_eff, target, misc);
    if (tid == 0) {
      int idx = misc[1] == 0x7FFFFFFFu ? cnt - 1 : (int)misc[1];       // rounding kept the mass below its target
      idx = max(idx, 0);
      st->cut_x = cand_x[idx];
      st->cut_c = cand_c[idx];
      st->kept_mass = mass_above + cand_w[idx];
      misc[5] = (uint32_t)idx;
    }
    __syncthreads();
  } else if (mode == 2) {
    // ---- 3. more than T_CAND equal logits: the cut is a column among them -------------------------------
    if (tid == 0) {
      const float w = __expf((lo - m) * inv_t);
      uint32_t want = k_eff - st->cnt_above;
      if (use_p) {
        const float need = (target - st->mass_above) / w;
        const uint32_t by_mass = need <= 1.f ? 1u : (need >= 4.0e9f ? 0xFFFFFFFFu : (uint32_t)ceilf(need));
        want = min(want, by_mass);
      }
      want = max(1u, min(want, st->pop));
      misc[2] = want;
      misc[3] = 0u;                                  // equal elements seen so far
      misc[4] = 0u;                                  // done flag
      st->kept_mass = st->mass_above + (float)want * w;
      st->cut_x = lo;
      st->cut_c = n - 1;
    }
    __syncthreads();
    const uint32_t want = misc[2];
    uint32_t* wave_cnt = misc + 8;
    for (int c0 = 0; c0 < n; c0 += T_CHUNK) {
      const int cb = c0 + tid * 4;
      uint32_t flags = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (cb + j < n && x[cb + j] == lo) flags |= 1u << j;
      const uint32_t mine = __popc(flags);
      uint32_t incl = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
      }
      if (lane == 63) wave_cnt[wave] = incl;
      __syncthreads();
      uint32_t before_me = misc[3] + incl - mine;
      uint32_t chunk_total = 0;
      for (int w = 0; w < T_WAVES; ++w) {
        if (w < wave) before_me += wave_cnt[w];
        chunk_total += wave_cnt[w];
      }
      if (before_me < want && before_me + mine >= want) {
        uint32_t seen = before_me;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (flags & (1u << j)) {
            if (++seen == want) st->cut_c = cb + j;
          }
        misc[4] = 1u;
      }
      __syncthreads();
      if (tid == 0) misc[3] += chunk_total;
      const bool done = misc[4] != 0u;
      __syncthreads();
      if (done) break;
    }
    __syncthreads();
  } else {
    // ---- everything in and above the interval is kept ---------------------------------------------------
    if (tid == 0) {
      st->cut_x = lo;
      st->cut_c = 0x7FFFFFFF;
      st->kept_mass = st->mass_above;
    }
    __syncthreads();
  }

  // ---- 4. the draw --------------------------------------------------------------------------------------
  const float cx = st->cut_x;
  const int cc = st->cut_c;
  Best best{kNegInf, 0.f, kNoColumn};
  if (all_in) {
    // every kept element is in the sorted list, positions 0 .. idx
    best = draw_from_list(cand_x, cand_c, (int)misc[5], inv_t, r, a.key0, a.key1, a.ctr2, a.ctr3);
  } else {
    for (int c0 = tid * 4; c0 < n; c0 += T_CHUNK) {
      uint4 words = uint4{0u, 0u, 0u, 0u};
      bool have = false;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + j;
        if (c < n) {
          const float v = x[c];
          if (v > cx || (v == cx && c <= cc)) {
            if (!have) {
              words = philox4x32_10(uint4{(uint32_t)(c0 >> 2), (uint32_t)r, a.ctr2, a.ctr3}, a.key0, a.key1);
              have = true;
            }
            const uint32_t w = j == 0 ? words.x : (j == 1 ? words.y : (j == 2 ? words.z : words.w));
            const float z = v * inv_t;
            const float p = z + gumbel_from_word(w);
            if (p > best.v) {                         // increasing columns: strict comparison keeps the lowest
              best.v = p;
              best.z = z;
              best.i = c;
            }
          }
        }
      }
    }
  }
  best = block_best(best, misc + 8);
  if (tid == 0) {
    a.token[r] = best.i;
    if (a.logprob) a.logprob[r] = (best.z - m * inv_t) - logf(st->kept_mass);
  }
}

// The short way, for a prefix of at most a few hundred columns.  The decode kernel left the largest value of
// every part of the row (256 base columns, 512 hyper columns).  Let L be the j-th largest of them: j different
// columns reach L, so the j-th element of the order is >= L, and every element >= L lies in a part whose
// largest value is >= L.  Only those parts are read again, their elements >= L collected, and the sorted list
// is then a prefix of the row's order that is at least j long: a top-k cut with k <= j, or a nucleus that
// closes inside the list, is decided on it exactly as on the whole row (total mass: from the row's
// log-sum-exp).  A row whose list overflows, or whose nucleus does not close inside it, sets redo[row].
// Returns whether the row was settled (uniform over the workgroup); a row that was not has redo[r] = 1.
// lds: L_LDS bytes.
constexpr int L_LDS = L_PARTS * 4 + 3 * T_CAND * 4 + 48 * 4 + 4 * (int)sizeof(Triple) + 16;
__device__ __forceinline__ bool list_row(const TruncArgs& a, int r, int rows, unsigned char* lds) {
  float* pm = reinterpret_cast<float*>(lds);                                     // [L_PARTS]
  float* cand_x = pm + L_PARTS;                                                  // [T_CAND]
  int* cand_c = reinterpret_cast<int*>(cand_x + T_CAND);                         // [T_CAND]
  float* cand_w = reinterpret_cast<float*>(cand_c + T_CAND);                     // [T_CAND]
  uint32_t* misc = reinterpret_cast<uint32_t*>(cand_w + T_CAND);                 // [48]
  Triple* xch = reinterpret_cast<Triple*>(misc + 48);                            // [4]
  float* row_stat = reinterpret_cast<float*>(xch + 4);                           // [2]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int C = min(max(a.size[r], 0), a.cap);
  const int n = a.V + C;
  const float* x = a.logits + (size_t)r * a.ld;
  const int n_parts = a.n_parts;
  const int depth = min(a.list_depth, n);
  uint32_t* hist = reinterpret_cast<uint32_t*>(cand_w);          // [4][256]: free until the work items are listed

  if (!a.stats_out)
    for (int i = tid; i < n_parts; i += T_THREADS) pm[i] = a.part_m[(size_t)r * n_parts + i];
  for (int i = tid; i < 4 * 256; i += T_THREADS) hist[i] = 0u;
  if (tid == 0) {
    misc[0] = 0u;            // list length
    misc[3] = 0u;            // work items
    misc[4] = 0u;            // mass of the list (float)
  }
  // the row's maximum and log-sum-exp: given, or merged here from the parts' (m, s, column) in the order of
  // logits_combine_kernel<256> (256 threads striding over the parts, a butterfly per wave, the four waves in turn)
  if (a.stats_out) {
    Triple tr = empty_triple();
    if (tid < 256) {
      const size_t base = (size_t)r * n_parts;
      for (int p = tid; p < n_parts; p += 256) {
        Triple o;
        o.m = a.part_m[base + p];
        o.s = a.part_s[base + p];
        o.i = a.part_i[base + p];
        pm[p] = o.m;                                  // (the one trip to memory serves both uses)
        merge_triple(tr, o);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        Triple o;
        o.m = __shfl_xor(tr.m, off);
        o.s = __shfl_xor(tr.s, off);
        o.i = __shfl_xor(tr.i, off);
        merge_triple(tr, o);
      }
      if (lane == 0) xch[wave] = tr;
    }
    __syncthreads();
    if (tid == 0) {
      Triple tr0 = xch[0];
#pragma unroll
      for (int w = 1; w < 4; ++w) merge_triple(tr0, xch[w]);
      row_stat[0] = tr0.m;
      row_stat[1] = tr0.m + logf(tr0.s);
      a.stats_out[r] = row_stat[0];
      a.stats_out[rows + r] = row_stat[1];
    }
  } else if (tid == 0) {
    row_stat[0] = a.row_max[r];
    row_stat[1] = a.row_lse[r];
  }
  __syncthreads();
  const float row_m = row_stat[0], row_l = row_stat[1];
  // the depth-th largest part maximum, by the digits of the maxima's order-preserving integer images (larger
  // float <=> larger key; -0 counts as +0): four passes of 8 bits, a 256-bin count each, every wave walks the
  // bins from the top for itself (the count of larger keys stays below depth until the digit's bin)
  bool ok = depth >= 1 && depth <= n_parts;          // uniform
  float level = -INFINITY;
  if (ok) {
    uint32_t key[L_PARTS / T_THREADS];
#pragma unroll
    for (int q = 0; q < L_PARTS / T_THREADS; ++q) {
      const int i = tid + q * T_THREADS;
      const uint32_t u = __float_as_uint((i < n_parts ? pm[i] : 0.f) + 0.0f);
      key[q] = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    }
    uint32_t prefix = 0u, rem = (uint32_t)depth;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      uint32_t* h = hist + pass * 256;
#pragma unroll
      for (int q = 0; q < L_PARTS / T_THREADS; ++q)
        if (tid + q * T_THREADS < n_parts && (pass == 0 || (key[q] >> (shift + 8)) == prefix))
          atomicAdd(&h[(key[q] >> shift) & 255u], 1u);
      __syncthreads();
      const uint4 cn = reinterpret_cast<const uint4*>(h)[lane];            // bins 4 lane .. 4 lane + 3
      const uint32_t own = cn.x + cn.y + cn.z + cn.w;
      uint32_t incl = own;                                                 // this lane's bins and all above
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_down(incl, off);
        if (lane + off < 64) incl += o;
      }
      const uint32_t a3 = incl - own, a2 = a3 + cn.w, a1 = a2 + cn.z, a0 = a1 + cn.y;   // keys above bin 3, 2, 1, 0
      int digit = -1;
      uint32_t left = 0u;
      if (a3 < rem && rem <= a3 + cn.w) { digit = 4 * lane + 3; left = rem - a3; }
      else if (a2 < rem && rem <= a2 + cn.z) { digit = 4 * lane + 2; left = rem - a2; }
      else if (a1 < rem && rem <= a1 + cn.y) { digit = 4 * lane + 1; left = rem - a1; }
      else if (a0 < rem && rem <= a0 + cn.x) { digit = 4 * lane; left = rem - a0; }
      const uint64_t who = __ballot(digit >= 0);                           // exactly one lane: rem <= the pass's keys
      const int src = who != 0ull ? __ffsll((long long)who) - 1 : 0;
      prefix = (prefix << 8) | (uint32_t)__shfl(digit >= 0 ? digit : 0, src);
      rem = __shfl(left, src);
    }
    level = __uint_as_float((prefix & 0x80000000u) ? (prefix & 0x7FFFFFFFu) : ~prefix);
    ok = level > -INFINITY;
  }
  __syncthreads();                                    // the counts are read: their words become the work items
  // no element weighs more than the largest one, exp(0) = 1 in the units of the masses, and the list comes out
  // about list_depth long: a nucleus alone that needs more mass than twice that many elements could carry
  // is not tried (a flat distribution; the passes over the whole row take it)
  if (a.top_k <= 0 && a.top_p * __expf((row_l - row_m) * a.inv_temperature) > (float)(2 * a.list_depth)) ok = false;
  const float L = ok ? level : INFINITY;
  // work items: runs of at most 256 columns of the parts that reach L (cand_c is free until the appends start,
  // and they start after the barrier; items are kept in cand_w, which the scan fills later)
  int* item_c0 = reinterpret_cast<int*>(cand_w);  // [<= 2 * L_PARTS = T_CAND]: a part has at most two runs
  if (ok) {
    for (int p = tid; p < n_parts; p += T_THREADS) {
      if (!(pm[p] >= L)) continue;
      int c0, c1;
      if (p < a.n_base_parts) {
        c0 = p * a.base_columns;
        c1 = min(c0 + a.base_columns, a.V);
      } else {
        c0 = a.V + (p - a.n_base_parts) * a.hyper_columns;
        c1 = min(c0 + a.hyper_columns, n);
      }
      const int pieces = (c1 - c0 + 255) >> 8;
      if (pieces > 0) {
        const uint32_t at = atomicAdd(&misc[3], (uint32_t)pieces);
        for (int q = 0; q < pieces; ++q) item_c0[at + q] = c0 + 256 * q;
      }
    }
  }
  __syncthreads();
  if (ok) {
    const int n_items = (int)misc[3];
    const float m0 = row_m;
    float mass = 0.f;                                // of what this lane appends
    constexpr int IPW = 8;                           // items per wave and round: 4 IPW independent loads in flight
    for (int it = 0; it < n_items; it += T_WAVES * IPW) {          // items dealt round-robin to the waves
      float v[4 * IPW];
      int cc[4 * IPW];
#pragma unroll
      for (int q = 0; q < IPW; ++q) {
        const int item = it + q * T_WAVES + wave;
        const bool have = item < n_items;            // wave-uniform
        const int c0 = have ? item_c0[item] : 0;
        int c1 = 0;                                  // the run ends with its part, after 256 columns at most
        if (have) {
          const int part_end = c0 < a.V ? min((c0 / a.base_columns + 1) * a.base_columns, a.V)
                                        : min(a.V + ((c0 - a.V) / a.hyper_columns + 1) * a.hyper_columns, n);
          c1 = min(c0 + 256, part_end);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int c = c0 + j * 64 + lane;
          cc[q * 4 + j] = c < c1 ? c : -1;
          v[q * 4 + j] = c < c1 ? x[c] : -INFINITY;
        }
      }
#pragma unroll
      for (int j = 0; j < 4 * IPW; ++j) {
        const bool take = cc[j] >= 0 && v[j] >= L;
        const uint64_t mask = __ballot(take);
        if (mask != 0ull) {
          uint32_t first = 0;
          if (lane == 0) first = atomicAdd(&misc[0], (uint32_t)__popcll(mask));
          first = __shfl(first, 0);
          const uint32_t slot = first + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
          if (take && slot < (uint32_t)T_CAND) {
            cand_x[slot] = v[j];
            cand_c[slot] = cc[j];
            mass += __expf((v[j] - m0) * a.inv_temperature);
          }
        }
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mass += __shfl_xor(mass, off);
    if (lane == 0) atomicAdd(reinterpret_cast<float*>(&misc[4]), mass);
  }
  __syncthreads();
  const uint32_t found = misc[0];
  ok = ok && found <= (uint32_t)T_CAND && found >= 1u;
  if (!ok) {
    if (tid == 0) a.redo[r] = 1;
    return false;
  }
  const int cnt = (int)found;
  const float m = row_m;
  const float inv_t = a.inv_temperature;
  const uint32_t k_eff = a.top_k > 0 ? (uint32_t)min(a.top_k, n) : (uint32_t)n;
  const float target = a.top_p < 1.0f ? a.top_p * __expf((row_l - m) * inv_t) : INFINITY;
  if (a.top_k <= 0 && cnt < n && __uint_as_float(misc[4]) < 0.999f * target) {
    if (tid == 0) a.redo[r] = 1;                     // a nucleus alone, and the whole list weighs too little
    return false;
  }
  sort_and_scan(cand_x, cand_c, cand_w, cnt, m, inv_t, 0u, 0.f, k_eff, target, misc);
  int idx;
  if (misc[1] != 0x7FFFFFFFu)
    idx = (int)misc[1];
  else if (cnt == n)
    idx = cnt - 1;                                   // the whole row is in the list and rounding kept the mass below p
  else {
    if (tid == 0) a.redo[r] = 1;                     // the cut lies beyond the list
    return false;
  }
  Best best = draw_from_list(cand_x, cand_c, idx, inv_t, r, a.key0, a.key1, a.ctr2, a.ctr3);
  best = block_best(best, misc + 8);
  if (tid == 0) {
    a.redo[r] = 0;
    a.token[r] = best.i;
    if (a.logprob) a.logprob[r] = (best.z - m * inv_t) - logf(cand_w[idx]);
  }
  return true;
}

__global__ void __launch_bounds__(T_THREADS) sample_truncated_kernel(TruncArgs a, const float* partial) {
  extern __shared__ __align__(16) unsigned char lds[];
  if (a.redo && a.redo[blockIdx.x] == 0) return;    // drawn by the list kernel
  truncated_row(a, partial, blockIdx.x, lds);
}

__global__ void __launch_bounds__(T_THREADS) sample_list_kernel(TruncArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  (void)list_row(a, blockIdx.x, gridDim.x, lds);
}

// Both in one launch: the workgroup of a row the list does not settle goes on to the passes over the whole row.
__global__ void __launch_bounds__(T_THREADS) sample_list_then_row_kernel(TruncArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  if (list_row(a, blockIdx.x, gridDim.x, lds)) return;
  __syncthreads();
  truncated_row(a, nullptr, blockIdx.x, lds);
}

}  // namespace

// Whether the selection starts with the short-list kernel (which then also merges the row's parts into the row
// maxima and log-sum-exps: the caller launches no merge of its own).
static bool list_first_for(const z2z_ctx* c, int n_parts, int32_t top_k, int base_columns) {
  int unit_base, unit_hyper;
  z2z_logits_decode_units(&unit_base, &unit_hyper);
  if (base_columns > 0) unit_base = base_columns;
  return c->opt_sample_kernel != 1 && n_parts <= L_PARTS && top_k <= L_DEPTH && unit_base <= 512 && unit_hyper <= 512;
}

bool z2z_sample_truncated_merges_parts(const z2z_ctx* c, int n_parts, int32_t top_k, int base_columns) {
  return list_first_for(c, n_parts, top_k, base_columns);
}

int z2z_launch_sample_truncated(z2z_ctx* c, const float* logits, float* row_stat, int32_t rows, int n_parts,
                                float* work, const z2z_sample_params* sp, int32_t top_k, float top_p,
                                int32_t* token, float* logprob, hipStream_t s, int base_columns) {
  (void)sp->temperature;                             // the stored values are scaled already
  TruncArgs a;
  memset(&a, 0, sizeof(a));
  a.logits = logits;
  a.size = c->st.size;
  a.row_max = row_stat;
  a.row_lse = row_stat + rows;
  a.part_m = c->part_m;
  a.part_s = c->part_s;
  a.part_i = c->part_i;
  a.n_parts = n_parts;
  z2z_logits_decode_units(&a.base_columns, &a.hyper_columns);
  if (base_columns > 0) a.base_columns = base_columns;   // the base parts came from another kernel's strips
  a.n_base_parts = (c->cfg.V + a.base_columns - 1) / a.base_columns;
  a.V = c->cfg.V;
  a.cap = c->cfg.cap;
  a.ld = c->cfg.V + c->cfg.cap;
  a.inv_temperature = 1.0f;
  a.top_k = top_k;
  a.top_p = top_p;
  a.key0 = (uint32_t)sp->seed;
  a.key1 = (uint32_t)(sp->seed >> 32);
  a.ctr2 = (uint32_t)sp->step;
  a.ctr3 = (uint32_t)(sp->step >> 32);
  a.token = token;
  a.logprob = logprob;
  a.redo = nullptr;
  a.list_depth = 0;
  float* partial = work + rows;                      // work: [rows] redo flags, then the first pass's bin totals
  // a short prefix first: rows it cannot settle are flagged, and only those take the passes over the whole row
  const bool list_first = list_first_for(c, n_parts, top_k, base_columns);
  if (list_first) {
    a.redo = reinterpret_cast<int32_t*>(work);
    a.list_depth = top_k > 0 ? top_k : L_DEPTH;
    a.stats_out = row_stat;
    if (top_k > 0) {
      // With a top-k the list settles every row but those with many equal logits at the cut: the rare row
      // that is left is finished by the same workgroup (it classifies its elements itself), one launch in all.
      hipLaunchKernelGGL(sample_list_then_row_kernel, dim3(rows), dim3(T_THREADS), T_LDS, s, a);
      Z2Z_HIP_TRY(hipGetLastError());
      return Z2Z_OK;
    }
    // A nucleus alone leaves whole batches of flat rows to the passes over the whole row: their first pass is
    // spread over T_SPLIT workgroups per row, in launches of their own.
    hipLaunchKernelGGL(sample_list_kernel, dim3(rows), dim3(T_THREADS), L_LDS, s, a);
    a.stats_out = nullptr;
  }
  hipLaunchKernelGGL(sample_first_pass_kernel, dim3(rows * T_SPLIT), dim3(T_THREADS), T_LDS, s, a, partial);
  hipLaunchKernelGGL(sample_truncated_kernel, dim3(rows), dim3(T_THREADS), T_LDS, s, a, partial);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

size_t z2z_sample_truncated_work_floats(int32_t rows) { return (size_t)rows * (1 + T_SPLIT * 2 * T_BINS); }

int z2z_sample_truncated_prepare(z2z_ctx* c) {
  if (c->lds_limit < T_LDS) return Z2Z_EUNSUPPORTED;
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sample_truncated_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, T_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sample_first_pass_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, T_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sample_list_then_row_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, T_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(sample_list_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, L_LDS));
  return Z2Z_OK;
}
