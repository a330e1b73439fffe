// Learned hyper-encoder for gfx950 (bf16): the network that turns the embeddings of a hypertoken's constituent
// base tokens, padded to M slots, into the hypertoken's vector (zip2zip paper, section 2.2; the attention and
// transformer rows of the hyper-encoder ablation table; the two-layer transformer of the training setup).
// The paper names the architectures only; what is computed here is the standard pre-norm encoder over the M
// slots, padding masked out as keys, mean of the real slots at the end:
//
//   X_i = E[y_i] + P_i;  A = LN1(X);  QKV = A Wqkv^T + b;  O = softmax(Q K^T / sqrt(d_head)) V per head;
//   Y = X + O Wo^T + bo;  Z = Y + GELU(LN2(Y) W1^T + b1) W2^T + b2  (transformer layers);  h = mean_i Z_i.
//
// All entries of a pass are batched, and only their real slots are rows: a one-workgroup scan over the entry
// lengths gives every entry its first row (padding slots and missing entries take no rows at all; a quarter
// of the M slots of a typical codebook is padding), the number of rows stays on the device and the kernels
// read it there.  Every dense layer is then one [rows, K] x [N, K]^T product on the bf16 MFMA kernel with
// bias / GELU / residual in its epilogue.  The kernels in this file are the bandwidth-bound rest: gather +
// LayerNorm (one wave per row, the row held in registers: read once), the L x L attention per entry and head
// (a wave per entry and 512 features: 64 lanes x 16 bytes, a head's dot products reduced across its lanes),
// and the final mean.  The residual stream (X, Y, Z) is fp32 from the gather to the final mean; the operands of
// the matrix products (LayerNorm outputs, q | k | v, attention outputs, the hidden layer) are bf16;
// accumulation and statistics are fp32.
#include "logits_common.h"

namespace {

using z2z_logits::bf16_bits_rne;

constexpr int E_KCH = 8;             // 16-byte chunks per lane of one row: d <= 64 * 8 * E_KCH = 4096
constexpr float E_EPS = 1e-5f;

struct RowMap {                      // which entries a pass covers, and where their rows sit
  const int32_t* size;               // [B] C_b
  const int32_t* ent_tokens;         // [B, cap, M]
  const int32_t* ent_len;            // [B, cap]
  const int32_t* first;              // [B] or nullptr
  int32_t last_n;                    // first == nullptr: 0 = entries from 0, n > 0 = the last n entries
  int32_t B, V, M, cap, d;
  int32_t u0, un;                    // entry units [u0, u0 + un) of every sequence
  // packed rows of this pass: entry unit bu = b * un + u owns rows [row0[bu], row0[bu + 1]), one per real slot;
  // row0[B * un] is the number of rows; row_slot[r] = bu * 8 + slot of row r
  int32_t* row0;
  int32_t* row_slot;
};

__device__ __forceinline__ int entry_of(const RowMap& m, int b, int u, int* C_out) {
  const int C = min(max(m.size[b], 0), m.cap);
  *C_out = C;
  const int base = m.first ? max(m.first[b], 0) : (m.last_n > 0 ? max(C - m.last_n, 0) : 0);
  return base + m.u0 + u;
}

__device__ __forceinline__ void unpack8(const uint4& x, float (&f)[8]) {
  f[0] = __uint_as_float(x.x << 16);
  f[1] = __uint_as_float(x.x & 0xFFFF0000u);
  f[2] = __uint_as_float(x.y << 16);
  f[3] = __uint_as_float(x.y & 0xFFFF0000u);
  f[4] = __uint_as_float(x.z << 16);
  f[5] = __uint_as_float(x.z & 0xFFFF0000u);
  f[6] = __uint_as_float(x.w << 16);
  f[7] = __uint_as_float(x.w & 0xFFFF0000u);
}

// 8 consecutive fp32 values of a residual-stream row (two 16-byte accesses)
__device__ __forceinline__ void load8(const float* p, float (&f)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
  f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}

__device__ __forceinline__ void store8(float* p, const float (&f)[8]) {
  *reinterpret_cast<float4*>(p) = float4{f[0], f[1], f[2], f[3]};
  *reinterpret_cast<float4*>(p + 4) = float4{f[4], f[5], f[6], f[7]};
}

__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  uint4 o;
  o.x = bf16_bits_rne(f[0]) | (bf16_bits_rne(f[1]) << 16);
  o.y = bf16_bits_rne(f[2]) | (bf16_bits_rne(f[3]) << 16);
  o.z = bf16_bits_rne(f[4]) | (bf16_bits_rne(f[5]) << 16);
  o.w = bf16_bits_rne(f[6]) | (bf16_bits_rne(f[7]) << 16);
  return o;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

__device__ __forceinline__ int entry_len(const RowMap& m, int b, int u) {
  int C;
  const int e = entry_of(m, b, u, &C);
  return e < C ? min(max(m.ent_len[(size_t)b * m.cap + e], 1), m.M) : 0;
}

// Rows of the pass: exclusive scan of the entry lengths over all entry units, one workgroup of 1024 threads,
// each taking a run of consecutive units.
__global__ void __launch_bounds__(1024) enc_rows_kernel(RowMap m, int n_units) {
  __shared__ int wave_tot[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (n_units + 1023) / 1024;
  const int b0 = tid * per, b1 = min(b0 + per, n_units);
  int mine = 0;
  for (int bu = b0; bu < b1; ++bu) mine += entry_len(m, bu / m.un, bu % m.un);
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  int base = incl - mine;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  for (int bu = b0; bu < b1; ++bu) {
    const int L = entry_len(m, bu / m.un, bu % m.un);
    m.row0[bu] = base;
    for (int i = 0; i < L; ++i) m.row_slot[base + i] = bu * 8 + i;
    base += L;
  }
  if (tid == 1023) {
    int total = 0;
    for (int w = 0; w < 16; ++w) total += wave_tot[w];
    m.row0[n_units] = total;
  }
}

// One wave per row.  The residual stream X is fp32 (the layers add to it without rounding; only what feeds a
// matrix product is bf16).  GATHER: X[r] = E[token] + P[slot] is formed and stored first.  Then
// A[r] = bf16(LN(X[r]) * gamma + beta), statistics in two steps: mean, then the mean of the squared deviations.
template <bool GATHER>
__global__ void __launch_bounds__(256) enc_norm_kernel(RowMap m, const uint4* E, const uint4* P, float* X, uint4* A,
                                                       const float* gamma, const float* beta, int n_units) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= m.row0[n_units]) return;
  const int n_chunks = m.d / 8;
  float* xr = X + (size_t)r * m.d;
  uint4* ar = A + (size_t)r * n_chunks;
  float x[E_KCH][8];
  if (GATHER) {
    const int rs = m.row_slot[r];
    const int i = rs & 7;
    const int bu = rs >> 3;
    const int b = bu / m.un, u = bu % m.un;
    int C;
    const int e = entry_of(m, b, u, &C);
    const int tok = min(max(m.ent_tokens[((size_t)b * m.cap + e) * m.M + i], 0), m.V - 1);
    const uint4* er = E + (size_t)tok * n_chunks;
#pragma unroll
    for (int k = 0; k < E_KCH; ++k) {
      const int c = lane + 64 * k;
      if (c < n_chunks) {
        float ev[8];
        unpack8(er[c], ev);
        if (P) {
          float pv[8];
          unpack8(P[(size_t)i * n_chunks + c], pv);
#pragma unroll
          for (int t = 0; t < 8; ++t) ev[t] += pv[t];
        }
        store8(xr + c * 8, ev);
#pragma unroll
        for (int t = 0; t < 8; ++t) x[k][t] = ev[t];
      }
    }
  } else {
#pragma unroll
    for (int k = 0; k < E_KCH; ++k) {
      const int c = lane + 64 * k;
      if (c < n_chunks) load8(xr + c * 8, x[k]);
    }
  }
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < E_KCH; ++k)
    if (lane + 64 * k < n_chunks) {
#pragma unroll
      for (int t = 0; t < 8; ++t) sum += x[k][t];
    }
  const float mean = wave_sum(sum) / (float)m.d;
  float sq = 0.f;
#pragma unroll
  for (int k = 0; k < E_KCH; ++k)
    if (lane + 64 * k < n_chunks) {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float dv = x[k][t] - mean;
        sq += dv * dv;
      }
    }
  const float rstd = rsqrtf(wave_sum(sq) / (float)m.d + E_EPS);
#pragma unroll
  for (int k = 0; k < E_KCH; ++k) {
    const int c = lane + 64 * k;
    if (c < n_chunks) {
      const float4 g0 = *reinterpret_cast<const float4*>(gamma + c * 8), g1 = *reinterpret_cast<const float4*>(gamma + c * 8 + 4);
      const float4 b0 = *reinterpret_cast<const float4*>(beta + c * 8), b1 = *reinterpret_cast<const float4*>(beta + c * 8 + 4);
      const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      const float bt[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
      float y[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) y[t] = (x[k][t] - mean) * rstd * g[t] + bt[t];
      ar[c] = pack8(y);
    }
  }
}

// Attention among the slots of one entry.  QKV [rows, 3d] holds q | k | v of every real slot; a wave takes
// one entry and 512 consecutive features (whole heads: the head width is a power of two of at most 512), lane
// l the 8 features of chunk l.  Scores are reduced over the lanes_per_head lanes of a head; the softmax runs
// over the entry's L rows.
__global__ void __launch_bounds__(256) enc_attention_kernel(RowMap m, const uint4* QKV, uint4* O, int lanes_per_head,
                                                            float scale, int groups, int n_units) {
  const int lane = threadIdx.x & 63;
  const long long wid = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int g = (int)(wid % groups);
  const long long bu = wid / groups;
  if (bu >= n_units) return;
  const int n_chunks = m.d / 8;
  const int c = g * 64 + lane;
  const bool active = c < n_chunks;
  const size_t r0 = (size_t)m.row0[bu];
  const int L = m.row0[bu + 1] - m.row0[bu];
  const uint4 zero = {0u, 0u, 0u, 0u};
  for (int i = 0; i < L; ++i) {
    float q[8];
    unpack8(active ? QKV[(r0 + i) * 3 * n_chunks + c] : zero, q);
    float s[Z2Z_MAX_M];
    float smax = -INFINITY;
#pragma unroll
    for (int j = 0; j < Z2Z_MAX_M; ++j) {
      s[j] = -INFINITY;
      if (j < L) {
        float k[8];
        unpack8(active ? QKV[(r0 + j) * 3 * n_chunks + n_chunks + c] : zero, k);
        float dot = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) dot += q[t] * k[t];
        for (int off = 1; off < lanes_per_head; off <<= 1) dot += __shfl_xor(dot, off);
        s[j] = dot * scale;
        smax = fmaxf(smax, s[j]);
      }
    }
    float den = 0.f;
#pragma unroll
    for (int j = 0; j < Z2Z_MAX_M; ++j) {
      s[j] = j < L ? __expf(s[j] - smax) : 0.f;
      den += s[j];
    }
    const float inv = 1.0f / den;
    float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < Z2Z_MAX_M; ++j) {
      if (j < L) {
        float v[8];
        unpack8(active ? QKV[(r0 + j) * 3 * n_chunks + 2 * n_chunks + c] : zero, v);
        const float p = s[j] * inv;
#pragma unroll
        for (int t = 0; t < 8; ++t) o[t] += p * v[t];
      }
    }
    if (active) O[(r0 + i) * n_chunks + c] = pack8(o);
  }
}

// h = mean of the entry's real slots of Z -> W_hyper[b, e]; one wave per entry.  Passes that start at entry 0
// (full mode) also zero the rows of missing entries.
__global__ void __launch_bounds__(256) enc_pool_kernel(RowMap m, const float* Z, uint4* W, int n_units, int zero_missing) {
  const int lane = threadIdx.x & 63;
  const long long bu = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (bu >= n_units) return;
  const int b = (int)(bu / m.un), u = (int)(bu % m.un);
  const int n_chunks = m.d / 8;
  int C;
  const int e = entry_of(m, b, u, &C);
  if (e >= m.cap) return;
  uint4* wrow = W + ((size_t)b * m.cap + e) * n_chunks;
  if (e >= C) {
    if (zero_missing) {
      const uint4 z = {0u, 0u, 0u, 0u};
      for (int c = lane; c < n_chunks; c += 64) wrow[c] = z;
    }
    return;
  }
  const int L = m.row0[bu + 1] - m.row0[bu];
  const float invL = 1.0f / (float)L;
  const size_t r0 = (size_t)m.row0[bu];
  for (int c = lane; c < n_chunks; c += 64) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < L; ++i) {
      float z[8];
      load8(Z + (r0 + i) * m.d + c * 8, z);
#pragma unroll
      for (int t = 0; t < 8; ++t) acc[t] += z[t];
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] *= invL;
    wrow[c] = pack8(acc);
  }
}

// ---------------------------------------------------------------------------------------------------------
// Backward pass (training f_phi: the loss reaches the encoder through every hypertoken vector, section 2.4).
// Reverse mode over the forward steps above.  Every product with a weight matrix, and every weight gradient
// (a product over the rows of the pass), runs on the same MFMA kernels from transposed bf16 copies; the kernels
// below are the bandwidth-bound rest.  Gradients between kernels are bf16, sums fp32.
// ---------------------------------------------------------------------------------------------------------

__global__ void __launch_bounds__(256) enc_fill_kernel(float* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}

// dX[r] = dW_hyper[b, e] / L for the L rows of every entry (h = mean of the real slots); one wave per entry.
__global__ void __launch_bounds__(256) enc_pool_backward_kernel(RowMap m, const uint4* dW, uint4* dX, int n_units) {
  const int lane = threadIdx.x & 63;
  const long long bu = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (bu >= n_units) return;
  const int L = m.row0[bu + 1] - m.row0[bu];
  if (L < 1) return;
  const int b = (int)(bu / m.un), u = (int)(bu % m.un);
  const int n_chunks = m.d / 8;
  int C;
  const int e = entry_of(m, b, u, &C);
  const uint4* wrow = dW + ((size_t)b * m.cap + e) * n_chunks;
  const float invL = 1.0f / (float)L;
  const size_t r0 = (size_t)m.row0[bu];
  for (int c = lane; c < n_chunks; c += 64) {
    float g[8];
    unpack8(wrow[c], g);
#pragma unroll
    for (int t = 0; t < 8; ++t) g[t] *= invL;
    const uint4 o = pack8(g);
    for (int i = 0; i < L; ++i) dX[(r0 + i) * n_chunks + c] = o;
  }
}

// (Float sums that several workgroups add to go through the hardware's float atomic add: every target here is
// ordinary device memory.)
// out[n] += sum over the pass's rows of G[r, n] (bias gradients).  A thread owns 8 columns and the rows
// stripe + E_CS_STRIPES * (lane group + 4 i); grid (ceil(N / 512), E_CS_STRIPES): few adds per address.
constexpr int E_CS_STRIPES = 32;
__global__ void __launch_bounds__(256) enc_colsum_kernel(const uint4* G, int n_chunks, const int32_t* rows_dev,
                                                         float* out) {
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rows = *rows_dev;
  if (c >= n_chunks) return;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const uint4 zero = {0u, 0u, 0u, 0u};
  const int step = 4 * E_CS_STRIPES;
  for (int r = blockIdx.y + E_CS_STRIPES * (threadIdx.x >> 6); r < rows; r += 4 * step) {   // four loads in flight
    const uint4 q0 = G[(size_t)r * n_chunks + c];
    const uint4 q1 = r + step < rows ? G[(size_t)(r + step) * n_chunks + c] : zero;
    const uint4 q2 = r + 2 * step < rows ? G[(size_t)(r + 2 * step) * n_chunks + c] : zero;
    const uint4 q3 = r + 3 * step < rows ? G[(size_t)(r + 3 * step) * n_chunks + c] : zero;
    float g[8];
    unpack8(q0, g);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] += g[t];
    unpack8(q1, g);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] += g[t];
    unpack8(q2, g);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] += g[t];
    unpack8(q3, g);
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] += g[t];
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) unsafeAtomicAdd(out + (size_t)c * 8 + t, acc[t]);
}

__device__ __forceinline__ float gelu_exact(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_slope(float x) {
  return 0.5f * (1.0f + erff(x * 0.70710678118654752f)) + x * 0.3989422804014327f * __expf(-0.5f * x * x);
}

// F = GELU(U) over the pass's rows (the training pass keeps U for the slope).
__global__ void __launch_bounds__(256) enc_gelu_kernel(const uint4* U, uint4* F, int n_chunks, const int32_t* rows_dev) {
  const size_t n = (size_t)*rows_dev * n_chunks;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    float u[8];
    unpack8(U[i], u);
#pragma unroll
    for (int t = 0; t < 8; ++t) u[t] = gelu_exact(u[t]);
    F[i] = pack8(u);
  }
}

// dU = dF * GELU'(U), in place over dF.
__global__ void __launch_bounds__(256) enc_gelu_backward_kernel(uint4* dF, const uint4* U, int n_chunks,
                                                                const int32_t* rows_dev) {
  const size_t n = (size_t)*rows_dev * n_chunks;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    float u[8], g[8];
    unpack8(U[i], u);
    unpack8(dF[i], g);
#pragma unroll
    for (int t = 0; t < 8; ++t) g[t] *= gelu_slope(u[t]);
    dF[i] = pack8(g);
  }
}

// LayerNorm backward: N = (x - mean) * rstd * gamma + beta.  out[r] = dres[r] + dx[r] with
//   g = dN * gamma;  dx = rstd * (g - mean(g) - xh * mean(g * xh)),  xh = (x - mean) * rstd.
// One wave per row as in the forward kernel: the row of X stays in registers, dN is streamed twice (the second
// time from cache).  The row's mean and rstd are left in stats[r] for the parameter gradients.
__global__ void __launch_bounds__(256) enc_norm_backward_kernel(const int32_t* rows_dev, int d, const uint4* dN,
                                                                const float* X, const float* gamma, const uint4* dres,
                                                                uint4* out, float2* stats) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= *rows_dev) return;
  const int n_chunks = d / 8;
  const float inv_d = 1.0f / (float)d;
  float x[E_KCH][8];
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < E_KCH; ++k) {
    const int c = lane + 64 * k;
    if (c < n_chunks) {
      load8(X + (size_t)r * d + c * 8, x[k]);
#pragma unroll
      for (int t = 0; t < 8; ++t) sum += x[k][t];
    }
  }
  const float mean = wave_sum(sum) * inv_d;
  float sq = 0.f;
#pragma unroll
  for (int k = 0; k < E_KCH; ++k)
    if (lane + 64 * k < n_chunks) {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float dv = x[k][t] - mean;
        sq += dv * dv;
      }
    }
  const float rstd = rsqrtf(wave_sum(sq) * inv_d + E_EPS);
  if (lane == 0) stats[r] = float2{mean, rstd};
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int k = 0; k < E_KCH; ++k) {
    const int c = lane + 64 * k;
    if (c < n_chunks) {
      float g[8];
      unpack8(dN[(size_t)r * n_chunks + c], g);
      const float4 g0 = *reinterpret_cast<const float4*>(gamma + c * 8), g1 = *reinterpret_cast<const float4*>(gamma + c * 8 + 4);
      const float gm[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float xh = (x[k][t] - mean) * rstd;
        x[k][t] = xh;
        s1 += g[t] * gm[t];
        s2 += g[t] * gm[t] * xh;
      }
    }
  }
  const float m1 = wave_sum(s1) * inv_d, m2 = wave_sum(s2) * inv_d;
#pragma unroll
  for (int k = 0; k < E_KCH; ++k) {
    const int c = lane + 64 * k;
    if (c < n_chunks) {
      float g[8], o[8];
      unpack8(dN[(size_t)r * n_chunks + c], g);
      unpack8(dres[(size_t)r * n_chunks + c], o);
      const float4 g0 = *reinterpret_cast<const float4*>(gamma + c * 8), g1 = *reinterpret_cast<const float4*>(gamma + c * 8 + 4);
      const float gm[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
      for (int t = 0; t < 8; ++t) o[t] += rstd * (g[t] * gm[t] - m1 - x[k][t] * m2);
      out[(size_t)r * n_chunks + c] = pack8(o);
    }
  }
}

// dgamma[n] += sum_r dN[r, n] * xh[r, n],  dbeta[n] += sum_r dN[r, n],  xh = (X - mean[r]) * rstd[r]: column sums
// in the shape of enc_colsum_kernel (a thread owns 8 columns and a strided set of rows).
__global__ void __launch_bounds__(256) enc_norm_param_grad_kernel(const uint4* dN, const float* X, const float2* stats,
                                                                  int n_chunks, const int32_t* rows_dev, float* dgamma,
                                                                  float* dbeta) {
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rows = *rows_dev;
  if (c >= n_chunks) return;
  float ag[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, ab[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int step = 4 * E_CS_STRIPES;
  for (int r = blockIdx.y + E_CS_STRIPES * (threadIdx.x >> 6); r < rows; r += 2 * step) {   // two rows in flight
    const bool two = r + step < rows;
    const int r2 = two ? r + step : r;
    const uint4 qg0 = dN[(size_t)r * n_chunks + c], qg1 = dN[(size_t)r2 * n_chunks + c];
    float g[8], x[8], x1[8];
    load8(X + ((size_t)r * n_chunks + c) * 8, x);
    load8(X + ((size_t)r2 * n_chunks + c) * 8, x1);
    const float2 st0 = stats[r], st1 = stats[r2];
    unpack8(qg0, g);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      ag[t] += g[t] * ((x[t] - st0.x) * st0.y);
      ab[t] += g[t];
    }
    if (two) {
      unpack8(qg1, g);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        ag[t] += g[t] * ((x1[t] - st1.x) * st1.y);
        ab[t] += g[t];
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    unsafeAtomicAdd(dgamma + (size_t)c * 8 + t, ag[t]);
    unsafeAtomicAdd(dbeta + (size_t)c * 8 + t, ab[t]);
  }
}

// Attention backward for one entry and 512 features (same split as the forward kernel).  Per query row i the
// probabilities p[i][.] are formed again from q and k; with dP[i][j] = dO_i . v_j and
// dS[i][j] = p[i][j] (dP[i][j] - sum_j' dP[i][j'] p[i][j']):  dq_i = scale * sum_j dS[i][j] k_j;
// dk_j += scale * dS[i][j] q_i;  dv_j += p[i][j] dO_i.  dQKV has the layout of QKV.
template <int MM>          // slots per entry the registers are sized for: 4 (the usual M = 3) or Z2Z_MAX_M
__global__ void __launch_bounds__(256) enc_attention_backward_kernel(RowMap m, const uint4* QKV, const uint4* dO,
                                                                     uint4* dQKV, int lanes_per_head, float scale,
                                                                     int groups, int n_units) {
  const int lane = threadIdx.x & 63;
  const long long wid = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int g = (int)(wid % groups);
  const long long bu = wid / groups;
  if (bu >= n_units) return;
  const int n_chunks = m.d / 8;
  const int c = g * 64 + lane;
  const bool active = c < n_chunks;
  const size_t r0 = (size_t)m.row0[bu];
  const int L = m.row0[bu + 1] - m.row0[bu];
  const uint4 zero = {0u, 0u, 0u, 0u};
  float dk[MM][8], dv[MM][8];
#pragma unroll
  for (int j = 0; j < MM; ++j)
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      dk[j][t] = 0.f;
      dv[j][t] = 0.f;
    }
  for (int i = 0; i < L; ++i) {
    float q[8], go[8];
    unpack8(active ? QKV[(r0 + i) * 3 * n_chunks + c] : zero, q);
    unpack8(active ? dO[(r0 + i) * n_chunks + c] : zero, go);
    float s[MM], dp[MM];
    float smax = -INFINITY;
#pragma unroll
    for (int j = 0; j < MM; ++j) {
      s[j] = -INFINITY;
      dp[j] = 0.f;
      if (j < L) {
        float k[8], v[8];
        unpack8(active ? QKV[(r0 + j) * 3 * n_chunks + n_chunks + c] : zero, k);
        unpack8(active ? QKV[(r0 + j) * 3 * n_chunks + 2 * n_chunks + c] : zero, v);
        float dot = 0.f, dot2 = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          dot += q[t] * k[t];
          dot2 += go[t] * v[t];
        }
        for (int off = 1; off < lanes_per_head; off <<= 1) {
          dot += __shfl_xor(dot, off);
          dot2 += __shfl_xor(dot2, off);
        }
        s[j] = dot * scale;
        dp[j] = dot2;
        smax = fmaxf(smax, s[j]);
      }
    }
    float den = 0.f;
#pragma unroll
    for (int j = 0; j < MM; ++j) {
      s[j] = j < L ? __expf(s[j] - smax) : 0.f;
      den += s[j];
    }
    const float inv = 1.0f / den;
    float dot_pp = 0.f;
#pragma unroll
    for (int j = 0; j < MM; ++j) {
      s[j] *= inv;                                   // p[i][j]
      dot_pp += s[j] * dp[j];
    }
    float dq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < MM; ++j) {
      if (j < L) {
        const float ds = s[j] * (dp[j] - dot_pp) * scale;
        float k[8];
        unpack8(active ? QKV[(r0 + j) * 3 * n_chunks + n_chunks + c] : zero, k);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          dq[t] += ds * k[t];
          dk[j][t] += ds * q[t];
          dv[j][t] += s[j] * go[t];
        }
      }
    }
    if (active) dQKV[(r0 + i) * 3 * n_chunks + c] = pack8(dq);
  }
#pragma unroll
  for (int j = 0; j < MM; ++j) {
    if (j < L && active) {
      dQKV[(r0 + j) * 3 * n_chunks + n_chunks + c] = pack8(dk[j]);
      dQKV[(r0 + j) * 3 * n_chunks + 2 * n_chunks + c] = pack8(dv[j]);
    }
  }
}

// The gradient at the encoder's input: dE[token of row r] += dX[r] (float atomics: tokens recur), and
// dP[slot of row r] += dX[r], the latter summed per slot over a stripe of 256 rows in registers first.
// Grid (ceil(d / 512), ceil(max rows / 256)); a thread owns features f0 + lane + 64 t (t < 8) of a block of 512,
// so that the 64 lanes of one atomic instruction cover 256 consecutive bytes, and every fourth row of the stripe.
__global__ void __launch_bounds__(256) enc_input_backward_kernel(RowMap m, const uint16_t* dX, float* dE, float* dP,
                                                                 int n_units) {
  const int f0 = blockIdx.x * 512 + (threadIdx.x & 63);
  const int rows = m.row0[n_units];
  const int r_begin = blockIdx.y * 256 + (threadIdx.x >> 6), r_end = min(rows, (int)(blockIdx.y + 1) * 256);
  if (r_begin >= r_end) return;
  float acc[Z2Z_MAX_M][8];
#pragma unroll
  for (int j = 0; j < Z2Z_MAX_M; ++j)
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[j][t] = 0.f;
  for (int r = r_begin; r < r_end; r += 4) {
    const int rs = m.row_slot[r];
    const int i = rs & 7;
    const int bu = rs >> 3;
    const int b = bu / m.un, u = bu % m.un;
    int C;
    const int e = entry_of(m, b, u, &C);
    const int tok = min(max(m.ent_tokens[((size_t)b * m.cap + e) * m.M + i], 0), m.V - 1);
    float g[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int f = f0 + 64 * t;
      g[t] = f < m.d ? __uint_as_float((uint32_t)dX[(size_t)r * m.d + f] << 16) : 0.f;
    }
    float* er = dE + (size_t)tok * m.d;
#pragma unroll
    for (int t = 0; t < 8; ++t)
      if (f0 + 64 * t < m.d) unsafeAtomicAdd(er + f0 + 64 * t, g[t]);
#pragma unroll
    for (int j = 0; j < Z2Z_MAX_M; ++j)
#pragma unroll
      for (int t = 0; t < 8; ++t) acc[j][t] += (i == j) ? g[t] : 0.f;
  }
  if (dP) {
#pragma unroll
    for (int j = 0; j < Z2Z_MAX_M; ++j)
      if (j < m.M) {
#pragma unroll
        for (int t = 0; t < 8; ++t)
          if (f0 + 64 * t < m.d) unsafeAtomicAdd(dP + (size_t)j * m.d + f0 + 64 * t, acc[j][t]);
      }
  }
}

__global__ void __launch_bounds__(256) enc_to_bf16_kernel(const float* in, uint16_t* out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    out[i] = (uint16_t)bf16_bits_rne(in[i]);
}

}  // namespace

bool z2z_hyper_encode_ok(const z2z_ctx* c, const z2z_encoder* enc) {
  const int d = c->cfg.d;
  if (c->cfg.dtype != Z2Z_BF16 || !c->fast_ready || d % 64 != 0 || d > 64 * 8 * E_KCH) return false;
  if (enc->n_heads < 1 || d % enc->n_heads != 0) return false;
  const int dh = d / enc->n_heads;
  if (dh < 8 || dh > 512 || (dh & (dh - 1)) != 0) return false;
  if (!enc->attention_only && (enc->d_ff < 64 || enc->d_ff % 64 != 0)) return false;
  return true;
}

int z2z_launch_hyper_encode(z2z_ctx* c, const void* E, const z2z_encoder* enc, void* W_hyper, const int32_t* first,
                            int32_t max_new, hipStream_t s) {
  const int B = c->cfg.B, M = c->cfg.M, cap = c->cfg.cap, d = c->cfg.d;
  if (cap == 0) return Z2Z_OK;
  const bool incremental = first || max_new > 0;
  const int units = incremental ? (max_new < 1 ? cap : (max_new < cap ? max_new : cap)) : cap;
  const int dff = enc->attention_only ? 0 : enc->d_ff;
  // rows per pass: all sequences, u_step entries each, M slots per entry
  long long u_step = 65536 / ((long long)B * M);
  if (u_step < 1) u_step = 1;
  if (u_step > units) u_step = units;
  const size_t R_max = (size_t)B * (size_t)u_step * M;
  const size_t n_units_max = (size_t)B * (size_t)u_step;
  const size_t index_bytes = ((n_units_max + 1 + R_max) * sizeof(int32_t) + 255) & ~(size_t)255;
  // per row: the stream X and Y in fp32 (2 x 4 bytes x d), A, O (d), QKV (3d) and F (d_ff) in bf16
  const size_t need = R_max * ((size_t)8 * d + ((size_t)2 * d + (size_t)3 * d + (size_t)dff) * 2) + index_bytes;
  if (need > c->enc_ws_bytes) {
    Z2Z_TRY_GROW(s);
    if (c->enc_ws) (void)hipFree(c->enc_ws);
    c->enc_ws = nullptr;
    c->enc_ws_bytes = 0;
    if (hipMalloc(&c->enc_ws, need) != hipSuccess) return Z2Z_ENOMEM;
    c->enc_ws_bytes = need;
  }
  int32_t* index = reinterpret_cast<int32_t*>(c->enc_ws);
  float* X = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(c->enc_ws) + index_bytes);
  float* Y = X + R_max * d;
  uint16_t* A = reinterpret_cast<uint16_t*>(Y + R_max * d);
  uint16_t* O = A + R_max * d;
  uint16_t* QKV = O + R_max * d;
  uint16_t* F = QKV + R_max * 3 * d;

  RowMap m;
  m.size = c->st.size;
  m.ent_tokens = c->st.ent_tokens;
  m.ent_len = c->st.ent_len;
  m.first = first;
  m.last_n = (!first && max_new > 0) ? max_new : 0;
  m.B = B;
  m.V = c->cfg.V;
  m.M = M;
  m.cap = cap;
  m.d = d;
  m.row0 = index;
  m.row_slot = index + n_units_max + 1;
  const int dh = d / enc->n_heads;
  const int groups = (d + 511) / 512;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int u0 = 0; u0 < units; u0 += (int)u_step) {
    m.u0 = u0;
    m.un = (int)(u0 + u_step <= units ? u_step : units - u0);
    const int n_units = B * m.un;
    const int R = n_units * M;                      // upper bound; the pass's row count is row0[n_units], on the device
    const int32_t* rows_dev = m.row0 + n_units;
    const unsigned row_blocks = (unsigned)((R + 3) / 4);
    hipLaunchKernelGGL(enc_rows_kernel, dim3(1), dim3(1024), 0, s, m, n_units);
    float* x = X;
    float* y = Y;
    for (int l = 0; l < enc->n_layers; ++l) {
      const z2z_encoder_layer& lay = enc->layers[l];
      if (l == 0)
        hipLaunchKernelGGL(enc_norm_kernel<true>, dim3(row_blocks), dim3(256), 0, s, m,
                           reinterpret_cast<const uint4*>(E), reinterpret_cast<const uint4*>(enc->pos), x,
                           reinterpret_cast<uint4*>(A), lay.ln1_g, lay.ln1_b, n_units);
      else
        hipLaunchKernelGGL(enc_norm_kernel<false>, dim3(row_blocks), dim3(256), 0, s, m, nullptr, nullptr, x,
                           reinterpret_cast<uint4*>(A), lay.ln1_g, lay.ln1_b, n_units);
      int rc = z2z_launch_linear(c, A, lay.w_qkv, lay.b_qkv, nullptr, 0, QKV, R, rows_dev, 3 * d, d, s);
      if (rc != Z2Z_OK) return rc;
      const long long att_waves = (long long)n_units * groups;
      hipLaunchKernelGGL(enc_attention_kernel, dim3((unsigned)((att_waves + 3) / 4)), dim3(256), 0, s, m,
                         reinterpret_cast<const uint4*>(QKV), reinterpret_cast<uint4*>(O), dh / 8, scale, groups,
                         n_units);
      rc = z2z_launch_linear(c, O, lay.w_o, lay.b_o, x, 0, y, R, rows_dev, d, d, s, nullptr, true);
      if (rc != Z2Z_OK) return rc;
      if (enc->attention_only) {
        float* t = x;
        x = y;
        y = t;
      } else {
        hipLaunchKernelGGL(enc_norm_kernel<false>, dim3(row_blocks), dim3(256), 0, s, m, nullptr, nullptr, y,
                           reinterpret_cast<uint4*>(A), lay.ln2_g, lay.ln2_b, n_units);
        rc = z2z_launch_linear(c, A, lay.w_1, lay.b_1, nullptr, 1, F, R, rows_dev, dff, d, s);
        if (rc != Z2Z_OK) return rc;
        rc = z2z_launch_linear(c, F, lay.w_2, lay.b_2, y, 0, x, R, rows_dev, d, dff, s, nullptr, true);
        if (rc != Z2Z_OK) return rc;
      }
    }
    hipLaunchKernelGGL(enc_pool_kernel, dim3((unsigned)((n_units + 3) / 4)), dim3(256), 0, s, m, x,
                       reinterpret_cast<uint4*>(W_hyper), n_units, incremental ? 0 : 1);
  }
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

namespace {

struct LayerSave {                   // what the training pass keeps of one layer: the stream (Xin, Y) [rows, d] fp32,
  float *Xin, *Y;                    // the operands of the matrix products [rows, .] bf16
  uint16_t *A, *QKV, *O, *N2, *U, *F;
};

int transpose_to(const void* in, void* out, int R, const int32_t* rows_dev, int C, int ld_in, int ld_out, hipStream_t s) {
  return z2z_launch_transpose(in, out, R, rows_dev, C, ld_in, ld_out, 1, 0, 0, s);
}

void colsum_to(const void* G, int N, int R, const int32_t* rows_dev, float* out, hipStream_t s) {
  (void)R;
  hipLaunchKernelGGL(enc_colsum_kernel, dim3((N / 8 + 63) / 64, E_CS_STRIPES), dim3(256), 0, s,
                     reinterpret_cast<const uint4*>(G), N / 8, rows_dev, out);
}

unsigned flat_grid(size_t n) {
  const size_t blocks = (n + 255) / 256;
  return (unsigned)(blocks < 1 ? 1 : (blocks > 65536 ? 65536 : blocks));
}

}  // namespace

// mode 0: forward (rows kept) + backward, pass by pass; mode 1: the forward alone, W_hyper written and the rows
// left in the work space; mode 2: the backward alone on the rows mode 1 left.  Modes 1 and 2 need all slot rows
// in one pass.
int z2z_launch_hyper_encode_train(z2z_ctx* c, int mode, const void* E, const z2z_encoder* enc, void* W_hyper,
                                  const void* dW_hyper, const z2z_encoder* grad, float* dE, hipStream_t s) {
  const int B = c->cfg.B, M = c->cfg.M, cap = c->cfg.cap, d = c->cfg.d;
  if (cap == 0) return Z2Z_OK;
  if (mode != 0 && (long long)B * cap * M > 65536) return Z2Z_EUNSUPPORTED;
  const int nl = enc->n_layers;
  const bool ffn = !enc->attention_only;
  const int dff = ffn ? enc->d_ff : 0;
  const int wide = 3 * d > dff ? 3 * d : dff;                   // widest activation
  long long u_step = 65536 / ((long long)B * M);
  if (u_step < 1) u_step = 1;
  if (u_step > cap) u_step = cap;
  const size_t R_max = (size_t)B * (size_t)u_step * M;
  const size_t Rp = (R_max + 127) / 128 * 128;                  // contraction length of the weight-gradient products
  const size_t n_units_max = (size_t)B * (size_t)u_step;
  const size_t index_bytes = ((n_units_max + 1 + R_max) * sizeof(int32_t) + 255) & ~(size_t)255;
  const size_t pos_bytes = ((size_t)Z2Z_MAX_M * d * sizeof(float) + 255) & ~(size_t)255;
  // in units of bf16 elements (an fp32 element counts as two): per layer what LayerSave names (Xin and Y fp32);
  // the last layer's output (fp32); the running gradients dX dY dN dO (d each), dQKV (3d), dF (d_ff); two
  // transposed operands [wide, Rp]; one transposed weight
  const size_t per_layer = R_max * ((size_t)10 * d + (size_t)2 * dff);
  const size_t elems = (size_t)nl * per_layer + R_max * ((size_t)7 * d + dff) + R_max * 2 * d + 2 * (size_t)wide * Rp +
                       (size_t)wide * d;
  const size_t nb_bytes = (R_max * sizeof(float2) + 255) & ~(size_t)255;   // mean and rstd of every row of a LayerNorm
  const size_t need = index_bytes + pos_bytes + nb_bytes + elems * 2;
  if (need > ((size_t)200 << 30)) return Z2Z_ENOMEM;
  // the rows a mode-1 call left are those of this encoder's shape only if the layout is the same
  if (mode == 2 && (!c->enc_kept || c->enc_kept_need != need || c->enc_kept_E != E)) return Z2Z_EINVAL;
  c->enc_kept = false;
  if (need > c->enc_bwd_ws_bytes) {
    Z2Z_TRY_GROW(s);
    if (c->enc_bwd_ws) (void)hipFree(c->enc_bwd_ws);
    c->enc_bwd_ws = nullptr;
    c->enc_bwd_ws_bytes = 0;
    if (hipMalloc(&c->enc_bwd_ws, need) != hipSuccess) return Z2Z_ENOMEM;
    c->enc_bwd_ws_bytes = need;
  }
  unsigned char* base = reinterpret_cast<unsigned char*>(c->enc_bwd_ws);
  int32_t* index = reinterpret_cast<int32_t*>(base);
  float* dP = reinterpret_cast<float*>(base + index_bytes);
  float2* ln_stats = reinterpret_cast<float2*>(base + index_bytes + pos_bytes);
  uint16_t* p = reinterpret_cast<uint16_t*>(base + index_bytes + pos_bytes + nb_bytes);
  auto take = [&](size_t n) {
    uint16_t* r = p;
    p += n;
    return r;
  };
  auto take_f32 = [&](size_t n) { return reinterpret_cast<float*>(take(2 * n)); };   // (every size is a multiple of 64 elements)
  LayerSave sv[Z2Z_MAX_ENCODER_LAYERS];
  for (int l = 0; l < nl; ++l) {
    sv[l].Xin = take_f32(R_max * d);
    sv[l].Y = take_f32(R_max * d);
    sv[l].A = take(R_max * d);
    sv[l].QKV = take(R_max * 3 * d);
    sv[l].O = take(R_max * d);
    sv[l].N2 = take(R_max * d);
    sv[l].U = take(R_max * (size_t)dff);
    sv[l].F = take(R_max * (size_t)dff);
  }
  float* Xout = take_f32(R_max * d);
  uint16_t* dX = take(R_max * d);
  uint16_t* dY = take(R_max * d);
  uint16_t* dN = take(R_max * d);
  uint16_t* dO = take(R_max * d);
  uint16_t* dQKV = take(R_max * 3 * d);
  uint16_t* dF = take(R_max * (size_t)dff);
  uint16_t* TA = take((size_t)wide * Rp);
  uint16_t* TB = take((size_t)wide * Rp);
  uint16_t* WT = take((size_t)wide * d);

  RowMap m;
  m.size = c->st.size;
  m.ent_tokens = c->st.ent_tokens;
  m.ent_len = c->st.ent_len;
  m.first = nullptr;
  m.last_n = 0;
  m.B = B;
  m.V = c->cfg.V;
  m.M = M;
  m.cap = cap;
  m.d = d;
  m.row0 = index;
  m.row_slot = index + n_units_max + 1;
  const int dh = d / enc->n_heads;
  const int groups = (d + 511) / 512;
  const float scale = 1.0f / sqrtf((float)dh);

  // vector gradients are sums over all passes: cleared once, added to by every pass
  auto clear = [&](const float* q, size_t n) {
    hipLaunchKernelGGL(enc_fill_kernel, dim3(flat_grid(n)), dim3(256), 0, s, const_cast<float*>(q), n);
  };
  for (int l = 0; l < nl && mode != 1; ++l) {
    const z2z_encoder_layer& g = grad->layers[l];
    clear(g.ln1_g, d);
    clear(g.ln1_b, d);
    clear(g.b_qkv, (size_t)3 * d);
    clear(g.b_o, d);
    if (ffn) {
      clear(g.ln2_g, d);
      clear(g.ln2_b, d);
      clear(g.b_1, dff);
      clear(g.b_2, d);
    }
  }
  if (mode != 1) clear(dP, (size_t)Z2Z_MAX_M * d);

  int rc;
#define Z2Z_TRY_RC(expr)      \
  do {                        \
    rc = (expr);              \
    if (rc != Z2Z_OK) return rc; \
  } while (0)

  int pass = 0;
  for (int u0 = 0; u0 < cap; u0 += (int)u_step, ++pass) {
    m.u0 = u0;
    m.un = (int)(u0 + u_step <= cap ? u_step : cap - u0);
    const int n_units = B * m.un;
    const int R = n_units * M;                       // upper bound; the real count is on the device
    const int Rk = (R + 127) / 128 * 128;            // contraction length of this pass's weight-gradient products
    const int32_t* rows_dev = m.row0 + n_units;
    const unsigned row_blocks = (unsigned)((R + 3) / 4);
    if (mode != 2) hipLaunchKernelGGL(enc_rows_kernel, dim3(1), dim3(1024), 0, s, m, n_units);

    // ---- forward, keeping every layer's intermediate rows ----
    for (int l = 0; l < nl && mode != 2; ++l) {
      const z2z_encoder_layer& lay = enc->layers[l];
      const LayerSave& v = sv[l];
      float* next = l + 1 < nl ? sv[l + 1].Xin : Xout;
      if (l == 0)
        hipLaunchKernelGGL(enc_norm_kernel<true>, dim3(row_blocks), dim3(256), 0, s, m,
                           reinterpret_cast<const uint4*>(E), reinterpret_cast<const uint4*>(enc->pos), v.Xin,
                           reinterpret_cast<uint4*>(v.A), lay.ln1_g, lay.ln1_b, n_units);
      else
        hipLaunchKernelGGL(enc_norm_kernel<false>, dim3(row_blocks), dim3(256), 0, s, m, nullptr, nullptr, v.Xin,
                           reinterpret_cast<uint4*>(v.A), lay.ln1_g, lay.ln1_b, n_units);
      Z2Z_TRY_RC(z2z_launch_linear(c, v.A, lay.w_qkv, lay.b_qkv, nullptr, 0, v.QKV, R, rows_dev, 3 * d, d, s));
      const long long att_waves = (long long)n_units * groups;
      hipLaunchKernelGGL(enc_attention_kernel, dim3((unsigned)((att_waves + 3) / 4)), dim3(256), 0, s, m,
                         reinterpret_cast<const uint4*>(v.QKV), reinterpret_cast<uint4*>(v.O), dh / 8, scale, groups,
                         n_units);
      float* y = ffn ? v.Y : next;
      Z2Z_TRY_RC(z2z_launch_linear(c, v.O, lay.w_o, lay.b_o, v.Xin, 0, y, R, rows_dev, d, d, s, nullptr, true));
      if (ffn) {
        hipLaunchKernelGGL(enc_norm_kernel<false>, dim3(row_blocks), dim3(256), 0, s, m, nullptr, nullptr, v.Y,
                           reinterpret_cast<uint4*>(v.N2), lay.ln2_g, lay.ln2_b, n_units);
        Z2Z_TRY_RC(z2z_launch_linear(c, v.N2, lay.w_1, lay.b_1, nullptr, 0, v.U, R, rows_dev, dff, d, s));
        hipLaunchKernelGGL(enc_gelu_kernel, dim3(flat_grid((size_t)R * dff / 8)), dim3(256), 0, s,
                           reinterpret_cast<const uint4*>(v.U), reinterpret_cast<uint4*>(v.F), dff / 8, rows_dev);
        Z2Z_TRY_RC(z2z_launch_linear(c, v.F, lay.w_2, lay.b_2, v.Y, 0, next, R, rows_dev, d, dff, s, nullptr, true));
      }
    }

    if (mode == 1) {
      hipLaunchKernelGGL(enc_pool_kernel, dim3((unsigned)((n_units + 3) / 4)), dim3(256), 0, s, m, Xout,
                         reinterpret_cast<uint4*>(W_hyper), n_units, 1);
      continue;
    }

    // ---- backward ----
    hipLaunchKernelGGL(enc_pool_backward_kernel, dim3((unsigned)((n_units + 3) / 4)), dim3(256), 0, s, m,
                       reinterpret_cast<const uint4*>(dW_hyper), reinterpret_cast<uint4*>(dX), n_units);
    auto norm_backward = [&](const uint16_t* dn, const float* x, const float* gamma, const uint16_t* dres,
                             uint16_t* out, const float* dgamma, const float* dbeta) {
      hipLaunchKernelGGL(enc_norm_backward_kernel, dim3(row_blocks), dim3(256), 0, s, rows_dev, d,
                         reinterpret_cast<const uint4*>(dn), x, gamma,
                         reinterpret_cast<const uint4*>(dres), reinterpret_cast<uint4*>(out), ln_stats);
      hipLaunchKernelGGL(enc_norm_param_grad_kernel, dim3((d / 8 + 63) / 64, E_CS_STRIPES), dim3(256), 0, s,
                         reinterpret_cast<const uint4*>(dn), x, ln_stats, d / 8, rows_dev,
                         const_cast<float*>(dgamma), const_cast<float*>(dbeta));
    };
    for (int l = nl - 1; l >= 0; --l) {
      const z2z_encoder_layer& lay = enc->layers[l];
      const z2z_encoder_layer& g = grad->layers[l];
      const LayerSave& v = sv[l];
      const void* acc = nullptr;                     // weight gradients of later passes add to the earlier ones
      uint16_t* dy = dX;                             // gradient at Y (attention layers: the layer's output)
      if (ffn) {
        colsum_to(dX, d, R, rows_dev, const_cast<float*>(g.b_2), s);
        Z2Z_TRY_RC(transpose_to(lay.w_2, WT, d, nullptr, dff, dff, d, s));                        // [dff, d]
        Z2Z_TRY_RC(z2z_launch_linear(c, dX, WT, nullptr, nullptr, 0, dF, R, rows_dev, dff, d, s));
        Z2Z_TRY_RC(transpose_to(dX, TA, R, rows_dev, d, d, Rk, s));
        Z2Z_TRY_RC(transpose_to(v.F, TB, R, rows_dev, dff, dff, Rk, s));
        acc = pass > 0 ? g.w_2 : nullptr;
        Z2Z_TRY_RC(z2z_launch_linear(c, TA, TB, nullptr, acc, 0, const_cast<void*>(g.w_2), d, nullptr, dff, Rk, s, rows_dev));
        hipLaunchKernelGGL(enc_gelu_backward_kernel, dim3(flat_grid((size_t)R * dff / 8)), dim3(256), 0, s,
                           reinterpret_cast<uint4*>(dF), reinterpret_cast<const uint4*>(v.U), dff / 8, rows_dev);
        colsum_to(dF, dff, R, rows_dev, const_cast<float*>(g.b_1), s);
        Z2Z_TRY_RC(transpose_to(dF, TA, R, rows_dev, dff, dff, Rk, s));
        Z2Z_TRY_RC(transpose_to(v.N2, TB, R, rows_dev, d, d, Rk, s));
        acc = pass > 0 ? g.w_1 : nullptr;
        Z2Z_TRY_RC(z2z_launch_linear(c, TA, TB, nullptr, acc, 0, const_cast<void*>(g.w_1), dff, nullptr, d, Rk, s, rows_dev));
        Z2Z_TRY_RC(transpose_to(lay.w_1, WT, dff, nullptr, d, d, dff, s));                        // [d, dff]
        Z2Z_TRY_RC(z2z_launch_linear(c, dF, WT, nullptr, nullptr, 0, dN, R, rows_dev, d, dff, s));
        norm_backward(dN, v.Y, lay.ln2_g, dX, dY, g.ln2_g, g.ln2_b);
        dy = dY;
      }
      colsum_to(dy, d, R, rows_dev, const_cast<float*>(g.b_o), s);
      Z2Z_TRY_RC(transpose_to(lay.w_o, WT, d, nullptr, d, d, d, s));
      Z2Z_TRY_RC(z2z_launch_linear(c, dy, WT, nullptr, nullptr, 0, dO, R, rows_dev, d, d, s));
      Z2Z_TRY_RC(transpose_to(dy, TA, R, rows_dev, d, d, Rk, s));
      Z2Z_TRY_RC(transpose_to(v.O, TB, R, rows_dev, d, d, Rk, s));
      acc = pass > 0 ? g.w_o : nullptr;
      Z2Z_TRY_RC(z2z_launch_linear(c, TA, TB, nullptr, acc, 0, const_cast<void*>(g.w_o), d, nullptr, d, Rk, s, rows_dev));
      const long long att_waves = (long long)n_units * groups;
      if (M <= 4)
        hipLaunchKernelGGL(enc_attention_backward_kernel<4>, dim3((unsigned)((att_waves + 3) / 4)), dim3(256), 0, s, m,
                           reinterpret_cast<const uint4*>(v.QKV), reinterpret_cast<const uint4*>(dO),
                           reinterpret_cast<uint4*>(dQKV), dh / 8, scale, groups, n_units);
      else
        hipLaunchKernelGGL(enc_attention_backward_kernel<Z2Z_MAX_M>, dim3((unsigned)((att_waves + 3) / 4)), dim3(256), 0,
                           s, m, reinterpret_cast<const uint4*>(v.QKV), reinterpret_cast<const uint4*>(dO),
                           reinterpret_cast<uint4*>(dQKV), dh / 8, scale, groups, n_units);
      colsum_to(dQKV, 3 * d, R, rows_dev, const_cast<float*>(g.b_qkv), s);
      Z2Z_TRY_RC(transpose_to(dQKV, TA, R, rows_dev, 3 * d, 3 * d, Rk, s));
      Z2Z_TRY_RC(transpose_to(v.A, TB, R, rows_dev, d, d, Rk, s));
      acc = pass > 0 ? g.w_qkv : nullptr;
      Z2Z_TRY_RC(z2z_launch_linear(c, TA, TB, nullptr, acc, 0, const_cast<void*>(g.w_qkv), 3 * d, nullptr, d, Rk, s, rows_dev));
      Z2Z_TRY_RC(transpose_to(lay.w_qkv, WT, 3 * d, nullptr, d, d, 3 * d, s));                    // [d, 3d]
      Z2Z_TRY_RC(z2z_launch_linear(c, dQKV, WT, nullptr, nullptr, 0, dN, R, rows_dev, d, 3 * d, s));
      norm_backward(dN, v.Xin, lay.ln1_g, dy, dX, g.ln1_g, g.ln1_b);
    }
    hipLaunchKernelGGL(enc_input_backward_kernel, dim3((d + 511) / 512, (R + 255) / 256), dim3(256), 0, s, m, dX, dE,
                       enc->pos ? dP : nullptr, n_units);
  }
#undef Z2Z_TRY_RC
  if (mode == 1) {
    Z2Z_HIP_TRY(hipGetLastError());
    c->enc_kept = true;
    c->enc_kept_need = need;
    c->enc_kept_E = E;
    return Z2Z_OK;
  }
  if (enc->pos)
    hipLaunchKernelGGL(enc_to_bf16_kernel, dim3(flat_grid((size_t)M * d)), dim3(256), 0, s, dP,
                       reinterpret_cast<uint16_t*>(const_cast<void*>(grad->pos)), (size_t)M * d);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}
