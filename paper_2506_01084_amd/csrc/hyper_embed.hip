// hyper_embed for gfx950: one wavefront per codebook entry, coalesced 16-byte row gathers.
//
// Section 2.2 of the zip2zip paper builds a hypertoken's vector from the embeddings of its
// constituent base tokens, padded to M slots; this is the parameter-free pooling of the
// hyper-encoder ablation ("Averaging"): padding contributes nothing and the divisor is the entry's
// own length.  The work is a gather of L rows of E plus one row written: bound by HBM bandwidth
// (popular rows are served by L2 / the memory-side cache).  Each lane owns 16-byte column chunks:
// a wave reads 1 KiB of a row per instruction, accumulates in fp32 in token order, and rounds once
// (nearest-even) to the storage type.
#include "z2z_internal.h"

namespace {

struct EmbedArgs {
  const void* E;
  void* W;
  const int32_t* size;        // [B] C_b
  const int32_t* ent_tokens;  // [B, cap, M]
  const int32_t* ent_len;     // [B, cap]
  const int32_t* first;       // [B] or nullptr
  int32_t last_n;             // first == nullptr: 0 = all of [0, cap), n > 0 = the last n entries only
  int32_t B, V, M, cap, d;
  int32_t units_per_seq;      // entry walkers assigned to each sequence
  int32_t split;              // waves that share one entry's row (each takes every split-th group of 64 chunks)
  int32_t pool;
  float coef[Z2Z_MAX_M + 1][Z2Z_MAX_M];
};

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

template <bool BF16>
__device__ __forceinline__ void embed_row(const EmbedArgs& a, const int32_t* toks, int L, size_t out_row, int lane,
                                          int part) {
  // elements per 16-byte chunk: 8 (bf16) or 4 (f32)
  constexpr int EPC = BF16 ? 8 : 4;
  const int n_chunks = a.d / EPC;
  const uint4* E = reinterpret_cast<const uint4*>(a.E);
  uint4* W = reinterpret_cast<uint4*>(a.W) + out_row * (size_t)n_chunks;
  int32_t t[Z2Z_MAX_M];
  float cf[Z2Z_MAX_M];
#pragma unroll
  for (int j = 0; j < Z2Z_MAX_M; ++j) {
    t[j] = j < L ? min(max(toks[j], 0), a.V - 1) : 0;
    cf[j] = a.pool == Z2Z_POOL_MEAN ? 1.0f : a.coef[L][j];   // mean: plain sum, divided by L at the end
  }
  const bool mean = a.pool == Z2Z_POOL_MEAN;
  const float fL = (float)L;
  for (int c = part * 64 + lane; c < n_chunks; c += 64 * a.split) {
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int j = 0; j < Z2Z_MAX_M; ++j) {
      if (j < L) {
        const uint4 x = E[(size_t)t[j] * n_chunks + c];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
        if (BF16) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[2 * e] = fmaf(cf[j], bf16_to_f32(xs[e] & 0xFFFFu), acc[2 * e]);
            acc[2 * e + 1] = fmaf(cf[j], bf16_to_f32(xs[e] >> 16), acc[2 * e + 1]);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] = fmaf(cf[j], __uint_as_float(xs[e]), acc[e]);
        }
      }
    }
    uint4 o;
    if (BF16) {
      uint32_t r[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = f32_to_bf16_rne(mean ? acc[e] / fL : acc[e]);
      o.x = r[0] | (r[1] << 16);
      o.y = r[2] | (r[3] << 16);
      o.z = r[4] | (r[5] << 16);
      o.w = r[6] | (r[7] << 16);
    } else {
      float r[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = mean ? acc[e] / fL : acc[e];
      o.x = __float_as_uint(r[0]);
      o.y = __float_as_uint(r[1]);
      o.z = __float_as_uint(r[2]);
      o.w = __float_as_uint(r[3]);
    }
    W[c] = o;
  }
}

// grid.x = B * units_per_seq * split / 4 (4 waves per block); walker u of sequence b visits entries
// e = e0 + u, e0 + u + units_per_seq, ...; `split` waves share a walker's rows (a handful of rows, as in a
// decode step, would otherwise be one long chain of loads per wave).  Full mode (first == nullptr,
// last_n == 0) covers [0, cap): rows below C_b are embedded, the others zeroed.  Incremental modes cover
// [first[b], C_b) or the last last_n entries only.
template <bool BF16>
__global__ void __launch_bounds__(256) hyper_embed_kernel(EmbedArgs a) {
  const int lane = threadIdx.x & 63;
  const long long wave_id = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int part = (int)(wave_id % a.split);
  const long long unit = wave_id / a.split;
  const int b = (int)(unit / a.units_per_seq);
  const int u = (int)(unit % a.units_per_seq);
  if (b >= a.B) return;
  const int C = min(a.size[b], a.cap);
  const bool full = a.first == nullptr && a.last_n == 0;
  const int e0 = full ? 0 : (a.first ? max(a.first[b], 0) : max(C - a.last_n, 0));
  const int e1 = full ? a.cap : C;
  constexpr int EPC = BF16 ? 8 : 4;
  const int n_chunks = a.d / EPC;
  for (int e = e0 + u; e < e1; e += a.units_per_seq) {
    const size_t row = (size_t)b * a.cap + e;
    if (e < C) {
      const int L = min(max(a.ent_len[row], 1), a.M);
      embed_row<BF16>(a, a.ent_tokens + row * a.M, L, row, lane, part);
    } else {
      uint4* W = reinterpret_cast<uint4*>(a.W) + row * (size_t)n_chunks;
      const uint4 z = {0u, 0u, 0u, 0u};
      for (int c = part * 64 + lane; c < n_chunks; c += 64 * a.split) W[c] = z;
    }
  }
}

}  // namespace

int z2z_launch_hyper_embed(z2z_ctx* c, const void* E, void* W_hyper, const int32_t* first, int32_t max_new,
                           hipStream_t s) {
  EmbedArgs a;
  a.E = E;
  a.W = W_hyper;
  a.size = c->st.size;
  a.ent_tokens = c->st.ent_tokens;
  a.ent_len = c->st.ent_len;
  a.first = first;
  a.last_n = (!first && max_new > 0) ? max_new : 0;
  a.B = c->cfg.B;
  a.V = c->cfg.V;
  a.M = c->cfg.M;
  a.cap = c->cfg.cap;
  a.d = c->cfg.d;
  a.pool = c->cfg.pool;
  for (int L = 0; L <= Z2Z_MAX_M; ++L)
    for (int j = 0; j < Z2Z_MAX_M; ++j) a.coef[L][j] = c->coef[L][j];
  if (c->cfg.cap == 0) return Z2Z_OK;
  const bool incremental = first || max_new > 0;
  int units = incremental ? (max_new < 1 ? c->cfg.cap : (max_new < c->cfg.cap ? max_new : c->cfg.cap)) : c->cfg.cap;
  a.units_per_seq = units;
  // few rows to embed: several waves per row (one group of 64 chunks each when the row is long enough)
  const int chunks = c->cfg.d / (c->cfg.dtype == Z2Z_BF16 ? 8 : 4);
  int split = 1;
  while (split < 8 && (long long)c->cfg.B * units * split < 1024 && chunks >= 128 * split) split *= 2;
  a.split = split;
  const long long total_units = (long long)c->cfg.B * units * split;
  const unsigned grid = (unsigned)((total_units + 3) / 4);
  if (c->cfg.dtype == Z2Z_BF16)
    hipLaunchKernelGGL(hyper_embed_kernel<true>, dim3(grid), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(hyper_embed_kernel<false>, dim3(grid), dim3(256), 0, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}
