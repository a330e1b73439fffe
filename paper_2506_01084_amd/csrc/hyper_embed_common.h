// The pooling of one codebook entry's constituent embeddings (section 2.2 of the zip2zip paper, the "Averaging"
// hyper-encoder: padding contributes nothing, the divisor is the entry's own length), shared by hyper_embed's
// kernel and the fused generation-step update.  A wave owns 16-byte column chunks of the row: 1 KiB of each
// constituent row per instruction, fp32 accumulation in token order, one rounding (nearest-even) to the
// storage type.
#pragma once

#include "z2z_internal.h"

namespace z2z_embed {

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

// The arguments every launch fills alike.
inline void fill_embed_args(const z2z_ctx* c, const void* E, void* W_hyper, EmbedArgs* a) {
  a->E = E;
  a->W = W_hyper;
  a->size = c->st.size;
  a->ent_tokens = c->st.ent_tokens;
  a->ent_len = c->st.ent_len;
  a->first = nullptr;
  a->last_n = 0;
  a->B = c->cfg.B;
  a->V = c->cfg.V;
  a->M = c->cfg.M;
  a->cap = c->cfg.cap;
  a->d = c->cfg.d;
  a->units_per_seq = 1;
  a->split = 1;
  a->pool = c->cfg.pool;
  for (int L = 0; L <= Z2Z_MAX_M; ++L)
    for (int j = 0; j < Z2Z_MAX_M; ++j) a->coef[L][j] = c->coef[L][j];
}

}  // namespace z2z_embed
