// Backward pass of the loss over the extended vocabulary (zip2zip paper, section 2.4, the objective over the
// compressed sequence): gradient into the hidden rows and both unembedding matrices, and through the pooling of
// the averaging hyper-encoder.
#include "logits_common.h"

#include <string.h>

#include <algorithm>

using namespace z2z_logits;

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
  if (!c->coef_dev) return Z2Z_EHIP;       // (allocated and filled by z2z_create)
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
  const size_t Vp = round_up(V, 64), capp = round_up(cap, 64), Np = round_up(rows_per_seq, 64);
  // The sequences go in chunks of n_seq, as many as the work-space limit allows (all of them at the sizes of
  // the benchmark configurations): dH and dW_hyper of a chunk are its own, dW_base of a later chunk adds to the
  // bf16 result of the earlier ones (one more rounding per chunk).
  // work space (bf16 unless noted), 256-byte aligned pieces
  size_t off = 0;
  size_t o_g, o_Pb, o_PbT, o_Ph, o_PhT, o_WbT, o_WhT, o_HT, o_HTs;
  auto take = [&](size_t bytes) { const size_t at = off; off += round_up(bytes, 256); return at; };
  auto layout = [&](int n_seq) {
    const size_t rc = (size_t)n_seq * rows_per_seq, rcp = round_up(rc, 64);
    off = 0;
    o_g = take(rc * 4);                              // float g[rows of the chunk]
    o_Pb = take(rc * Vp * 2);                        // dZ, base columns      [rows, Vp]
    o_PbT = take((size_t)V * rcp * 2);               // its transpose         [V, rows_p]
    o_Ph = take(rc * capp * 2);                      // dZ, hyper columns     [rows, capp]
    o_PhT = take((size_t)n_seq * cap * Np * 2);      // per sequence          [n_seq][cap, Np]
    o_WbT = take((size_t)d * Vp * 2);                // W_base^T              [d, Vp]
    o_WhT = take((size_t)n_seq * d * capp * 2);      // W_hyper[b]^T          [n_seq][d, capp]
    o_HT = take((size_t)d * rcp * 2);                // H^T                   [d, rows_p]
    o_HTs = take((size_t)n_seq * d * Np * 2);        // H[b]^T                [n_seq][d, Np]
    return off;
  };
  const size_t limit = (size_t)200 << 30;
  int n_seq = B;
  if (c->opt_backward_chunk > 0 && c->opt_backward_chunk < n_seq) n_seq = c->opt_backward_chunk;
  while (n_seq > 1 && layout(n_seq) > limit) n_seq = (n_seq + 1) / 2;
  if (layout(n_seq) > limit) return Z2Z_ENOMEM;      // one sequence alone does not fit
  if (off > c->bwd_ws_bytes) {
    Z2Z_TRY_GROW(s);
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
  const int strip = c->opt_logits_strip > 0 ? c->opt_logits_strip : 4;
  const uint16_t* H16 = reinterpret_cast<const uint16_t*>(H);
  const uint16_t* Wh16 = reinterpret_cast<const uint16_t*>(W_hyper);

  int rc = z2z_launch_transpose(W_base, WbT, V, nullptr, d, d, (int)Vp, 1, 0, 0, s);
  if (rc != Z2Z_OK) return rc;
  for (int b0 = 0; b0 < B; b0 += n_seq) {
    const int nb = b0 + n_seq <= B ? n_seq : B - b0;
    const int r0 = b0 * rows_per_seq, rows_c = nb * rows_per_seq;
    const size_t rows_p = round_up(rows_c, 64);
    const uint16_t* Hc = H16 + (size_t)r0 * d;
    const uint16_t* Whc = Wh16 + (size_t)b0 * cap * d;
    hipLaunchKernelGGL(row_grad_kernel, dim3((rows_c + 255) / 256), dim3(256), 0, s, targets + r0,
                       grad_nll ? grad_nll + r0 : nullptr, c->st.size + b0, rows_c, rows_per_seq, V, cap, g);
    // ---- dZ: the forward kernel with the probability epilogue -------------------------------------------
    LogitsArgs a;
    memset(&a, 0, sizeof(a));
    a.H = Hc;
    a.rows = rows_c;
    a.rows_per_seq = rows_per_seq;
    a.d = d;
    a.map_lr = a.map_ls = a.map_xr = a.map_xs = a.map_sb_r = 1;
    a.lse = lse + r0;
    a.row_grad = g;
    a.targets = targets + r0;
    int ns = 0;
    a.out = Pb;
    a.ldo = (int)Vp;
    rc = z2z_launch_logits_part(c, false, true, a, W_base, V, 0, 0, strip, rows_c, rows_per_seq, &ns, false, s, true);
    if (rc != Z2Z_OK) return rc;
    if (cap > 0) {
      const size_t n16 = (size_t)rows_c * capp * 2 / 16;
      hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)std::min<size_t>((n16 + 255) / 256, 4096)), dim3(256), 0, s,
                         reinterpret_cast<uint4*>(Ph), n16);
      a.out = Ph;
      a.ldo = (int)capp;
      rc = z2z_launch_logits_part(c, true, true, a, Whc, cap, V, 0, strip, rows_c, rows_per_seq, &ns, false, s, true, b0,
                                  nb);
      if (rc != Z2Z_OK) return rc;
    }
    // ---- transposed copies -----------------------------------------------------------------------------------
    if ((rc = z2z_launch_transpose(Hc, HT, rows_c, nullptr, d, d, (int)rows_p, 1, 0, 0, s)) != Z2Z_OK) return rc;
    if ((rc = z2z_launch_transpose(Pb, PbT, rows_c, nullptr, V, (int)Vp, (int)rows_p, 1, 0, 0, s)) != Z2Z_OK) return rc;
    if (cap > 0) {
      if ((rc = z2z_launch_transpose(Whc, WhT, cap, nullptr, d, d, (int)capp, nb, (size_t)cap * d, (size_t)d * capp, s)) != Z2Z_OK) return rc;
      if ((rc = z2z_launch_transpose(Hc, HTs, rows_per_seq, nullptr, d, d, (int)Np, nb, (size_t)rows_per_seq * d, (size_t)d * Np, s)) != Z2Z_OK) return rc;
      if ((rc = z2z_launch_transpose(Ph, PhT, rows_per_seq, nullptr, cap, (int)capp, (int)Np, nb, (size_t)rows_per_seq * capp, (size_t)cap * Np, s)) != Z2Z_OK) return rc;
    }
    // ---- the products ------------------------------------------------------------------------------------------
    uint16_t* dHc = reinterpret_cast<uint16_t*>(dH) + (size_t)r0 * d;
    if ((rc = z2z_launch_linear(c, Pb, WbT, nullptr, nullptr, 0, dHc, rows_c, nullptr, d, (int)Vp, s)) != Z2Z_OK) return rc;
    if ((rc = z2z_launch_linear(c, PbT, HT, nullptr, b0 > 0 ? dW_base : nullptr, 0, dW_base, V, nullptr, d, (int)rows_p, s)) != Z2Z_OK) return rc;
    for (int b = 0; b < nb && cap > 0; ++b) {
      uint16_t* dH_b = dHc + (size_t)b * rows_per_seq * d;
      const uint16_t* Ph_b = reinterpret_cast<const uint16_t*>(Ph) + (size_t)b * rows_per_seq * capp;
      const uint16_t* WhT_b = reinterpret_cast<const uint16_t*>(WhT) + (size_t)b * d * capp;
      if ((rc = z2z_launch_linear(c, Ph_b, WhT_b, nullptr, dH_b, 0, dH_b, rows_per_seq, nullptr, d, (int)capp, s)) != Z2Z_OK) return rc;
      const uint16_t* PhT_b = reinterpret_cast<const uint16_t*>(PhT) + (size_t)b * cap * Np;
      const uint16_t* HTs_b = reinterpret_cast<const uint16_t*>(HTs) + (size_t)b * d * Np;
      uint16_t* dWh_b = reinterpret_cast<uint16_t*>(dW_hyper) + (size_t)(b0 + b) * cap * d;
      if ((rc = z2z_launch_linear(c, PhT_b, HTs_b, nullptr, nullptr, 0, dWh_b, cap, nullptr, d, (int)Np, s)) != Z2Z_OK) return rc;
    }
  }
  return Z2Z_OK;
}
