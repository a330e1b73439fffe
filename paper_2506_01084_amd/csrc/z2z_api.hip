// C ABI of libz2z: argument checks, context life cycle, option and timing plumbing.
// Every entry point validates on the host, then hands over to a launcher; nothing here computes.
#include "z2z_internal.h"

#include <math.h>
#include <new>
#include <string.h>

#include "logits_common.h"
#include "logits_mid.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

void free_ctx(z2z_ctx* c) {
  if (!c) return;
  (void)hipFree(c->st.size);
  (void)hipFree(c->st.prev_code);
  (void)hipFree(c->st.prev_len);
  (void)hipFree(c->st.rounds);
  (void)hipFree(c->st.ent_tokens);
  (void)hipFree(c->st.ent_len);
  (void)hipFree(c->st.slots);
  (void)hipFree(c->part_m);
  (void)hipFree(c->part_s);
  (void)hipFree(c->part_i);
  (void)hipFree(c->part_v);
  (void)hipFree(c->part_l);
  (void)hipFree(c->sample_logits);
  (void)hipFree(c->row_max);
  (void)hipFree(c->enc_ws);
  (void)hipFree(c->enc_bwd_ws);
  (void)hipFree(c->bwd_ws);
  (void)hipFree(c->coef_dev);
  (void)hipFree(c->prune_prefix);
  (void)hipFree(c->skinny_partial);
  if (c->ev_created) {
    for (int i = 0; i < Z2Z_MAX_TIMED; ++i) {
      (void)hipEventDestroy(c->ev_start[i]);
      (void)hipEventDestroy(c->ev_stop[i]);
    }
  }
  delete c;
}

}  // namespace

extern "C" {

Z2Z_API int z2z_create(z2z_ctx** out, const z2z_config* cfg) {
  if (!out || !cfg) return Z2Z_EINVAL;
  *out = nullptr;
  if (cfg->B < 1 || cfg->V < 1 || cfg->M < 1 || cfg->M > Z2Z_MAX_M) return Z2Z_EINVAL;
  if (cfg->cap < 0 || cfg->cap > Z2Z_MAX_CAP) return Z2Z_EINVAL;
  if ((long long)cfg->V + cfg->cap > (1LL << 24)) return Z2Z_EUNSUPPORTED;   // codes are packed in 24 bits
  if (cfg->dtype != Z2Z_F32 && cfg->dtype != Z2Z_BF16) return Z2Z_EUNSUPPORTED;
  if (cfg->pool != Z2Z_POOL_MEAN && cfg->pool != Z2Z_POOL_WEIGHTED) return Z2Z_EUNSUPPORTED;
  const int epc = cfg->dtype == Z2Z_BF16 ? 8 : 4;
  if (cfg->d < epc || cfg->d % epc != 0) return Z2Z_EINVAL;
  for (int j = 0; j < cfg->M; ++j)
    if (!isfinite(cfg->w[j])) return Z2Z_EINVAL;

  z2z_ctx* c = new (std::nothrow) z2z_ctx();
  if (!c) return Z2Z_ENOMEM;
  memset(c, 0, sizeof(*c));
  c->cfg = *cfg;
  if (hipGetDevice(&c->device) != hipSuccess) {
    delete c;
    return Z2Z_EHIP;
  }
  int lds = 0, cus = 0;
  if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, c->device) != hipSuccess) lds = 65536;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess) cus = 256;
  c->lds_limit = lds > 160 * 1024 ? 160 * 1024 : lds;
  c->num_cu = cus;

  // pooling coefficients: coef[L][j] = 1/L or softmax(w[0..L))_j, computed in double
  for (int L = 1; L <= Z2Z_MAX_M; ++L) {
    double mx = -INFINITY, sum = 0.0;
    for (int j = 0; j < L; ++j) mx = cfg->w[j] > mx ? cfg->w[j] : mx;
    for (int j = 0; j < L; ++j) sum += exp((double)cfg->w[j] - mx);
    for (int j = 0; j < L; ++j)
      c->coef[L][j] = cfg->pool == Z2Z_POOL_MEAN ? (float)(1.0 / L) : (float)(exp((double)cfg->w[j] - mx) / sum);
  }

  LzwState& st = c->st;
  st.V = cfg->V;
  st.M = cfg->M;
  st.cap = cfg->cap;
  if (z2z_lzw_prepare(c) != Z2Z_OK) {   // sizes the hash table (st.nslots) for this device
    delete c;
    return Z2Z_EHIP;
  }
  const size_t B = (size_t)cfg->B;
  const size_t capn = cfg->cap > 0 ? (size_t)cfg->cap : 1;
  bool ok = true;
  ok = ok && hipMalloc(&st.size, B * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&st.prev_code, B * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&st.prev_len, B * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&st.rounds, B * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMemset(st.rounds, 0, B * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&st.ent_tokens, B * capn * cfg->M * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&st.ent_len, B * capn * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&st.slots, B * (size_t)st.nslots * sizeof(unsigned long long)) == hipSuccess;
  // fixed-size work buffers of calls that must not allocate on a stream: pruning's prefix map, and the pooling
  // coefficients on the device (the pooling's backward pass)
  ok = ok && hipMalloc(&c->prune_prefix, B * capn * sizeof(int32_t)) == hipSuccess;
  ok = ok && hipMalloc(&c->coef_dev, sizeof(c->coef)) == hipSuccess;
  ok = ok && hipMemcpy(c->coef_dev, c->coef, sizeof(c->coef), hipMemcpyHostToDevice) == hipSuccess;
  if (!ok) {
    free_ctx(c);
    return Z2Z_ENOMEM;
  }
  if (z2z_static_scratch_prepare(c) != Z2Z_OK) {   // the allocation-free entry point's array on this device
    free_ctx(c);
    return Z2Z_EHIP;
  }
  c->fast_ready = z2z_logits_fast_prepare(c) == Z2Z_OK;
  c->mid_ready = z2z_logits_mid_prepare(c) == Z2Z_OK;
  c->skinny_ready = z2z_logits_decode_prepare(c) == Z2Z_OK;      // the kernel itself; decode_ready: for this shape
  c->decode_ready = z2z_logits_decode_ok(c) && c->skinny_ready;
  c->trunc_ready = c->decode_ready && z2z_sample_truncated_prepare(c) == Z2Z_OK;
  if (z2z_launch_lzw_reset(c, nullptr) != Z2Z_OK ||
      hipStreamSynchronize(nullptr) != hipSuccess) {
    free_ctx(c);
    return Z2Z_EHIP;
  }
  *out = c;
  return Z2Z_OK;
}

Z2Z_API int z2z_destroy(z2z_ctx* ctx) {
  if (!ctx) return Z2Z_EINVAL;
  (void)hipDeviceSynchronize();
  free_ctx(ctx);
  return Z2Z_OK;
}

Z2Z_API int z2z_reset(z2z_ctx* ctx, void* stream) {
  if (!ctx) return Z2Z_EINVAL;
  return z2z_launch_lzw_reset(ctx, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_lzw_encode(z2z_ctx* ctx, const int32_t* d_tokens, const int32_t* d_lens, int32_t stride,
                           int32_t flags, int32_t* d_codes, int32_t* d_n_codes, int32_t out_stride,
                           int32_t* d_status, void* stream) {
  if (!ctx || !d_n_codes || !d_status) return Z2Z_EINVAL;
  if (stride < 0 || out_stride < 0) return Z2Z_EINVAL;
  if ((stride > 0 && !d_tokens) || (out_stride > 0 && !d_codes)) return Z2Z_EINVAL;
  if (flags != Z2Z_APPEND && flags != Z2Z_RESET) return Z2Z_EINVAL;
  return z2z_launch_lzw_encode(ctx, d_tokens, d_lens, stride, flags, d_codes, d_n_codes, out_stride, d_status,
                               static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_lzw_decode(z2z_ctx* ctx, const int32_t* d_codes, const int32_t* d_n_codes, int32_t stride,
                           int32_t flags, int32_t* d_tokens, int32_t* d_n_tokens, int32_t out_stride,
                           int32_t* d_status, void* stream) {
  if (!ctx || !d_n_tokens || !d_status) return Z2Z_EINVAL;
  if (stride < 0 || out_stride < 0) return Z2Z_EINVAL;
  if (stride > 0 && !d_codes) return Z2Z_EINVAL;
  if (out_stride > 0 && !d_tokens) return Z2Z_EINVAL;
  if (out_stride == 0 && d_tokens) return Z2Z_EINVAL;
  if (flags != Z2Z_APPEND && flags != Z2Z_RESET) return Z2Z_EINVAL;
  return z2z_launch_lzw_decode(ctx, d_codes, d_n_codes, stride, flags, d_tokens, d_n_tokens, out_stride, d_status,
                               static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_codebook(z2z_ctx* ctx, const int32_t** d_entries, const int32_t** d_entry_len,
                         const int32_t** d_size) {
  if (!ctx) return Z2Z_EINVAL;
  if (d_entries) *d_entries = ctx->st.ent_tokens;
  if (d_entry_len) *d_entry_len = ctx->st.ent_len;
  if (d_size) *d_size = ctx->st.size;
  return Z2Z_OK;
}

Z2Z_API int z2z_step_update(z2z_ctx* ctx, const int32_t* d_codes, int32_t stride, const void* d_E, void* d_W_hyper,
                            int32_t* d_n_tokens, int32_t* d_status, void* stream) {
  if (!ctx || !d_codes || !d_n_tokens || !d_status || stride < 1) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && (!d_E || !d_W_hyper)) return Z2Z_EINVAL;
  if (!aligned16(d_E) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  return z2z_launch_step_update(ctx, d_codes, stride, d_E, d_W_hyper, d_n_tokens, d_status,
                                static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_lzw_rounds(z2z_ctx* ctx, const int32_t** d_rounds) {
  if (!ctx || !d_rounds) return Z2Z_EINVAL;
  *d_rounds = ctx->st.rounds;
  return Z2Z_OK;
}

Z2Z_API int z2z_codebook_usage(z2z_ctx* ctx, const int32_t* d_codes, const int32_t* d_n_codes, int32_t stride,
                               int32_t* d_usage, void* stream) {
  if (!ctx || stride < 0 || (stride > 0 && !d_codes)) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_usage) return Z2Z_EINVAL;
  if (ctx->cfg.cap == 0 || stride == 0) return Z2Z_OK;
  return z2z_launch_codebook_usage(ctx, d_codes, d_n_codes, stride, d_usage, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_codebook_prune(z2z_ctx* ctx, const int32_t* d_keep, int32_t* d_new_id, int32_t* d_n_kept,
                               void* stream) {
  if (!ctx || !d_n_kept) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && (!d_keep || !d_new_id)) return Z2Z_EINVAL;
  return z2z_launch_codebook_prune(ctx, d_keep, d_new_id, d_n_kept, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_codebook_prefill(z2z_ctx* ctx, const int32_t* d_phrases, const int32_t* d_phrase_len,
                                 const int32_t* d_counts, int32_t n_max, int32_t flags, int32_t* d_n_added,
                                 int32_t* d_status, void* stream) {
  if (!ctx || !d_n_added || !d_status || n_max < 0) return Z2Z_EINVAL;
  if (n_max > 0 && (!d_phrases || !d_phrase_len)) return Z2Z_EINVAL;
  if (flags != Z2Z_RESET && flags != Z2Z_APPEND) return Z2Z_EINVAL;
  return z2z_launch_codebook_prefill(ctx, d_phrases, d_phrase_len, d_counts, n_max, flags, d_n_added, d_status,
                                     static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_hyper_embed(z2z_ctx* ctx, const void* d_E, void* d_W_hyper, const int32_t* d_first,
                            int32_t max_new, void* stream) {
  if (!ctx || !d_E) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_W_hyper) return Z2Z_EINVAL;
  if (!aligned16(d_E) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  return z2z_launch_hyper_embed(ctx, d_E, d_W_hyper, d_first, max_new, static_cast<hipStream_t>(stream));
}

namespace {

// every pointer a layer of the description must carry, present and 16-byte aligned
bool encoder_pointers_ok(const z2z_encoder* enc) {
  if (!enc || !enc->layers) return false;
  if (enc->n_layers < 1 || enc->n_layers > Z2Z_MAX_ENCODER_LAYERS) return false;
  if (!aligned16(enc->pos)) return false;
  for (int l = 0; l < enc->n_layers; ++l) {
    const z2z_encoder_layer& y = enc->layers[l];
    const void* always[] = {y.ln1_g, y.ln1_b, y.w_qkv, y.b_qkv, y.w_o, y.b_o};
    for (const void* p : always)
      if (!p || !aligned16(p)) return false;
    if (!enc->attention_only) {
      const void* ffn[] = {y.ln2_g, y.ln2_b, y.w_1, y.b_1, y.w_2, y.b_2};
      for (const void* p : ffn)
        if (!p || !aligned16(p)) return false;
    }
  }
  return true;
}

}  // namespace

Z2Z_API int z2z_hyper_encode(z2z_ctx* ctx, const void* d_E, const z2z_encoder* enc, void* d_W_hyper,
                             const int32_t* d_first, int32_t max_new, void* stream) {
  if (!ctx || !d_E || !encoder_pointers_ok(enc)) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_W_hyper) return Z2Z_EINVAL;
  if (!aligned16(d_E) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  if (!z2z_hyper_encode_ok(ctx, enc)) return Z2Z_EUNSUPPORTED;
  return z2z_launch_hyper_encode(ctx, d_E, enc, d_W_hyper, d_first, max_new, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_hyper_encode_keep(z2z_ctx* ctx, const void* d_E, const z2z_encoder* enc, void* d_W_hyper, void* stream) {
  if (!ctx || !d_E || !encoder_pointers_ok(enc)) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_W_hyper) return Z2Z_EINVAL;
  if (!aligned16(d_E) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  if (!z2z_hyper_encode_ok(ctx, enc)) return Z2Z_EUNSUPPORTED;
  return z2z_launch_hyper_encode_train(ctx, 1, d_E, enc, d_W_hyper, nullptr, nullptr, nullptr,
                                       static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_hyper_encode_backward(z2z_ctx* ctx, const void* d_E, const z2z_encoder* enc, const void* d_dW_hyper,
                                      const z2z_encoder* grad, float* d_dE, int32_t flags, void* stream) {
  if (!ctx || !d_E || !d_dE || !encoder_pointers_ok(enc) || !encoder_pointers_ok(grad)) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_dW_hyper) return Z2Z_EINVAL;
  if (grad->n_layers != enc->n_layers || (enc->pos && !grad->pos)) return Z2Z_EINVAL;
  if (flags & ~Z2Z_ENC_KEPT) return Z2Z_EINVAL;
  if (!aligned16(d_E) || !aligned16(d_dW_hyper) || !aligned16(d_dE)) return Z2Z_EINVAL;
  if (!z2z_hyper_encode_ok(ctx, enc)) return Z2Z_EUNSUPPORTED;
  return z2z_launch_hyper_encode_train(ctx, (flags & Z2Z_ENC_KEPT) ? 2 : 0, d_E, enc, nullptr, d_dW_hyper, grad, d_dE,
                                       static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_extended_logits(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                                const void* d_W_base, const void* d_W_hyper, int32_t* d_argmax, float* d_max,
                                float* d_lse, float* d_logits, void* stream) {
  if (!ctx || !d_H || !d_W_base) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_W_hyper) return Z2Z_EINVAL;
  if (rows_per_seq < 1 || rows < 1) return Z2Z_EINVAL;
  if ((long long)rows_per_seq * ctx->cfg.B != (long long)rows) return Z2Z_EINVAL;
  if (!aligned16(d_H) || !aligned16(d_W_base) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  return z2z_launch_extended_logits(ctx, d_H, rows, rows_per_seq, d_W_base, d_W_hyper, d_argmax, d_max, d_lse,
                                    d_logits, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_extended_logits_static(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                                       const void* d_W_base, const void* d_W_hyper, int32_t* d_argmax,
                                       float* d_max, float* d_lse, float* d_logits, void* stream) {
  if (!ctx || !d_H || !d_W_base) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_W_hyper) return Z2Z_EINVAL;
  if (rows_per_seq < 1 || rows < 1) return Z2Z_EINVAL;
  if ((long long)rows_per_seq * ctx->cfg.B != (long long)rows) return Z2Z_EINVAL;
  if (!aligned16(d_H) || !aligned16(d_W_base) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  return z2z_launch_extended_logits(ctx, d_H, rows, rows_per_seq, d_W_base, d_W_hyper, d_argmax, d_max, d_lse,
                                    d_logits, static_cast<hipStream_t>(stream), true);
}

Z2Z_API int z2z_extended_sample(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                                const void* d_W_base, const void* d_W_hyper, float temperature, int32_t top_k,
                                float top_p, uint64_t seed, uint64_t step, int32_t* d_token, float* d_logprob,
                                void* stream) {
  if (!ctx || !d_H || !d_W_base || !d_token) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_W_hyper) return Z2Z_EINVAL;
  if (rows_per_seq < 1 || rows < 1) return Z2Z_EINVAL;
  if ((long long)rows_per_seq * ctx->cfg.B != (long long)rows) return Z2Z_EINVAL;
  if (!(temperature > 0.f) || !(temperature < 3.0e38f)) return Z2Z_EINVAL;
  if (!(top_p > 0.f)) return Z2Z_EINVAL;          // also rejects NaN; >= 1 switches the filter off
  if (!aligned16(d_H) || !aligned16(d_W_base) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  return z2z_launch_extended_sample(ctx, d_H, rows, rows_per_seq, d_W_base, d_W_hyper, temperature, top_k, top_p,
                                    seed, step, d_token, d_logprob, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_extended_nll(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq, const void* d_W_base,
                             const void* d_W_hyper, const int32_t* d_targets, float* d_nll, float* d_lse,
                             void* stream) {
  if (!ctx || !d_H || !d_W_base || !d_targets || !d_nll || !d_lse) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_W_hyper) return Z2Z_EINVAL;
  if (rows_per_seq < 1 || rows < 1) return Z2Z_EINVAL;
  if ((long long)rows_per_seq * ctx->cfg.B != (long long)rows) return Z2Z_EINVAL;
  if (!aligned16(d_H) || !aligned16(d_W_base) || !aligned16(d_W_hyper)) return Z2Z_EINVAL;
  return z2z_launch_extended_nll(ctx, d_H, rows, rows_per_seq, d_W_base, d_W_hyper, d_targets, d_nll, d_lse,
                                 static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_extended_nll_backward(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                                      const void* d_W_base, const void* d_W_hyper, const int32_t* d_targets,
                                      const float* d_lse, const float* d_grad_nll, void* d_dH, void* d_dW_base,
                                      void* d_dW_hyper, void* stream) {
  if (!ctx || !d_H || !d_W_base || !d_targets || !d_lse || !d_dH || !d_dW_base) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && (!d_W_hyper || !d_dW_hyper)) return Z2Z_EINVAL;
  if (rows_per_seq < 1 || rows < 1) return Z2Z_EINVAL;
  if ((long long)rows_per_seq * ctx->cfg.B != (long long)rows) return Z2Z_EINVAL;
  if (!aligned16(d_H) || !aligned16(d_W_base) || !aligned16(d_W_hyper) || !aligned16(d_dH) || !aligned16(d_dW_base) ||
      !aligned16(d_dW_hyper))
    return Z2Z_EINVAL;
  return z2z_launch_extended_nll_backward(ctx, d_H, rows, rows_per_seq, d_W_base, d_W_hyper, d_targets, d_lse,
                                          d_grad_nll, d_dH, d_dW_base, d_dW_hyper, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_hyper_embed_backward(z2z_ctx* ctx, const void* d_dW_hyper, float* d_dE, void* stream) {
  if (!ctx || !d_dE) return Z2Z_EINVAL;
  if (ctx->cfg.cap > 0 && !d_dW_hyper) return Z2Z_EINVAL;
  if (ctx->cfg.dtype != Z2Z_BF16) return Z2Z_EUNSUPPORTED;
  return z2z_launch_hyper_embed_backward(ctx, d_dW_hyper, d_dE, static_cast<hipStream_t>(stream));
}

Z2Z_API int z2z_set_option(z2z_ctx* ctx, int32_t key, int32_t value) {
  if (!ctx) return Z2Z_EINVAL;
  switch (key) {
    case Z2Z_OPT_LOGITS_KERNEL: ctx->opt_logits_kernel = value; return Z2Z_OK;
    case Z2Z_OPT_LOGITS_STRIP:
      if (value < 0) return Z2Z_EINVAL;
      ctx->opt_logits_strip = value;
      return Z2Z_OK;
    case Z2Z_OPT_LZW_KERNEL: ctx->opt_lzw_kernel = value; return Z2Z_OK;
    case Z2Z_OPT_DECODE_KERNEL: ctx->opt_decode_kernel = value; return Z2Z_OK;
    case Z2Z_OPT_SAMPLE_KERNEL: ctx->opt_sample_kernel = value; return Z2Z_OK;
    case Z2Z_OPT_BACKWARD_CHUNK:
      if (value < 0) return Z2Z_EINVAL;
      ctx->opt_backward_chunk = value;
      return Z2Z_OK;
    case Z2Z_OPT_LOGITS_MAP:
      if (value != 0 && ((value & 0xFF) < 1 || ((value >> 8) & 0xFF) < 1 || ((value >> 16) & 0xFF) < 1 ||
                         ((value >> 24) & 0xFF) < 1 || ((value >> 16) & 0xFF) * ((value >> 24) & 0xFF) != 8))
        return Z2Z_EINVAL;
      ctx->opt_logits_map = value;
      return Z2Z_OK;
    case Z2Z_OPT_TIMING:
      if (value && !ctx->ev_created) {
        for (int i = 0; i < Z2Z_MAX_TIMED; ++i) {
          if (hipEventCreate(&ctx->ev_start[i]) != hipSuccess || hipEventCreate(&ctx->ev_stop[i]) != hipSuccess)
            return Z2Z_EHIP;
        }
        ctx->ev_created = 1;
      }
      ctx->opt_timing = value ? 1 : 0;
      return Z2Z_OK;
    default: return Z2Z_EINVAL;
  }
}

Z2Z_API int z2z_read_timing(z2z_ctx* ctx, float* total_ms, int32_t* launches) {
  if (!ctx || !total_ms || !launches) return Z2Z_EINVAL;
  float sum = 0.f;
  for (int i = 0; i < ctx->n_timed; ++i) {
    if (hipEventSynchronize(ctx->ev_stop[i]) != hipSuccess) return Z2Z_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i]) != hipSuccess) return Z2Z_EHIP;
    sum += ms;
  }
  *total_ms = sum;
  *launches = ctx->n_timed;
  ctx->n_timed = 0;
  return Z2Z_OK;
}

Z2Z_API int z2z_read_launches(const z2z_ctx* ctx, int64_t* counts) {
  if (!ctx || !counts) return Z2Z_EINVAL;
  for (int i = 0; i < Z2Z_N_KERNEL_FAMILIES; ++i) counts[i] = ctx->n_launch[i];
  return Z2Z_OK;
}

Z2Z_API const char* z2z_strerror(int code) {
  switch (code) {
    case Z2Z_OK: return "ok";
    case Z2Z_EINVAL: return "invalid argument";
    case Z2Z_ENOMEM: return "out of device or host memory";
    case Z2Z_EHIP: return "HIP runtime error";
    case Z2Z_EUNSUPPORTED: return "unsupported dtype or pooling kind";
    case Z2Z_ELIMIT: return "beyond the fixed scratch size of the allocation-free entry point";
    case Z2Z_ECAPTURE: return "a work buffer would have to grow while the stream is being captured";
    default: return "unknown error";
  }
}

}  // extern "C"
