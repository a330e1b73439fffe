// Internal declarations shared by the translation units of libz2z (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "z2z.h"

#define Z2Z_API __attribute__((visibility("default")))
#define Z2Z_MAX_TIMED 1024

// Per-sequence codebook storage, all in device global memory and owned by the context.
//   size[b]                    number of entries C_b
//   prev_code[b], prev_len[b]  last phrase emitted / consumed (-1, 0 = none)
//   ent_tokens[b][e][0..M)     flattened base tokens of entry e, -1 padded
//   ent_len[b][e]              its length (0 = unused)
//   slots[b][h]                open-addressing hash table over the trie edges, one 64-bit word per slot:
//                              parent code (24 bits) | last token (24 bits) | entry index (16 bits); all
//                              ones = empty.  Hence V + cap <= 2^24.
struct LzwState {
  int32_t* size;
  int32_t* prev_code;
  int32_t* prev_len;
  int32_t* rounds;           // [B] rounds the latest parse kernel took for the sequence (instrumentation)
  int32_t* ent_tokens;
  int32_t* ent_len;
  unsigned long long* slots;
  int32_t V, M, cap, nslots;
  int32_t slots_fit_lds;     // the table of one sequence fits the LDS of a CU
};

// Where the tile kernels leave their partial (max, sum-exp, argmax) triples: three arrays of `capacity`
// elements each.  Either the context's growable buffers or a device's static array.
struct z2z_parts {
  float* m;
  float* s;
  int32_t* i;
  size_t capacity;
};

struct z2z_ctx {
  z2z_config cfg;
  int device;
  int lds_limit;           // bytes of LDS one workgroup may use on this device
  int num_cu;
  LzwState st;
  float coef[Z2Z_MAX_M + 1][Z2Z_MAX_M];   // coef[L][j]: pooling coefficient of token j of a length-L entry
  // extended_logits scratch: partial (max, sum-exp, argmax) per (part, row)
  float* part_m;
  float* part_s;
  int32_t* part_i;
  size_t part_capacity;    // elements in each of the three arrays
  // extended_sample scratch: best perturbed value and the scaled logit at that column (its column is part_i)
  float* part_v;
  float* part_l;
  size_t part_vl_capacity;
  // truncated sampling: the rows' logits as the decode kernel stores them, and the row maxima
  float* sample_logits;
  float* row_max;
  size_t sample_logits_capacity;   // floats
  int trunc_ready;
  // hyper_encode work space: the activations of one pass (bf16)
  void* enc_ws;
  size_t enc_ws_bytes;
  // backward pass of the loss: dZ, the transposed operand copies (bf16), the row gradients
  void* enc_bwd_ws;        // saved activations and gradients of the learned encoder's backward pass
  size_t enc_bwd_ws_bytes;
  bool enc_kept;           // the work space holds the rows of a z2z_hyper_encode_keep call ...
  size_t enc_kept_need;    // ... laid out for this size ...
  const void* enc_kept_E;  // ... computed from this embedding matrix
  void* bwd_ws;
  size_t bwd_ws_bytes;
  void* prune_prefix;      // codebook pruning: every entry's prefix entry (scratch, [B, cap] int32)
  void* coef_dev;          // the pooling coefficients on the device (pooling backward)
  // dense layers on few rows with K split over workgroups: the partial tiles
  void* skinny_partial;
  size_t skinny_partial_bytes;
  // options
  int opt_backward_chunk;
  int opt_logits_kernel, opt_logits_strip, opt_lzw_kernel, opt_decode_kernel, opt_timing, opt_logits_map,
      opt_sample_kernel;
  int decode_ready;        // the decode-step logits kernel can be launched for this configuration
  int skinny_ready;        // the decode-step kernel's LDS fits this device (dense layers on few rows use it)
  int fast_ready;          // the 128 KiB-LDS bf16 logits kernel can be launched on this device
  int mid_ready;           // the weight-streaming kernel for up to 192 hidden rows can be launched on this device
  // timing record
  hipEvent_t ev_start[Z2Z_MAX_TIMED];
  hipEvent_t ev_stop[Z2Z_MAX_TIMED];
  int n_timed;
  int ev_created;
  long long n_launch[Z2Z_N_KERNEL_FAMILIES];   // launches enqueued per logits kernel family
};

// launchers (each validates nothing: the C-ABI layer has done so)
int z2z_lzw_prepare(z2z_ctx* c);   // raises the dynamic-LDS ceiling of the parse kernels
int z2z_launch_lzw_reset(z2z_ctx* c, hipStream_t s);
int z2z_launch_lzw_encode(z2z_ctx* c, const int32_t* tokens, const int32_t* lens, int32_t stride, int32_t flags,
                          int32_t* codes, int32_t* n_codes, int32_t out_stride, int32_t* status, hipStream_t s);
int z2z_launch_lzw_decode(z2z_ctx* c, const int32_t* codes, const int32_t* n_codes, int32_t stride, int32_t flags,
                          int32_t* tokens, int32_t* n_tokens, int32_t out_stride, int32_t* status, hipStream_t s);
int z2z_launch_step_update(z2z_ctx* c, const int32_t* codes, int32_t stride, const void* E, void* W_hyper,
                           int32_t* n_tokens, int32_t* status, hipStream_t s);
int z2z_launch_codebook_usage(z2z_ctx* c, const int32_t* codes, const int32_t* n_codes, int32_t stride, int32_t* usage,
                              hipStream_t s);
int z2z_launch_codebook_prune(z2z_ctx* c, const int32_t* keep, int32_t* new_id, int32_t* n_kept, hipStream_t s);
int z2z_launch_codebook_prefill(z2z_ctx* c, const int32_t* phrases, const int32_t* phrase_len, const int32_t* counts,
                                int32_t n_max, int32_t flags, int32_t* n_added, int32_t* status, hipStream_t s);
int z2z_launch_hyper_embed(z2z_ctx* c, const void* E, void* W_hyper, const int32_t* first, int32_t max_new,
                           hipStream_t s);
// use_static: the partial triples go to the device's static array (nothing is allocated; Z2Z_ELIMIT when they
// do not fit) instead of the context's growable buffers
int z2z_launch_extended_logits(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                               const void* W_hyper, int32_t* argmax, float* mx, float* lse, float* logits,
                               hipStream_t s, bool use_static = false);
int z2z_static_scratch_prepare(z2z_ctx* c);   // z2z_create: look up the static array's address on c->device
int z2z_launch_extended_sample(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                               const void* W_hyper, float temperature, int32_t top_k, float top_p, uint64_t seed,
                               uint64_t step, int32_t* token, float* logprob, hipStream_t s);
int z2z_sample_truncated_prepare(z2z_ctx* c);
int z2z_launch_extended_nll_backward(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                                     const void* W_hyper, const int32_t* targets, const float* lse,
                                     const float* grad_nll, void* dH, void* dW_base, void* dW_hyper, hipStream_t s);
int z2z_launch_hyper_embed_backward(z2z_ctx* c, const void* dW_hyper, float* dE, hipStream_t s);
bool z2z_hyper_encode_ok(const z2z_ctx* c, const z2z_encoder* enc);
int z2z_launch_hyper_encode(z2z_ctx* c, const void* E, const z2z_encoder* enc, void* W_hyper, const int32_t* first,
                            int32_t max_new, hipStream_t s);
int z2z_launch_hyper_encode_train(z2z_ctx* c, int mode, const void* E, const z2z_encoder* enc, void* W_hyper,
                                  const void* dW_hyper, const z2z_encoder* grad, float* dE, hipStream_t s);
int z2z_launch_extended_nll(z2z_ctx* c, const void* H, int32_t rows, int32_t rows_per_seq, const void* W_base,
                            const void* W_hyper, const int32_t* targets, float* nll, float* lse, hipStream_t s);

// A work buffer that has to grow is freed and allocated again (hipFree / hipMalloc: the device synchronises that
// once).  A stream capture does not survive that, so under capture the call is refused instead, before anything
// is freed: the caller makes one eager call at the shape first.
inline int z2z_can_allocate(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) return Z2Z_EHIP;
  return st == hipStreamCaptureStatusNone ? Z2Z_OK : Z2Z_ECAPTURE;
}
#define Z2Z_TRY_GROW(s)                        \
  do {                                         \
    int _g = z2z_can_allocate(s);              \
    if (_g != Z2Z_OK) return _g;               \
  } while (0)

#define Z2Z_HIP_TRY(expr)                      \
  do {                                         \
    hipError_t _e = (expr);                    \
    if (_e != hipSuccess) return Z2Z_EHIP;     \
  } while (0)
