/*
 * z2z.h -- C ABI of the zip2zip dynamic-vocabulary hot path for AMD MI355X (gfx950).
 *
 * The operations follow the paper's statement of the method (arxiv 2506.01084):
 *   lzw_encode       section 2.1 "LZW Algorithm"; section 2.3 step 2 (compress base tokens to hypertokens)
 *   lzw_decode       section 2.1 property (2) "self-contained"; section 2.3 steps 11-12 (decompress);
 *                    in append mode it is the per-step codebook update of steps 9-10
 *   hyper_embed      section 2.2 (hyper-encoder over the constituent base embeddings, padded to M);
 *                    "Averaging" row of the hyper-encoder ablation table; "Hyper-Embedding Cache"
 *   extended_logits  section 2.3 steps 7-9 (hyper rows appended to the LM head, joint softmax, pick)
 *   extended_sample  the same with the pick drawn from the softmax at a temperature (step 9)
 *   extended_nll     section 2.4 (next-token objective over compressed sequences): -log p(target) per row
 *
 * Conventions
 *   - Every pointer named d_* is DEVICE memory owned by the caller; it must stay valid until the
 *     work enqueued on `stream` has finished.  Pointers without the prefix are host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     and return without synchronising, except z2z_create / z2z_destroy.
 *   - One context serves B independent sequences (section 2.4: each document is compressed on its
 *     own).  The context owns each sequence's codebook; all calls read the same codebook,
 *     so the embedding side and the unembedding side always see the same hypertoken set
 *     (section 2.3, "Consistent Vocabulary Updates").
 *   - IDs: 0..V-1 are base tokens; V+i is codebook entry i of that sequence, in creation order.
 *   - Return value: 0 on success, a negative Z2Z_E* code when an argument is rejected on the host
 *     (nothing is enqueued then).  Data errors are reported per sequence in d_status (bit flags);
 *     a sequence with an error stops at the offending element, the others are unaffected.
 *   - Work buffers.  Some calls keep library-owned work space in the context (the partial reductions of
 *     extended_logits / extended_sample, the stored logits of filtered sampling, the learned encoder's
 *     activations, the backward passes' work space).  Each is allocated by the first call that needs it and
 *     grows when a later call needs more: such a call frees and allocates on the device (hipFree / hipMalloc,
 *     which synchronise the device that once) before it enqueues; every other call only enqueues.  While
 *     `stream` is being captured into a graph a buffer cannot grow: the call returns Z2Z_ECAPTURE and
 *     enqueues nothing -- make one eager call at the same shape before capturing, or use
 *     z2z_extended_logits_static, which never allocates.
 *   - Calls on one context must be issued from one host thread at a time, and work of one context
 *     must be ordered (same stream, or synchronised by the caller).
 */
#ifndef Z2Z_H
#define Z2Z_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct z2z_ctx z2z_ctx;

enum { Z2Z_F32 = 0, Z2Z_BF16 = 1 };                 /* storage type of E, W_base, W_hyper, H        */
enum { Z2Z_POOL_MEAN = 0, Z2Z_POOL_WEIGHTED = 1 };  /* hyper_embed pooling kind                      */
enum { Z2Z_APPEND = 0, Z2Z_RESET = 1 };             /* lzw_* flags: continue, or empty codebook first */

enum {                                              /* host-side argument errors                      */
  Z2Z_OK = 0, Z2Z_EINVAL = -1, Z2Z_ENOMEM = -2, Z2Z_EHIP = -3, Z2Z_EUNSUPPORTED = -4,
  Z2Z_ELIMIT = -5,                                  /* beyond a fixed limit of an allocation-free call */
  Z2Z_ECAPTURE = -6                                 /* a work buffer would have to grow under stream capture */
};
enum {                                              /* per-sequence data status bits                  */
  Z2Z_ST_OK = 0,
  Z2Z_ST_BAD_TOKEN = 1,   /* base-token ID outside [0, V)                                            */
  Z2Z_ST_BAD_CODE = 2,    /* code that names no existing entry (a "non-existing hypertoken")          */
  Z2Z_ST_OVERFLOW = 4     /* output row too short for the result                                      */
};

#define Z2Z_MAX_M 8
#define Z2Z_MAX_CAP 65535

typedef struct {
  int32_t B;      /* sequences served by the context, >= 1                                            */
  int32_t V;      /* base vocabulary size, >= 1, V + cap <= 2^24 (else Z2Z_EUNSUPPORTED)              */
  int32_t M;      /* maximum merge size (base tokens per hypertoken), 1..Z2Z_MAX_M                    */
  int32_t cap;    /* codebook capacity per sequence, 0..Z2Z_MAX_CAP; a full codebook is frozen        */
  int32_t d;      /* embedding width, multiple of 8 (bf16) or 4 (f32)                                 */
  int32_t dtype;  /* Z2Z_F32 or Z2Z_BF16                                                              */
  int32_t pool;   /* Z2Z_POOL_MEAN or Z2Z_POOL_WEIGHTED                                               */
  float w[Z2Z_MAX_M]; /* WEIGHTED: raw position weights; an entry of length L uses softmax(w[0..L))   */
} z2z_config;

/* Create / destroy a context on the current HIP device.  Allocates the codebook storage
 * (about cap * (4*M + 20) bytes per sequence) and empties it.  Synchronous. */
int z2z_create(z2z_ctx** out, const z2z_config* cfg);
int z2z_destroy(z2z_ctx* ctx);

/* Empty all codebooks and forget the previous phrase of every sequence. */
int z2z_reset(z2z_ctx* ctx, void* stream);

/* lzw_encode.  Greedy longest-match parse of each sequence against its growing codebook:
 * a match is extended while phrase+next token is an entry and the phrase is shorter than M; when
 * it ends its ID is emitted and phrase+next token becomes entry number C (if it spans <= M tokens
 * and C < cap).  The last phrase of the call is emitted too (adding nothing).  With Z2Z_APPEND the
 * codebook continues from earlier calls, and the entry "last emitted phrase + first token of this
 * call" is added first if it is legal and not present yet (what a decoder of the joined code
 * stream would add).
 *   d_tokens  [B, stride] int32, row b holds d_lens[b] valid IDs (d_lens NULL: every row has `stride`)
 *   d_codes   [B, out_stride] int32 out; d_n_codes [B] int32 out (number of codes written)
 *   d_status  [B] int32 out (Z2Z_ST_* bits); BAD_TOKEN ends the sequence just before that token
 */
int z2z_lzw_encode(z2z_ctx* ctx, const int32_t* d_tokens, const int32_t* d_lens, int32_t stride,
                   int32_t flags, int32_t* d_codes, int32_t* d_n_codes, int32_t out_stride,
                   int32_t* d_status, void* stream);

/* lzw_decode.  Inverse of lzw_encode; rebuilds the same codebook from the codes alone.  For each
 * code: resolve its phrase (base token, existing entry, or the one not-yet-defined entry textbook
 * LZW allows: previous phrase + its own first token); then add "previous phrase + first token of
 * this phrase" as entry C if the previous phrase is shorter than M, C < cap, and that phrase is
 * not an entry already.  With Z2Z_APPEND and one code per sequence this is the decode-step update
 * (at most one new entry per sequence per step).
 *   d_codes   [B, stride] int32, d_n_codes [B] (NULL: every row has `stride`)
 *   d_tokens  [B, out_stride] int32 out (may be NULL with out_stride 0: only update the codebook;
 *             nothing is written and OVERFLOW is not raised); d_n_tokens [B] out (tokens produced)
 *   d_status  [B] out; BAD_CODE / OVERFLOW end the sequence before the offending code
 */
int z2z_lzw_decode(z2z_ctx* ctx, const int32_t* d_codes, const int32_t* d_n_codes, int32_t stride,
                   int32_t flags, int32_t* d_tokens, int32_t* d_n_tokens, int32_t out_stride,
                   int32_t* d_status, void* stream);

/* Borrowed read-only device views of the codebooks, valid until z2z_destroy:
 *   entries   [B, cap, M] int32, the flattened base tokens of each entry, padded with -1
 *   entry_len [B, cap]    int32 (0 for unused slots)
 *   size      [B]         int32 C_b, the number of entries
 * Any of the three out-pointers may be NULL. */
int z2z_codebook(z2z_ctx* ctx, const int32_t** d_entries, const int32_t** d_entry_len,
                 const int32_t** d_size);

/* The codebook side of one generation step in one launch (section 2.3, steps 9-10: the sampled code extends
 * the codebook; "Hyper-Embedding Cache": only the new hypertoken's vector is computed).  Exactly
 *   z2z_lzw_decode(ctx, d_codes, d_ones, stride, Z2Z_APPEND, NULL, d_n_tokens, 0, d_status, stream) with d_ones = 1
 *   for every sequence (ONE code each: the code of sequence b is d_codes[b * stride]), followed by
 *   z2z_hyper_embed(ctx, d_E, d_W_hyper, NULL, 1, stream)
 * with the same results bit for bit: the codebook update of the step, then the newest entry's row of the
 * hyper-embedding cache (recomputed also when the step added no entry; nothing is written when the codebook is
 * empty).  A decode loop saves a launch per step with it.
 *   d_codes [B, stride] int32 (column 0 is read); d_n_tokens [B], d_status [B] out as for z2z_lzw_decode */
int z2z_step_update(z2z_ctx* ctx, const int32_t* d_codes, int32_t stride, const void* d_E, void* d_W_hyper,
                    int32_t* d_n_tokens, int32_t* d_status, void* stream);

/* Instrumentation: a borrowed device view [B] int32 of how many rounds the latest z2z_lzw_encode or
 * z2z_lzw_decode call took for each sequence.  The parse kernels (section 2.1's sequential loop, restructured)
 * take the elements of a sequence in rounds of up to 64 (one wave) or 256 (four waves) and cut a round at the
 * first element that depends on an entry made inside it; the serial chain of a call is its rounds, so
 * kernel time / rounds is the latency the parse is bound by.  Valid until z2z_destroy. */
int z2z_lzw_rounds(z2z_ctx* ctx, const int32_t** d_rounds);

/* Codebook prefilling (the paper's discussion, "Codebook Management Strategy", item 2: seeding the codebook
 * with phrases expected to occur, ahead of the input).  The paper names the idea only; the operation here:
 * phrase i of sequence b becomes entry C_b (ID V + C_b) if it has 2..M tokens, all in [0, V), its prefix
 * without the last token is a base token or an entry already (the codebook stays prefix-closed, which the
 * parse relies on), it is not an entry yet, and the codebook is not full.  The first phrase that fails ends
 * that sequence's prefill: BAD_TOKEN (length or token out of range), BAD_CODE (prefix unknown, or a
 * duplicate), OVERFLOW (codebook full); entries added before it stay.  Afterwards no phrase is pending:
 * z2z_lzw_encode / z2z_lzw_decode continue with Z2Z_APPEND, and both sides of a round trip must prefill alike.
 *   d_phrases    [B, n_max, M] int32 (tokens beyond a phrase's length are ignored)
 *   d_phrase_len [B, n_max] int32;  d_counts [B] int32 or NULL (= n_max phrases for every sequence)
 *   flags        Z2Z_RESET: start from empty codebooks; Z2Z_APPEND: add to what is there
 *   d_n_added    [B] int32 out;  d_status [B] int32 out */
int z2z_codebook_prefill(z2z_ctx* ctx, const int32_t* d_phrases, const int32_t* d_phrase_len,
                         const int32_t* d_counts, int32_t n_max, int32_t flags, int32_t* d_n_added,
                         int32_t* d_status, void* stream);

/* Entry usage: d_usage[b, e] += the number of codes of sequence b's stream that name entry e (the statistic
 * behind the paper's remark that only about a quarter of the hypertokens are reused; what a retention policy
 * looks at).  d_codes [B, stride], d_n_codes [B] or NULL, d_usage [B, cap] int32, accumulated (zero it first). */
int z2z_codebook_usage(z2z_ctx* ctx, const int32_t* d_codes, const int32_t* d_n_codes, int32_t stride,
                       int32_t* d_usage, void* stream);

/* Pruning / selective retention (the paper's discussion, "Codebook Management Strategy", item 1; the idea is
 * named, no rule is given).  The operation here: entry e of sequence b stays iff d_keep[b, e] != 0 and its
 * prefix without the last token is a base token or an entry that stays (the codebook remains prefix-closed:
 * dropping an entry drops its extensions).  The survivors keep their order and are renumbered from V; no phrase
 * is pending afterwards.  Codes emitted before the call name the old numbering: d_new_id maps them.  Both sides
 * of a round trip must prune alike, and the hyper-embedding cache has to be rebuilt (z2z_hyper_embed).
 *   d_keep   [B, cap] int32 (entries at and beyond C_b are ignored)
 *   d_new_id [B, cap] int32 out: new entry index of old entry e, -1 = dropped (entries beyond C_b: untouched)
 *   d_n_kept [B] int32 out: the new C_b */
int z2z_codebook_prune(z2z_ctx* ctx, const int32_t* d_keep, int32_t* d_new_id, int32_t* d_n_kept, void* stream);

/* hyper_embed.  W_hyper[b, e, :] = sum_j a_j * E[t_j, :] over the L tokens of entry e of sequence b,
 * a_j = 1/L (MEAN) or softmax(w[0..L))_j (WEIGHTED); padding slots contribute nothing and are not
 * in the divisor.  fp32 accumulation in token order, one round-to-nearest-even to the storage type.
 *   d_E       [V, d]       dtype of the context
 *   d_W_hyper [B, cap, d]  same dtype, out.  This buffer is the hyper-embedding cache.
 *   d_first   [B] int32 or NULL, and max_new, select the rows to (re)compute:
 *             NULL, max_new <= 0: entries [0, C_b), and rows [C_b, cap) are zeroed;
 *             NULL, max_new >= 1: the last max_new entries [max(C_b - max_new, 0), C_b) only, all other
 *                                 rows untouched (recomputing a row gives the same bits, so a decode loop
 *                                 that adds at most one entry per step keeps the cache current with
 *                                 max_new = 1 and no snapshot of the sizes);
 *             non-NULL:           entries [d_first[b], C_b) only, all other rows untouched; max_new is
 *                                 an upper bound the caller expects for C_b - d_first[b] (it sizes the
 *                                 launch; any value >= 1 is correct, a tight one is faster, <= 0 = cap).
 */
int z2z_hyper_embed(z2z_ctx* ctx, const void* d_E, void* d_W_hyper, const int32_t* d_first,
                    int32_t max_new, void* stream);

/* hyper_encode: the learned hyper-encoder f_phi of section 2.2 (the attention and transformer rows of the
 * hyper-encoder ablation table; the training setup uses two transformer layers, M = 3).  The paper names the
 * architectures only; computed here is the standard pre-norm encoder over an entry's M padded slots:
 *   X_i = E[y_i] + pos[i]                                   (real slots i < L; pos may be NULL)
 *   A = LayerNorm(X; ln1);  q|k|v = A w_qkv^T + b_qkv;  per head: O = softmax(q k^T / sqrt(d / n_heads)) v,
 *   padding slots masked out as keys;  Y = X + O w_o^T + b_o                       (an attention layer)
 *   Z = Y + GELU(LayerNorm(Y; ln2) w_1^T + b_1) w_2^T + b_2   (GELU with erf)      (a transformer layer)
 *   W_hyper[b, e, :] = mean over the real slots of the last layer's output.
 * LayerNorm: over the d features, biased variance, eps = 1e-5.  Matrices are bf16 [out, in] row-major, vectors
 * float; every pointer is a device pointer, 16-byte aligned, borrowed for the call; the structs themselves
 * are host memory.  Activations between the layers' steps are rounded to bf16, sums are fp32.
 *   d_E, d_W_hyper, d_first, max_new: as for z2z_hyper_embed, except that with d_first the entries
 *   [d_first[b], min(C_b, d_first[b] + max_new)) are computed (max_new <= 0: up to cap).
 * Requires a bf16 context, d a multiple of 64 and at most 4096, d / n_heads a power of two in [8, 512], d_ff a
 * multiple of 64, 1 <= n_layers <= Z2Z_MAX_ENCODER_LAYERS; anything else returns Z2Z_EUNSUPPORTED or
 * Z2Z_EINVAL.  Work space (activations of up to 65536 slot rows) is library scratch, allocated by the first
 * call at a size. */
#define Z2Z_MAX_ENCODER_LAYERS 8
typedef struct z2z_encoder_layer {
  const float* ln1_g;   /* [d]  */
  const float* ln1_b;   /* [d]  */
  const void* w_qkv;    /* [3d, d]: rows 0..d-1 query, d..2d-1 key, 2d..3d-1 value projections */
  const float* b_qkv;   /* [3d] */
  const void* w_o;      /* [d, d] */
  const float* b_o;     /* [d]  */
  const float* ln2_g;   /* [d]      transformer layers only (ignored when attention_only) */
  const float* ln2_b;   /* [d]      */
  const void* w_1;      /* [d_ff, d] */
  const float* b_1;     /* [d_ff]   */
  const void* w_2;      /* [d, d_ff] */
  const float* b_2;     /* [d]      */
} z2z_encoder_layer;
typedef struct z2z_encoder {
  int32_t n_layers;
  int32_t n_heads;
  int32_t d_ff;             /* width of the feed-forward block (ignored when attention_only) */
  int32_t attention_only;   /* 1: every layer is the attention layer alone */
  const void* pos;          /* [M, d] bf16 learned slot positions, or NULL */
  const z2z_encoder_layer* layers;   /* host array of n_layers */
} z2z_encoder;
int z2z_hyper_encode(z2z_ctx* ctx, const void* d_E, const z2z_encoder* encoder, void* d_W_hyper,
                     const int32_t* d_first, int32_t max_new, void* stream);

/* Backward of z2z_hyper_encode over ALL existing entries (training f_phi, section 2.4: the loss over the
 * compressed sequence reaches the hyper-encoder through every hypertoken vector): the gradient of
 *   L = sum_{b, e < C_b, k} d_dW_hyper[b, e, k] * W_hyper[b, e, k]
 * with respect to every parameter of the encoder, the slot positions and the embedding rows.
 *   d_dW_hyper [B, cap, d] bf16: dL / dW_hyper (e.g. from z2z_extended_nll_backward); rows >= C_b are ignored
 *   grad       a second description with the shape of `encoder` whose pointers name the device buffers that
 *              RECEIVE the gradients (the call writes through them although the struct declares them const):
 *              matrices and pos bf16, vectors float, all overwritten; n_heads, d_ff, attention_only of `grad`
 *              are not read; grad->pos is required when encoder->pos is given
 *   d_dE       [V, d] float, ACCUMULATED into (tokens recur across entries; the caller clears it)
 *   flags      0, or Z2Z_ENC_KEPT: use the rows the latest z2z_hyper_encode_keep call on this context left
 *              instead of running the forward pass again.  The caller guarantees that d_E's contents and the
 *              encoder's parameters are unchanged since that call; the library checks that such a call was the
 *              context's latest use of this work space, with the same d_E and an encoder of the same shape, and
 *              that no call that can change a codebook (lzw_encode / lzw_decode / reset / prefill / prune) was
 *              made since (else Z2Z_EINVAL).  A backward call consumes the kept rows.
 * Without the flag the call runs the forward pass again, keeping every layer's rows, then reverse mode over the
 * same steps; activations and gradients between kernels are bf16, sums fp32; passes of up to 65536 slot rows
 * (matrix gradients of later passes add to the bf16 result of the earlier ones).  Work space (about
 * 2 * (n_layers * (8 d + 2 d_ff) + 8 d + d_ff + 2 max(3 d, d_ff)) bytes per slot row) is library scratch,
 * Z2Z_ENOMEM beyond 200 GB.  Restrictions and errors as for z2z_hyper_encode. */
#define Z2Z_ENC_KEPT 1
int z2z_hyper_encode_backward(z2z_ctx* ctx, const void* d_E, const z2z_encoder* encoder, const void* d_dW_hyper,
                              const z2z_encoder* grad, float* d_dE, int32_t flags, void* stream);

/* z2z_hyper_encode over all entries (d_first = NULL, max_new = 0) for a training step: same network, and the rows
 * of every layer stay in the work space of z2z_hyper_encode_backward, whose Z2Z_ENC_KEPT flag then skips the
 * forward pass (a third of its time).  The feed-forward pre-activation is rounded to bf16 before the GELU here
 * (it is kept for the slope), so results can differ from z2z_hyper_encode's in the last bf16 bit.  Needs all
 * slot rows in one pass: B * cap * M <= 65536, else Z2Z_EUNSUPPORTED.  Other restrictions, errors and the work
 * space as for z2z_hyper_encode_backward. */
int z2z_hyper_encode_keep(z2z_ctx* ctx, const void* d_E, const z2z_encoder* encoder, void* d_W_hyper, void* stream);

/* extended_logits.  For row r of sequence b = r / rows_per_seq:
 *   logit[r, v] = sum_k H[r,k] * W[v,k],  W = W_base for v < V, W_hyper[b, v-V] for V <= v < V + C_b;
 * slots at and beyond C_b are not columns (never predicted).  Products of the stored values,
 * fp32 accumulation.  Per row the joint softmax is reduced on the fly to
 *   d_argmax[r] (lowest index among equal maxima), d_max[r], d_lse[r] = ln sum_v exp(logit[r,v]).
 *   d_H [rows, d]; rows must be B * rows_per_seq; d_W_base [V, d]; d_W_hyper [B, cap, d]
 *   d_logits  NULL, or [rows, V + cap] float32 out: the full logits, -inf in unused slots
 *             (for small shapes only: the reduction above never needs it).
 * The partial reductions go through a work buffer of the context (see "Work buffers" above: it grows when a
 * call needs more than any earlier one, Z2Z_ECAPTURE if that happens under stream capture).
 */
int z2z_extended_logits(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                        const void* d_W_base, const void* d_W_hyper, int32_t* d_argmax, float* d_max,
                        float* d_lse, float* d_logits, void* stream);

/* z2z_extended_logits for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results;
 * the difference is where the partial reductions go: into a static device array of the library
 * (3 * Z2Z_STATIC_PARTS * 4 bytes = 48 MiB, held by every GPU the library runs on until the process ends)
 * instead of the context's growable buffer.  The call allocates and frees nothing, on the device or through
 * any library.  A call needs parts * rows elements, parts = strips of the base vocabulary + strips (or units)
 * of the hyper vocabulary as the launch plan cuts them (one decode step at V = 128256, cap = 4096, 64
 * sequences: 509 * 64; a prefill of 32768 rows at V = 128256, cap = 2048: 128 * 32768 = Z2Z_STATIC_PARTS);
 * a call that needs more returns Z2Z_ELIMIT and enqueues nothing.  Nothing in the array has to start at zero
 * (every element a call reads it has written before).  All contexts on one GPU share that GPU's array: calls
 * that may overlap in time on one GPU (different streams, different contexts) race -- order them. */
#define Z2Z_STATIC_PARTS (1 << 22)
int z2z_extended_logits_static(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                               const void* d_W_base, const void* d_W_hyper, int32_t* d_argmax, float* d_max,
                               float* d_lse, float* d_logits, void* stream);

/* extended_sample.  The generation step's pick when it is a draw rather than the maximum (section 2.3,
 * steps 8-9: the next token comes from the joint distribution over base tokens and hypertokens):
 *   d_token[r] ~ softmax(logit[r, :] / temperature), over the same columns as z2z_extended_logits.
 * Gumbel-max: d_token[r] = argmax_v (logit[r, v] / temperature - ln(-ln u[r, v])) (lowest v among equal
 * maxima), which has exactly that distribution.  u[r, v] is a pure function of (seed, step, r, v): word
 * v & 3 of Philox4x32-10 (Salmon et al., SC'11) with counter (v >> 2, r, step low, step high) and key
 * (seed low, seed high), u = ((word >> 9) + 0.5) * 2^-23.  The same (seed, step) gives the same draws; a
 * generation loop passes its step number.
 * Filters (the usual top-k / nucleus truncation): order the columns by logit, largest first, equal logits by
 * lower column; with q = softmax(logit / temperature) over all existing columns keep the first
 * n = min(top_k, n_p) columns, n_p the smallest prefix whose q sums to at least top_p (both filters look at the
 * full distribution; at least one column is kept); the draw is the same argmax restricted to the kept
 * columns, i.e. a draw from q renormalised on them.  top_k <= 0 and top_p >= 1 switch a filter off; with both
 * off nothing is stored, otherwise the rows' scaled logits go through rows * (V + cap) floats of library
 * scratch (allocated by the first such call at a size: make one call before capturing into a graph).
 *   d_token   [rows] int32 out
 *   d_logprob [rows] float out or NULL: ln of the drawn token's probability under the (renormalised)
 *             distribution it was drawn from
 *   temperature  > 0 and finite, top_p > 0 (else Z2Z_EINVAL)
 * Built for the generation step: rows_per_seq must be 1 and the context bf16 with d a multiple of 128 and
 * d <= 4096; anything else returns Z2Z_EUNSUPPORTED.  Scratch as for z2z_extended_logits.
 */
int z2z_extended_sample(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                        const void* d_W_base, const void* d_W_hyper, float temperature, int32_t top_k,
                        float top_p, uint64_t seed, uint64_t step, int32_t* d_token, float* d_logprob,
                        void* stream);

/* extended_nll.  The per-position term of the training objective over compressed sequences (section 2.4,
 * the next-token loss on z = LZW(y)): for hidden row r with target code t = d_targets[r],
 *   d_nll[r] = d_lse[r] - logit[r, t],   d_lse[r] = ln sum_v exp(logit[r, v])
 * over the same columns as z2z_extended_logits.  t < V is a base token, V <= t < V + C_b entry t - V of the
 * row's sequence; t < 0 marks a position without a target (d_nll = 0); a t that names no existing column
 * has probability zero (d_nll = +inf).  Any shape and storage type z2z_extended_logits takes.
 *   d_targets [rows] int32; d_nll [rows] float out; d_lse [rows] float out (both required)
 */
int z2z_extended_nll(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                     const void* d_W_base, const void* d_W_hyper, const int32_t* d_targets, float* d_nll,
                     float* d_lse, void* stream);

/* Backward of z2z_extended_nll (the training objective of section 2.4, second displayed equation, over the
 * compressed sequence): the gradient of  L = sum_r grad_nll[r] * nll[r]  with respect to the hidden rows and
 * both unembedding matrices.  With p = softmax(logit[r, :]) over the existing columns and t = target[r],
 *   dZ[r, v] = grad_nll[r] * (p[v] - [v == t]);   dH = dZ [W_base ; W_hyper[b]];   dW_base = dZ[:, :V]^T H;
 *   dW_hyper[b] = dZ[rows of b, V:]^T H[rows of b]   (rows at and beyond C_b: 0).
 * Rows without a target (t < 0) and rows whose target names no existing column contribute nothing.
 *   d_lse      [rows] float: the log-sum-exp z2z_extended_nll returned for the same inputs
 *   d_grad_nll [rows] float or NULL (= 1 for every row)
 *   d_dH [rows, d], d_dW_base [V, d], d_dW_hyper [B, cap, d]: out, bf16 (overwritten, not accumulated)
 * dZ is rounded to bf16 once and the four products accumulate in fp32.  bf16 contexts with d a multiple of 64;
 * anything else returns Z2Z_EUNSUPPORTED.  Work space: 2 * rows * (V + cap) bf16 for dZ and its transpose plus
 * one transposed copy of H, W_base and W_hyper, library scratch.  Beyond 200 GB the sequences go in chunks (halved
 * until a chunk fits; dW_base of a later chunk adds to the bf16 result of the earlier ones); Z2Z_ENOMEM if one
 * sequence alone does not fit. */
int z2z_extended_nll_backward(z2z_ctx* ctx, const void* d_H, int32_t rows, int32_t rows_per_seq,
                              const void* d_W_base, const void* d_W_hyper, const int32_t* d_targets,
                              const float* d_lse, const float* d_grad_nll, void* d_dH, void* d_dW_base,
                              void* d_dW_hyper, void* stream);

/* Backward of z2z_hyper_embed (the pooling is linear in E):  dE[t_j, :] += a_j * dW_hyper[b, e, :]  for every
 * token t_j of every existing entry, with the coefficients a_j of the forward pass.
 *   d_dW_hyper [B, cap, d] bf16;  d_dE [V, d] float, ACCUMULATED into (zero it first for the plain gradient).
 * Float atomics: the order of the additions, and so the last bits, vary from run to run.  bf16 contexts. */
int z2z_hyper_embed_backward(z2z_ctx* ctx, const void* d_dW_hyper, float* d_dE, void* stream);

/* Tuning knobs (kernel variants and tile schedule) and instrumentation; unknown keys return
 * Z2Z_EINVAL. */
enum {
  Z2Z_OPT_LOGITS_KERNEL = 1,   /* 0 = automatic; 1 = the general tile kernel everywhere; 2, 3 = MEASUREMENT
                                  PROBES of the bf16 MFMA tile kernel's base part, whose outputs are not the
                                  logits' reduction: 2 = no operand requests after the first two K slabs,
                                  3 = the MFMA stream alone (no requests, no LDS reads, one fold per strip);
                                  4 = the bf16 MFMA tile kernel also for the base part of calls with at most
                                  192 hidden rows, which otherwise goes to the weight-streaming kernel */
  Z2Z_OPT_LOGITS_STRIP = 2,    /* vocabulary tiles swept per workgroup, 0 = automatic               */
  Z2Z_OPT_LZW_KERNEL = 3,      /* 0 = automatic, >0 = force a variant (2: table in global memory, 3: one
                                  code per step in the decoder, 4: one wave per sequence in the encoder) */
  Z2Z_OPT_DECODE_KERNEL = 4,   /* 0 = automatic, >0 = force a variant                               */
  Z2Z_OPT_LOGITS_MAP = 6,      /* workgroup -> tile order of the bf16 MFMA kernel's base part, packed
                                  lr | ls << 8 | xr << 16 | xs << 24: each of the 8 XCDs walks blocks of
                                  lr row tiles x ls strips, the XCDs' blocks lie xr x xs (xr * xs = 8)
                                  inside one super block; 0 = automatic                              */
  Z2Z_OPT_SAMPLE_KERNEL = 7,   /* filtered sampling: 0 = automatic, 1 = always select the kept prefix by
                                  passes over the whole row (no short list from the largest parts)   */
  Z2Z_OPT_BACKWARD_CHUNK = 8,  /* z2z_extended_nll_backward: at most this many sequences per pass, 0 = as many as
                                  the 200 GB work-space limit allows                                  */
  Z2Z_OPT_TIMING = 5           /* 1 = bracket the dominant kernel of every z2z_extended_logits call
                                  with HIP events on the call's stream (at most 1024 calls are kept
                                  between two z2z_read_timing calls); 0 = off (default)             */
};
int z2z_set_option(z2z_ctx* ctx, int32_t key, int32_t value);

/* Sum of the event-measured durations (milliseconds) of the dominant extended_logits kernel over
 * the calls made since the last read, and their number.  Synchronises on the recorded events and
 * clears the record.  `total_ms` / `launches` are host pointers. */
int z2z_read_timing(z2z_ctx* ctx, float* total_ms, int32_t* launches);

/* Instrumentation: how many launches of each logits kernel family this context has enqueued since it
 * was created (host-side counters; nothing is read from the device).  Tests use it to make sure that a
 * call ran on the kernel they mean to check; a profile can be matched against it.
 *   counts[Z2Z_KERNEL_TILE_BASE]   bf16 MFMA tile kernel, base-vocabulary launches (any epilogue)
 *   counts[Z2Z_KERNEL_TILE_HYPER]  bf16 MFMA tile kernel, per-sequence hyper-vocabulary launches
 *   counts[Z2Z_KERNEL_GENERAL]     the general tile kernel (fp32, d not a multiple of 64, full logits)
 *   counts[Z2Z_KERNEL_DECODE]      the one-row-per-sequence (bandwidth-bound) kernel
 *   counts[Z2Z_KERNEL_MID]         the weight-streaming kernel for the base part of calls with up to 192 hidden rows
 * `counts` is a host array of Z2Z_N_KERNEL_FAMILIES elements. */
enum { Z2Z_KERNEL_TILE_BASE = 0, Z2Z_KERNEL_TILE_HYPER = 1, Z2Z_KERNEL_GENERAL = 2, Z2Z_KERNEL_DECODE = 3,
       Z2Z_KERNEL_MID = 4, Z2Z_N_KERNEL_FAMILIES = 5 };
int z2z_read_launches(const z2z_ctx* ctx, int64_t* counts);

const char* z2z_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* Z2Z_H */
