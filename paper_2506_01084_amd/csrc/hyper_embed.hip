// hyper_embed for gfx950: one wavefront per codebook entry, coalesced 16-byte row gathers.
//
// Section 2.2 of the zip2zip paper builds a hypertoken's vector from the embeddings of its
// constituent base tokens, padded to M slots; this is the parameter-free pooling of the
// hyper-encoder ablation ("Averaging"): padding contributes nothing and the divisor is the entry's
// own length.  The work is a gather of L rows of E plus one row written: bound by HBM bandwidth
// (popular rows are served by L2 / the memory-side cache).  Each lane owns 16-byte column chunks:
// a wave reads 1 KiB of a row per instruction, accumulates in fp32 in token order, and rounds once
// (nearest-even) to the storage type.
#include "hyper_embed_common.h"

namespace {

using namespace z2z_embed;

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
  fill_embed_args(c, E, W_hyper, &a);
  a.first = first;
  a.last_n = (!first && max_new > 0) ? max_new : 0;
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
