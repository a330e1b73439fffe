// Batched token-level LZW for gfx950: one wavefront (64 lanes) per sequence.
//
// The parse of one sequence is a serial dependency chain (section 2.1 of the zip2zip paper: every
// step looks up "current phrase + next token" in the codebook built so far), so the unit of
// parallelism is the sequence.  The codebook is a trie stored as a hash table over its edges
// (parent code, token) -> entry index.  The wave keeps the hash slots -- and, when they fit, the
// edge keys -- of its sequence in LDS for the whole call; tokens are read 64 at a time with one
// coalesced load and handed out with readlane; emitted codes are collected in a lane-distributed
// register and written 64 at a time.  All control flow is wave-uniform.
#include "z2z_internal.h"

namespace {

constexpr int kWave = 64;

struct LzwArgs {
  LzwState st;
  const int32_t* in;       // tokens (encode) or codes (decode), [B, stride]
  const int32_t* in_len;   // [B] or nullptr
  int32_t stride;
  int32_t flags;
  int32_t* out;            // codes (encode) or tokens (decode), [B, out_stride]
  int32_t* out_n;          // [B]
  int32_t out_stride;
  int32_t* status;         // [B]
  int32_t lds_slots;       // 1: hash slots live in LDS during the call
  int32_t lds_keys;        // 1: edge keys live in LDS during the call
};

__device__ __forceinline__ uint32_t edge_hash(int32_t parent, int32_t tok) {
  uint32_t h = (uint32_t)parent * 0x9E3779B1u + (uint32_t)tok * 0x85EBCA77u;
  h ^= h >> 15;
  h *= 0x2C1B3C6Du;
  h ^= h >> 12;
  h *= 0x297A2D39u;
  h ^= h >> 15;
  return h;
}

__device__ __forceinline__ unsigned long long edge_key(int32_t parent, int32_t tok) {
  return ((unsigned long long)(uint32_t)parent << 32) | (unsigned long long)(uint32_t)tok;
}

struct Table {
  uint16_t* slots;             // LDS or global (generic pointer)
  unsigned long long* keys;    // LDS or global (generic pointer)
  uint32_t mask;
};

// Linear probing.  Returns the entry index, or -1 with *free_pos = the empty slot the probe ended
// at (-1 if the table has no empty slot, which cannot happen while nslots >= 2*cap).
__device__ __forceinline__ int table_find(const Table& t, int32_t parent, int32_t tok, int* free_pos) {
  const unsigned long long key = edge_key(parent, tok);
  uint32_t pos = edge_hash(parent, tok) & t.mask;
  for (uint32_t probe = 0; probe <= t.mask; ++probe) {
    // every lane reads the same address; readfirstlane keeps the chain in scalar registers
    const uint32_t s = __builtin_amdgcn_readfirstlane((uint32_t)t.slots[pos]);
    if (s == Z2Z_EMPTY_SLOT) {
      *free_pos = (int)pos;
      return -1;
    }
    if (__builtin_amdgcn_readfirstlane((int)(t.keys[s] == key))) return (int)s;
    pos = (pos + 1) & t.mask;
  }
  *free_pos = -1;
  return -1;
}

// Shared set-up: bring the sequence's table into LDS (or clear it on RESET).
__device__ __forceinline__ void table_open(const LzwArgs& a, int b, int lane, unsigned char* smem, bool reset,
                                           int C, Table* t) {
  const LzwState& st = a.st;
  uint16_t* g_slots = st.slots + (size_t)b * st.nslots;
  unsigned long long* g_keys = st.keys + (size_t)b * st.cap;
  uint16_t* l_slots = reinterpret_cast<uint16_t*>(smem);
  unsigned long long* l_keys = reinterpret_cast<unsigned long long*>(smem + (size_t)st.nslots * sizeof(uint16_t));
  t->mask = (uint32_t)st.nslots - 1u;
  t->slots = a.lds_slots ? l_slots : g_slots;
  t->keys = a.lds_keys ? l_keys : g_keys;
  // nslots is a power of two >= 64, so the table is a whole number of 4-byte words
  uint32_t* dst32 = reinterpret_cast<uint32_t*>(t->slots);
  const int nwords = st.nslots / 2;
  if (reset) {
    for (int i = lane; i < nwords; i += kWave) dst32[i] = 0xFFFFFFFFu;
  } else {
    if (a.lds_slots) {
      const uint32_t* src32 = reinterpret_cast<const uint32_t*>(g_slots);
      for (int i = lane; i < nwords; i += kWave) dst32[i] = src32[i];
    }
    if (a.lds_keys) {
      for (int i = lane; i < C; i += kWave) l_keys[i] = g_keys[i];
    }
  }
  __syncthreads();
}

// Shared tear-down: write the LDS-resident parts back so that later calls see them.
__device__ __forceinline__ void table_close(const LzwArgs& a, int b, int lane, const Table& t, int C) {
  const LzwState& st = a.st;
  __syncthreads();
  if (a.lds_slots) {
    uint32_t* g32 = reinterpret_cast<uint32_t*>(st.slots + (size_t)b * st.nslots);
    const uint32_t* l32 = reinterpret_cast<const uint32_t*>(t.slots);
    for (int i = lane; i < st.nslots / 2; i += kWave) g32[i] = l32[i];
  }
  if (a.lds_keys) {
    unsigned long long* g_keys = st.keys + (size_t)b * st.cap;
    for (int i = lane; i < C; i += kWave) g_keys[i] = t.keys[i];
  }
}

// Add the edge (parent, tok) as entry C.  `ph` holds, in lane j, token j of the parent phrase
// (plen tokens); the new entry's flattened row is that phrase followed by tok.
__device__ __forceinline__ void table_insert(const LzwArgs& a, int b, int lane, const Table& t, int free_pos, int C,
                                             int32_t parent, int32_t tok, int32_t ph, int plen) {
  const LzwState& st = a.st;
  if (lane == 0) {
    t.slots[free_pos] = (uint16_t)C;
    t.keys[C] = edge_key(parent, tok);
    st.ent_len[(size_t)b * st.cap + C] = plen + 1;
  }
  if (lane < st.M) {
    const int32_t v = lane < plen ? ph : (lane == plen ? tok : -1);
    st.ent_tokens[((size_t)b * st.cap + C) * st.M + lane] = v;
  }
}

// ------------------------------------------------------------------------------------------------
// encode
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kWave) lzw_encode_kernel(LzwArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;

  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  int prev = reset ? -1 : __builtin_amdgcn_readfirstlane(st.prev_code[b]);
  int prev_len = reset ? 0 : __builtin_amdgcn_readfirstlane(st.prev_len[b]);

  Table t;
  table_open(a, b, lane, smem, reset, C, &t);

  // tokens of the previous phrase (lane j = token j), needed only for the first entry of an append
  int32_t ph = -1;
  if (prev >= 0) {
    if (prev < V) {
      ph = lane == 0 ? prev : -1;
    } else if (lane < M) {
      ph = st.ent_tokens[((size_t)b * cap + (prev - V)) * M + lane];
    }
  }

  const int n = a.in_len ? min(max(__builtin_amdgcn_readfirstlane(a.in_len[b]), 0), a.stride) : a.stride;
  const int32_t* in = a.in + (size_t)b * a.stride;
  int32_t* out = a.out + (size_t)b * a.out_stride;

  int status = 0;
  int w = -1, wlen = 0;      // current phrase: its code and its length (w < 0: none yet in this call)
  int n_out = 0;
  int32_t out_reg = 0;       // lane (n_out % 64) holds the code emitted at position n_out
  bool stop = false;

  for (int base = 0; base < n && !stop; base += kWave) {
    const int cnt = min(kWave, n - base);
    const int32_t tok_reg = lane < cnt ? in[base + lane] : 0;
    for (int j = 0; j < cnt; ++j) {
      const int32_t c = __builtin_amdgcn_readlane(tok_reg, j);
      if (c < 0 || c >= V) {
        status |= Z2Z_ST_BAD_TOKEN;
        stop = true;
        break;
      }
      int free_pos = -1;
      bool emit = false;
      if (w >= 0 && wlen < M) {
        const int idx = table_find(t, w, c, &free_pos);
        if (idx >= 0) {               // the match grows
          w = V + idx;
          if (lane == wlen) ph = c;
          ++wlen;
          continue;
        }
        emit = true;
      } else if (w >= 0) {            // phrase already has M tokens: it ends here, nothing is added
        emit = true;
      } else if (prev >= 0 && prev_len < M && C < cap) {
        // first token of an appended chunk: the entry the earlier flush could not add
        const int idx = table_find(t, prev, c, &free_pos);
        if (idx < 0 && free_pos >= 0) {
          table_insert(a, b, lane, t, free_pos, C, prev, c, ph, prev_len);
          ++C;
        }
      }
      if (emit) {
        if (n_out >= a.out_stride) {
          status |= Z2Z_ST_OVERFLOW;
          stop = true;
          w = -1;
          break;
        }
        if (lane == (n_out & (kWave - 1))) out_reg = w;
        ++n_out;
        if ((n_out & (kWave - 1)) == 0) out[n_out - kWave + lane] = out_reg;
        prev = w;
        prev_len = wlen;
        if (wlen < M && C < cap && free_pos >= 0) {
          table_insert(a, b, lane, t, free_pos, C, w, c, ph, wlen);
          ++C;
        }
      }
      w = c;
      wlen = 1;
      if (lane == 0) ph = c;
    }
  }
  if (w >= 0) {                       // flush the pending phrase; no entry is added
    if (n_out >= a.out_stride) {
      status |= Z2Z_ST_OVERFLOW;
    } else {
      if (lane == (n_out & (kWave - 1))) out_reg = w;
      ++n_out;
      if ((n_out & (kWave - 1)) == 0) out[n_out - kWave + lane] = out_reg;
      prev = w;
      prev_len = wlen;
    }
  }
  const int tail = n_out & (kWave - 1);
  if (tail != 0 && lane < tail) out[n_out - tail + lane] = out_reg;

  table_close(a, b, lane, t, C);
  if (lane == 0) {
    st.size[b] = C;
    st.prev_code[b] = prev;
    st.prev_len[b] = prev_len;
    a.out_n[b] = n_out;
    a.status[b] = status;
  }
}

// ------------------------------------------------------------------------------------------------
// decode
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kWave) lzw_decode_kernel(LzwArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;

  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  int prev = reset ? -1 : __builtin_amdgcn_readfirstlane(st.prev_code[b]);
  int prev_len = reset ? 0 : __builtin_amdgcn_readfirstlane(st.prev_len[b]);

  Table t;
  table_open(a, b, lane, smem, reset, C, &t);

  int32_t ph = -1;                    // tokens of the previous phrase, lane j = token j
  if (prev >= 0) {
    if (prev < V) {
      ph = lane == 0 ? prev : -1;
    } else if (lane < M) {
      ph = st.ent_tokens[((size_t)b * cap + (prev - V)) * M + lane];
    }
  }

  const int n = a.in_len ? min(max(__builtin_amdgcn_readfirstlane(a.in_len[b]), 0), a.stride) : a.stride;
  const int32_t* in = a.in + (size_t)b * a.stride;
  int32_t* out = a.out ? a.out + (size_t)b * a.out_stride : nullptr;

  int status = 0;
  int n_out = 0;
  bool stop = false;

  for (int base = 0; base < n && !stop; base += kWave) {
    const int cnt = min(kWave, n - base);
    const int32_t code_reg = lane < cnt ? in[base + lane] : 0;
    for (int j = 0; j < cnt; ++j) {
      const int32_t k = __builtin_amdgcn_readlane(code_reg, j);
      int32_t cur = -1;               // tokens of this code's phrase, lane j = token j
      int cur_len = 0;
      int free_pos = -1;
      bool looked_up = false;         // (prev, first) already probed and found absent
      if (k >= 0 && k < V) {
        cur = lane == 0 ? k : -1;
        cur_len = 1;
      } else if (k >= V && k - V < C) {
        if (lane < M) cur = st.ent_tokens[((size_t)b * cap + (k - V)) * M + lane];
        cur_len = __popcll(__ballot(cur >= 0));
      } else if (k >= V && k - V == C && prev >= 0 && prev_len < M && C < cap) {
        // the entry the encoder made in the step just before using it: previous phrase + its first token
        const int32_t pf = __builtin_amdgcn_readlane(ph, 0);
        const int idx = table_find(t, prev, pf, &free_pos);
        if (idx >= 0 || free_pos < 0) {
          status |= Z2Z_ST_BAD_CODE;
          stop = true;
          break;
        }
        cur = lane < prev_len ? ph : (lane == prev_len ? pf : -1);
        cur_len = prev_len + 1;
        looked_up = true;
      } else {
        status |= Z2Z_ST_BAD_CODE;
        stop = true;
        break;
      }
      if (out != nullptr && n_out + cur_len > a.out_stride) {
        status |= Z2Z_ST_OVERFLOW;
        stop = true;
        break;
      }
      const int32_t first = __builtin_amdgcn_readlane(cur, 0);
      if (prev >= 0 && prev_len < M && C < cap) {
        int idx = -1;
        if (!looked_up) idx = table_find(t, prev, first, &free_pos);
        if (idx < 0 && free_pos >= 0) {
          table_insert(a, b, lane, t, free_pos, C, prev, first, ph, prev_len);
          ++C;
        }
      }
      if (out != nullptr && lane < cur_len) out[n_out + lane] = cur;
      n_out += cur_len;
      prev = k;
      prev_len = cur_len;
      ph = cur;
    }
  }

  table_close(a, b, lane, t, C);
  if (lane == 0) {
    st.size[b] = C;
    st.prev_code[b] = prev;
    st.prev_len[b] = prev_len;
    a.out_n[b] = n_out;
    a.status[b] = status;
  }
}

// Empty every codebook.  grid = B, block = 256.
__global__ void lzw_reset_kernel(LzwState st) {
  const int b = blockIdx.x;
  uint32_t* s32 = reinterpret_cast<uint32_t*>(st.slots + (size_t)b * st.nslots);
  for (int i = threadIdx.x; i < st.nslots / 2; i += blockDim.x) s32[i] = 0xFFFFFFFFu;
  for (int i = threadIdx.x; i < st.cap; i += blockDim.x) st.ent_len[(size_t)b * st.cap + i] = 0;
  for (size_t i = threadIdx.x; i < (size_t)st.cap * st.M; i += blockDim.x)
    st.ent_tokens[(size_t)b * st.cap * st.M + i] = -1;
  if (threadIdx.x == 0) {
    st.size[b] = 0;
    st.prev_code[b] = -1;
    st.prev_len[b] = 0;
  }
}

// Clear the entry rows of a sequence that a RESET encode/decode is about to refill, so that rows
// at and beyond the new size read as unused.  grid = B, block = 256.
__global__ void lzw_clear_entries_kernel(LzwState st) {
  const int b = blockIdx.x;
  const int C = st.size[b];
  for (int i = threadIdx.x; i < C; i += blockDim.x) st.ent_len[(size_t)b * st.cap + i] = 0;
  for (size_t i = threadIdx.x; i < (size_t)C * st.M; i += blockDim.x)
    st.ent_tokens[(size_t)b * st.cap * st.M + i] = -1;
}

void plan_lds(const z2z_ctx* c, int32_t stride, int32_t flags, LzwArgs* a, size_t* smem) {
  const size_t slot_bytes = (size_t)c->st.nslots * sizeof(uint16_t);
  const size_t key_bytes = (size_t)c->st.cap * sizeof(unsigned long long);
  const size_t limit = (size_t)c->lds_limit;
  a->lds_slots = 0;
  a->lds_keys = 0;
  *smem = 0;
  // a short append (a decode step) touches a handful of slots: probing global memory directly
  // is cheaper than staging the table
  const bool tiny_append = !(flags & Z2Z_RESET) && stride <= 64;
  if (c->opt_lzw_kernel == 2 || tiny_append) return;
  if (slot_bytes <= limit) {
    a->lds_slots = 1;
    *smem = slot_bytes;
    if (slot_bytes + key_bytes <= limit) {
      a->lds_keys = 1;
      *smem = slot_bytes + key_bytes;
    }
  }
}

}  // namespace

int z2z_launch_lzw_reset(z2z_ctx* c, hipStream_t s) {
  hipLaunchKernelGGL(lzw_reset_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_lzw_encode(z2z_ctx* c, const int32_t* tokens, const int32_t* lens, int32_t stride, int32_t flags,
                          int32_t* codes, int32_t* n_codes, int32_t out_stride, int32_t* status, hipStream_t s) {
  LzwArgs a;
  a.st = c->st;
  a.in = tokens;
  a.in_len = lens;
  a.stride = stride;
  a.flags = flags;
  a.out = codes;
  a.out_n = n_codes;
  a.out_stride = out_stride;
  a.status = status;
  size_t smem = 0;
  plan_lds(c, stride, flags, &a, &smem);
  if (flags & Z2Z_RESET) {
    hipLaunchKernelGGL(lzw_clear_entries_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
    if (!a.lds_slots) hipLaunchKernelGGL(lzw_reset_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
  }
  hipLaunchKernelGGL(lzw_encode_kernel, dim3(c->cfg.B), dim3(kWave), smem, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_lzw_decode(z2z_ctx* c, const int32_t* codes, const int32_t* n_codes, int32_t stride, int32_t flags,
                          int32_t* tokens, int32_t* n_tokens, int32_t out_stride, int32_t* status, hipStream_t s) {
  LzwArgs a;
  a.st = c->st;
  a.in = codes;
  a.in_len = n_codes;
  a.stride = stride;
  a.flags = flags;
  a.out = tokens;
  a.out_n = n_tokens;
  a.out_stride = out_stride;
  a.status = status;
  size_t smem = 0;
  plan_lds(c, stride, flags, &a, &smem);
  if (flags & Z2Z_RESET) {
    hipLaunchKernelGGL(lzw_clear_entries_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
    if (!a.lds_slots) hipLaunchKernelGGL(lzw_reset_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
  }
  hipLaunchKernelGGL(lzw_decode_kernel, dim3(c->cfg.B), dim3(kWave), smem, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// Raise the dynamic-LDS ceiling of the two parse kernels to what the device allows.
int z2z_lzw_prepare(z2z_ctx* c) {
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(lzw_encode_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(lzw_decode_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit));
  return Z2Z_OK;
}
