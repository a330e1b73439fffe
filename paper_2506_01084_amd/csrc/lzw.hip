// Batched token-level LZW for gfx950: one wavefront (64 lanes) per sequence.
//
// The parse of one sequence is a serial dependency chain (section 2.1 of the zip2zip paper: every
// step looks up "current phrase + next token" in the codebook built so far), so the unit of
// parallelism across workgroups is the sequence.  Inside a sequence the 64 lanes work on 64 consecutive
// positions (encoder) or codes (decoder) at once against the codebook as it stood when the round began,
// and the round is cut short at the first element that depends on an entry made inside the round; the
// kernels' own comments give the argument why the result is that of the one-element-at-a-time loop.
//
// The codebook is a trie stored as a hash table over its edges: one 64-bit slot = parent code (24 bits)
// | token (24 bits) | entry index (16 bits), two slots per bucket, so a probe is one 16-byte LDS read and
// two compares.  The wave keeps the table of its sequence in LDS for the whole call (4 slots per entry
// when the 160 KiB of a CU allow, at least 1.25); the decoder also keeps (length, first token) of every
// entry there when it fits.  Tokens and codes are staged in LDS 2048 at a time.  Control flow is
// wave-uniform (ballots, scalar registers).
#include "hyper_embed_common.h"

#include <string.h>

namespace {

constexpr int kWave = 64;
typedef unsigned long long u64;
constexpr u64 kEmpty = ~0ull;

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
  int32_t lds_ef;          // decode, LDS variant: 1 = (length, first token) of the entries live in LDS too
  int32_t in_step;         // one-code-at-a-time decoder only: > 0 = row distance of `in` (else `stride`)
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

__device__ __forceinline__ u64 edge_bits(int32_t parent, int32_t tok) {
  return ((u64)(uint32_t)parent << 40) | ((u64)(uint32_t)tok << 16);
}

extern __shared__ __align__(16) u64 lds_slots[];   // LDS variant: the sequence's hash table (+ entry info)

// The hash table of one sequence, in LDS (LDS = true; indexes the shared array directly so that probes
// are ds_read_b64) or in global memory (huge capacities, and short appends that touch a few slots).
template <bool LDS>
struct Table {
  u64* g;           // global slots of this sequence
  uint32_t n;       // number of slots

  // Slots are probed in pairs ("buckets", n is even) so that the per-lane lookup tests two slots with
  // one 16-byte LDS read.  The first kJumps buckets of a probe sequence are `step` buckets apart (a
  // second hash: no clustering, so the longest of 64 simultaneous probes stays short), the rest follow
  // one by one, which reaches every bucket whatever n is.  A lookup ends at the first empty slot.
  static constexpr uint32_t kJumps = 8;
  __device__ __forceinline__ void probe_init(int32_t parent, int32_t tok, uint32_t* bucket, uint32_t* step) const {
    const uint32_t h = edge_hash(parent, tok);
    const uint32_t nb = n >> 1;
    *bucket = __umulhi(h, nb);
    *step = 1 + __umulhi(h * 0x9E3779B1u + 0x7F4A7C15u, nb - 1);       // 1 .. nb-1
  }
  __device__ __forceinline__ uint32_t probe_next(uint32_t bucket, uint32_t step, uint32_t i) const {
    const uint32_t nb = n >> 1;
    bucket += i < kJumps ? step : 1;
    return bucket >= nb ? bucket - nb : bucket;
  }
  __device__ __forceinline__ u64 load(uint32_t pos) const {
    // (the global table is read past the vector L1 everywhere: slots are claimed with atomics, which do not
    // update that cache, so a line it holds can be stale)
    const u64 v = LDS ? lds_slots[pos] : __hip_atomic_load(&g[pos], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // every lane reads the same address; readfirstlane keeps the chain in scalar registers
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((u64)hi << 32) | lo;
  }
  __device__ __forceinline__ void store(uint32_t pos, u64 v) const {
    if (LDS)
      lds_slots[pos] = v;
    else
      __hip_atomic_store(&g[pos], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // Returns the entry index, or -1 with *free_pos = the empty slot the probe ended at (-1 if the
  // table has no empty slot, which cannot happen while n > cap).
  __device__ __forceinline__ int find(int32_t parent, int32_t tok, int* free_pos) const {
    const u64 key = edge_bits(parent, tok);
    uint32_t bucket, step;
    probe_init(parent, tok, &bucket, &step);
    const uint32_t n_probe = (n >> 1) + kJumps;
    for (uint32_t i = 0; i < n_probe; ++i) {
      for (uint32_t k = 0; k < 2; ++k) {
        const uint32_t pos = 2 * bucket + k;
        const u64 s = load(pos);
        if (s == kEmpty) {
          *free_pos = (int)pos;
          return -1;
        }
        if ((s & ~0xFFFFull) == key) return (int)(s & 0xFFFFull);
      }
      bucket = probe_next(bucket, step, i);
    }
    *free_pos = -1;
    return -1;
  }
  // The same probe, per lane (each lane looks up its own edge; no scalar broadcast).  The global table
  // is read past the vector L1: slots are claimed with atomics, which do not update that cache.
  __device__ __forceinline__ int find_lane(int32_t parent, int32_t tok) const {
    const u64 key = edge_bits(parent, tok);
    uint32_t bucket, step;
    probe_init(parent, tok, &bucket, &step);
    const uint32_t n_probe = (n >> 1) + kJumps;
    for (uint32_t i = 0; i < n_probe; ++i) {
      u64 s0, s1;
      if (LDS) {
        const ulonglong2 two = *reinterpret_cast<const ulonglong2*>(&lds_slots[2 * bucket]);
        s0 = two.x;
        s1 = two.y;
      } else {
        s0 = __hip_atomic_load(&g[2 * bucket], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s1 = __hip_atomic_load(&g[2 * bucket + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (s0 == kEmpty) return -1;
      if ((s0 & ~0xFFFFull) == key) return (int)(s0 & 0xFFFFull);
      if (s1 == kEmpty) return -1;
      if ((s1 & ~0xFFFFull) == key) return (int)(s1 & 0xFFFFull);
      bucket = probe_next(bucket, step, i);
    }
    return -1;
  }
  // Per-lane insertion of an edge known to be absent: claim the first empty slot of the probe
  // sequence with a compare-and-swap (several lanes insert at once).
  __device__ __forceinline__ void insert_lane(int32_t parent, int32_t tok, int idx) const {
    const u64 val = edge_bits(parent, tok) | (u64)(uint32_t)idx;
    uint32_t bucket, step;
    probe_init(parent, tok, &bucket, &step);
    const uint32_t n_probe = (n >> 1) + kJumps;
    for (uint32_t i = 0; i < n_probe; ++i) {
      u64* slot = LDS ? &lds_slots[2 * bucket] : &g[2 * bucket];
      if (atomicCAS(slot, kEmpty, val) == kEmpty) return;
      if (atomicCAS(slot + 1, kEmpty, val) == kEmpty) return;
      bucket = probe_next(bucket, step, i);
    }
  }
};

// A workgroup barrier that other waves' reads PAST the vector L1 may rely on.  Between the waves of a workgroup
// plain stores and plain loads are ordered by the L1 they share, and the barrier does not wait for the stores
// to leave it; a load that goes straight to L2 (load_fresh, the table's atomic loads) could overtake a store of
// another wave that is still on its way there.  So the stores are awaited before the barrier.
__device__ __forceinline__ void sync_after_global_stores() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

// The one-wave helpers (table_open / table_close, lzw_encode_rounds, lzw_decode_rounds) are run by exactly one
// wave: the whole workgroup of the 64-thread kernels, or wave 0 of a four-wave kernel on a short appended call
// after the other three have returned.  What they need between their steps is that the lanes' earlier LDS and
// global accesses have completed, not a meeting of waves, so they never execute a workgroup barrier: a fence at
// workgroup scope (the waits for the outstanding memory operations) and a wave barrier (keeps the compiler from
// moving memory operations across).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
}

template <bool LDS>
__device__ __forceinline__ void table_open(const LzwArgs& a, int b, int lane, bool reset, Table<LDS>* t) {
  const LzwState& st = a.st;
  t->g = st.slots + (size_t)b * st.nslots;
  t->n = (uint32_t)st.nslots;
  if (LDS) {
    if (reset) {
      for (int i = lane; i < st.nslots; i += kWave) lds_slots[i] = kEmpty;
    } else {
      for (int i = lane; i < st.nslots; i += kWave) lds_slots[i] = t->g[i];
    }
    wave_sync();
  } else if (reset) {
    // plain stores; the probes read past the L1 (atomic loads), so the stores are awaited first
    for (int i = lane; i < st.nslots; i += kWave) t->g[i] = kEmpty;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wave_sync();
  }
}

template <bool LDS>
__device__ __forceinline__ void table_close(const LzwArgs& a, int lane, const Table<LDS>& t) {
  if (LDS) {
    wave_sync();
    for (int i = lane; i < a.st.nslots; i += kWave) t.g[i] = lds_slots[i];
  }
}

// Add the edge (parent, tok) as entry C.  `ph` holds, in lane j, token j of the parent phrase (plen
// tokens); the new entry's flattened row is that phrase followed by tok.
template <bool LDS>
__device__ __forceinline__ void table_insert(const LzwArgs& a, int b, int lane, const Table<LDS>& t, int free_pos,
                                             int C, int32_t parent, int32_t tok, int32_t ph, int plen) {
  const LzwState& st = a.st;
  if (lane == 0) {
    t.store((uint32_t)free_pos, edge_bits(parent, tok) | (u64)(uint32_t)C);
    st.ent_len[(size_t)b * st.cap + C] = plen + 1;
  }
  if (lane < st.M) {
    const int32_t v = lane < plen ? ph : (lane == plen ? tok : -1);
    st.ent_tokens[((size_t)b * st.cap + C) * st.M + lane] = v;
  }
}

// ------------------------------------------------------------------------------------------------
// encode
//
// The serial chain of the parse is cut into rounds of 64 positions whose work is done by the 64 lanes
// side by side; nothing in a round is a per-token scalar loop.
//   1. lane j follows, for the phrase that would start at position pos + j, the chain of lookups
//      token -> (code, next token) -> ... against the table as it stands at the start of the round
//      (at most M-1 probes, all lanes at once).  This gives L0[j], the length of that match.
//   2. the true phrase starts are the positions reached from 0 by j -> j + L0[j]; six rounds of pointer
//      doubling (each lane carries the 64-bit set of positions its chain visits) give lane 0 the set.
//   3. a start whose match may still grow (length < M, a next token exists) proposes the edge
//      (its code, next token); the proposals of the round get consecutive entry numbers in position
//      order while the codebook has room.
//   4. what step 1 cannot see is an entry made earlier in this same round.  A phrase is longer than
//      L0 exactly when its proposed edge equals an edge proposed by an earlier start of the round, so
//      the round is cut at the first such repeat (found with a small LDS hash filter keyed by edge,
//      keeping the lowest position): everything before the cut is exact, and the next round starts at
//      the cut with the new entries in the table.  A cut is never at position 0, so every round emits
//      at least one phrase.
//   5. the starts before the cut store their codes, insert their edges (compare-and-swap on the slot)
//      and write their flattened rows from the staged tokens.
// Greedy longest match and the order of entry creation are those of the one-token-at-a-time parse: a
// lookup that hit at the start of the round still hits later, and a new entry only matters to later
// starts.  Tokens are staged in LDS kTokBuf at a time, so a round reads no global memory.
// ------------------------------------------------------------------------------------------------
constexpr int kTokBuf = 2048;                 // tokens staged in LDS per refill
constexpr int kFilter = 512;                  // slots of the per-round repeat filter (<= 64 keys)
constexpr int kEncStaticLds = kTokBuf * 4 + kFilter * 8;

__device__ __forceinline__ void lds_order() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// The first lane whose proposed edge (parent, tok) repeats the edge of an earlier lane that inserts
// (kWave if there is none).  `cand` lanes propose, the `inserter` ones among them (a prefix of the
// candidates in lane order) have room to insert.  `filter` is an empty LDS hash set on entry and on exit.
__device__ __forceinline__ int first_repeat(u64* filter, int lane, bool cand, bool inserter, int32_t parent,
                                            int32_t tok) {
  const u64 key = edge_bits(parent, tok);
  const uint32_t h0 = (edge_hash(parent, tok) >> 20) & (kFilter - 1);
  int own = -1;
  bool same = false;                                // met its own edge in the filter
  if (inserter) {
    const u64 val = key | (u64)lane;
    uint32_t h = h0;
    for (int probe = 0; probe < kFilter; ++probe) {
      const u64 old = atomicCAS(&filter[h], kEmpty, val);
      if (old == kEmpty) {
        own = (int)h;
        break;
      }
      if ((old & ~0xFFFFull) == key) {
        atomicMin(&filter[h], val);                 // same edge: keep the lowest lane
        same = true;
        break;
      }
      h = (h + 1) & (kFilter - 1);
    }
  }
  lds_order();
  u64 dup_mask = 0;
  // No inserter met its edge: all inserted edges differ.  A proposal without room can then only
  // repeat an inserted one, which the lookup below finds; with room for all there is none.
  if (__ballot(same) != 0 || __ballot(cand && !inserter) != 0) {
    int fpos = kWave;
    if (cand) {
      uint32_t h = h0;
      for (int probe = 0; probe < kFilter; ++probe) {
        const u64 sl = filter[h];
        if (sl == kEmpty) break;
        if ((sl & ~0xFFFFull) == key) {
          fpos = (int)(sl & 0xFFFFull);
          break;
        }
        h = (h + 1) & (kFilter - 1);
      }
    }
    dup_mask = __ballot(cand && fpos < lane);
    lds_order();
  }
  if (own >= 0) filter[own] = kEmpty;               // leave the filter empty for the next round
  lds_order();
  return dup_mask ? __builtin_ctzll(dup_mask) : kWave;
}

template <bool LDS>
__device__ __forceinline__ void lzw_encode_rounds(const LzwArgs& a, int32_t* tokbuf, u64* filter) {
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;

  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  int prev = reset ? -1 : __builtin_amdgcn_readfirstlane(st.prev_code[b]);
  int prev_len = reset ? 0 : __builtin_amdgcn_readfirstlane(st.prev_len[b]);

  Table<LDS> t;
  table_open<LDS>(a, b, lane, reset, &t);
  for (int i = lane; i < kFilter; i += kWave) filter[i] = kEmpty;

  const int n = a.in_len ? min(max(__builtin_amdgcn_readfirstlane(a.in_len[b]), 0), a.stride) : a.stride;
  const int32_t* in = a.in + (size_t)b * a.stride;
  int32_t* out = a.out + (size_t)b * a.out_stride;
  int32_t* ent_tokens = st.ent_tokens + (size_t)b * cap * M;
  int32_t* ent_len = st.ent_len + (size_t)b * cap;

  int status = 0;
  int n_out = 0;

  // An appended call: the entry "last emitted phrase + first token of this call", which the earlier
  // flush could not add, is added now if it is legal and absent.
  if (n > 0 && prev >= 0 && prev_len < M && C < cap) {
    const int32_t c = __builtin_amdgcn_readfirstlane(in[0]);
    if (c >= 0 && c < V) {
      int free_pos = -1;
      const int idx = t.find(prev, c, &free_pos);
      if (idx < 0 && free_pos >= 0) {
        int32_t ph = -1;        // lane j = token j of the previous phrase
        if (prev < V) {
          ph = lane == 0 ? prev : -1;
        } else if (lane < M) {
          ph = ent_tokens[(size_t)(prev - V) * M + lane];
        }
        table_insert<LDS>(a, b, lane, t, free_pos, C, prev, c, ph, prev_len);
        ++C;
      }
    }
    wave_sync();
  }

  const u64 lanes_below = (1ull << lane) - 1;
  int cbase = 0;                      // tokbuf holds positions [cbase, cbase + kTokBuf)
  bool filled = false;
  bool stop = false;
  int pos = 0;                        // first position not yet covered by an emitted phrase
  int n_rounds = 0;
  while (pos < n && !stop) {
    ++n_rounds;
    // a round touches positions pos .. pos + 63 + M
    if (!filled || (pos + kWave + M > cbase + kTokBuf && cbase + kTokBuf < n)) {
      cbase = pos;
      filled = true;
      const int cnt = min(kTokBuf, n - cbase);
      for (int i = lane; i < cnt; i += kWave) {
        const int32_t v = in[cbase + i];
        tokbuf[i] = (v >= 0 && v < V) ? v : -2;
      }
      lds_order();
    }
    const int rel = pos - cbase + lane;
    auto tk = [&](int d) -> int32_t {           // token class at position pos + lane + d, -1 past the end
      return pos + lane + d < n ? tokbuf[rel + d] : -1;
    };

    // ---- 1. chains against the table of the round's start ---------------------------------------
    const int32_t tok0 = tk(0);
    int L0 = tok0 >= 0 ? 1 : 0;
    int32_t cfin = tok0;
    int32_t nxt = tk(1);              // always the token that follows this lane's match
    for (int d = 1; d < M; ++d) {
      int idx = -1;
      if (L0 == d && nxt >= 0) idx = t.find_lane(cfin, nxt);
      if (__ballot(idx >= 0) == 0) break;
      if (idx >= 0) {
        cfin = V + idx;
        L0 = d + 1;
        nxt = tk(d + 1);
      }
    }

    // ---- 2. phrase starts: positions reachable from 0 ---------------------------------------------
    const int avail = min(kWave, n - pos);
    int jump = (L0 > 0 && lane + L0 < kWave) ? lane + L0 : kWave;
    uint32_t r_lo = lane < 32 ? 1u << lane : 0u, r_hi = lane < 32 ? 0u : 1u << (lane - 32);
#pragma unroll
    for (int k = 0; k < 6; ++k) {
      const int src = jump & (kWave - 1);
      const uint32_t o_lo = __shfl(r_lo, src), o_hi = __shfl(r_hi, src);
      const int o_jump = __shfl(jump, src);
      if (jump < kWave) {
        r_lo |= o_lo;
        r_hi |= o_hi;
        jump = o_jump;
      }
    }
    const u64 S = ((u64)(uint32_t)__builtin_amdgcn_readfirstlane(r_hi) << 32) |
                  (u64)(uint32_t)__builtin_amdgcn_readfirstlane(r_lo);
    const bool start = ((S >> lane) & 1) != 0 && lane < avail;
    const int prank = __popcll(S & lanes_below);          // phrases of the round before this one

    // ---- 3. limits of the round, proposals -------------------------------------------------------
    const u64 bad_mask = __ballot(start && tok0 == -2);
    const u64 ovf_mask = __ballot(start && n_out + prank >= a.out_stride);
    const int bad_pos = bad_mask ? __builtin_ctzll(bad_mask) : kWave;
    const int ovf_pos = ovf_mask ? __builtin_ctzll(ovf_mask) : kWave;
    const bool cand = start && tok0 >= 0 && L0 < M && nxt >= 0;
    const u64 cand_mask = __ballot(cand);
    const int rank = __popcll(cand_mask & lanes_below);
    const int room = cap - C;
    const bool inserter = cand && rank < room;

    // ---- 4. first repeat of a proposed edge --------------------------------------------------------
    int cut = kWave;
    if (room > 0 && (cand_mask & (cand_mask - 1)) != 0) cut = first_repeat(filter, lane, cand, inserter, cfin, nxt);

    // ---- 5. publish ---------------------------------------------------------------------------------
    const int limit = min(min(avail, cut), min(bad_pos, ovf_pos));
    if (bad_pos < kWave && limit == bad_pos) {
      status |= Z2Z_ST_BAD_TOKEN;     // the sequence ends just before this token
      stop = true;
    } else if (ovf_pos < kWave && limit == ovf_pos) {
      status |= Z2Z_ST_OVERFLOW;
      stop = true;
    }
    const bool valid = start && lane < limit;
    const u64 valid_mask = __ballot(valid);
    if (valid) out[n_out + prank] = cfin;
    const bool ins = valid && inserter;
    if (ins) {
      const int idx = C + rank;
      t.insert_lane(cfin, nxt, idx);
      int32_t* row = ent_tokens + (size_t)idx * M;
      for (int k = 0; k < M; ++k) row[k] = k <= L0 ? tokbuf[rel + k] : -1;
      ent_len[idx] = L0 + 1;
    }
    lds_order();
    C += __popcll(__ballot(ins));
    if (valid_mask) {
      const int last = 63 - __builtin_clzll(valid_mask);
      prev = __builtin_amdgcn_readlane(cfin, last);
      prev_len = __builtin_amdgcn_readlane(L0, last);
      n_out += __popcll(valid_mask);
      pos += last + prev_len;
    } else {
      stop = true;                    // only reached with a limit of 0 (bad token or no room at the first start)
    }
  }

  table_close<LDS>(a, lane, t);
  if (lane == 0) {
    st.size[b] = C;
    st.prev_code[b] = prev;
    st.prev_len[b] = prev_len;
    st.rounds[b] = n_rounds;
    a.out_n[b] = n_out;
    a.status[b] = status;
  }
}

// Number of elements of sequence b in this call.
__device__ __forceinline__ int call_length(const LzwArgs& a, int b) {
  return a.in_len ? min(max(__builtin_amdgcn_readfirstlane(a.in_len[b]), 0), a.stride) : a.stride;
}

// A short appended call touches a handful of slots: probing the table where it lives, in global memory,
// is cheaper than staging all of it in LDS and writing it back (the length is known only on the device,
// so the LDS kernels take this decision per sequence).
constexpr int kShortAppend = 64;

template <bool LDS>
__global__ void __launch_bounds__(kWave) lzw_encode_kernel(LzwArgs a) {
  __shared__ int32_t tokbuf[kTokBuf];         // token classes: >= 0 valid ID, -2 out of range
  __shared__ u64 filter[kFilter];
  if (LDS && !(a.flags & Z2Z_RESET) && call_length(a, blockIdx.x) <= kShortAppend)
    lzw_encode_rounds<false>(a, tokbuf, filter);
  else
    lzw_encode_rounds<LDS>(a, tokbuf, filter);
}

// ------------------------------------------------------------------------------------------------
// encode, four waves per sequence
//
// With few sequences in a call the machine is nearly empty and a sequence's parse time is what counts: the
// same rounds, 256 positions wide.  Each of the four waves takes a window of 64 positions and does steps 1
// and 2 of the round on it, now keeping for every lane also where its chain leaves the window (the offset at
// which it enters the next one, or "it ends here").  The per-lane (visited set, exit) pairs go to LDS; after a
// barrier every wave walks the four windows from position 0 (four dependent LDS reads) and knows the phrase
// starts of the whole round.  Limits, proposal ranks and the publishing of codes are the same with prefix
// counts over the waves' ballots (exchanged through LDS), the repeat filter is one LDS hash set for all 256
// positions (insert, barrier, look up, barrier; the first repeat by an LDS atomic minimum), and the table
// insertions of a round are visible to the next round's chains after the round's last barrier.
// ------------------------------------------------------------------------------------------------
constexpr int kWide = 4;
constexpr int kWideLanes = kWide * kWave;
constexpr int kWideFilter = 2048;             // slots of the repeat filter (<= 64 * kWide keys)
struct WideShared {
  u64 sets[kWide][kWave];
  int32_t exits[kWide][kWave];
  u64 cand_mask[kWide], valid_mask[kWide], ins_mask[kWide];
  int32_t bad_pos[kWide], ovf_pos[kWide], last_code[kWide], last_len[kWide];
  int32_t cut;
};
constexpr int kWideStaticLds = kTokBuf * 4 + kWideFilter * 8 + (int)sizeof(WideShared) + 512;   // + alignment slack

template <bool LDS>
__global__ void __launch_bounds__(kWideLanes) lzw_encode_wide_kernel(LzwArgs a) {
  __shared__ int32_t tokbuf[kTokBuf];
  __shared__ u64 filter[kWideFilter];
  __shared__ WideShared sh;
  // a short appended call (its length is known on the device only): one wave, probing the table where it
  // lives; the other waves leave (the one-wave helper executes no workgroup barrier: see wave_sync)
  if (!(a.flags & Z2Z_RESET) && call_length(a, blockIdx.x) <= kShortAppend) {
    if (threadIdx.x < kWave) lzw_encode_rounds<false>(a, tokbuf, filter);
    return;
  }
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;

  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  int prev = reset ? -1 : __builtin_amdgcn_readfirstlane(st.prev_code[b]);
  int prev_len = reset ? 0 : __builtin_amdgcn_readfirstlane(st.prev_len[b]);

  Table<LDS> t;
  t.g = st.slots + (size_t)b * st.nslots;
  t.n = (uint32_t)st.nslots;
  if (LDS) {
    for (int i = tid; i < st.nslots; i += kWideLanes) lds_slots[i] = reset ? kEmpty : t.g[i];
  } else if (reset) {
    for (int i = tid; i < st.nslots; i += kWideLanes) t.g[i] = kEmpty;
  }
  for (int i = tid; i < kWideFilter; i += kWideLanes) filter[i] = kEmpty;
  if (tid == 0) sh.cut = kWideLanes;
  sync_after_global_stores();        // (the table cleared in global memory is read past the L1)

  const int n = call_length(a, b);
  const int32_t* in = a.in + (size_t)b * a.stride;
  int32_t* out = a.out + (size_t)b * a.out_stride;
  int32_t* ent_tokens = st.ent_tokens + (size_t)b * cap * M;
  int32_t* ent_len = st.ent_len + (size_t)b * cap;

  int status = 0;
  int n_out = 0;

  // an appended call: the entry "last emitted phrase + first token of this call" (see lzw_encode_rounds)
  if (n > 0 && prev >= 0 && prev_len < M && C < cap) {
    const int32_t c = __builtin_amdgcn_readfirstlane(in[0]);
    if (c >= 0 && c < V) {
      int free_pos = -1;
      const int idx = t.find(prev, c, &free_pos);
      __syncthreads();     // every wave has looked before wave 0 inserts (else a late wave finds the new edge)
      if (idx < 0 && free_pos >= 0) {
        if (w == 0) {
          int32_t ph = -1;
          if (prev < V) {
            ph = lane == 0 ? prev : -1;
          } else if (lane < M) {
            ph = ent_tokens[(size_t)(prev - V) * M + lane];
          }
          table_insert<LDS>(a, b, lane, t, free_pos, C, prev, c, ph, prev_len);
        }
        ++C;
      }
    }
    sync_after_global_stores();
  }

  const u64 lanes_below = (1ull << lane) - 1;
  const int gpos = w * kWave + lane;      // position of this thread in the round
  int cbase = 0;
  bool filled = false;
  bool stop = false;
  int pos = 0;
  int n_rounds = 0;
  while (pos < n && !stop) {
    ++n_rounds;
    if (!filled || (pos + kWideLanes + M > cbase + kTokBuf && cbase + kTokBuf < n)) {
      cbase = pos;
      filled = true;
      const int cnt = min(kTokBuf, n - cbase);
      for (int i = tid; i < cnt; i += kWideLanes) {
        const int32_t v = in[cbase + i];
        tokbuf[i] = (v >= 0 && v < V) ? v : -2;
      }
      __syncthreads();
    }
    const int rel = pos - cbase + gpos;
    auto tk = [&](int d) -> int32_t { return pos + gpos + d < n ? tokbuf[rel + d] : -1; };

    // ---- 1. chains against the table of the round's start ---------------------------------------
    const int32_t tok0 = tk(0);
    int L0 = tok0 >= 0 ? 1 : 0;
    int32_t cfin = tok0;
    int32_t nxt = tk(1);
    for (int d = 1; d < M; ++d) {
      int idx = -1;
      if (L0 == d && nxt >= 0) idx = t.find_lane(cfin, nxt);
      if (__ballot(idx >= 0) == 0) break;
      if (idx >= 0) {
        cfin = V + idx;
        L0 = d + 1;
        nxt = tk(d + 1);
      }
    }

    // ---- 2. the window's chains: visited positions and where they leave the window ----------------
    int jump = (L0 > 0 && lane + L0 < kWave) ? lane + L0 : kWave;
    int ex = (L0 > 0 && lane + L0 >= kWave) ? lane + L0 - kWave : -1;
    uint32_t r_lo = lane < 32 ? 1u << lane : 0u, r_hi = lane < 32 ? 0u : 1u << (lane - 32);
#pragma unroll
    for (int k = 0; k < 6; ++k) {
      const int src = jump & (kWave - 1);
      const uint32_t o_lo = __shfl(r_lo, src), o_hi = __shfl(r_hi, src);
      const int o_jump = __shfl(jump, src), o_ex = __shfl(ex, src);
      if (jump < kWave) {
        r_lo |= o_lo;
        r_hi |= o_hi;
        ex = o_ex;
        jump = o_jump;
      }
    }
    sh.sets[w][lane] = ((u64)r_hi << 32) | r_lo;
    sh.exits[w][lane] = ex;
    __syncthreads();
    // the round's phrase starts: walk the windows from position 0
    u64 S_mine = 0;
    int starts_before = 0;                      // phrase starts in the windows before this wave's
    {
      int e = 0;
      for (int ww = 0; ww < kWide; ++ww) {
        u64 S = 0;
        if (e >= 0) {
          S = sh.sets[ww][e];
          e = sh.exits[ww][e];
        }
        const int avail_w = min(kWave, n - pos - ww * kWave);      // positions of window ww that exist
        if (avail_w < kWave) S = avail_w <= 0 ? 0 : (S & ((1ull << avail_w) - 1));
        if (ww < w) starts_before += __popcll(S);
        if (ww == w) S_mine = S;
      }
    }
    const int avail = min(kWideLanes, n - pos);
    const bool start = ((S_mine >> lane) & 1) != 0;
    const int prank = starts_before + __popcll(S_mine & lanes_below);

    // ---- 3. limits of the round, proposals -------------------------------------------------------
    const u64 bad_mask = __ballot(start && tok0 == -2);
    const u64 ovf_mask = __ballot(start && n_out + prank >= a.out_stride);
    const bool cand = start && tok0 >= 0 && L0 < M && nxt >= 0;
    const u64 cand_mask = __ballot(cand);
    if (lane == 0) {
      sh.bad_pos[w] = bad_mask ? w * kWave + __builtin_ctzll(bad_mask) : kWideLanes;
      sh.ovf_pos[w] = ovf_mask ? w * kWave + __builtin_ctzll(ovf_mask) : kWideLanes;
      sh.cand_mask[w] = cand_mask;
    }
    __syncthreads();
    int bad_pos = kWideLanes, ovf_pos = kWideLanes, cand_before = 0, cand_total = 0;
    for (int ww = 0; ww < kWide; ++ww) {
      bad_pos = min(bad_pos, sh.bad_pos[ww]);
      ovf_pos = min(ovf_pos, sh.ovf_pos[ww]);
      const int cnt = __popcll(sh.cand_mask[ww]);
      if (ww < w) cand_before += cnt;
      cand_total += cnt;
    }
    const int rank = cand_before + __popcll(cand_mask & lanes_below);
    const int room = cap - C;
    const bool inserter = cand && rank < room;

    // ---- 4. first repeat of a proposed edge (one filter for the whole round) ------------------------
    int cut = kWideLanes;
    if (room > 0 && cand_total >= 2) {              // uniform over the workgroup
      const u64 key = edge_bits(cfin, nxt);
      const uint32_t h0 = (edge_hash(cfin, nxt) >> 20) & (kWideFilter - 1);
      int own = -1;
      if (inserter) {
        const u64 val = key | (u64)gpos;
        uint32_t h = h0;
        for (int probe = 0; probe < kWideFilter; ++probe) {
          const u64 old = atomicCAS(&filter[h], kEmpty, val);
          if (old == kEmpty) {
            own = (int)h;
            break;
          }
          if ((old & ~0xFFFFull) == key) {
            atomicMin(&filter[h], val);             // same edge: keep the lowest position
            break;
          }
          h = (h + 1) & (kWideFilter - 1);
        }
      }
      __syncthreads();
      int fpos = kWideLanes;
      if (cand) {
        uint32_t h = h0;
        for (int probe = 0; probe < kWideFilter; ++probe) {
          const u64 sl = filter[h];
          if (sl == kEmpty) break;
          if ((sl & ~0xFFFFull) == key) {
            fpos = (int)(sl & 0xFFFFull);
            break;
          }
          h = (h + 1) & (kWideFilter - 1);
        }
      }
      const u64 dup_mask = __ballot(cand && fpos < gpos);
      if (dup_mask && lane == 0) atomicMin(&sh.cut, w * kWave + __builtin_ctzll(dup_mask));
      __syncthreads();
      cut = sh.cut;
      if (own >= 0) filter[own] = kEmpty;           // leave the filter empty for the next round
    }

    // ---- 5. publish ---------------------------------------------------------------------------------
    const int limit = min(min(avail, cut), min(bad_pos, ovf_pos));
    if (bad_pos < kWideLanes && limit == bad_pos) {
      status |= Z2Z_ST_BAD_TOKEN;
      stop = true;
    } else if (ovf_pos < kWideLanes && limit == ovf_pos) {
      status |= Z2Z_ST_OVERFLOW;
      stop = true;
    }
    const bool valid = start && gpos < limit;
    const u64 valid_mask = __ballot(valid);
    if (valid) out[n_out + prank] = cfin;
    const bool ins = valid && inserter;
    if (ins) {
      const int idx = C + rank;
      t.insert_lane(cfin, nxt, idx);
      int32_t* row = ent_tokens + (size_t)idx * M;
      for (int k = 0; k < M; ++k) row[k] = k <= L0 ? tokbuf[rel + k] : -1;
      ent_len[idx] = L0 + 1;
    }
    const u64 ins_mask = __ballot(ins);
    if (valid_mask) {
      const int last = 63 - __builtin_clzll(valid_mask);
      const int lc = __builtin_amdgcn_readlane(cfin, last), ll = __builtin_amdgcn_readlane(L0, last);
      if (lane == 0) {
        sh.last_code[w] = lc;
        sh.last_len[w] = ll;
      }
    }
    if (lane == 0) {
      sh.valid_mask[w] = valid_mask;
      sh.ins_mask[w] = ins_mask;
    }
    sync_after_global_stores();
    if (tid == 0) sh.cut = kWideLanes;              // everybody has read it; next written after two more barriers
    int last_w = -1;
    for (int ww = 0; ww < kWide; ++ww) {
      const u64 vm = sh.valid_mask[ww];
      C += __popcll(sh.ins_mask[ww]);
      n_out += __popcll(vm);
      if (vm) last_w = ww;
    }
    if (last_w >= 0) {
      const int last = 63 - __builtin_clzll(sh.valid_mask[last_w]);
      prev = sh.last_code[last_w];
      prev_len = sh.last_len[last_w];
      pos += last_w * kWave + last + prev_len;
    } else {
      stop = true;
    }
    __syncthreads();                                // the exchange arrays are free for the next round
  }

  if (LDS) {
    __syncthreads();
    for (int i = tid; i < st.nslots; i += kWideLanes) t.g[i] = lds_slots[i];
  }
  if (tid == 0) {
    st.size[b] = C;
    st.prev_code[b] = prev;
    st.prev_len[b] = prev_len;
    st.rounds[b] = n_rounds;
    a.out_n[b] = n_out;
    a.status[b] = status;
  }
}

// ------------------------------------------------------------------------------------------------
// decode
// ------------------------------------------------------------------------------------------------
// (length, first token) of an entry packed in 32 bits: length in the top 4 bits.
__device__ __forceinline__ uint32_t pack_ef(int len, int32_t first) { return ((uint32_t)len << 28) | (uint32_t)first; }

// One code at a time (the textbook loop, wave-uniform): used for short appended calls, where a
// round of the kernel below would be mostly empty.
// (a read past the vector L1 of data another wave of the workgroup wrote earlier in the launch)
__device__ __forceinline__ int32_t load_fresh_i32(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <bool LDS>
__device__ __forceinline__ void lzw_decode_serial_body(const LzwArgs& a, int b, int lane) {
  const LzwState& st = a.st;
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;
  const bool ef_lds = LDS && a.lds_ef;
  uint32_t* ef = reinterpret_cast<uint32_t*>(lds_slots + st.nslots);   // [cap], valid when ef_lds
  int32_t* ent_tokens = st.ent_tokens + (size_t)b * cap * M;
  int32_t* ent_len = st.ent_len + (size_t)b * cap;

  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  int prev = reset ? -1 : __builtin_amdgcn_readfirstlane(st.prev_code[b]);
  int prev_len = reset ? 0 : __builtin_amdgcn_readfirstlane(st.prev_len[b]);
  int prev_first = prev < 0 ? 0 : (prev < V ? prev : __builtin_amdgcn_readfirstlane(ent_tokens[(size_t)(prev - V) * M]));

  Table<LDS> t;
  if (ef_lds && !reset) {
    for (int i = lane; i < C; i += kWave) ef[i] = pack_ef(ent_len[i], ent_tokens[(size_t)i * M]);
  }
  table_open<LDS>(a, b, lane, reset, &t);

  const int n = a.in_len ? min(max(__builtin_amdgcn_readfirstlane(a.in_len[b]), 0), a.stride) : a.stride;
  const int32_t* in = a.in + (size_t)b * (a.in_step > 0 ? a.in_step : a.stride);
  int32_t* out = a.out ? a.out + (size_t)b * a.out_stride : nullptr;

  int status = 0;
  int n_out = 0;
  bool stop = false;

  for (int base = 0; base < n && !stop; base += kWave) {
    const int cnt = min(kWave, n - base);
    const int32_t code_reg = lane < cnt ? in[base + lane] : 0;
    // ---- serial part: (length, first token) of each code and the codebook update, all in LDS and
    //      scalar registers.  Lane j keeps what the parallel part needs for code j: where its tokens
    //      go, and the entry (if any) that code j caused.
    int my_off = 0, my_len = 0;
    int new_idx = -1, new_parent = 0, new_tok = 0, new_plen = 0;
    int done = 0;                     // codes of this chunk accepted
    for (int j = 0; j < cnt; ++j) {
      const int32_t k = __builtin_amdgcn_readlane(code_reg, j);
      int cur_len = 0;
      int32_t first = 0;
      int free_pos = -1;
      bool fresh = false;             // the code names the entry made in this very step
      if (k >= 0 && k < V) {
        cur_len = 1;
        first = k;
      } else if (k >= V && k - V < C) {
        uint32_t e;
        if (ef_lds)
          e = ef[k - V];
        else
          e = pack_ef(ent_len[k - V], ent_tokens[(size_t)(k - V) * M]);
        e = __builtin_amdgcn_readfirstlane(e);
        cur_len = (int)(e >> 28);
        first = (int32_t)(e & 0x0FFFFFFFu);
      } else if (k >= V && k - V == C && prev >= 0 && prev_len < M && C < cap) {
        // previous phrase + its own first token, which must not exist yet
        const int idx = t.find(prev, prev_first, &free_pos);
        if (idx >= 0 || free_pos < 0) {
          status |= Z2Z_ST_BAD_CODE;
          stop = true;
          break;
        }
        cur_len = prev_len + 1;
        first = prev_first;
        fresh = true;
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
      if (prev >= 0 && prev_len < M && C < cap) {
        int idx = -1;
        if (!fresh) idx = t.find(prev, first, &free_pos);
        if (idx < 0 && free_pos >= 0) {
          if (lane == 0) {
            t.store((uint32_t)free_pos, edge_bits(prev, first) | (u64)(uint32_t)C);
            if (ef_lds) {
              ef[C] = pack_ef(prev_len + 1, prev_first);
            } else {
              // no LDS copy: a later code of this chunk may already name this entry, and its length
              // and first token are then read from memory before the rows are completed below
              ent_len[C] = prev_len + 1;
              ent_tokens[(size_t)C * M] = prev_first;
            }
          }
          if (lane == j) {
            new_idx = C;
            new_parent = prev;
            new_tok = first;
            new_plen = prev_len;
          }
          ++C;
        }
      }
      if (lane == j) {
        my_off = n_out;
        my_len = cur_len;
      }
      n_out += cur_len;
      prev = k;
      prev_len = cur_len;
      prev_first = first;
      ++done;
    }
    // ---- parallel part 1: write the flattened rows of the entries made in this chunk, shortest
    //      parents first (a parent made in this chunk is shorter than its child, so it is complete
    //      by the time the child copies it)
    for (int L = 1; L < M; ++L) {
      if (new_idx >= 0 && new_plen == L) {
        int32_t* row = ent_tokens + (size_t)new_idx * M;
        if (new_parent < V) {
          row[0] = new_parent;
        } else {
          const int32_t* prow = ent_tokens + (size_t)(new_parent - V) * M;
          for (int i = 0; i < L; ++i) row[i] = prow[i];
        }
        row[L] = new_tok;
        for (int i = L + 1; i < M; ++i) row[i] = -1;
        ent_len[new_idx] = L + 1;
      }
      wave_sync();                    // one wave: orders this level's stores before the next level's loads
    }
    // ---- parallel part 2: lane j writes the tokens of code j
    if (out != nullptr && lane < done) {
      const int32_t k = code_reg;
      if (k < V) {
        out[my_off] = k;
      } else {
        const int32_t* row = ent_tokens + (size_t)(k - V) * M;
        for (int i = 0; i < my_len; ++i) out[my_off + i] = row[i];
      }
    }
  }

  table_close<LDS>(a, lane, t);
  if (lane == 0) {
    st.size[b] = C;
    st.prev_code[b] = prev;
    st.prev_len[b] = prev_len;
    st.rounds[b] = n;                 // one code per step
    a.out_n[b] = n_out;
    a.status[b] = status;
  }
}

template <bool LDS>
__global__ void __launch_bounds__(kWave) lzw_decode_serial_kernel(LzwArgs a) {
  lzw_decode_serial_body<LDS>(a, blockIdx.x, threadIdx.x);
}

// One generation step's codebook side in one launch (section 2.3, steps 9-10; "Hyper-Embedding Cache"): wave 0
// of the workgroup applies the sequence's new code to its codebook (the one-code-at-a-time update above, table
// in global memory), then all waves pool the newest entry's constituent embeddings into its row of the cache --
// what an appended z2z_lzw_decode of one code followed by z2z_hyper_embed of the last entry do in two launches.
// The newest entry is pooled whether or not this step made it (the row comes out bit-identical).
constexpr int kStepWaves = 8;
template <bool BF16>
__global__ void __launch_bounds__(kStepWaves * kWave) lzw_step_update_kernel(LzwArgs a, z2z_embed::EmbedArgs ea) {
  const int b = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (w == 0) lzw_decode_serial_body<false>(a, b, lane);
  sync_after_global_stores();          // the entry's row and the size are in memory before the other waves read them
  const int C = min(__builtin_amdgcn_readfirstlane(load_fresh_i32(a.st.size + b)), a.st.cap);
  if (C <= 0) return;
  const size_t row = (size_t)b * a.st.cap + (C - 1);
  const int L = min(max(__builtin_amdgcn_readfirstlane(load_fresh_i32(a.st.ent_len + row)), 1), a.st.M);
  int32_t toks[Z2Z_MAX_M];
#pragma unroll
  for (int j = 0; j < Z2Z_MAX_M; ++j) toks[j] = j < L ? load_fresh_i32(a.st.ent_tokens + row * a.st.M + j) : 0;
  if (w < ea.split) z2z_embed::embed_row<BF16>(ea, toks, L, row, lane, w);
}

// Entry data written earlier in the same launch is read past the vector L1.
__device__ __forceinline__ int32_t load_fresh(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Rounds of up to 63 codes, one code per lane; lane 0 stands for the code before the round (its phrase
// is the parent of the entry the first code of the round may cause).
//   1. (length, first token) of every code whose entry existed when the round began; the round ends
//      before the first code that names a later entry (or no entry at all).  If that is the very first
//      code of the round it is taken alone, the textbook way (the one not-yet-defined code, or an error).
//   2. code i proposes the edge (code i-1, first token of code i) if code i-1 is shorter than M; the
//      table is probed for all proposals at once; absent ones get consecutive entry numbers while the
//      codebook has room.  As in the encoder the round is cut at the first proposal that repeats an
//      earlier one of the same round (only streams that no greedy parse produced have such repeats).
//   3. token offsets are a prefix sum of the lengths (lengths are < 16: four ballots); the round is cut
//      before the first code whose tokens do not fit.
//   4. the lanes before the cut insert their edges, lane i-1 writes the flattened row of the entry that
//      code i caused (its own tokens + that first token), and every lane writes its tokens.
template <bool LDS>
__device__ __forceinline__ void lzw_decode_rounds(const LzwArgs& a, int32_t* codebuf, u64* filter) {
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;
  const bool ef_lds = LDS && a.lds_ef;
  uint32_t* ef = reinterpret_cast<uint32_t*>(lds_slots + st.nslots);   // [cap], valid when ef_lds
  int32_t* ent_tokens = st.ent_tokens + (size_t)b * cap * M;
  int32_t* ent_len = st.ent_len + (size_t)b * cap;

  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  int prev = reset ? -1 : __builtin_amdgcn_readfirstlane(st.prev_code[b]);
  int prev_len = reset ? 0 : __builtin_amdgcn_readfirstlane(st.prev_len[b]);

  Table<LDS> t;
  if (ef_lds && !reset) {
    for (int i = lane; i < C; i += kWave) ef[i] = pack_ef(ent_len[i], ent_tokens[(size_t)i * M]);
  }
  table_open<LDS>(a, b, lane, reset, &t);
  for (int i = lane; i < kFilter; i += kWave) filter[i] = kEmpty;

  const int n = a.in_len ? min(max(__builtin_amdgcn_readfirstlane(a.in_len[b]), 0), a.stride) : a.stride;
  const int32_t* in = a.in + (size_t)b * a.stride;
  int32_t* out = a.out ? a.out + (size_t)b * a.out_stride : nullptr;

  const u64 lanes_upto = lane == 63 ? ~0ull : (2ull << lane) - 1;     // lanes 0..lane
  const u64 lanes_below = (1ull << lane) - 1;
  int status = 0;
  int n_out = 0;
  bool stop = false;
  int cbase = 0;                      // codebuf holds codes [cbase, cbase + kTokBuf)
  bool filled = false;
  int cpos = 0;                       // codes consumed
  int n_rounds = 0;
  while (cpos < n && !stop) {
    ++n_rounds;
    if (!filled || (cpos + kWave > cbase + kTokBuf && cbase + kTokBuf < n)) {
      cbase = cpos;
      filled = true;
      const int cnt = min(kTokBuf, n - cbase);
      for (int i = lane; i < cnt; i += kWave) codebuf[i] = in[cbase + i];
      lds_order();
    }
    // ---- 1. the codes of the round ------------------------------------------------------------------
    const int ci = cpos + lane - 1;
    const bool present = lane == 0 ? prev >= 0 : ci < n;
    const int32_t k = lane == 0 ? prev : (ci < n ? codebuf[ci - cbase] : -1);
    int len = 0;
    int32_t first = 0;
    bool known = false;
    if (present && k >= 0 && k < V) {
      len = 1;
      first = k;
      known = true;
    } else if (present && k >= V && k - V < C) {
      const uint32_t e = ef_lds ? ef[k - V]
                                : pack_ef(load_fresh(&ent_len[k - V]), load_fresh(&ent_tokens[(size_t)(k - V) * M]));
      len = (int)(e >> 28);
      first = (int32_t)(e & 0x0FFFFFFFu);
      known = true;
    }
    const u64 hard_mask = __ballot(present && !known);          // never lane 0
    const int hard_pos = hard_mask ? __builtin_ctzll(hard_mask) : kWave;

    if (hard_pos == 1) {
      // the first code of the round names no entry of the codebook as it stands: it is either
      // "previous phrase + its own first token", which must be legal and absent, or an error
      const int32_t k1 = __builtin_amdgcn_readlane(k, 1);
      bool ok = false;
      if (k1 >= V && k1 - V == C && prev >= 0 && prev_len < M && C < cap) {
        const int32_t pf = __builtin_amdgcn_readlane(first, 0);
        int free_pos = -1;
        const int idx = t.find(prev, pf, &free_pos);
        if (idx < 0 && free_pos >= 0) {
          const int cur_len = prev_len + 1;
          if (out != nullptr && n_out + cur_len > a.out_stride) {
            status |= Z2Z_ST_OVERFLOW;
            stop = true;
          } else {
            int32_t tokj = -1;        // lane j: token j of the new phrase
            if (lane < prev_len) tokj = prev < V ? prev : load_fresh(&ent_tokens[(size_t)(prev - V) * M + lane]);
            if (lane == prev_len) tokj = pf;
            if (lane == 0) {
              t.store((uint32_t)free_pos, edge_bits(prev, pf) | (u64)(uint32_t)C);
              if (ef_lds) ef[C] = pack_ef(cur_len, pf);
              ent_len[C] = cur_len;
            }
            if (lane < M) ent_tokens[(size_t)C * M + lane] = tokj;
            if (out != nullptr && lane < cur_len) out[n_out + lane] = tokj;
            prev = k1;
            prev_len = cur_len;
            ++C;
            n_out += cur_len;
            ++cpos;
          }
          ok = true;
        }
      }
      if (!ok) {
        status |= Z2Z_ST_BAD_CODE;
        stop = true;
      }
      wave_sync();                    // the new row is in memory before a later round reads it
      continue;
    }

    // ---- 2. proposals --------------------------------------------------------------------------------
    const int limit0 = min(hard_pos, min(kWave, n - cpos + 1));  // lanes 1 .. limit0-1 hold known codes
    const int32_t pk = __shfl_up(k, 1);
    const int plen = __shfl_up(len, 1);
    const int32_t pfirst = __shfl_up(first, 1);
    const bool pknown = __shfl_up((int)known, 1) != 0;
    const int room = cap - C;
    const bool prop = lane >= 1 && lane < limit0 && pknown && plen < M && room > 0;
    int found = -1;
    if (prop) found = t.find_lane(pk, first);
    const bool cand = prop && found < 0;
    const u64 cand_mask = __ballot(cand);
    const int rank = __popcll(cand_mask & lanes_below);
    const bool inserter = cand && rank < room;
    int cut = kWave;
    if ((cand_mask & (cand_mask - 1)) != 0) cut = first_repeat(filter, lane, cand, inserter, pk, first);

    // ---- 3. token offsets -------------------------------------------------------------------------------
    const int mylen = (lane >= 1 && lane < limit0) ? len : 0;
    int incl = 0;                     // tokens of codes 1 .. lane of the round
#pragma unroll
    for (int bit = 0; bit < 4; ++bit) incl += __popcll(__ballot((mylen >> bit) & 1) & lanes_upto) << bit;
    const u64 ovf_mask = __ballot(out != nullptr && mylen > 0 && n_out + incl > a.out_stride);
    const int ovf_pos = ovf_mask ? __builtin_ctzll(ovf_mask) : kWave;
    const int limit = min(limit0, min(cut, ovf_pos));
    if (ovf_pos < kWave && limit == ovf_pos) {
      status |= Z2Z_ST_OVERFLOW;
      stop = true;
    }

    // ---- 4. publish ---------------------------------------------------------------------------------------
    const bool valid = lane >= 1 && lane < limit;
    const bool ins = valid && inserter;
    const int idx = C + rank;
    if (ins) {
      t.insert_lane(pk, first, idx);
      if (ef_lds) ef[idx] = pack_ef(plen + 1, pfirst);
    }
    // the tokens of this lane's own code (lane 0: of the code before the round)
    int32_t T[Z2Z_MAX_M];
#pragma unroll
    for (int j = 0; j < Z2Z_MAX_M; ++j) T[j] = -1;
    if (lane < limit && known) {
      if (k < V) {
        T[0] = k;
      } else {
        const int32_t* row = ent_tokens + (size_t)(k - V) * M;
#pragma unroll
        for (int j = 0; j < Z2Z_MAX_M; ++j)
          if (j < len) T[j] = load_fresh(&row[j]);
      }
    }
    // the entry caused by the next lane's code: this lane's tokens + that code's first token
    const bool s_ins = __shfl_down((int)ins, 1) != 0 && lane < kWave - 1;
    const int s_idx = __shfl_down(idx, 1);
    const int32_t s_first = __shfl_down(first, 1);
    if (s_ins) {
      int32_t* row = ent_tokens + (size_t)s_idx * M;
#pragma unroll
      for (int j = 0; j < Z2Z_MAX_M; ++j)
        if (j < M) row[j] = j < len ? T[j] : (j == len ? s_first : -1);
      ent_len[s_idx] = len + 1;
    }
    if (valid && out != nullptr) {
      int32_t* dst = out + n_out + incl - len;
#pragma unroll
      for (int j = 0; j < Z2Z_MAX_M; ++j)
        if (j < len) dst[j] = T[j];
    }
    C += __popcll(__ballot(ins));
    if (limit >= 2) {
      const int last = limit - 1;
      prev = __builtin_amdgcn_readlane(k, last);
      prev_len = __builtin_amdgcn_readlane(len, last);
      n_out += __builtin_amdgcn_readlane(incl, last);
      cpos += last;
    } else {
      stop = true;                    // only reached when the first code of the round does not fit
    }
    wave_sync();                      // rows written above are in memory before a later round reads them
  }

  table_close<LDS>(a, lane, t);
  if (lane == 0) {
    st.size[b] = C;
    st.prev_code[b] = prev;
    st.prev_len[b] = prev_len;
    st.rounds[b] = n_rounds;
    a.out_n[b] = n_out;
    a.status[b] = status;
  }
}

template <bool LDS>
__global__ void __launch_bounds__(kWave) lzw_decode_kernel(LzwArgs a) {
  __shared__ int32_t codebuf[kTokBuf];
  __shared__ u64 filter[kFilter];
  if (LDS && !(a.flags & Z2Z_RESET) && call_length(a, blockIdx.x) <= kShortAppend)
    lzw_decode_rounds<false>(a, codebuf, filter);
  else
    lzw_decode_rounds<LDS>(a, codebuf, filter);
}

// ------------------------------------------------------------------------------------------------
// decode, four waves per sequence (few long sequences: see the encoder's counterpart)
//
// A round takes up to 255 codes: global lane g = 64 * wave + lane holds code cpos + g - 1, global lane 0 the code
// before the round.  The steps are those of lzw_decode_rounds; what crosses a window boundary goes through LDS:
// the first code that names no entry yet (minimum over the waves), the (code, length, first token) of every
// window's last lane for the next window's first proposal, proposal ranks and token offsets as prefix counts
// over the waves, one repeat filter for the round.  A lane that inserts writes the new entry's row itself (the
// previous code's tokens, which are older than the round, plus its own first token), so no registers cross
// the boundary.  The one code that may name the entry it creates is taken alone at the head of a round by
// every wave alike, wave 0 doing the stores.
// ------------------------------------------------------------------------------------------------
struct WideDecShared {
  int32_t hard[kWide], edge_k[kWide], edge_len[kWide], edge_first[kWide], edge_known[kWide];
  int32_t k1, first0;
  u64 cand_mask[kWide];
  int32_t lensum[kWide], ovf[kWide], ins_cnt[kWide];
  int32_t last_k, last_len, last_incl;
  int32_t cut;
};
static_assert(sizeof(WideDecShared) <= sizeof(WideShared), "the decoder's exchange area fits the encoder's LDS budget");

template <bool LDS>
__global__ void __launch_bounds__(kWideLanes) lzw_decode_wide_kernel(LzwArgs a) {
  __shared__ int32_t codebuf[kTokBuf];
  __shared__ u64 filter[kWideFilter];
  __shared__ WideDecShared sh;
  if (!(a.flags & Z2Z_RESET) && call_length(a, blockIdx.x) <= kShortAppend) {      // see the encoder
    if (threadIdx.x < kWave) lzw_decode_rounds<false>(a, codebuf, filter);
    return;
  }
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = tid;                                 // global lane of the round
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;
  const bool ef_lds = LDS && a.lds_ef;
  uint32_t* ef = reinterpret_cast<uint32_t*>(lds_slots + st.nslots);
  int32_t* ent_tokens = st.ent_tokens + (size_t)b * cap * M;
  int32_t* ent_len = st.ent_len + (size_t)b * cap;

  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  int prev = reset ? -1 : __builtin_amdgcn_readfirstlane(st.prev_code[b]);
  int prev_len = reset ? 0 : __builtin_amdgcn_readfirstlane(st.prev_len[b]);

  Table<LDS> t;
  t.g = st.slots + (size_t)b * st.nslots;
  t.n = (uint32_t)st.nslots;
  if (ef_lds && !reset) {
    for (int i = tid; i < C; i += kWideLanes) ef[i] = pack_ef(ent_len[i], ent_tokens[(size_t)i * M]);
  }
  if (LDS) {
    for (int i = tid; i < st.nslots; i += kWideLanes) lds_slots[i] = reset ? kEmpty : t.g[i];
  } else if (reset) {
    for (int i = tid; i < st.nslots; i += kWideLanes) t.g[i] = kEmpty;
  }
  for (int i = tid; i < kWideFilter; i += kWideLanes) filter[i] = kEmpty;
  if (tid == 0) sh.cut = kWideLanes;
  sync_after_global_stores();        // (the table cleared in global memory is read past the L1)

  const int n = call_length(a, b);
  const int32_t* in = a.in + (size_t)b * a.stride;
  int32_t* out = a.out ? a.out + (size_t)b * a.out_stride : nullptr;

  const u64 lanes_upto = lane == 63 ? ~0ull : (2ull << lane) - 1;
  const u64 lanes_below = (1ull << lane) - 1;
  int status = 0;
  int n_out = 0;
  bool stop = false;
  int cbase = 0;
  bool filled = false;
  int cpos = 0;
  int n_rounds = 0;
  while (cpos < n && !stop) {
    ++n_rounds;
    if (!filled || (cpos + kWideLanes > cbase + kTokBuf && cbase + kTokBuf < n)) {
      cbase = cpos;
      filled = true;
      const int cnt = min(kTokBuf, n - cbase);
      for (int i = tid; i < cnt; i += kWideLanes) codebuf[i] = in[cbase + i];
      __syncthreads();
    }
    // ---- 1. the codes of the round ------------------------------------------------------------------
    const int ci = cpos + g - 1;
    const bool present = g == 0 ? prev >= 0 : ci < n;
    const int32_t k = g == 0 ? prev : (ci < n ? codebuf[ci - cbase] : -1);
    int len = 0;
    int32_t first = 0;
    bool known = false;
    if (present && k >= 0 && k < V) {
      len = 1;
      first = k;
      known = true;
    } else if (present && k >= V && k - V < C) {
      const uint32_t e = ef_lds ? ef[k - V]
                                : pack_ef(load_fresh(&ent_len[k - V]), load_fresh(&ent_tokens[(size_t)(k - V) * M]));
      len = (int)(e >> 28);
      first = (int32_t)(e & 0x0FFFFFFFu);
      known = true;
    }
    const u64 hard_mask = __ballot(present && !known);            // never global lane 0
    if (lane == 0) sh.hard[w] = hard_mask ? w * kWave + __builtin_ctzll(hard_mask) : kWideLanes;
    if (lane == kWave - 1) {
      sh.edge_k[w] = k;
      sh.edge_len[w] = len;
      sh.edge_first[w] = first;
      sh.edge_known[w] = known ? 1 : 0;
    }
    if (tid == 0) sh.first0 = first;
    if (tid == 1) sh.k1 = k;
    __syncthreads();
    int hard_pos = kWideLanes;
    for (int ww = 0; ww < kWide; ++ww) hard_pos = min(hard_pos, sh.hard[ww]);

    if (hard_pos == 1) {
      // the first code of the round names no entry of the codebook as it stands: "previous phrase + its own
      // first token", legal and absent, or an error.  Every wave takes the same decisions (hence the barrier between the
      // lookup and the store); wave 0 stores.
      const int32_t k1 = sh.k1;
      bool ok = false;
      if (k1 >= V && k1 - V == C && prev >= 0 && prev_len < M && C < cap) {
        const int32_t pf = sh.first0;
        int free_pos = -1;
        const int idx = t.find(prev, pf, &free_pos);
        __syncthreads();   // every wave has looked before wave 0 stores (else a late wave finds the new edge)
        if (idx < 0 && free_pos >= 0) {
          const int cur_len = prev_len + 1;
          if (out != nullptr && n_out + cur_len > a.out_stride) {
            status |= Z2Z_ST_OVERFLOW;
            stop = true;
          } else {
            if (w == 0) {
              int32_t tokj = -1;        // lane j: token j of the new phrase
              if (lane < prev_len) tokj = prev < V ? prev : load_fresh(&ent_tokens[(size_t)(prev - V) * M + lane]);
              if (lane == prev_len) tokj = pf;
              if (lane == 0) {
                t.store((uint32_t)free_pos, edge_bits(prev, pf) | (u64)(uint32_t)C);
                if (ef_lds) ef[C] = pack_ef(cur_len, pf);
                ent_len[C] = cur_len;
              }
              if (lane < M) ent_tokens[(size_t)C * M + lane] = tokj;
              if (out != nullptr && lane < cur_len) out[n_out + lane] = tokj;
            }
            prev = k1;
            prev_len = cur_len;
            ++C;
            n_out += cur_len;
            ++cpos;
          }
          ok = true;
        }
      }
      if (!ok) {
        status |= Z2Z_ST_BAD_CODE;
        stop = true;
      }
      sync_after_global_stores();
      continue;
    }

    // ---- 2. proposals --------------------------------------------------------------------------------
    const int limit0 = min(hard_pos, min(kWideLanes, n - cpos + 1));   // global lanes 1 .. limit0-1 hold known codes
    int32_t pk = __shfl_up(k, 1);
    int plen = __shfl_up(len, 1);
    int32_t pfirst = __shfl_up(first, 1);
    bool pknown = __shfl_up((int)known, 1) != 0;
    if (lane == 0 && w > 0) {
      pk = sh.edge_k[w - 1];
      plen = sh.edge_len[w - 1];
      pfirst = sh.edge_first[w - 1];
      pknown = sh.edge_known[w - 1] != 0;
    }
    const int room = cap - C;
    const bool prop = g >= 1 && g < limit0 && pknown && plen < M && room > 0;
    int found = -1;
    if (prop) found = t.find_lane(pk, first);
    const bool cand = prop && found < 0;
    const u64 cand_mask = __ballot(cand);
    // token offsets inside the window
    const int mylen = (g >= 1 && g < limit0) ? len : 0;
    int incl = 0;
#pragma unroll
    for (int bit = 0; bit < 4; ++bit) incl += __popcll(__ballot((mylen >> bit) & 1) & lanes_upto) << bit;
    if (lane == 0) sh.cand_mask[w] = cand_mask;
    if (lane == kWave - 1) sh.lensum[w] = incl;
    __syncthreads();
    int cand_before = 0, cand_total = 0, len_before = 0;
    for (int ww = 0; ww < kWide; ++ww) {
      const int cnt = __popcll(sh.cand_mask[ww]);
      if (ww < w) {
        cand_before += cnt;
        len_before += sh.lensum[ww];
      }
      cand_total += cnt;
    }
    const int rank = cand_before + __popcll(cand_mask & lanes_below);
    const bool inserter = cand && rank < room;
    incl += len_before;                               // tokens of codes 1 .. g of the round
    const u64 ovf_mask = __ballot(out != nullptr && mylen > 0 && n_out + incl > a.out_stride);
    if (lane == 0) sh.ovf[w] = ovf_mask ? w * kWave + __builtin_ctzll(ovf_mask) : kWideLanes;
    // first repeat of a proposed edge: insert phase
    const bool filtering = cand_total >= 2;           // uniform
    const u64 key = edge_bits(pk, first);
    const uint32_t h0 = (edge_hash(pk, first) >> 20) & (kWideFilter - 1);
    int own = -1;
    if (filtering && inserter) {
      const u64 val = key | (u64)g;
      uint32_t h = h0;
      for (int probe = 0; probe < kWideFilter; ++probe) {
        const u64 old = atomicCAS(&filter[h], kEmpty, val);
        if (old == kEmpty) {
          own = (int)h;
          break;
        }
        if ((old & ~0xFFFFull) == key) {
          atomicMin(&filter[h], val);
          break;
        }
        h = (h + 1) & (kWideFilter - 1);
      }
    }
    __syncthreads();
    if (filtering) {
      int fpos = kWideLanes;
      if (cand) {
        uint32_t h = h0;
        for (int probe = 0; probe < kWideFilter; ++probe) {
          const u64 sl = filter[h];
          if (sl == kEmpty) break;
          if ((sl & ~0xFFFFull) == key) {
            fpos = (int)(sl & 0xFFFFull);
            break;
          }
          h = (h + 1) & (kWideFilter - 1);
        }
      }
      const u64 dup_mask = __ballot(cand && fpos < g);
      if (dup_mask && lane == 0) atomicMin(&sh.cut, w * kWave + __builtin_ctzll(dup_mask));
    }
    __syncthreads();
    const int cut = sh.cut;
    if (own >= 0) filter[own] = kEmpty;
    int ovf_pos = kWideLanes;
    for (int ww = 0; ww < kWide; ++ww) ovf_pos = min(ovf_pos, sh.ovf[ww]);
    const int limit = min(limit0, min(cut, ovf_pos));
    if (ovf_pos < kWideLanes && limit == ovf_pos) {
      status |= Z2Z_ST_OVERFLOW;
      stop = true;
    }

    // ---- 3. publish ---------------------------------------------------------------------------------------
    const bool valid = g >= 1 && g < limit;
    const bool ins = valid && inserter;
    if (ins) {
      const int idx = C + rank;
      t.insert_lane(pk, first, idx);
      if (ef_lds) ef[idx] = pack_ef(plen + 1, pfirst);
      // the new entry's row: the previous code's tokens (older than the round) and this code's first token
      int32_t* row = ent_tokens + (size_t)idx * M;
      for (int j = 0; j < M; ++j) {
        int32_t v = -1;
        if (j < plen) v = pk < V ? pk : load_fresh(&ent_tokens[(size_t)(pk - V) * M + j]);
        if (j == plen) v = first;
        row[j] = v;
      }
      ent_len[idx] = plen + 1;
    }
    if (valid && out != nullptr) {
      int32_t* dst = out + n_out + incl - len;
      if (k < V) {
        dst[0] = k;
      } else {
        const int32_t* row = ent_tokens + (size_t)(k - V) * M;
        for (int j = 0; j < len; ++j) dst[j] = load_fresh(&row[j]);
      }
    }
    const u64 ins_mask = __ballot(ins);
    if (lane == 0) sh.ins_cnt[w] = __popcll(ins_mask);
    if (limit >= 2 && g == limit - 1) {
      sh.last_k = k;
      sh.last_len = len;
      sh.last_incl = incl;
    }
    sync_after_global_stores();
    for (int ww = 0; ww < kWide; ++ww) C += sh.ins_cnt[ww];
    if (limit >= 2) {
      prev = sh.last_k;
      prev_len = sh.last_len;
      n_out += sh.last_incl;
      cpos += limit - 1;
    } else {
      stop = true;
    }
    if (tid == 0) sh.cut = kWideLanes;
    sync_after_global_stores();                  // rows written above are in memory, the exchange area is free
  }

  if (LDS) {
    for (int i = tid; i < st.nslots; i += kWideLanes) t.g[i] = lds_slots[i];
  }
  if (tid == 0) {
    st.size[b] = C;
    st.prev_code[b] = prev;
    st.prev_len[b] = prev_len;
    st.rounds[b] = n_rounds;
    a.out_n[b] = n_out;
    a.status[b] = status;
  }
}

// Empty every codebook.  grid = B, block = 256.
__global__ void lzw_reset_kernel(LzwState st) {
  const int b = blockIdx.x;
  for (int i = threadIdx.x; i < st.nslots; i += blockDim.x) st.slots[(size_t)b * st.nslots + i] = kEmpty;
  for (int i = threadIdx.x; i < st.cap; i += blockDim.x) st.ent_len[(size_t)b * st.cap + i] = 0;
  for (size_t i = threadIdx.x; i < (size_t)st.cap * st.M; i += blockDim.x)
    st.ent_tokens[(size_t)b * st.cap * st.M + i] = -1;
  if (threadIdx.x == 0) {
    st.size[b] = 0;
    st.prev_code[b] = -1;
    st.prev_len[b] = 0;
  }
}

// Clear the entry rows of a sequence that a RESET encode/decode is about to refill, so that rows at
// and beyond the new size read as unused.  grid = B, block = 256.
__global__ void lzw_clear_entries_kernel(LzwState st) {
  const int b = blockIdx.x;
  const int C = st.size[b];
  for (int i = threadIdx.x; i < C; i += blockDim.x) st.ent_len[(size_t)b * st.cap + i] = 0;
  for (size_t i = threadIdx.x; i < (size_t)C * st.M; i += blockDim.x)
    st.ent_tokens[(size_t)b * st.cap * st.M + i] = -1;
}

// Which table variant a call uses, and how much LDS it needs.
void plan(const z2z_ctx* c, int32_t stride, int32_t flags, bool decode, bool* lds, LzwArgs* a, size_t* smem) {
  const size_t slot_bytes = (size_t)c->st.nslots * sizeof(u64);
  const size_t ef_bytes = (size_t)c->st.cap * sizeof(uint32_t);
  const size_t limit = (size_t)c->lds_limit - kEncStaticLds;
  // a short append (a decode step) touches a handful of slots: probing global memory directly is
  // cheaper than staging the table
  const bool tiny_append = !(flags & Z2Z_RESET) && stride <= 64;
  // with thousands of sequences the LDS a table takes limits a CU to a few waves; probing the table in
  // global memory (L2) with the CU full of waves is then faster (measured crossover between 512 and 2048
  // sequences of 4096 tokens)
  const bool crowd = c->cfg.B >= 1024;
  *lds = c->st.slots_fit_lds && !tiny_append && !crowd && c->opt_lzw_kernel != 2;
  a->lds_ef = 0;
  *smem = 0;
  if (*lds) {
    *smem = slot_bytes;
    if (decode && slot_bytes + ef_bytes <= limit) {
      a->lds_ef = 1;
      *smem += ef_bytes;
    }
  }
}

// How often each entry is named by a code stream: usage[b][e] += number of codes equal to V + e (codes of base
// tokens and codes that name no entry are skipped).  One workgroup per sequence.
__global__ void __launch_bounds__(256) lzw_usage_kernel(LzwState st, const int32_t* codes, const int32_t* n_codes,
                                                        int stride, int32_t* usage) {
  const int b = blockIdx.x;
  const int n = n_codes ? min(max(n_codes[b], 0), stride) : stride;
  const int C = min(max(st.size[b], 0), st.cap);
  for (int i = threadIdx.x; i < n; i += 256) {
    const int e = codes[(size_t)b * stride + i] - st.V;
    if (e >= 0 && e < C) atomicAdd(&usage[(size_t)b * st.cap + e], 1);
  }
}

// Pruning / selective retention (zip2zip paper, discussion, "Codebook Management Strategy", item 1): entry e
// stays iff keep[e] != 0 and its prefix without the last token is a base token or an entry that stays; the
// survivors keep their order and are renumbered.  One wave per sequence, wave-uniform, in two sweeps over the
// entries in creation order (a prefix is always older than its extensions): the first walks the trie as it
// is to find every entry's prefix and decides who stays (new_id: new index or -1; prefix: scratch); the
// second empties the table, moves the survivors' rows down and inserts their edges under the new numbers.
__global__ void __launch_bounds__(kWave) lzw_prune_kernel(LzwArgs a, const int32_t* keep, int32_t* new_id, int32_t* prefix) {
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int V = st.V, M = st.M, cap = st.cap;
  const int C = min(max(__builtin_amdgcn_readfirstlane(st.size[b]), 0), cap);
  int32_t* ent_tokens = st.ent_tokens + (size_t)b * cap * M;
  int32_t* ent_len = st.ent_len + (size_t)b * cap;
  const int32_t* kp = keep + (size_t)b * cap;
  int32_t* nid = new_id + (size_t)b * cap;
  int32_t* pre = prefix + (size_t)b * cap;
  Table<false> t;
  table_open<false>(a, b, lane, false, &t);
  int kept = 0;
  for (int e = 0; e < C; ++e) {
    const int L = min(max(__builtin_amdgcn_readfirstlane(ent_len[e]), 2), M);
    const int32_t tok = lane < L ? ent_tokens[(size_t)e * M + lane] : 0;
    int32_t code = __builtin_amdgcn_readlane(tok, 0);
    for (int j = 1; j < L - 1; ++j) {
      int fp;
      code = V + t.find(code, __builtin_amdgcn_readlane(tok, j), &fp);     // exists: the codebook is prefix-closed
    }
    const int p = L == 2 ? -1 : code - V;
    // (read past the vector L1: the line may have been cached before lane 0 wrote this element)
    const int pn = p < 0 ? 0 : __builtin_amdgcn_readfirstlane(__hip_atomic_load(&nid[p], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    const bool stays = __builtin_amdgcn_readfirstlane(kp[e]) != 0 && pn >= 0;
    if (lane == 0) {
      nid[e] = stays ? kept : -1;
      pre[e] = p;
    }
    kept += stays ? 1 : 0;
    __syncthreads();                                 // nid[e] is read by the entries that extend e
  }
  for (int i = lane; i < st.nslots; i += kWave) t.g[i] = kEmpty;
  sync_after_global_stores();                        // the re-insert sweep probes the cleared table past the L1
  for (int e = 0; e < C; ++e) {
    const int n = __builtin_amdgcn_readfirstlane(__hip_atomic_load(&nid[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (n < 0) continue;
    const int L = min(max(__builtin_amdgcn_readfirstlane(ent_len[e]), 2), M);
    const int32_t tok = lane < M ? ent_tokens[(size_t)e * M + lane] : -1;
    const int p = __builtin_amdgcn_readfirstlane(__hip_atomic_load(&pre[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    const int32_t parent = p < 0 ? __builtin_amdgcn_readlane(tok, 0)
                                 : V + __builtin_amdgcn_readfirstlane(__hip_atomic_load(&nid[p], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    int free_pos = -1;
    t.find(parent, __builtin_amdgcn_readlane(tok, L - 1), &free_pos);
    __syncthreads();                                 // row e is read before row n <= e is overwritten
    if (lane == 0) {
      t.store((uint32_t)free_pos, edge_bits(parent, __builtin_amdgcn_readlane(tok, L - 1)) | (u64)(uint32_t)n);
      ent_len[n] = L;
    }
    if (lane < M) ent_tokens[(size_t)n * M + lane] = tok;
    __syncthreads();
  }
  for (int e = kept + lane; e < C; e += kWave) ent_len[e] = 0;            // the rows above the survivors are unused again
  for (int i = kept * M + lane; i < C * M; i += kWave) ent_tokens[i] = -1;
  if (lane == 0) {
    st.size[b] = kept;
    st.prev_code[b] = -1;
    st.prev_len[b] = 0;
    a.out_n[b] = kept;
  }
}

// Codebook prefilling: the given phrases become entries, in order, before any input is parsed (zip2zip
// paper, discussion, "Codebook Management Strategy", item 2).  A phrase is taken if it keeps the codebook what
// the parse kernels rely on: 2..M tokens, all in [0, V), its prefix without the last token a base token or an
// entry already, itself not an entry yet, and the codebook not full; the first phrase that is not ends the
// sequence's prefill with a status bit.  One wave per sequence, wave-uniform scalar walk of the trie in the
// global table.  a.in = phrases [B, stride, M], a.in_len = [B] counts or nullptr, a.out = phrase lengths
// [B, stride], a.out_n = [B] entries added.
__global__ void __launch_bounds__(kWave) lzw_prefill_kernel(LzwArgs a) {
  const LzwState& st = a.st;
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int V = st.V, M = st.M, cap = st.cap;
  const bool reset = (a.flags & Z2Z_RESET) != 0;
  int C = reset ? 0 : __builtin_amdgcn_readfirstlane(st.size[b]);
  Table<false> t;
  table_open<false>(a, b, lane, reset, &t);
  const int n = call_length(a, b);
  const int32_t* phrases = a.in + (size_t)b * a.stride * M;
  const int32_t* lens = a.out + (size_t)b * a.stride;
  int status = 0, added = 0;
  for (int i = 0; i < n; ++i) {
    const int L = __builtin_amdgcn_readfirstlane(lens[i]);
    if (L < 2 || L > M) {
      status |= Z2Z_ST_BAD_TOKEN;
      break;
    }
    const int32_t tok = lane < L ? phrases[(size_t)i * M + lane] : 0;      // lane j = token j
    if (__any(lane < L && (tok < 0 || tok >= V))) {
      status |= Z2Z_ST_BAD_TOKEN;
      break;
    }
    int32_t code = __builtin_amdgcn_readlane(tok, 0);
    bool known = true;
    for (int j = 1; j < L - 1 && known; ++j) {
      int fp;
      const int idx = t.find(code, __builtin_amdgcn_readlane(tok, j), &fp);
      known = idx >= 0;
      code = V + idx;
    }
    int free_pos = -1;
    const int32_t last = __builtin_amdgcn_readlane(tok, L - 1);
    if (!known || t.find(code, last, &free_pos) >= 0 || free_pos < 0) {
      status |= Z2Z_ST_BAD_CODE;                     // prefix unknown, or the phrase is an entry already
      break;
    }
    if (C >= cap) {
      status |= Z2Z_ST_OVERFLOW;
      break;
    }
    table_insert<false>(a, b, lane, t, free_pos, C, code, last, tok, L - 1);
    ++C;
    ++added;
    __syncthreads();                                 // the slot is visible to the next phrase's walk
  }
  if (lane == 0) {
    st.size[b] = C;
    st.prev_code[b] = -1;                            // the parse starts afresh: no pending phrase
    st.prev_len[b] = 0;
    a.out_n[b] = added;
    a.status[b] = status;
  }
}

}  // namespace

int z2z_launch_lzw_reset(z2z_ctx* c, hipStream_t s) {
  c->enc_kept = false;   // the rows a keeping encoder pass left behind belong to the codebook as it was
  hipLaunchKernelGGL(lzw_reset_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_codebook_usage(z2z_ctx* c, const int32_t* codes, const int32_t* n_codes, int32_t stride, int32_t* usage,
                              hipStream_t s) {
  hipLaunchKernelGGL(lzw_usage_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st, codes, n_codes, stride, usage);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_codebook_prune(z2z_ctx* c, const int32_t* keep, int32_t* new_id, int32_t* n_kept, hipStream_t s) {
  c->enc_kept = false;   // the rows a keeping encoder pass left behind belong to the codebook as it was
  if (!c->prune_prefix && c->cfg.cap > 0) return Z2Z_EHIP;       // (allocated by z2z_create)
  LzwArgs a;
  memset(&a, 0, sizeof(a));
  a.st = c->st;
  a.out_n = n_kept;
  hipLaunchKernelGGL(lzw_prune_kernel, dim3(c->cfg.B), dim3(kWave), 0, s, a, keep, new_id,
                     reinterpret_cast<int32_t*>(c->prune_prefix));
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_codebook_prefill(z2z_ctx* c, const int32_t* phrases, const int32_t* phrase_len, const int32_t* counts,
                                int32_t n_max, int32_t flags, int32_t* n_added, int32_t* status, hipStream_t s) {
  c->enc_kept = false;   // the rows a keeping encoder pass left behind belong to the codebook as it was
  LzwArgs a;
  memset(&a, 0, sizeof(a));
  a.st = c->st;
  a.in = phrases;
  a.in_len = counts;
  a.stride = n_max;
  a.flags = flags;
  a.out = const_cast<int32_t*>(phrase_len);          // read only
  a.out_n = n_added;
  a.out_stride = n_max;
  a.status = status;
  a.lds_ef = 0;
  if (flags & Z2Z_RESET) hipLaunchKernelGGL(lzw_clear_entries_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
  hipLaunchKernelGGL(lzw_prefill_kernel, dim3(c->cfg.B), dim3(kWave), 0, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// Four waves per sequence beat one as long as the machine is not full of sequences anyway: measured faster up
// to 1024 sequences of 4096 tokens (B = 512: encode 218 -> 155 us, decode 168 -> 120 us), about equal at 1024
// tokens, slower from 2048 sequences on.
static bool wide_pays(int B, int stride) {
  return stride >= 512 && (B <= 256 || (B <= 1024 && stride >= 2048));
}

int z2z_launch_lzw_encode(z2z_ctx* c, const int32_t* tokens, const int32_t* lens, int32_t stride, int32_t flags,
                          int32_t* codes, int32_t* n_codes, int32_t out_stride, int32_t* status, hipStream_t s) {
  c->enc_kept = false;   // the rows a keeping encoder pass left behind belong to the codebook as it was
  LzwArgs a;
  memset(&a, 0, sizeof(a));
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
  bool lds = false;
  plan(c, stride, flags, false, &lds, &a, &smem);
  if (flags & Z2Z_RESET) hipLaunchKernelGGL(lzw_clear_entries_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
  // few long sequences: four waves per sequence (the machine is nearly empty, a sequence's parse time counts)
  const bool wide = wide_pays(c->cfg.B, stride) && c->opt_lzw_kernel != 4 &&
                    (!lds || smem + kWideStaticLds <= (size_t)c->lds_limit);
  if (wide && lds)
    hipLaunchKernelGGL(lzw_encode_wide_kernel<true>, dim3(c->cfg.B), dim3(kWideLanes), smem, s, a);
  else if (wide)
    hipLaunchKernelGGL(lzw_encode_wide_kernel<false>, dim3(c->cfg.B), dim3(kWideLanes), 0, s, a);
  else if (lds)
    hipLaunchKernelGGL(lzw_encode_kernel<true>, dim3(c->cfg.B), dim3(kWave), smem, s, a);
  else
    hipLaunchKernelGGL(lzw_encode_kernel<false>, dim3(c->cfg.B), dim3(kWave), 0, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_lzw_decode(z2z_ctx* c, const int32_t* codes, const int32_t* n_codes, int32_t stride, int32_t flags,
                          int32_t* tokens, int32_t* n_tokens, int32_t out_stride, int32_t* status, hipStream_t s) {
  c->enc_kept = false;   // the rows a keeping encoder pass left behind belong to the codebook as it was
  LzwArgs a;
  memset(&a, 0, sizeof(a));
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
  bool lds = false;
  plan(c, stride, flags, true, &lds, &a, &smem);
  if (flags & Z2Z_RESET) hipLaunchKernelGGL(lzw_clear_entries_kernel, dim3(c->cfg.B), dim3(256), 0, s, c->st);
  const bool serial = stride <= 8 || c->opt_lzw_kernel == 3;
  const bool wide = !serial && wide_pays(c->cfg.B, stride) && c->opt_lzw_kernel != 4 &&
                    (!lds || smem + kWideStaticLds <= (size_t)c->lds_limit);
  if (wide && lds)
    hipLaunchKernelGGL(lzw_decode_wide_kernel<true>, dim3(c->cfg.B), dim3(kWideLanes), smem, s, a);
  else if (wide)
    hipLaunchKernelGGL(lzw_decode_wide_kernel<false>, dim3(c->cfg.B), dim3(kWideLanes), 0, s, a);
  else if (serial && lds)
    hipLaunchKernelGGL(lzw_decode_serial_kernel<true>, dim3(c->cfg.B), dim3(kWave), smem, s, a);
  else if (serial)
    hipLaunchKernelGGL(lzw_decode_serial_kernel<false>, dim3(c->cfg.B), dim3(kWave), 0, s, a);
  else if (lds)
    hipLaunchKernelGGL(lzw_decode_kernel<true>, dim3(c->cfg.B), dim3(kWave), smem, s, a);
  else
    hipLaunchKernelGGL(lzw_decode_kernel<false>, dim3(c->cfg.B), dim3(kWave), 0, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_launch_step_update(z2z_ctx* c, const int32_t* codes, int32_t stride, const void* E, void* W_hyper,
                           int32_t* n_tokens, int32_t* status, hipStream_t s) {
  c->enc_kept = false;
  LzwArgs a;
  memset(&a, 0, sizeof(a));
  a.st = c->st;
  a.in = codes;
  a.in_len = nullptr;
  a.stride = 1;                         // one code per sequence; `stride` is the distance between them
  a.flags = Z2Z_APPEND;
  a.out = nullptr;
  a.out_n = n_tokens;
  a.out_stride = 0;
  a.status = status;
  a.lds_ef = 0;
  a.in_step = stride;
  z2z_embed::EmbedArgs ea;
  z2z_embed::fill_embed_args(c, E, W_hyper, &ea);
  const int chunks = c->cfg.d / (c->cfg.dtype == Z2Z_BF16 ? 8 : 4);
  int split = 1;
  while (split < kStepWaves && chunks >= 128 * split) split *= 2;    // a wave takes at least 64 chunks of the row
  ea.split = split;
  if (c->cfg.dtype == Z2Z_BF16)
    hipLaunchKernelGGL(lzw_step_update_kernel<true>, dim3(c->cfg.B), dim3(kStepWaves * kWave), 0, s, a, ea);
  else
    hipLaunchKernelGGL(lzw_step_update_kernel<false>, dim3(c->cfg.B), dim3(kStepWaves * kWave), 0, s, a, ea);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

// Size the hash table for the device's LDS and raise the dynamic-LDS ceiling of the parse kernels.
// Load factor at a full codebook is at most 0.8 (at least 1.25 slots per entry; 2 or 4 when LDS allows).
int z2z_lzw_prepare(z2z_ctx* c) {
  LzwState& st = c->st;
  const int cap = st.cap;
  const int want4 = 4 * cap < 64 ? 64 : 4 * cap;
  const int want = 2 * cap < 64 ? 64 : 2 * cap;
  const int floor125 = cap + cap / 4 + 1;
  const int lds_slots = (c->lds_limit - kEncStaticLds) / (int)sizeof(u64);   // the encoder's own LDS comes first
  // With fewer sequences than CUs a workgroup has its CU to itself and the roomier table (shorter probe
  // sequences) is free; with many, LDS decides how many sequences a CU works on at once.
  const bool roomy = c->cfg.B < 256;
  if (roomy && want4 + cap / 2 <= lds_slots) {        // room left for the decoder's entry info
    st.nslots = want4;
    st.slots_fit_lds = 1;
  } else if (want <= lds_slots) {
    st.nslots = want;
    st.slots_fit_lds = 1;
  } else if (floor125 <= lds_slots) {
    st.nslots = lds_slots;
    st.slots_fit_lds = 1;
  } else {
    st.nslots = want;
    st.slots_fit_lds = 0;
  }
  st.nslots &= ~1;                                     // even: probe sequences start on slot pairs
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(lzw_encode_kernel<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit - kEncStaticLds));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(lzw_encode_wide_kernel<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit - kWideStaticLds));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(lzw_decode_wide_kernel<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit - kWideStaticLds));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(lzw_decode_kernel<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit - kEncStaticLds));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(lzw_decode_serial_kernel<true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, c->lds_limit - kEncStaticLds));
  return Z2Z_OK;
}
