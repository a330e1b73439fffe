// extended_logits, bf16 MFMA kernel for gfx950 (d a multiple of 64), one wave per SIMD.
//
// Workgroup tile 256 (vocabulary rows, MFMA "A") x 256 (hidden rows, MFMA "B"), 4 waves in a 2 x 2 grid,
// each wave 128 x 128 = 4 x 4 blocks of v_mfma_f32_32x32x16_bf16 (256 accumulator registers per lane):
// per 16-deep k-step a wave reads 8 operand fragments from LDS for 16 MFMAs.  With one wave per SIMD all
// overlap is inside the instruction stream: the fragments of k-step t+1 are read while the MFMAs of
// k-step t run, and the global->LDS requests of slab s+2 are handed out one pair at a time between the
// MFMAs that follow the hand-over of slab s.  (F_WAVES = 8 builds the same kernel with two waves per SIMD,
// each 128 x 64; measured equal, so the default stays at the layout with the larger register tiles.)
//
// K advances in slabs of 64 elements (128 bytes per row, four k-steps): the global -> LDS stream moves
// whole 128-byte lines, which it does markedly faster than half lines (measured on a bare streaming
// kernel: 14-22 TB/s against 12-15 TB/s out of L2).  Both operand tiles of a slab (2 x 32 KiB) go straight
// from global memory into LDS (16-byte global_load ... lds), two stages.  Once per slab, in the middle of
// its last k-step, the waves meet at a barrier: at that point everybody has read the slab completely (its
// stage is refilled with slab s+2) and slab s+1 has landed (its first fragments are read next).  The stream
// runs on across the vocabulary tiles of a strip.  The refill requests are spread over the following
// ~35 MFMAs: issued as one burst they back up the memory pipeline, the wave then stalls on its next
// request, and a stalled wave issues no MFMAs (measured: 28.9 ms as a burst, 26.3 ms spread, 22.9 ms with
// no requests at all on the 32768 x 4096 x 128256 problem); spread over the whole slab they would land
// too late for the next hand-over.
//
// LDS layout of an operand tile: row r = 128 bytes = 8 chunks of 16 B; chunk c is stored at position
// c ^ ((r >> 1) & 7).  The LDS has 64 four-byte banks and serves a 16-byte-per-lane read 16 lanes at a
// time; an MFMA operand read has 16 consecutive lanes on 16 consecutive rows at one logical chunk, whose
// bank group is (r & 1) * 8 + position -- all 16 distinct with this swizzle.
//
// In the 32x32 result block a lane holds 16 vocabulary entries of one hidden row, so the running
// (max, sum-exp, argmax) of the joint softmax (zip2zip paper, section 2.3, step 8) lives in registers
// and crosses lanes once per strip.
#include "logits_common.h"

namespace {

using namespace z2z_logits;

constexpr int FT = 256;                   // tile edge, vocabulary and hidden rows
constexpr int F_SLAB = 128;               // bytes per row per K slab (64 bf16)
constexpr int F_OPER = FT * F_SLAB;       // one operand tile of one slab: 32 KiB
constexpr int F_STAGE = 2 * F_OPER;       // A + B
constexpr int F_NSTAGE = 2;
constexpr int F_LDS = F_NSTAGE * F_STAGE; // 128 KiB
#ifndef F_WAVES
#define F_WAVES 4
#endif
constexpr int F_THREADS = 64 * F_WAVES;
// waves: 2 along the vocabulary rows (128 each: 4 MFMA blocks), F_WAVES / 2 along the hidden rows
constexpr int F_NI = 4;
constexpr int F_WR = F_WAVES / 2;
constexpr int F_NJ = FT / (F_WR * 32);                 // MFMA blocks of a wave along the hidden rows
constexpr int F_KSTEP = F_NI * F_NJ;                   // MFMAs of a wave per k-step
constexpr int F_PAIRS = 32 / F_WAVES;                  // request pairs (8 rows of A + 8 rows of B) per wave and slab
#ifndef F_SPREAD
#define F_SPREAD (F_WAVES == 4 ? 5 : 4)
#endif
// Pacing of the two operand paths inside the MFMA stream.  With one wave per SIMD, and the four waves of a
// workgroup in step (they meet at a barrier every slab), whatever a wave issues as a burst arrives at the LDS or
// at the memory pipeline together with the other waves' bursts, and the MFMAs wait behind it.  Measured on the
// 32768 x 4096 x 128256 problem, same box, each step on top of the previous one: fragment reads of the next
// k-step one per MFMA instead of eight ahead of the k-step: -2.1 %; the same for the first k-step of the next slab
// after the hand-over barrier: -1.4 %; the two requests of a pair two MFMAs apart (a request every 2-3 MFMAs)
// instead of back to back every five: -0.7 %.  Closer spacing of the requests (every 1.5 MFMAs) or wider (every 3,
// 3.5) is slower, and so are reads that start right at the first MFMA of a k-step.
//   F_LDS_SPREAD       1 = read n of the next k-step goes out after MFMA F_RD_FIRST + n * F_RD_EVERY of the
//                      current one (in the order of first use), 0 = all eight ahead of the k-step
//   F_HANDOVER_SPREAD  1 = the same for the reads that follow the hand-over barrier
//   F_SPLIT_PAIR       n > 0 = the hidden-row request of a pair goes out n MFMAs after the vocabulary-row one
#ifndef F_LDS_SPREAD
#define F_LDS_SPREAD 1
#endif
#ifndef F_SPLIT_PAIR
#define F_SPLIT_PAIR 2
#endif
#ifndef F_HANDOVER_SPREAD
#define F_HANDOVER_SPREAD 1
#endif
#ifndef F_RD_FIRST
#define F_RD_FIRST 3
#endif
#ifndef F_RD_EVERY
#define F_RD_EVERY 1
#endif
// Request pair i goes out after the MFMA with window index 1 + i * F_SPREAD, counted from the slab
// hand-over: first the rest of the hand-over k-step (F_KSTEP - F_NJ MFMAs), then the first three k-steps
// of the next slab.
#ifndef F_ROTATE_FEW
#define F_ROTATE_FEW 1                   // 0: the rotated-K instances (see the kernel) are never launched
#endif
#ifndef F_HO_ROWS
#define F_HO_ROWS 1
#endif
#ifndef F_HO_RD_FIRST
#define F_HO_RD_FIRST F_RD_FIRST
#endif
constexpr int F_REST = F_KSTEP - F_HO_ROWS * F_NJ;   // MFMAs of the hand-over k-step that follow the barrier
static_assert(!F_LDS_SPREAD || !F_HANDOVER_SPREAD || F_HO_RD_FIRST + (F_NI + F_NJ - 1) * F_RD_EVERY < F_REST,
              "the reads after the hand-over must all go out before the k-step ends");
static_assert(!F_LDS_SPREAD || F_RD_FIRST + (F_NI + F_NJ - 1) * F_RD_EVERY < F_KSTEP, "reads of a k-step must fit it");
constexpr int F_LAST_IN_HANDOVER = (F_REST - 2) / F_SPREAD;          // last pair issued before the slab ends
static_assert(F_LAST_IN_HANDOVER < F_PAIRS, "spread too small for this layout");
static_assert(1 + (F_PAIRS - 1) * F_SPREAD < F_REST + 3 * F_KSTEP, "all pairs must be out before the next hand-over");
constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }

// 16 bytes per lane, global -> LDS without passing through registers: address = 64-bit scalar base +
// 32-bit per-lane offset; the LDS address is the wave-uniform byte offset in M0 plus 16 * lane.  Inline
// assembly on purpose: the compiler cannot tell the LDS stages apart and would make every LDS read wait
// for all outstanding direct loads.  Completion is awaited explicitly (s_waitcnt vmcnt) before the
// barrier that publishes a stage.  One wait state is required between the write of M0 and its use.
// M0 is written as stage base + constant in one scalar instruction: with one wave per SIMD every
// instruction issued between two MFMAs counts, and the request stream is the bulk of them.
template <int LDS_IMM>
__device__ __forceinline__ void load16_to_lds(const unsigned char* base, uint32_t lane_offset, uint32_t lds_stage_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_offset), "s"(base), "s"(lds_stage_base), "n"(LDS_IMM)
               : "memory", "scc");   // M0 is reserved: the compiler keeps nothing in it across statements
}

__device__ __forceinline__ uint32_t lds_offset_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// Workgroup id -> (row tile, strip) for the base part; returns false when the id maps to no work.
__device__ __forceinline__ bool map_base(const LogitsArgs& a, int bid, int* rt, int* st) {
  const int xcd = bid & 7;
  const int j = bid >> 3;
  const int per = a.map_lr * a.map_ls;
  const int g = j / per;
  const int within = j - g * per;
  const int lr = within % a.map_lr;
  const int ls = within / a.map_lr;
  const int xr = xcd % a.map_xr;
  const int xs = xcd / a.map_xr;
  const int sb_r = g % a.map_sb_r;
  const int sb_s = g / a.map_sb_r;
  *rt = (sb_r * a.map_xr + xr) * a.map_lr + lr;
  *st = (sb_s * a.map_xs + xs) * a.map_ls + ls;
  return *rt < a.row_tiles && *st < a.n_strips;
}

// Linear mode when the number of rows is known on the device only.  Workgroup ids go round-robin over the 8
// XCDs; an XCD walks blocks of map_lr row tiles x map_ls weight tiles ("strips" of one tile), the weight
// tiles of a row block before the next row block.  What an XCD owns is decided here, on the device, from the
// row count: if the weight tiles divide evenly among the XCDs (map_xs = 8), XCD x owns the weight tiles
// x, x + 8, ... and every row tile -- equal shares whatever the count is; otherwise row tile t belongs to XCD
// t mod 8 (shares differ by one row tile at most).  The grid is sized for the rows laid out.
__device__ __forceinline__ bool map_rows_dev(const LogitsArgs& a, int bid, int row_tiles_now, int* rt, int* st) {
  const int xcd = bid & 7;
  const int j = bid >> 3;
  const int per = a.map_lr * a.map_ls;
  const int blk = j / per;
  const int within = j - blk * per;
  const int lr = within % a.map_lr;
  const int ls = within / a.map_lr;
  const int sblk = blk % a.strip_blocks;
  const int rblk = blk / a.strip_blocks;
  if (a.map_xs == 8) {
    *rt = rblk * a.map_lr + lr;
    *st = (sblk * a.map_ls + ls) * 8 + xcd;
  } else {
    *rt = (rblk * a.map_lr + lr) * 8 + xcd;
    *st = sblk * a.map_ls + ls;
  }
  return *rt < row_tiles_now && *st < a.n_strips;
}

struct Frags {
  uint4 a[F_NI];
  uint4 b[F_NJ];
};

// MODE 8 and 9 are measurement probes of the base part (their results are NOT the logits' reduction): 8 stops
// requesting operands after the first two slabs (the matrix cores, the LDS reads and the fold run as usual on
// those two slabs' values), 9 also stops reading LDS and folds once per strip -- the MFMA stream alone.  They
// bracket what the operand stream costs and give the clock the matrix cores alone are left with.
// ROT (base part with a single row tile: up to 256 hidden rows): nobody shares a workgroup's weight tiles, so the
// strips walk K from different slabs, wrapping round.  With all of them at the same
// slab every request in flight goes to the same 128-byte column of rows a power of two apart, and with it to the
// same few memory channels.  (With many row tiles the workgroups that share operands through L2 and the
// memory-side cache must stay in step: there the rotation costs 1-2 %, and so does its arithmetic alone; with two
// row tiles it is level or 1 % slower.  A decode step of 256 sequences: 646 -> 634 us, with a filtered draw 704 -> 675.)
template <int MODE, bool ROT = false>
__global__ void __launch_bounds__(F_THREADS) logits_fast_kernel(LogitsArgs a) {
  constexpr bool PROBE_NOREQ = MODE == 8 || MODE == 9;
  constexpr bool PROBE_MFMA = MODE == 9;
  extern __shared__ __align__(1024) unsigned char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wv = wave & 1;    // which 128 vocabulary rows of the tile
  const int wr = wave >> 1;   // which F_NJ * 32 hidden rows of the tile

  int rt, st;
  int r0, r_end, n_valid;
  const unsigned char* Wp = reinterpret_cast<const unsigned char*>(a.W);
  const size_t row_bytes = (size_t)a.d * 2;
  if (MODE == 1 || MODE == 4) {
    if ((int)blockIdx.x >= a.n_work) return;
    rt = blockIdx.x / a.n_strips;
    // workgroup ids go round-robin over the 8 XCDs, and the strips beyond a sequence's C_b are empty: with the
    // strip taken straight from the id, the XCDs that own the low strips would do all the work (config 5: 9 of 16
    // strips exist, XCD 0 owned two of them, the others one).  Rotating by the row tile deals them out evenly.
    st = (int)((blockIdx.x + (unsigned)rt) % (unsigned)a.n_strips);
    const int b = rt / a.row_tiles;
    r0 = b * a.rows_per_seq + (rt % a.row_tiles) * FT;
    r_end = (b + 1) * a.rows_per_seq;
    n_valid = min(max(a.size[b], 0), a.w_rows);
    Wp += (size_t)b * a.w_rows * row_bytes;
  } else if (MODE == 5) {
    // few tiles, K split: workgroup -> (K part, row tile, weight tile)
    r_end = a.rows_dev ? min(a.rows, *a.rows_dev) : a.rows;
    const int t = blockIdx.x / a.ksplit;
    rt = t % a.row_tiles;
    st = t / a.row_tiles;
    if (st >= a.n_strips) return;
    r0 = rt * FT;
    if (r0 >= r_end) return;
    n_valid = a.w_rows;
  } else {
    r_end = a.rows;
    if (MODE == 2 && a.rows_dev) r_end = min(r_end, *a.rows_dev);
    if (MODE == 2 && a.strip_blocks > 0) {
      if (!map_rows_dev(a, blockIdx.x, (r_end + FT - 1) / FT, &rt, &st)) return;
    } else {
      if (!map_base(a, blockIdx.x, &rt, &st)) return;
    }
    r0 = rt * FT;
    if (r0 >= r_end) return;                       // a tile beyond the rows that exist
    n_valid = a.w_rows;
  }
  const unsigned char* Hp = reinterpret_cast<const unsigned char*>(a.H) + (size_t)r0 * row_bytes;
  const int ks = MODE == 5 ? (int)(blockIdx.x % a.ksplit) : 0;
  if (MODE == 5) {                                   // this part's slabs start here in every row
    Wp += (size_t)ks * a.slabs_per_part * F_SLAB;
    Hp += (size_t)ks * a.slabs_per_part * F_SLAB;
  }
  const int vt0 = st * a.strip;
  const int vt_end = min(min(vt0 + a.strip, a.n_vtiles), (n_valid + FT - 1) / FT);
  const int n_tiles = vt_end - vt0;          // vocabulary tiles this workgroup sweeps (may be <= 0)
  int n_slabs = MODE == 5 ? min(a.slabs_per_part, (int)(row_bytes / F_SLAB) - ks * a.slabs_per_part)
                          : (int)(row_bytes / F_SLAB);
  if (MODE == 2 && a.k_dev) n_slabs = max(1, min(n_slabs, (*a.k_dev * 2 + F_SLAB - 1) / F_SLAB));

  Triple run[F_NJ];
  Draw draw[F_NJ];                                   // MODE 6 only
#pragma unroll
  for (int j = 0; j < F_NJ; ++j) {
    run[j] = empty_triple();
    draw[j] = empty_draw();
  }

  // ---- loader: lane l of wave w, instruction i moves the chunk that lands at LDS byte
  //      ((w * F_PAIRS + i) * 8 + (l >> 3)) * 128 + (l & 7) * 16 of the operand tile; offsets are relative to
  //      the first row of the tile, rows past the last valid one are clamped onto it ------------------
  const uint32_t lds_base = lds_offset_of(lds);
  const int ld_row = lane >> 3;                                  // row inside the 8-row group
  const int limB = r_end - 1 - r0;                               // last valid hidden row of the tile
  const unsigned char* Wtile = Wp;
  int limA = 0;                                                  // last valid vocabulary row of the tile
  // per-lane global byte offsets of the 8 row groups a wave requests (swizzled chunk folded in); rows
  // past the last valid one are clamped onto it.  B's never change, A's change with the tile.
  auto row_offset = [&](int i, int lim) -> uint32_t {
    const int row = (wave * F_PAIRS + i) * 8 + ld_row;
    const int chunk16 = ((lane & 7) ^ ((row >> 1) & 7)) * 16;
    return (uint32_t)(min(row, lim) * (int)row_bytes + chunk16);
  };
  uint32_t voffA[F_PAIRS], voffB[F_PAIRS];
#pragma unroll
  for (int i = 0; i < F_PAIRS; ++i) voffB[i] = row_offset(i, limB);
  auto set_tile = [&](int vt) {
    Wtile = Wp + (size_t)vt * FT * row_bytes;
    limA = n_valid - 1 - vt * FT;
#pragma unroll
    for (int i = 0; i < F_PAIRS; ++i) voffA[i] = row_offset(i, limA);
  };
  // request the slab that follows (lslab, lvt) in the stream, if any, and advance the cursor.  A request
  // is 16 instructions per wave; issue_rows<i>() issues the pair for row group i so that the caller can
  // place the pairs between MFMAs.
  int lslab = 0, lvt = vt0;
  uint32_t isA = 0;                          // LDS destination (operand A) of the slab being requested
  const unsigned char* is_ga = Wp;
  const unsigned char* is_gb = Hp;
  const int rot = ROT ? st % n_slabs : 0;
  auto issue_begin = [&](int stage) {
    isA = lds_base + stage * F_STAGE + wave * (F_PAIRS * 1024);
    if (lvt < vt_end) {                      // else: keep the last valid source
      int sl = lslab;
      if (ROT) {
        sl += rot;
        if (sl >= n_slabs) sl -= n_slabs;
      }
      is_ga = Wtile + (size_t)sl * F_SLAB;
      is_gb = Hp + (size_t)sl * F_SLAB;
    }
  };
#define Z2Z_ISSUE_PAIR(i)                                             \
  do {                                                                \
    load16_to_lds<(i) * 1024>(is_ga, voffA[i], isA);                  \
    load16_to_lds<F_OPER + (i) * 1024>(is_gb, voffB[i], isA);         \
  } while (0)
#define Z2Z_ISSUE_A(i) load16_to_lds<(i) * 1024>(is_ga, voffA[i], isA)
#define Z2Z_ISSUE_B(i) load16_to_lds<F_OPER + (i) * 1024>(is_gb, voffB[i], isA)
  auto issue_end = [&]() {
    if (lvt < vt_end && ++lslab == n_slabs) {
      lslab = 0;
      ++lvt;
      if (lvt < vt_end) set_tile(lvt);
    }
  };
  // ---- MFMA operand addresses (bytes inside an operand tile), swizzle folded in ---------------------
  const int sw = (lane >> 1) & 7;   // ((row >> 1) & 7) of every row this lane reads
  const int half = lane >> 5;
  const int offA0 = (wv * 128 + (lane & 31)) * F_SLAB;
  const int offB0 = (wr * (F_NJ * 32) + (lane & 31)) * F_SLAB;
  auto read_frags = [&](Frags& f, int stage, int q) {
    const unsigned char* A = lds + stage * F_STAGE + offA0 + (((2 * q + half) ^ sw) << 4);
    const unsigned char* Bt = lds + stage * F_STAGE + F_OPER + offB0 + (((2 * q + half) ^ sw) << 4);
#pragma unroll
    for (int i = 0; i < F_NI; ++i) f.a[i] = *reinterpret_cast<const uint4*>(A + i * 32 * F_SLAB);
#pragma unroll
    for (int j = 0; j < F_NJ; ++j) f.b[j] = *reinterpret_cast<const uint4*>(Bt + j * 32 * F_SLAB);
  };

  // one fragment of a k-step, so that the reads of the next k-step can be handed out between the MFMAs of the
  // current one; n counts them in the order the MFMAs (vocabulary block i outer, hidden-row block j inner) first
  // need them: b0, a0, b1 .. b(NJ-1), a1 .. a(NI-1)
  auto read_one = [&](Frags& f, int stage, int q, int n) {
    const int base = stage * F_STAGE + (((2 * q + half) ^ sw) << 4);
    const bool is_a = n == 1 || n > F_NJ;
    const int idx = n == 0 ? 0 : (n == 1 ? 0 : (n <= F_NJ ? n - 1 : n - F_NJ));
    if (is_a)
      f.a[idx] = *reinterpret_cast<const uint4*>(lds + base + offA0 + idx * 32 * F_SLAB);
    else
      f.b[idx] = *reinterpret_cast<const uint4*>(lds + base + F_OPER + offB0 + idx * 32 * F_SLAB);
  };

  f32x16 acc[F_NI][F_NJ];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < F_NI; ++i)
#pragma unroll
      for (int j = 0; j < F_NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  };
  // pair i of the request in progress (switch: the LDS offset is an instruction literal)
  auto issue_pair = [&](int i) {
    switch (i) {
      case 0: Z2Z_ISSUE_PAIR(0); break;
      case 1: Z2Z_ISSUE_PAIR(1); break;
      case 2: Z2Z_ISSUE_PAIR(2); break;
#if F_WAVES == 4
      case 3: Z2Z_ISSUE_PAIR(3); break;
      case 4: Z2Z_ISSUE_PAIR(4); break;
      case 5: Z2Z_ISSUE_PAIR(5); break;
      case 6: Z2Z_ISSUE_PAIR(6); break;
      default: Z2Z_ISSUE_PAIR(7); break;
#else
      default: Z2Z_ISSUE_PAIR(3); break;
#endif
    }
  };
  // The MFMAs of blocks [i_lo, i_hi) x [0, F_NJ); w0 = window index of the first one.  After an MFMA
  // whose window index is 1 + i * F_SPREAD, request pair i is issued (fenced, so that it stays there: a
  // burst of requests backs up the memory pipeline, and a wave that cannot issue its request cannot issue
  // MFMAs either).
  // the two requests of pair i on their own (F_SPLIT_PAIR: the hidden-row half goes out a few MFMAs after the other)
  auto issue_a = [&](int i) {
    switch (i) {
      case 0: Z2Z_ISSUE_A(0); break;
      case 1: Z2Z_ISSUE_A(1); break;
      case 2: Z2Z_ISSUE_A(2); break;
#if F_WAVES == 4
      case 3: Z2Z_ISSUE_A(3); break;
      case 4: Z2Z_ISSUE_A(4); break;
      case 5: Z2Z_ISSUE_A(5); break;
      case 6: Z2Z_ISSUE_A(6); break;
      default: Z2Z_ISSUE_A(7); break;
#else
      default: Z2Z_ISSUE_A(3); break;
#endif
    }
  };
  // The MFMAs of blocks [i_lo, i_hi) x [0, F_NJ); w0 = window index of the first one.  After an MFMA
  // whose window index is 1 + i * F_SPREAD, request pair i is issued (fenced, so that it stays there: a
  // burst of requests backs up the memory pipeline, and a wave that cannot issue its request cannot issue
  // MFMAs either).
  auto issue_b = [&](int i) {
    switch (i) {
      case 0: Z2Z_ISSUE_B(0); break;
      case 1: Z2Z_ISSUE_B(1); break;
      case 2: Z2Z_ISSUE_B(2); break;
#if F_WAVES == 4
      case 3: Z2Z_ISSUE_B(3); break;
      case 4: Z2Z_ISSUE_B(4); break;
      case 5: Z2Z_ISSUE_B(5); break;
      case 6: Z2Z_ISSUE_B(6); break;
      default: Z2Z_ISSUE_B(7); break;
#else
      default: Z2Z_ISSUE_B(3); break;
#endif
    }
  };
  // The MFMAs of blocks [i_lo, i_hi) x [0, F_NJ); w0 = window index of the first one.  After an MFMA
  // whose window index is 1 + i * F_SPREAD, request pair i is issued (fenced, so that it stays there: a
  // burst of requests backs up the memory pipeline, and a wave that cannot issue its request cannot issue
  // MFMAs either).
  // `nf` (may be null): the fragments of the k-step (nstage, nq) are read into it, one read after every
  // F_RD_EVERY-th MFMA starting at MFMA F_RD_FIRST of this call
  auto mfma_rows = [&](const Frags& f, int i_lo, int i_hi, int w0, Frags* nf = nullptr, int nstage = 0, int nq = 0,
                       int rd_first = F_RD_FIRST) {
#pragma unroll
    for (int i = i_lo; i < i_hi; ++i)
#pragma unroll
      for (int j = 0; j < F_NJ; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i]),
                                                            __builtin_bit_cast(bf16x8, f.b[j]), acc[i][j], 0, 0, 0);
        const int local = (i - i_lo) * F_NJ + j;
        if (F_LDS_SPREAD && nf != nullptr && local >= rd_first && (local - rd_first) % F_RD_EVERY == 0 &&
            (local - rd_first) / F_RD_EVERY < F_NI + F_NJ) {
          __builtin_amdgcn_sched_barrier(0);
          read_one(*nf, nstage, nq, (local - rd_first) / F_RD_EVERY);
          __builtin_amdgcn_sched_barrier(0);
        }
        const int w = w0 + (i - i_lo) * F_NJ + j;
        if (!PROBE_NOREQ && F_SPLIT_PAIR == 0 && w >= 1 && (w - 1) % F_SPREAD == 0 && (w - 1) / F_SPREAD < F_PAIRS) {
          __builtin_amdgcn_sched_barrier(0);
          issue_pair((w - 1) / F_SPREAD);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (!PROBE_NOREQ && F_SPLIT_PAIR > 0 && w >= 1 && (w - 1) % F_SPREAD == 0 && (w - 1) / F_SPREAD < F_PAIRS) {
          __builtin_amdgcn_sched_barrier(0);
          issue_a((w - 1) / F_SPREAD);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (!PROBE_NOREQ && F_SPLIT_PAIR > 0 && w >= 1 + F_SPLIT_PAIR && (w - 1 - F_SPLIT_PAIR) % F_SPREAD == 0 &&
            (w - 1 - F_SPLIT_PAIR) / F_SPREAD < F_PAIRS) {
          __builtin_amdgcn_sched_barrier(0);
          issue_b((w - 1 - F_SPLIT_PAIR) / F_SPREAD);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
  };

  if (n_tiles > 0) {
    zero_acc();
    set_tile(vt0);
    // prologue: slab 0 requested in full, of slab 1 the pairs that a hand-over k-step issues (the rest
    // follows during the first three k-steps, as for every later slab); slab 0 landed and visible, its
    // first fragments on the way
    issue_begin(0);
#pragma unroll
    for (int i = 0; i < F_PAIRS; ++i) issue_pair(i);
    issue_end();
    issue_begin(1);
#pragma unroll
    for (int i = 0; i <= (PROBE_NOREQ ? F_PAIRS - 1 : F_LAST_IN_HANDOVER); ++i) issue_pair(i);
    if (PROBE_NOREQ)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    else
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * (F_LAST_IN_HANDOVER + 1)));   // all of slab 0
    __syncthreads();
    Frags f0, f1;
    read_frags(f0, 0, 0);
    if (PROBE_MFMA) read_frags(f1, 0, 1);
    int g = 0;
    for (int vt = vt0; vt < vt_end; ++vt) {
      for (int slab = 0; slab < n_slabs; ++slab, ++g) {
        const int stage = g & 1;
        if (F_LDS_SPREAD && !PROBE_MFMA) {
          // the fragments of k-step q + 1 are read between the MFMAs of k-step q (as one burst per wave the four
          // waves' reads arrive at the LDS together, right after a barrier, and the MFMAs wait behind them)
          mfma_rows(f0, 0, F_NI, F_REST, &f1, stage, 1);
          mfma_rows(f1, 0, F_NI, F_REST + F_KSTEP, &f0, stage, 2);
          mfma_rows(f0, 0, F_NI, F_REST + 2 * F_KSTEP, &f1, stage, 3);
        } else {
          if (!PROBE_MFMA) read_frags(f1, stage, 1);
          mfma_rows(f0, 0, F_NI, F_REST);
          if (!PROBE_MFMA) read_frags(f0, stage, 2);
          mfma_rows(f1, 0, F_NI, F_REST + F_KSTEP);
          if (!PROBE_MFMA) read_frags(f1, stage, 3);
          mfma_rows(f0, 0, F_NI, F_REST + 2 * F_KSTEP);
        }
        if (!PROBE_NOREQ) issue_end();          // the request for slab g+1 is out in full
        // last k-step: a quarter of its MFMAs, then the slab hand-over.  It is the same for every slab,
        // the last ones included (no test inside the loop): past the end of the stream the requests
        // re-read the last slab into a stage nobody reads again.
        mfma_rows(f1, 0, F_HO_ROWS, 1000);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // slab g+1 (the only one in flight) has landed
        __syncthreads();                            // slab g+1 visible to all; everyone has read slab g
        if (!PROBE_NOREQ) issue_begin(stage);       // refill this stage with slab g+2
        if (F_LDS_SPREAD && F_HANDOVER_SPREAD && !PROBE_MFMA) {
          mfma_rows(f1, F_HO_ROWS, F_NI, 0, &f0, stage ^ 1, 0, F_HO_RD_FIRST);
        } else {
          if (!PROBE_MFMA) read_frags(f0, stage ^ 1, 0);
          mfma_rows(f1, F_HO_ROWS, F_NI, 0);
        }
      }
      // ---- this vocabulary tile is complete: fold its 128 x 128 logits into the running triples ------
      const int v0 = vt * FT;
      if (MODE == 2) {
        if (a.stream_f32)
          store_tile_f32<F_NI, F_NJ>(acc, a, r0 + wr * (F_NJ * 32), r_end, v0 + wv * 128 + half * 4, n_valid);
        else
          store_tile<F_NI, F_NJ>(acc, a, r0 + wr * (F_NJ * 32), r_end, v0 + wv * 128 + half * 4, n_valid);
      }
      else if (MODE == 5)
        store_partial_tile<F_NI, F_NJ>(acc, a.partial + (size_t)ks * a.rows * a.ldo, a.ldo, r0 + wr * (F_NJ * 32), r_end,
                                       v0 + wv * 128 + half * 4, n_valid);
      else if (MODE == 3 || MODE == 4)
        store_prob_tile<F_NI, F_NJ>(acc, a, r0 + wr * (F_NJ * 32), r_end, v0 + wv * 128 + half * 4, n_valid);
      else if (MODE == 6)
        fold_tile_sample<F_NI, F_NJ>(acc, run, draw, a, r0 + wr * (F_NJ * 32), v0 + wv * 128 + half * 4, n_valid);
      else if (MODE == 7)
        fold_tile_store<F_NI, F_NJ>(acc, run, a, r0 + wr * (F_NJ * 32), r_end, v0 + wv * 128 + half * 4, n_valid);
      else if (!PROBE_MFMA)
        fold_tile<F_NI, F_NJ>(acc, run, v0 + wv * 128 + half * 4, a.col0, n_valid, v0 + FT > n_valid);
      if (!PROBE_MFMA) zero_acc();
    }
    if (PROBE_MFMA) fold_tile_impl<F_NI, F_NJ, false>(acc, run, vt0 * FT + wv * 128 + half * 4, a.col0, n_valid);
  }

  if (MODE >= 2 && MODE <= 5) {
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): the requests past the end of the stream land in LDS
    return;
  }
  // ---- end of strip: lanes l and l+32 hold the same hidden row; then the two vocabulary halves ------
#pragma unroll
  for (int j = 0; j < F_NJ; ++j) {
    Triple o;
    o.m = __shfl_xor(run[j].m, 32);
    o.s = __shfl_xor(run[j].s, 32);
    o.i = __shfl_xor(run[j].i, 32);
    merge_triple(run[j], o);
    if (MODE == 6) {
      Draw od;
      od.v = __shfl_xor(draw[j].v, 32);
      od.l = __shfl_xor(draw[j].l, 32);
      od.i = __shfl_xor(draw[j].i, 32);
      merge_draw(draw[j], od);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the requests past the end of the stream too
  __syncthreads();                                 // every wave is done with the operand stages
  Triple* xch = reinterpret_cast<Triple*>(lds);    // [256 hidden rows of the tile]
  Draw* xdr = reinterpret_cast<Draw*>(xch + FT);
  const int hrow0 = wr * (F_NJ * 32);
  if (wv == 1 && lane < 32) {
#pragma unroll
    for (int j = 0; j < F_NJ; ++j) {
      xch[hrow0 + j * 32 + lane] = run[j];
      if (MODE == 6) xdr[hrow0 + j * 32 + lane] = draw[j];
    }
  }
  __syncthreads();
  if (wv == 0 && lane < 32) {
#pragma unroll
    for (int j = 0; j < F_NJ; ++j) {
      merge_triple(run[j], xch[hrow0 + j * 32 + lane]);
      const int hrow = r0 + hrow0 + j * 32 + lane;
      if (hrow < r_end) {
        const size_t p = (size_t)hrow * a.n_parts + a.part0 + st;
        a.part_m[p] = run[j].m;
        a.part_s[p] = run[j].s;
        if (MODE == 6) {
          merge_draw(draw[j], xdr[hrow0 + j * 32 + lane]);
          a.part_v[p] = draw[j].v;
          a.part_l[p] = draw[j].l;
          a.part_i[p] = draw[j].i;
        } else {
          a.part_i[p] = run[j].i;
        }
      }
    }
  }
}

}  // namespace

int z2z_launch_logits_fast(int mode, const LogitsArgs& a, unsigned grid, hipStream_t s) {
  const bool rot = F_ROTATE_FEW && a.row_tiles == 1;
  if (rot && mode == 0)
    hipLaunchKernelGGL((logits_fast_kernel<0, true>), dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (rot && mode == 6)
    hipLaunchKernelGGL((logits_fast_kernel<6, true>), dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (rot && mode == 7)
    hipLaunchKernelGGL((logits_fast_kernel<7, true>), dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 9)
    hipLaunchKernelGGL(logits_fast_kernel<9>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 8)
    hipLaunchKernelGGL(logits_fast_kernel<8>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 7)
    hipLaunchKernelGGL(logits_fast_kernel<7>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 6)
    hipLaunchKernelGGL(logits_fast_kernel<6>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 5)
    hipLaunchKernelGGL(logits_fast_kernel<5>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 4)
    hipLaunchKernelGGL(logits_fast_kernel<4>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 3)
    hipLaunchKernelGGL(logits_fast_kernel<3>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 2)
    hipLaunchKernelGGL(logits_fast_kernel<2>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else if (mode == 1)
    hipLaunchKernelGGL(logits_fast_kernel<1>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  else
    hipLaunchKernelGGL(logits_fast_kernel<0>, dim3(grid), dim3(F_THREADS), F_LDS, s, a);
  Z2Z_HIP_TRY(hipGetLastError());
  return Z2Z_OK;
}

int z2z_logits_fast_prepare(z2z_ctx* c) {
  if (c->lds_limit < F_LDS) return Z2Z_EUNSUPPORTED;
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<0>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<1>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<2>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<3>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<4>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<5>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<6>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<7>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<8>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<9>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<0, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<6, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  Z2Z_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(logits_fast_kernel<7, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, F_LDS));
  return Z2Z_OK;
}
