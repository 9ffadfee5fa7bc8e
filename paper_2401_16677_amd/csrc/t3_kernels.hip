// Device code of the fused sliced-GEMM + reduce-scatter-reduction path for gfx950 (CDNA4).
//
// A persistent workgroup produces BM x BN output tiles with v_mfma_f32_16x16x32_bf16.  K-slabs of
// 64 bf16 of A and B are copied global -> LDS without passing through registers
// (global_load_lds_dwordx4) into two or three stages, ahead of the slab being multiplied; LDS
// rows are XOR-swizzled so that the MFMA operand reads are bank-conflict free.
//
// The 256 x 256 tile (B stored N x K, A stored M x K) runs on four wavefronts of 128 x 128, one
// per SIMD, with a hand-ordered main loop: every operand read and slab copy has its place
// between the products.  The other shapes and layouts run on eight (or, 128 x 128, four)
// wavefronts with a compiler-scheduled loop.
//
// The reduction of Sec. 4.3 of the T3 paper (op-and-store into the buffer that also receives
// the upstream partial) is done by starting the accumulators from the incoming partial, so a
// tile is read once and written once; both moves use full 128-byte lines and are transposed to
// and from the accumulator layout through LDS.  A persistent workgroup requests the next
// tile's incoming partial right behind the current tile's stores.
//
// A persistent launch whose last round of tiles would fill at most half the chip computes each
// of those tiles as two halves of K on two workgroups (balanced tail, see work_item).
//
// Included by t3_api.hip only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#ifndef T3_MH
#define T3_MH 2            // row passes per MFMA k-step of a 128-row wavefront tile (2 or 4)
#endif
#ifndef T3_AGENTS
#define T3_AGENTS 32          // release workgroups per forwarded chunk (multiple of 8)
#endif

namespace t3k {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *global_void_ptr;

constexpr int kThreads = 256;
constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr int kSpinLimit = 1 << 22;   // polls of a release workgroup before it gives up
constexpr int kTimelineItems = 16;     // pieces of work per workgroup a timeline records
constexpr int kTailSlots = 256;       // tiles a balanced tail can split (flag words behind the tracker state)

constexpr uint32_t kFlagStep0StoreOnly = 1u;
constexpr uint32_t kFlagFwdDirect = 2u;
constexpr uint32_t kFlagTwoWriters = 4u;
constexpr uint32_t kFlagFwdBf16 = 8u;

enum Mode { kModeGemm = 0, kModeFused = 1 };
enum Role { kRoleNone = 0, kRoleTile = 1, kRoleRelease = 2 };

// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt << 4 | lgkmcnt << 8 | vmcnt[5:4] << 14)
constexpr int kWaitVm0 = 0x0F70;
constexpr int kWaitLgkm0 = 0xF0FF;    // and-mask that turns a wait into "... and lgkmcnt(0)"
constexpr int kWaitAll = 0;
__host__ __device__ constexpr int wait_vm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// Everything a kernel needs, passed by value.
struct Plan {
  const uint16_t *A;
  const uint16_t *B;
  const float *C;    // reduce kernel input
  float *R;          // fused / reduce: incoming in, sums out.  gemm: the C output
  float *fwd;
  uint32_t *track;
  int64_t lda, ldb, ldr, ldc;
  int64_t limit;     // tiles with issue index >= limit do nothing
  int64_t begin;     // nor do tiles with issue index < begin
  int32_t M, N, K, P, rank, W, own;
  int32_t Mt, Wt, tpc;                 // the grid of WORKGROUP tiles: rows, columns, tiles per chunk
  // The tracked tile may be half a workgroup tile high (128 x 256 tracked, 256 x 256 computed):
  // then pair_m == 2, a workgroup tile covers the tracked tiles 2 mi and 2 mi + 1 of its column
  // (consecutive in the issue order) and counts as many as exist.  Otherwise pair_m == 1 and
  // the two grids are the same.
  int32_t pair_m, Mt_t, tpc_t;         // tracked tile rows and tracked tiles per chunk
  int32_t xcd_nbm, xcd_bmk, xcd_bnk;   // XCD grouping of a stage's tiles; xcd_nbm == 0: none
  int32_t agents, lag, rows_per_agent; // release workgroups per chunk, their lag in stages
  int32_t expected_done;               // grid positions of this launch that do work
  int32_t total_blocks;                // grid positions (tiles and release work) of the launch
  int32_t resident;                    // tile workgroups the chip holds at once
  int32_t upd_first, upd_rest;         // updates expected per element of chunk order[0] / the others
  int32_t split_k;                     // >= 1: workgroups that share a tile, each taking a part of K (Sec. 7.7)
  int32_t stagger_blocks, stagger_groups, stagger_ticks;   // start-up phase offsets (see stagger_start)
  int32_t k_groups;                    // > 1: workgroup w starts its K loop (w % k_groups) / k_groups of the way in
  int32_t nt_out;                      // results leave with the streaming hint (hand-ordered kernel)
  // Timeline (a profiling aid, normally null): workgroup w < timeline_wgs writes, for its i-th
  // piece of work, i < kTimelineItems, four wall-clock readings (100 MHz) at
  // timeline[(w * kTimelineItems + i) * 4 + ...]: piece taken; accumulators set up (the
  // incoming partial in place); main loop done; results handed to the memory system.
  uint64_t *timeline;
  int32_t timeline_wgs;
  // Balanced tail (persistent launches): the last tail_r grid positions, which would keep only
  // tail_r of the workgroups busy for a whole tile time, are each split into two halves of K
  // (see work_item).  0: off.  tail_q = full rounds of the grid before them; tail_flags = one
  // word per split tile, 0 between launches.
  int32_t tail_r, tail_q;
  uint32_t *tail_flags;
  uint32_t flags;
};

struct Tile {
  int s, c, mi, nj;
};

// Tracker state (uint32 words): two banks of { counter[P] ready[P] queue[P] queue_len done },
// then the globals { gen, error }.  A launch works in bank gen & 1; the last workgroup of the
// launch to finish clears the other bank and increments gen, so the next launch starts from a
// clean bank without a reset kernel in between, and the caller finds the results of the launch
// that just ended in bank (gen - 1) & 1.
__device__ inline int trk_bank_words(int P) { return 3 * P + 2; }
struct Trk {
  uint32_t *counter, *ready, *queue, *queue_len, *done;   // this launch's bank
  uint32_t *other;                                         // the bank to clear at the end
  uint32_t *gen, *error;
};
__device__ inline Trk trk_open(const Plan &p) {
  Trk t;
  t.gen = p.track + 2 * trk_bank_words(p.P);
  t.error = t.gen + 1;
  // (the same in every lane: made uniform so that the bank pointers live in scalar registers)
  const uint32_t g = __builtin_amdgcn_readfirstlane(
      __hip_atomic_load(t.gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  uint32_t *b = p.track + (g & 1u) * trk_bank_words(p.P);
  t.counter = b;
  t.ready = b + p.P;
  t.queue = b + 2 * p.P;
  t.queue_len = b + 3 * p.P;
  t.done = b + 3 * p.P + 1;
  t.other = p.track + ((g & 1u) ^ 1u) * trk_bank_words(p.P);
  return t;
}
__device__ inline void trk_clear_bank(uint32_t *b, int P) {
  for (int i = 0; i < 3 * P + 2; ++i)
    __hip_atomic_store(&b[i], (i >= 2 * P && i < 3 * P) ? kEmpty : 0u, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
// Called by thread 0 of every workgroup that did work, as its last act; d = the value its
// increment of `done` returned.
__device__ inline void trk_close_if_last(const Plan &p, const Trk &t, uint32_t d) {
  if (d + 1u == (uint32_t)p.expected_done) {
    trk_clear_bank(t.other, p.P);
    __hip_atomic_fetch_add(t.gen, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
__device__ inline void trk_workgroup_done(const Plan &p, const Trk &t) {
  trk_close_if_last(
      p, t, __hip_atomic_fetch_add(t.done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// Index j of a tile inside its stage -> tile.  Workgroups are dealt round-robin to the 8 XCDs,
// so workgroup j of a stage lands on XCD j % 8; that XCD gets a compact block of
// xcd_bmk x xcd_bnk tiles which share A rows and B columns in its L2.
__device__ inline bool decode_tile(const Plan &p, int s, int j, Tile &tl) {
  int mi, nj;
  if (p.xcd_nbm) {
    const int x = j & 7, i = j >> 3;
    const int bxm = x % p.xcd_nbm, bxn = x / p.xcd_nbm;
    mi = bxm * p.xcd_bmk + i % p.xcd_bmk;
    nj = bxn * p.xcd_bnk + i / p.xcd_bmk;
  } else {
    mi = j % p.Mt;
    nj = j / p.Mt;
  }
  // issue index of the (first) tracked tile
  const int64_t t = (int64_t)s * p.tpc_t + (int64_t)nj * p.Mt_t + (int64_t)mi * p.pair_m;
  int c = p.rank + s;
  if (c >= p.P) c -= p.P;
  tl.s = s;
  tl.c = c;
  tl.mi = mi;
  tl.nj = nj;
  return t >= p.begin && t < p.limit;
}

// Grid layout: the tiles of stage 0, 1, ... in order; after the tiles of stage s come the
// `agents` release workgroups of forward slot s - lag (a chunk whose tiles were all dispatched
// at least `lag` stages earlier); slots not served that way follow the last stage.
__device__ inline int decode_block(const Plan &p, int b, Tile &tl, int &slot, int &agent) {
  int base = 0;
  for (int s = 0; s < p.P; ++s) {
    if (b < base + p.tpc) return decode_tile(p, s, b - base, tl) ? kRoleTile : kRoleNone;
    base += p.tpc;
    const int sl = s - p.lag;
    if (p.agents && sl >= 0 && sl <= p.P - 2) {
      if (b < base + p.agents) {
        slot = sl;
        agent = b - base;
        return kRoleRelease;
      }
      base += p.agents;
    }
  }
  if (!p.agents) return kRoleNone;
  const int rem = b - base;
  slot = max(0, p.P - p.lag) + rem / p.agents;
  agent = rem % p.agents;
  return slot <= p.P - 2 ? kRoleRelease : kRoleNone;
}

// The it-th piece of work of a persistent workgroup: grid position `blk`, part `part` of
// `nparts` parts of K.  Without a balanced tail, workgroup w of G takes positions w, w + G, ...
// (split-K: `split_k` consecutive positions share a tile).
//
// Balanced tail.  With T = q G + r positions, 0 < r <= G / 2, the last round would run r tiles on
// r workgroups while the others idle.  Instead each of those r tiles is cut into two halves of
// K.  Half the workgroups are "early": early workgroup number i < r computes the first half of
// tile q G + i BEFORE its q whole tiles, starting from the incoming partial as any tile does,
// and stores the partial sums where the tile's result belongs.  The others are "late": late
// workgroup number i < r computes the second half AFTER its q whole tiles, starting from those
// partial sums, and stores and counts the tile.  Each workgroup then has at most q + 1/2 tiles
// of work, and the first half is q tile times old when the second half asks for it (a flag per
// tile says it is there; see the wait in the kernel).
//
// Workgroups 0 .. r-1 are early, r .. 2r-1 late; the early workgroup of a tile has the lower
// index: it was dispatched first and waits for nothing, so the late one's wait ends.  Early and
// late workgroups run half a tile time apart for the whole launch, and every XCD has both kinds
// (r is normally a multiple of 8, so the two halves of a tile even run on the same XCD): that
// spread of phases measures 5 % faster than whole XCDs running early or late.
template <int TAIL>
__device__ inline bool work_item(const Plan &p, int it, int &blk, int &part, int &nparts) {
  const int G = (int)gridDim.x, w = (int)blockIdx.x;
  if (TAIL && p.tail_r) {
    nparts = 1;
    part = 0;
    const bool early = w < p.tail_r;
    const int i = early ? w : w - p.tail_r;
    if (early) {
      if (it == 0) {
        blk = p.tail_q * G + i;
        nparts = 2;
        return true;
      }
      blk = w + (it - 1) * G;
      return it <= p.tail_q;
    }
    if (it < p.tail_q) {
      blk = w + it * G;
      return true;
    }
    if (it == p.tail_q && !early && i < p.tail_r) {
      blk = p.tail_q * G + i;
      part = 1;
      nparts = 2;
      return true;
    }
    return false;
  }
  // (positions fit 31 bits, the launch code sees to that)
  const uint32_t pos = (uint32_t)w + (uint32_t)it * (uint32_t)G;
  if (pos >= (uint32_t)p.total_blocks * (uint32_t)p.split_k) return false;
  blk = (int)(pos / (uint32_t)p.split_k);
  part = (int)(pos - (uint32_t)blk * (uint32_t)p.split_k);
  nparts = p.split_k;
  return true;
}

// Phase offsets at start-up.  All workgroups of the first wave of tiles start together and would
// reach their reduction traffic (incoming tile in, sums out) together, an HBM-bound burst during
// which no matrix core works.  The first `stagger_blocks` workgroups are put into
// `stagger_groups` phase groups; group g starts g * stagger_ticks (100 MHz ticks) late.  A
// persistent workgroup keeps its offset through all its tiles (every tile takes the same time);
// with one workgroup per grid position, later ones are dispatched as earlier ones retire.
__device__ inline void stagger_start(const Plan &p) {
  const int b = blockIdx.x;
  if (b >= p.stagger_blocks) return;
  const int grp = ((b >> 3) + (b >> 8)) % p.stagger_groups;
  if (!grp) return;
  const uint64_t t0 = wall_clock64(), wait = (uint64_t)grp * (uint64_t)p.stagger_ticks;
  while (wall_clock64() - t0 < wait) __builtin_amdgcn_s_sleep(8);
}

// Stores that are visible to every XCD once acknowledged: agent scope, i.e. the sc1 bit, which
// writes through the issuing XCD's L2.  (Plain and non-temporal stores stay in that L2 until a
// release fence writes the whole cache back.)
__device__ inline void store_agent(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store_agent(f32x4 *p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}
// Tile results and the incoming partial are accessed through buffer instructions: uniform
// descriptor, 32-bit byte offset of the lane, uniform offset of the block.  They are issued as
// compiler builtins, not inline assembly, so that the compiler keeps the required distance
// between an MFMA and a store that reads its result.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kAuxNt = 2, kAuxSc1 = 16;     // cache-policy bits of the buffer builtins on gfx94x/gfx950
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ inline void store_agent(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t blk_off, f32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)lane_off, (int)blk_off, kAuxSc1);
}
// (NT: with the streaming hint as well: the lines do not stay in the XCD's L2, where slabs of A
// and B are better kept)
template <bool NT>
__device__ inline void store_agent_hint(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t blk_off, f32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)lane_off, (int)blk_off,
                                         NT ? (kAuxSc1 | kAuxNt) : kAuxSc1);
}
__device__ inline f32x4 load_stream(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t blk_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)blk_off, kAuxNt));
}

// fp32 -> bfloat16, round to nearest even (v_cvt_pk_bf16_f32): the 16-bit format a forward slot
// may hold (activations under mixed precision, Sec. 5.2).
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
__device__ inline u32x2 pack_bf16(f32x4 v) {
  return __builtin_bit_cast(u32x2, __builtin_convertvector(v, bf16x4));
}
__device__ inline u32x4 pack_bf16(f32x4 lo, f32x4 hi) {
  const u32x2 a = pack_bf16(lo), b = pack_bf16(hi);
  return u32x4{a[0], a[1], b[0], b[1]};
}

// Rows r0, r0 + step, ... < r_end of chunk c of R into forward slot `slot`, one wavefront per
// row, 16 bytes per lane: the copy a trigger starts (Sec. 4.2.2).  The slot holds fp32, or
// bfloat16 under kFlagFwdBf16.
__device__ inline f32x4 load_agent(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t row_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)row_off, kAuxSc1 | kAuxNt));
}
__device__ inline void copy_chunk_rows(const Plan &p, int slot, int c, int r0, int r_end, int step) {
  const int lane = threadIdx.x & 63;
  // R is read with agent-scope loads: they see the producers' write-through stores, so no cache
  // has to be invalidated first (which would cost every workgroup of the XCD its slabs in L2)
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.R, (uint32_t)p.M * (uint32_t)p.ldr * 4u);
  const uint32_t col_off = (uint32_t)c * (uint32_t)p.W * 4u;
  if (p.flags & kFlagFwdBf16) {
    const int W8 = p.W >> 3;
    for (int r = r0; r < r_end; r += step) {
      const uint32_t row_off = (uint32_t)r * (uint32_t)p.ldr * 4u + col_off;
      u32x4 *dst = (u32x4 *)((uint16_t *)p.fwd + ((int64_t)slot * p.M + r) * p.W);
      for (int c0 = lane; c0 < W8; c0 += 2 * 64) {
        f32x4 v[4];
#pragma unroll
        for (int u = 0; u < 2; ++u)
          if (c0 + u * 64 < W8) {
            v[2 * u] = load_agent(rs, (uint32_t)(c0 + u * 64) * 32u, row_off);
            v[2 * u + 1] = load_agent(rs, (uint32_t)(c0 + u * 64) * 32u + 16u, row_off);
          }
#pragma unroll
        for (int u = 0; u < 2; ++u)
          if (c0 + u * 64 < W8)
            __builtin_nontemporal_store(pack_bf16(v[2 * u], v[2 * u + 1]), dst + c0 + u * 64);
      }
    }
    return;
  }
  const int W4 = p.W >> 2;
  for (int r = r0; r < r_end; r += step) {
    const uint32_t row_off = (uint32_t)r * (uint32_t)p.ldr * 4u + col_off;
    f32x4 *dst = (f32x4 *)(p.fwd + ((int64_t)slot * p.M + r) * p.W);
    for (int c0 = lane; c0 < W4; c0 += 4 * 64) {
      f32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c0 + u * 64 < W4) v[u] = load_agent(rs, (uint32_t)(c0 + u * 64) * 16u, row_off);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c0 + u * 64 < W4) __builtin_nontemporal_store(v[u], dst + c0 + u * 64);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Track & trigger (Sec. 4.2).  Called by all threads of a workgroup after the tile's stores
// have been issued.  Tile results are written with agent-scope stores; once they have been
// acknowledged (vmcnt == 0 in every wavefront, then the barrier) the tile is counted.  A
// device-scope release fence instead would write back the whole L2 for every tile and costs
// several times the reduction itself.
__device__ inline void track_count(const Plan &p, const Trk &t, int c, int n = 1);
__device__ inline void track_tile(const Plan &p, const Trk &t, int c, int n = 1) {
  __builtin_amdgcn_s_waitcnt(kWaitAll);
  __syncthreads();
  track_count(p, t, c, n);
}
// The counting itself, once every wavefront's stores of the tile are known to be acknowledged
// and a barrier has passed.
// (n: tracked tiles the workgroup's tile covers)
__device__ inline void track_count(const Plan &p, const Trk &t, int c, int n) {
  if (threadIdx.x == 0) {
    // both increments are in flight together: one round trip at the end of a tile, not two
    const uint32_t old = __hip_atomic_fetch_add(&t.counter[c], (uint32_t)n, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t d = __hip_atomic_fetch_add(t.done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // threshold = tracked regions of the chunk x updates expected per element (Sec. 4.2.1)
    const uint32_t threshold = (uint32_t)p.tpc_t * (uint32_t)(c == p.rank ? p.upd_first : p.upd_rest);
    if (old + (uint32_t)n == threshold) {         // the landing that reaches the threshold triggers
      if (c != p.own) {
        const uint32_t pos = __hip_atomic_fetch_add(t.queue_len, 1u, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&t.queue[pos], (uint32_t)c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      // The flag is what publishes: a release store, so the queue entry above and everything this
      // workgroup made visible before the barrier that precedes the count are ordered before it.
      // (queue_len alone publishes nothing: it may run ahead of the entry it reserves.)
      __hip_atomic_store(&t.ready[c], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    trk_close_if_last(p, t, d);
  }
}

// Release of a triggered chunk into its forward slot (the DMA of Sec. 4.2.2): workgroup `agent`
// of `agents` waits for the chunk's ready flag and copies its share of rows.  Every tile of the
// chunk was dispatched before this workgroup (lower block index), so the wait ends; should it
// not (a broken launch), the workgroup gives up after kSpinLimit polls and raises the error word.
__device__ inline void release_chunk(const Plan &p, int slot, int agent, uint32_t *sh) {
  if ((int64_t)(slot + 1) * p.tpc_t > p.limit || (int64_t)slot * p.tpc_t < p.begin)
    return;                                              // this chunk will not complete
  const Trk t = trk_open(p);
  int c = p.rank + slot;
  if (c >= p.P) c -= p.P;
  if (threadIdx.x == 0) {
    int spins = 0;
    while (__hip_atomic_load(&t.ready[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u &&
           ++spins < kSpinLimit)
      __builtin_amdgcn_s_sleep(16);
    const uint32_t ok = spins < kSpinLimit;
    if (!ok) __hip_atomic_fetch_or(t.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *sh = ok;
  }
  __syncthreads();
  if (!*sh) {            // gave up: still count as finished so that the launch closes its bank
    if (threadIdx.x == 0) trk_workgroup_done(p, t);
    return;
  }
  copy_chunk_rows(p, slot, c, agent * p.rows_per_agent + (int)(threadIdx.x >> 6),
                  min(p.M, (agent + 1) * p.rows_per_agent), (int)(blockDim.x >> 6));
  __builtin_amdgcn_s_waitcnt(kWaitAll);
  __syncthreads();
  if (threadIdx.x == 0) trk_workgroup_done(p, t);
}

// ---------------------------------------------------------------------------------------------
// LDS layout of one stage: BM rows of A then BN rows of B; a row holds the 64 bf16 of one tile
// row of the K-slab (128 bytes = 8 chunks of 16).  Row r keeps chunk k at position k ^ swz(r),
// which makes both the 1-KiB linear writes of the global->LDS copies (8 rows each) and the MFMA
// operand reads (16 consecutive rows, one chunk) bank-conflict free.
__device__ inline int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

constexpr int kBK = 64;               // bf16 elements of K per slab
constexpr int kRowBytes = kBK * 2;    // one LDS row
constexpr int kCPR = 8;               // 16-byte chunks per row
constexpr int kRPC = 8;               // rows filled by one 1-KiB copy

// sched_group_barrier masks
constexpr int kSchedMfma = 0x008, kSchedDsRead = 0x100;

// Instruction order of one MFMA k-step: the operand reads of each of its MH row passes (AREADS
// for the row blocks; FN + EXTRA more in the first), each followed by that pass's FMH * FN products.
template <int MH, int FMH, int FN, int EXTRA, int AREADS = FMH>
__device__ inline void sched_kstep() {
  __builtin_amdgcn_sched_group_barrier(kSchedDsRead, AREADS + FN + EXTRA, 0);
  __builtin_amdgcn_sched_group_barrier(kSchedMfma, FMH * FN, 0);
  if constexpr (MH >= 2) {
    __builtin_amdgcn_sched_group_barrier(kSchedDsRead, AREADS, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, FMH * FN, 0);
  }
  if constexpr (MH == 4) {
    __builtin_amdgcn_sched_group_barrier(kSchedDsRead, AREADS, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, FMH * FN, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedDsRead, AREADS, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, FMH * FN, 0);
  }
}

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), so that the
// index can be used where a constant is required (instruction offsets, which register).
template <int I, int N, typename F>
__device__ __forceinline__ void static_for_impl(F &f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for_impl<I + 1, N>(f);
  }
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F f) {
  static_for_impl<0, N>(f);
}

// The memory instructions of the hand-ordered main loop, one volatile statement each: they are
// emitted in exactly the order written, and the waits they need are written out as well.  The
// products stay compiler builtins (the compiler must know them to keep the distances the
// hardware requires around them) and are fenced into place with scheduling barriers.
template <int OFF>
__device__ __forceinline__ void asm_ds_read_b128(bf16x8 &dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// "The 8 + 8 operands of a k-step have landed": the wait carries them as in/out operands, so
// that no product that uses them can be moved above it.
__device__ __forceinline__ void asm_wait_operands(bf16x8 (&a)[8], bf16x8 (&b)[8]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]),
                 "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7])
               :
               : "memory");
}

constexpr int kRingSlots = 4;         // 1-KiB LDS slots per wavefront for transposing pairs: two pairs

// WAVES_M x WAVES_N wavefronts per workgroup, each producing a (BM/WAVES_M) x (BN/WAVES_N)
// block of the tile out of 16 x 16 MFMA blocks; NSTAGE LDS stages, NSTAGE-1 slabs in flight.
//
// The products are formed transposed (the B rows go in as the MFMA's first operand, the A rows
// as its second), so that a lane ends up holding, per block, one output row and FOUR
// CONSECUTIVE COLUMNS: the incoming partial is read and the sum written with 16-byte accesses.
//
// BKN = 1: B is stored K x N with N contiguous (the layout of the backward-pass GEMMs).  Its
// stage region then holds 64 k-rows of BN values; the MFMA operand (8 consecutive k for one n
// per lane) is fetched with the transposing LDS read ds_read_b64_tr_b16: in each block of 16
// lanes, lane i supplies the address of 4 consecutive n of k-row i / 4 (n offset 4 (i % 4)) and
// receives, for n = i, the values of the block's 4 k-rows.  32-byte pieces of a k-row sit at
// position (piece ^ sw(k)), sw(k) = (k & 3) | ((k >> 3) & 1) << 2, which spreads the 8 k-rows
// that 32 lanes read together over all banks.  K must be a multiple of 64 in this layout.
//
// AKM = 1: A is stored K x M with M contiguous (the transposed operand of the backward-pass
// GEMMs, Sec. 5.2): the same arrangement on the A side -- its stage region holds 64 k-rows of BM
// values, pieces swizzled the same way, operands fetched with the transposing read.  K must be
// a multiple of 64 and M a multiple of 8.
//
// TAIL = 1: the variant that can balance the tail of a persistent launch (see work_item).
// TAIL = 2: that variant of the fused kernel with the reduction and the tracking taken out: the
// plain GEMM with a balanced tail (the plain kernel's own TAIL = 1 variant of the hand-ordered
// loop does not fit the register file).
template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE, int MODE, int BKN, int AKM = 0, int TAIL = 0>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N)
__attribute__((amdgpu_waves_per_eu((BM / WAVES_M) * (BN / WAVES_N) > 8192 ? 1 : 2)))
void gemm_tile_kernel(const Plan p) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;   // wavefront tile
  constexpr int FM = WM / 16, FN = WN / 16;     // 16x16 MFMA blocks per wavefront
  constexpr int MH = FM > 4 ? T3_MH : 1;        // a k-step is taken in MH passes over the rows,
  constexpr int FMH = FM / MH;                  //   FMH row blocks each, to bound operand registers
  constexpr int KS = kBK / 32;                  // MFMA k-steps per slab
  constexpr int US = KS * MH;                   // micro-steps (row pass of a k-step) per slab
  constexpr int NA = BM / kRPC / NW, NB = BN / kRPC / NW;   // copies per wavefront per slab
  constexpr int NL = NA + NB;
  constexpr int NBLK = FM * FN;
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  constexpr int kBOff = BM * kRowBytes;
  static_assert(NA * kRPC * NW == BM && NB * kRPC * NW == BN, "copies must tile the slab");
  static_assert(NSTAGE >= 2 && (NSTAGE - 2) * NL < 64, "vmcnt range");
  static_assert(KS == 2, "the loop body is written as two k-steps");
  static_assert(NL % MH == 0, "a slab's copies are split evenly over the first k-step's passes");
  static_assert((FN & (FN - 1)) == 0, "block index -> (row block, column block) by shifts");
  static_assert(NSTAGE * kStageBytes <= 160 * 1024, "LDS");

  // Four wavefronts of 128 x 128 (one per SIMD) run the hand-ordered main loop and add the
  // incoming partial on the way out; B stored N x K only.
  constexpr bool kAsmLoop = (NW == 4 && FM == 8 && FN == 8 && NSTAGE == 2 && !BKN && !AKM);
  // Their pair transpositions get LDS of their own (4 KiB per wavefront) behind the stages.
  constexpr int kScrOff = kAsmLoop ? NSTAGE * kStageBytes : 0;
  static_assert(kScrOff + NW * kRingSlots * 1024 <= 160 * 1024, "LDS");

  __shared__ __attribute__((aligned(1024))) char lds[NSTAGE * kStageBytes + (kAsmLoop ? NW * kRingSlots * 1024 : 0)];

  // Persistent workgroups: workgroup w takes grid positions w, w + gridDim.x, ... in order (a
  // position is a tile or a piece of release work).  The tracking of a finished tile is
  // deferred into the next tile: by the first barrier of that tile's main loop every
  // wavefront has waited for its stores (they are older than the slab copies waited for
  // there), so the acknowledgement wait costs nothing.
  // (TAIL == 2: the fused kernel's code run as a plain GEMM with a balanced tail -- no incoming
  // partial, nothing tracked, output through R)
  static_assert(TAIL != 2 || MODE == kModeFused, "the plain variant is cut from the fused kernel");
  bool plain = false;
  if constexpr (TAIL == 2) {
    // always, but not known to the compiler: as compile-time facts (accumulators always start
    // from zero, nothing tracked, no next tile's partial to request) they lead its register
    // allocation of the hand-ordered loop to spill, as they do in the plain kernel itself
    int yes = 1;
    asm volatile("" : "+s"(yes));
    plain = yes != 0;
  }
  const bool tracked = MODE == kModeFused && !plain;
  Trk trk;
  if (tracked) trk = trk_open(p);              // reads gen now; used when tiles are done
  if (p.stagger_groups > 1) stagger_start(p);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  int pending_c = -1;                          // chunk of a tile whose stores are issued but not counted
  int pending_n = 1;                           //   and the tracked tiles it covers
  int pending_half = -1;                       // first half of a split tile whose stores are issued but not announced
  // to be called after a barrier that every wavefront reached with its stores acknowledged
  auto settle_pending = [&]() {
    if (tracked && pending_c >= 0) track_count(p, trk, pending_c, pending_n);
    // (relaxed, like the counting: what orders it behind the partial sums is that they were
    // written through and acknowledged before the barrier; a release would write back the L2)
    if (TAIL && pending_half >= 0 && threadIdx.x == 0)
      __hip_atomic_store(&p.tail_flags[pending_half], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    pending_c = pending_half = -1;
  };
  auto flush_pending = [&]() {
    if ((tracked && pending_c >= 0) || (TAIL && pending_half >= 0)) {
      __builtin_amdgcn_s_waitcnt(kWaitAll);
      __syncthreads();
      settle_pending();
    }
  };

  // (not in the eight-wavefront 256 x 256 kernels: they have no register to spare)
  constexpr bool kTimeline = !(NW == 8 && FM == 8);
  auto stamp = [&](int it, int k) {
    if (kTimeline && p.timeline && threadIdx.x == 0 && (int)blockIdx.x < p.timeline_wgs && it < kTimelineItems)
      p.timeline[((size_t)blockIdx.x * kTimelineItems + it) * 4 + k] = wall_clock64();
  };

  // The accumulators live across tiles: the hand-ordered kernel fills them with the NEXT tile's
  // incoming partial while the current tile's sums are on their way out (`have_in`).
  f32x4 acc[BM / WAVES_M / 16][BN / WAVES_N / 16];
  bool have_in = false;
  for (int it = 0;; ++it) {
  // Parts of K (split-K in two-writer mode; the two halves of a balanced tail's tiles): part j
  // takes K-slabs [j q, (j+1) q) of the K / 64 full ones, the last part also what is left over
  int blk, part, nparts;
  if (!work_item<TAIL>(p, it, blk, part, nparts)) break;
  stamp(it, 0);
  const int part_slabs = (p.K / kBK) / nparts;
  const int k0 = part * part_slabs * kBK;
  const int Kpart = (part == nparts - 1) ? p.K - k0 : part_slabs * kBK;
  const bool half0 = TAIL && p.tail_r && nparts == 2 && part == 0;   // partial sums out, nothing counted
  const bool half1 = TAIL && p.tail_r && nparts == 2 && part == 1;   // starts from those partial sums
  const int tail_idx = blk - p.tail_q * (int)gridDim.x;
  const char *const Ap = (const char *)p.A + (AKM ? (int64_t)k0 * p.lda * 2 : (int64_t)k0 * 2);
  const char *const Bp = (const char *)p.B + (BKN ? (int64_t)k0 * p.ldb * 2 : (int64_t)k0 * 2);
  Tile tl;
  int slot = 0, agent = 0;
  const int role = decode_block(p, blk, tl, slot, agent);
  if (role != kRoleTile) {
    flush_pending();                           // release work may wait for the very tile we finished
    // the release role never touches the stages: its one shared word lives there
    if (role == kRoleRelease && MODE == kModeFused) {
      __syncthreads();
      release_chunk(p, slot, agent, (uint32_t *)lds);
    }
    continue;
  }
  if (half1 && threadIdx.x == 0) {
    // The first half was computed by a workgroup with a lower index as its first piece of work
    // and waits for nothing, so this wait ends (normally at once: that was q tile times ago).
    int spins = 0;
    while (__hip_atomic_load(&p.tail_flags[tail_idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u &&
           ++spins < kSpinLimit)
      __builtin_amdgcn_s_sleep(16);
    if (tracked && spins >= kSpinLimit)
      __hip_atomic_fetch_or(trk.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // (this workgroup is the flag's only reader: cleared for the next launch)
    __hip_atomic_store(&p.tail_flags[tail_idx], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();                             // the previous tile's epilogue is done with the LDS

  const int m0 = tl.mi * BM;
  const int col_lo = tl.c * p.W;                 // chunk bounds in N
  const int col_hi = col_lo + p.W;
  const int n0 = col_lo + tl.nj * BN;

  const int nkf = Kpart / kBK;                   // full slabs
  const int ktail = Kpart - nkf * kBK;           // leftover elements of K (a multiple of 8)
  // Workgroups that run on different XCDs walk K from different starting slabs (and wrap
  // around): at any moment the chip then reads 8 different K ranges of A and B instead of one,
  // which spreads the traffic over the memory channels, and what one XCD misses in its L2
  // another has usually brought into the memory-side cache already.  Workgroups of one XCD
  // (same index modulo the group count) keep the same offset, so they still share slabs in L2.
  const int koff = p.k_groups > 1
                       ? (int)(((uint32_t)(blockIdx.x % (uint32_t)p.k_groups) * (uint32_t)nkf) / (uint32_t)p.k_groups)
                       : 0;
  // ---- global -> LDS copy addressing.  Copy q of this wavefront fills 8 LDS rows (1 KiB):
  // lane l lands in row l / 8, position l % 8, so it must fetch chunk (l % 8) ^ swz(row).
  const int cp_row = lane / kCPR;
  uint32_t offA[NA], offB[NB];                   // byte offsets, rows clamped into range
  auto chunk_of = [&](int rows_per_wave, int q) {  // the k-chunk copy q of this lane fetches
    return (lane % kCPR) ^ swz(wave * rows_per_wave + q * kRPC + cp_row);
  };
  constexpr int kARowBytes = BM * 2;             // (AKM) one k-row of the A region
  constexpr int kSwMaskA = (BM / 16 < 8 ? BM / 16 : 8) - 1;
#pragma unroll
  for (int q = 0; q < NA; ++q) {
    if (AKM) {
      // as for B stored K x N below: copy (wave * NA + q) fills 1 KiB of the A region, lane l
      // lands in k-row L / kARowBytes at 16-byte position cp = half (cp & 1) of piece (cp >> 1) ^ sw(k)
      const int L = (wave * NA + q) * 1024 + lane * 16;
      const int k = L / kARowBytes, cp = (L % kARowBytes) / 16;
      const int sw = ((k & 3) | (((k >> 3) & 1) << 2)) & kSwMaskA;
      const int mcol = (((cp >> 1) ^ sw) * 2 + (cp & 1)) * 8;
      offA[q] = (uint32_t)((k * p.lda + min(m0 + mcol, p.M - 8)) * 2);
    } else {
      const int r = wave * (BM / NW) + q * kRPC + cp_row;
      offA[q] = (uint32_t)((min(m0 + r, p.M - 1) * p.lda + chunk_of(BM / NW, q) * 8) * 2);
    }
  }
  constexpr int kBRowBytes = BN * 2;             // (BKN) one k-row of the B region
  constexpr int kSwMask = (BN / 16 < 8 ? BN / 16 : 8) - 1;
#pragma unroll
  for (int q = 0; q < NB; ++q) {
    if (BKN) {
      // copy (wave * NB + q) fills bytes [1024 (wave NB + q), +1024) of the B region: lane l
      // lands in k-row L / kBRowBytes at 16-byte position cp, which holds half (cp & 1) of
      // 32-byte piece (cp >> 1) ^ sw(k)
      const int L = (wave * NB + q) * 1024 + lane * 16;
      const int k = L / kBRowBytes, cp = (L % kBRowBytes) / 16;
      const int sw = ((k & 3) | (((k >> 3) & 1) << 2)) & kSwMask;
      const int ncol = (((cp >> 1) ^ sw) * 2 + (cp & 1)) * 8;
      offB[q] = (uint32_t)((k * p.ldb + min(n0 + ncol, col_hi - 8)) * 2);
    } else {
      const int r = wave * (BN / NW) + q * kRPC + cp_row;
      offB[q] = (uint32_t)((min(n0 + r, col_hi - 1) * p.ldb + chunk_of(BN / NW, q) * 8) * 2);
    }
  }
  const int ldsA_w = wave * (BM / NW) * kRowBytes;            // this wavefront's rows, stage 0
  const int ldsB_w = kBOff + wave * (BN / NW) * kRowBytes;

  // The copies are issued as inline assembly: the compiler would otherwise wait for every
  // outstanding global->LDS copy (vmcnt(0)) before any LDS read, which defeats the prefetch.
  // Waits for them are therefore explicit (s_waitcnt below).  Copies [q0, q1) of the slab's
  // NA + NB are issued by one call, so that a slab's copies can be spread over its micro-steps
  // (all eight wavefronts issuing all of theirs at once stalls them on the memory pipeline).
  // They write m0 (the LDS destination of the copy) and say so in their clobber lists, so the
  // compiler never assumes a value of its own survives them; it flags every clobber of that
  // register as "reserved", which is exactly what is meant here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_ptr)lds;
  auto issue_copies = [&](int kt, int stage, int q0, int q1) {
    kt += koff;                                   // slab kt of this workgroup's walk over K
    if (kt >= nkf) kt -= nkf;
    const char *a = Ap + (AKM ? (int64_t)kt * kBK * p.lda * 2 : (int64_t)kt * (kBK * 2));
    const char *b = Bp + (BKN ? (int64_t)kt * kBK * p.ldb * 2 : (int64_t)kt * (kBK * 2));
    const uint32_t dst = lds_base + stage * kStageBytes;
#pragma unroll
    for (int q = 0; q < NA; ++q)
      if (q >= q0 && q < q1)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(dst + ldsA_w + q * 1024), "v"(offA[q]), "s"(a)
                     : "memory", "m0");
#pragma unroll
    for (int q = 0; q < NB; ++q)
      if (NA + q >= q0 && NA + q < q1)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(dst + ldsB_w + q * 1024), "v"(offB[q]), "s"(b)
                     : "memory", "m0");
  };
#pragma clang diagnostic pop
  auto issue_slab = [&](int kt, int stage) { issue_copies(kt, stage, 0, NL); };

  // ---- MFMA operand addressing (v_mfma_f32_16x16x32_bf16): lane reads row (lane & 15) of a
  // 16-row block, k-chunk 4*kk + (lane >> 4) of k-step kk.
  const int fr = lane & 15, fq = lane >> 4, fs = swz(fr);
  int fragA[KS], fragB[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const int pos = ((4 * kk + fq) ^ fs) * 16;
    fragA[kk] = (wm * WM + fr) * kRowBytes + pos;
    fragB[kk] = kBOff + (wn * WN + fr) * kRowBytes + pos;
  }
  // (BKN) this lane's address parts of the transposing reads: k-row 8 (lane >> 4) + (fr >> 2) of
  // a k-step's 32 (+ 4 for the second read), 8 bytes at n offset 4 (fr & 3) of 32-byte piece
  // (wn WN / 16 + j) ^ sw
  const int trB = kBOff + (8 * fq + (fr >> 2)) * kBRowBytes + (fr & 3) * 8;
  const int trSw = ((fr >> 2) | ((fq & 1) << 2)) & kSwMask;
  const int trA = (8 * fq + (fr >> 2)) * kARowBytes + (fr & 3) * 8;        // (AKM) the same for A
  const int trSwA = ((fr >> 2) | ((fq & 1) << 2)) & kSwMaskA;

  // NSTAGE-1 slabs are always in flight.  Past the last slab the copies are repeated into
  // stages nobody reads any more, so every wait below is for the same number of younger copies.
  if (nkf > 0) issue_slab(0, 0);
  if (kAsmLoop && nkf > 0) issue_slab(min(1, nkf - 1), 1);   // (its scratch is not in the stages)

  // ---- accumulators start from the incoming partial (fused) or zero.
  // Block (i, j), element e of this lane: row 16*i + (lane & 15), column 16*j + 4*(lane >> 4) + e
  // of the wavefront tile.  Per 16-byte access 4 lanes cover 64 contiguous bytes of a row.
  const bool store_only = (MODE == kModeGemm) || plain || ((p.flags & kFlagStep0StoreOnly) && tl.s == 0);
  const bool to_fwd = (MODE == kModeFused) && (p.flags & kFlagFwdDirect) && tl.c != p.own;
  // two writers (Sec. 4.1): the tile is ADDED into R with atomics, as the upstream update is
  const bool two_writers = (MODE == kModeFused) && (p.flags & kFlagTwoWriters);
  const int rw0 = m0 + wm * WM, cw0 = n0 + wn * WN;          // wavefront tile origin (uniform)
  const bool full = (rw0 + WM <= p.M) && (cw0 + WN <= col_hi);
  // where the tile's result goes (uniform): R, C, or the chunk's forward slot
  const float *out_base;
  uint32_t ld_out;
  int col_org;            // column the base's rows start at
  if (to_fwd) {
    ld_out = (uint32_t)p.W;
    out_base = p.fwd + (int64_t)tl.s * p.M * p.W;
    col_org = col_lo;
  } else {
    ld_out = (uint32_t)((MODE == kModeGemm) ? p.ldc : p.ldr);
    out_base = p.R;
    col_org = 0;
  }
  // ---- "pairs".  Global accesses that touch half a 128-byte line per row (what one 16 x 16
  // block in the accumulator layout amounts to) run at a third of the rate of full lines, so
  // the incoming partial and the results move in units of one PAIR = two neighbouring blocks =
  // 16 rows x 32 columns = two instructions of 8 rows x 128 bytes each, and are transposed to
  // and from the accumulator layout in LDS.  A pair occupies two 1-KiB slots (rows 0-7, rows
  // 8-15); in a slot, the lane that a linear access maps to position (rp, pp) = (lane / 8,
  // lane % 8) holds row r = rp (first slot) or rp ^ 1 (second slot), 16-byte chunk pp ^ r: with
  // that swizzle both the linear side and the accumulator side are bank-conflict free.
  constexpr int UJ = FN / 2;                     // pairs per row of blocks
  struct PairLane {
    int row[2], col[2];   // row / column (in the pair) of the linear side's two instructions
    int acc[2];           // byte offset (in the pair's two slots) of the lane's 16 bytes of block 0 / 1
  };
  auto pair_lane = [](int ln) {
    PairLane u;
    const int rp = ln >> 3, pp = ln & 7;
    u.row[0] = rp;
    u.row[1] = 8 + (rp ^ 1);
    u.col[0] = 4 * (pp ^ rp);
    u.col[1] = 4 * (pp ^ rp ^ 1);
    const int m = ln & 15, q = ln >> 4, h = m >> 3, r = m & 7, rq = h ? (r ^ 1) : r;
    u.acc[0] = h * 1024 + rq * 128 + (q ^ r) * 16;
    u.acc[1] = h * 1024 + rq * 128 + ((4 + q) ^ r) * 16;
    return u;
  };
  const PairLane ul = pair_lane(lane);           // (for the loads just below; the epilogue recomputes it)
  const int *u_acc = ul.acc;

  constexpr int NPAIR = NBLK / 2;
  static_assert(FN % 2 == 0, "pairs");
  // Every access to R, C or a forward slot is (uniform base) + (32-bit byte offset of the lane),
  // the offset formed per block when it is needed: byte sizes of these arrays stay below 4 GiB.
  if (!have_in) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // The incoming partial: every pair as two full-line accesses (8 rows x 128 bytes), all in
  // flight together, landing in the pair's accumulator registers; then pair by pair through LDS
  // into the accumulator layout, so that the products accumulate on top of it.  (The scratch is
  // the last stage, which no copy touches before the main loop's first barrier; the hand-ordered
  // kernel has scratch of its own.)
  // (AGENT: the data was written by another workgroup of this launch, with agent-scope stores,
  // and is read with agent-scope loads; src / ld_in / org: the array, its leading dimension and
  // the column its rows start at)
  auto in_pairs_load = [&](auto AGENT, const PairLane &ul, const float *src, uint32_t ld_in, int org, int m_lo,
                           int n_lo, int col_end, bool whole) {
    const int *u_row = ul.row, *u_col = ul.col;
    const __amdgpu_buffer_rsrc_t in_rsrc = make_rsrc(src, (uint32_t)p.M * ld_in * 4u);
    uint32_t in_l[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
      in_l[h] = ((uint32_t)(m_lo + u_row[h]) * ld_in + (uint32_t)(n_lo - org + u_col[h])) * 4u;
#pragma unroll
    for (int t = 0; t < NPAIR; ++t) {
      const int i = t / UJ, jj = t % UJ;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
        if (whole || (m_lo + 16 * i + u_row[h] < p.M && n_lo + 32 * jj + u_col[h] < col_end)) {
          const uint32_t blk_off = ((uint32_t)(16 * i) * ld_in + (uint32_t)(32 * jj)) * 4u;
          v = decltype(AGENT)::value ? load_agent(in_rsrc, in_l[h], blk_off) : load_stream(in_rsrc, in_l[h], blk_off);
        }
        acc[i][2 * jj + h] = v;
      }
    }
  };
  auto in_pairs_transpose = [&]() {
    char *scr = lds + (kAsmLoop ? kScrOff : (NSTAGE - 1) * kStageBytes) + wave * (kRingSlots * 1024);
#pragma unroll
    for (int t = 0; t < NPAIR; ++t) {
      const int i = t / UJ, jj = t % UJ;
      char *slot = scr + ((2 * t) & (kRingSlots - 1)) * 1024;
      *(f32x4 *)(slot + lane * 16) = acc[i][2 * jj];
      *(f32x4 *)(slot + 1024 + lane * 16) = acc[i][2 * jj + 1];
      acc[i][2 * jj] = *(const f32x4 *)(slot + u_acc[0]);
      acc[i][2 * jj + 1] = *(const f32x4 *)(slot + u_acc[1]);
      if (t % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
  };
  // A persistent workgroup of the hand-ordered kernel requests the NEXT tile's incoming partial
  // at the end of a tile's epilogue, right behind that tile's stores (`have_in`): the loads are
  // then on their way while the workgroup decodes its next position and requests its first slabs.
  if (half1) {
    // the second half of a split tile starts from the first half's partial sums, which sit
    // where the result will go
    in_pairs_load(std::true_type{}, ul, out_base, ld_out, col_org, rw0, cw0, col_hi, full);
    in_pairs_transpose();
  } else if (MODE == kModeFused && !store_only && !two_writers) {
    if (!have_in) in_pairs_load(std::false_type{}, ul, p.R, (uint32_t)p.ldr, 0, rw0, cw0, col_hi, full);
    in_pairs_transpose();
  }
  have_in = false;
  stamp(it, 1);

  if constexpr (kAsmLoop) {
  // ---- main loop, hand-ordered.  One wavefront per SIMD: nobody else fills the matrix pipe while
  // this one waits, so no wait may be exposed.  Two LDS stages, two sets of operand registers.  A
  // k-step is 64 products; the 16 operand reads of the next k-step go out one per three
  // products, early enough to have landed when the k-step ends, and the 16 copies of the slab
  // after next one per three products of a slab's second k-step.  One barrier per slab:
  //   second k-step of slab t  | reads: first k-step of slab t+1  | copies: slab t+2 -> stage of t
  //   first k-step of slab t+1 | reads: second k-step of slab t+1
  //   wait for own reads and copies, barrier   (slab t+2 visible; all are done reading slab t+1)
  if (nkf > 0) {
    bf16x8 xa[2][FM], xb[2][FN];
    uint32_t adA[KS], adB[KS];                   // this lane's operand rows of k-step kk, stage 0
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      adA[kk] = lds_base + fragA[kk];
      adB[kk] = lds_base + fragB[kk];
    }
    // read r of a k-step's FM + FN, in the order the products need them: B block 0, A block 0,
    // the other B blocks, the other A blocks
    auto read_op = [&](auto R, auto SET, uint32_t a_addr, uint32_t b_addr) {
      constexpr int r = decltype(R)::value, set = decltype(SET)::value;
      if constexpr (r == 0) asm_ds_read_b128<0>(xb[set][0], b_addr);
      else if constexpr (r == 1) asm_ds_read_b128<0>(xa[set][0], a_addr);
      else if constexpr (r <= FN) asm_ds_read_b128<(r - 1) * 16 * kRowBytes>(xb[set][r - 1], b_addr);
      else asm_ds_read_b128<(r - FN) * 16 * kRowBytes>(xa[set][r - FN], a_addr);
    };
    // One k-step: the products of operand set CS.  READS: the next k-step's operands go into the
    // other set from (a_addr, b_addr).  COPIES: slab kt_c goes into stage st_c.
    auto kstep = [&](auto CS, auto READS, auto COPIES, uint32_t a_addr, uint32_t b_addr, int kt_c, int st_c) {
      constexpr int cs = decltype(CS)::value;
      asm_wait_operands(xa[cs], xb[cs]);                      // this k-step's operands have landed
      __builtin_amdgcn_sched_barrier(0);
      static_for<FM * FN>([&](auto Mi) {
        constexpr int m = decltype(Mi)::value, i = m / FN, j = m % FN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xb[cs][j], xa[cs][i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);                    // nothing moves across: the order is as written
        if constexpr (decltype(READS)::value && m % 3 == 0 && m / 3 < FM + FN) {
          read_op(std::integral_constant<int, m / 3>{}, std::integral_constant<int, cs ^ 1>{}, a_addr, b_addr);
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (decltype(COPIES)::value && m % 3 == 1 && m / 3 < NL) {
          issue_copies(kt_c, st_c, m / 3, m / 3 + 1);
          __builtin_amdgcn_sched_barrier(0);
        }
      });
    };
    using std::false_type;
    using std::true_type;
    constexpr std::integral_constant<int, 0> set0{};
    constexpr std::integral_constant<int, 1> set1{};

    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NL) : "memory");   // slab 0 landed (slab 1 may be on its way)
    __builtin_amdgcn_s_barrier();
    static_for<FM + FN>([&](auto R) { read_op(R, set0, adA[0], adB[0]); });
    kstep(set0, true_type{}, false_type{}, adA[1], adB[1], 0, 0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                  // slab 1 visible
    settle_pending();                              // the previous tile's stores are acknowledged too:
                                                   //   every wavefront has just waited for vmcnt(0)
    uint32_t so = 0;                               // byte offset of the stage that holds slab kt
    for (int kt = 0; kt < nkf - 2; ++kt) {
      const uint32_t sn = so ^ (uint32_t)kStageBytes;
      kstep(set1, true_type{}, true_type{}, adA[0] + sn, adB[0] + sn, kt + 2, (int)(so / kStageBytes));
      kstep(set0, true_type{}, false_type{}, adA[1] + sn, adB[1] + sn, 0, 0);
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      so = sn;
    }
    if (nkf > 1) {                                 // slab nkf-2's second k-step, slab nkf-1's first
      const uint32_t sn = so ^ (uint32_t)kStageBytes;
      kstep(set1, true_type{}, false_type{}, adA[0] + sn, adB[0] + sn, 0, 0);
      kstep(set0, true_type{}, false_type{}, adA[1] + sn, adB[1] + sn, 0, 0);
    }
    kstep(set1, false_type{}, false_type{}, 0u, 0u, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  }
  if constexpr (!kAsmLoop) {
  if (nkf > 0) {
#pragma unroll
    for (int st = 1; st < NSTAGE - 1; ++st) issue_slab(min(st, nkf - 1), st);
  }

  }
  // Two sets of operand registers.  Micro-step u = (k-step kk, row pass h) reads FMH row blocks
  // of A (set u & 1) and, on the first pass of a k-step, the FN column blocks of B (set kk & 1),
  // while the products of micro-step u-1 are issued.
  bf16x8 fa[2][FMH], fb[2][FN];
  auto read_u = [&](int u, int stage_off) {
    const int kk = u / MH, h = u % MH;
#pragma unroll
    for (int i = 0; i < FMH; ++i) {
      if (AKM) {
        typedef __attribute__((ext_vector_type(4))) short s16x4;
        typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;
        const char *a0 = lds + stage_off + trA + 32 * kk * kARowBytes +
                         (((wm * (WM / 16) + h * FMH + i) ^ trSwA) << 5);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_void_ptr)a0);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_void_ptr)(a0 + 4 * kARowBytes));
        typedef __attribute__((ext_vector_type(8))) short s16x8;
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        fa[u & 1][i] = __builtin_bit_cast(bf16x8, both);
      } else {
        fa[u & 1][i] = *(const bf16x8 *)(lds + stage_off + fragA[kk] + (h * FMH + i) * 16 * kRowBytes);
      }
    }
    if (h == 0) {
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        if (BKN) {
          typedef __attribute__((ext_vector_type(4))) short s16x4;
          typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;
          const char *a0 = lds + stage_off + trB + 32 * kk * kBRowBytes + (((wn * (WN / 16) + j) ^ trSw) << 5);
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_void_ptr)a0);
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_void_ptr)(a0 + 4 * kBRowBytes));
          typedef __attribute__((ext_vector_type(8))) short s16x8;
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          fb[kk & 1][j] = __builtin_bit_cast(bf16x8, both);
        } else {
          fb[kk & 1][j] = *(const bf16x8 *)(lds + stage_off + fragB[kk] + j * 16 * kRowBytes);
        }
      }
    }
  };
  auto mfma_u = [&](int u) {
    const int kk = u / MH, h = u % MH;
#pragma unroll
    for (int i = 0; i < FMH; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        acc[h * FMH + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[kk & 1][j], fa[u & 1][i],
                                                                      acc[h * FMH + i][j], 0, 0, 0);
  };

  if constexpr (!kAsmLoop) {
  // ---- main loop: slab kt is multiplied while the next NSTAGE-1 slabs are in flight.  The
  // products of a slab's last micro-step are issued after the next barrier, under the next
  // slab's first LDS reads.  An iteration is: wait + barrier; k-step 0, with the next slab's
  // copies spread over its row passes; k-step 1.
  constexpr int kWaitSlab = wait_vm((NSTAGE - 2) * NL);
  if (nkf > 0) {
    // Slab 0 (and the incoming partial) landed -- and this wavefront's LDS accesses are done: the
    // transposition of the incoming partial used the last stage as scratch, and the copies issued
    // right after this barrier refill that stage.  A copy that finds its line in L1 can land
    // within a hundred clocks, before a read or write still waiting in a busy LDS queue (two
    // workgroups share the unit): the read then returns slab data, the late write ruins the slab.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitSlab & kWaitLgkm0);
    __builtin_amdgcn_s_barrier();
    settle_pending();                              // (also older: the previous tile's stores)
    issue_slab(min(NSTAGE - 1, nkf - 1), NSTAGE - 1);
    read_u(0, 0);
#pragma unroll
    for (int u = 1; u < US; ++u) {
      read_u(u, 0);
      mfma_u(u - 1);
    }
    int stage = 1;
    for (int kt = 1; kt < nkf; ++kt) {
      const int so = stage * kStageBytes;
      const int kt_next = min(kt + NSTAGE - 1, nkf - 1);
      const int st_next = stage >= 1 ? stage - 1 : NSTAGE - 1;
      asm volatile("" ::: "memory");               // LDS reads above stay above the barrier
      __builtin_amdgcn_s_waitcnt(kWaitSlab & kWaitLgkm0);   // own copies of slab kt landed, own LDS reads done
      __builtin_amdgcn_s_barrier();                // everyone's; all are done with the stage refilled next
#pragma unroll
      for (int u = 0; u < MH; ++u) {               // k-step 0
        read_u(u, so);
        issue_copies(kt_next, st_next, u * NL / MH, (u + 1) * NL / MH);
        mfma_u((u + US - 1) % US);                 // u == 0: last micro-step of slab kt-1
      }
      sched_kstep<MH, FMH, FN, BKN ? FN : 0, AKM ? 2 * FMH : FMH>();   // (the transposing reads are two per block)
#pragma unroll
      for (int u = MH; u < US; ++u) {              // k-step 1
        read_u(u, so);
        mfma_u(u - 1);
      }
      sched_kstep<MH, FMH, FN, BKN ? FN : 0, AKM ? 2 * FMH : FMH>();   // (the transposing reads are two per block)
      stage = stage == NSTAGE - 1 ? 0 : stage + 1;
    }
    mfma_u(US - 1);
    __builtin_amdgcn_s_waitcnt(kWaitVm0);          // drain the repeated copies
  }
  }
  asm volatile("" ::: "memory");

  if (ktail) {
    // ragged end of K: through registers, chunks past K zeroed, into stage 0
    __syncthreads();
    const int64_t kb = (int64_t)nkf * (kBK * 2);
    const uint4 zero = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int q = 0; q < NA; ++q) {
      if (AKM) break;                              // (no ragged K in this layout)
      uint4 v = zero;
      if (chunk_of(BM / NW, q) * 8 < ktail) v = *(const uint4 *)(Ap + kb + offA[q]);
      *(uint4 *)(lds + ldsA_w + q * 1024 + lane * 16) = v;
      if (q % 2 == 1) __builtin_amdgcn_sched_barrier(0);   // two loads in flight, not all: registers
    }
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      if (BKN) break;                              // (no ragged K in this layout)
      uint4 v = zero;
      if (chunk_of(BN / NW, q) * 8 < ktail) v = *(const uint4 *)(Bp + kb + offB[q]);
      *(uint4 *)(lds + ldsB_w + q * 1024 + lane * 16) = v;
      if (q % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    // both k-steps, whatever ktail is: the zeroed chunks add nothing
#pragma unroll
    for (int u = 0; u < US; ++u) {
      read_u(u, 0);
      mfma_u(u);
    }
  }

  stamp(it, 2);
  // ---- epilogue: the tile leaves in whole 128-byte lines, agent-scope (write-through) stores
  if constexpr (kAsmLoop) {
    // Pair by pair through this wavefront's own 4 KiB of LDS: written in the accumulator layout,
    // read back linearly, stored 8 rows x 128 bytes per instruction.  (Two-writer mode and
    // bfloat16 forward slots written directly are served by the eight-wavefront kernel.)
    const __amdgpu_buffer_rsrc_t out_rsrc = make_rsrc(out_base, (uint32_t)p.M * ld_out * 4u);
    char *scr = lds + kScrOff + wave * (kRingSlots * 1024);
    int lane_e = lane;                             // recomputed here rather than kept through the main loop
    asm volatile("" : "+v"(lane_e));
    const PairLane ue = pair_lane(lane_e);
    const int *u_row = ue.row, *u_col = ue.col, *u_acc = ue.acc;
    uint32_t out_u[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
      out_u[h] = ((uint32_t)(rw0 + u_row[h]) * ld_out + (uint32_t)(cw0 - col_org + u_col[h])) * 4u;
    // the next grid position of this workgroup: if it is a tile that takes an incoming partial,
    // its accumulator blocks are requested once this tile's sums have been stored
    bool next_in = false, next_full = false;
    int next_rw0 = 0, next_cw0 = 0, next_col_hi = 0;
    int blk_n, part_n, nparts_n;
    if (MODE == kModeFused && !plain && work_item<TAIL>(p, it + 1, blk_n, part_n, nparts_n) && nparts_n == 1) {
      Tile tn;
      int slot_n = 0, agent_n = 0;
      if (decode_block(p, blk_n, tn, slot_n, agent_n) == kRoleTile &&
          !((p.flags & kFlagStep0StoreOnly) && tn.s == 0)) {
        next_in = true;
        next_col_hi = tn.c * p.W + p.W;
        next_rw0 = tn.mi * BM + wm * WM;
        next_cw0 = tn.c * p.W + tn.nj * BN + wn * WN;
        next_full = (next_rw0 + WM <= p.M) && (next_cw0 + WN <= next_col_hi);
      }
    }
    auto store_pairs = [&](auto NT) {
#pragma unroll
      for (int t = 0; t < NPAIR; ++t) {
        const int i = t / UJ, jj = t % UJ;
        char *slot = scr + ((2 * t) & (kRingSlots - 1)) * 1024;
        *(f32x4 *)(slot + u_acc[0]) = acc[i][2 * jj];
        *(f32x4 *)(slot + u_acc[1]) = acc[i][2 * jj + 1];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const f32x4 v = *(const f32x4 *)(slot + h * 1024 + lane_e * 16);
          if (full || (rw0 + 16 * i + u_row[h] < p.M && cw0 + 32 * jj + u_col[h] < col_hi))
            store_agent_hint<decltype(NT)::value>(out_rsrc, out_u[h],
                                                  ((uint32_t)(16 * i) * ld_out + (uint32_t)(32 * jj)) * 4u, v);
        }
        // keep the scheduler from running many pairs ahead: it would park their values in registers
        if (t % 2 == 1) __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (p.nt_out) store_pairs(std::true_type{});
    else store_pairs(std::false_type{});
    // (after the last store, not between the stores: reads and writes that alternate cost the
    // memory more than a burst of each)
    if (next_in) {
      __builtin_amdgcn_sched_barrier(0);
      in_pairs_load(std::false_type{}, ue, p.R, (uint32_t)p.ldr, 0, next_rw0, next_cw0, next_col_hi, next_full);
    }
    have_in = next_in;
  } else if (to_fwd && (p.flags & kFlagFwdBf16)) {
    // Forward slot in bfloat16: a row of the wavefront tile (64 columns) is one 128-byte line.
    // Row of blocks by row of blocks through LDS: the lane's four rounded sums of each block
    // (8 bytes) go to row (lane & 15), columns 16 j + 4 (lane >> 4) of a 16-row x 128-byte
    // image, 16-byte chunk k of row r kept at position k ^ ((r >> 1) & 7) (both sides free of
    // bank conflicts); read back linearly, each store instruction covers 8 rows x 128 bytes.
    static_assert(FN == 4, "a wavefront tile is 64 columns wide");
    __syncthreads();
    char *scr = lds + wave * (kRingSlots * 1024);
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    const int arow = lane_e & 15, aq = lane_e >> 4;
    int w_off[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j)
      w_off[j] = arow * 128 + (((2 * j + (aq >> 1)) ^ ((arow >> 1) & 7)) << 4) + ((aq & 1) << 3);
    const __amdgpu_buffer_rsrc_t o16 =
        make_rsrc((const uint16_t *)p.fwd + (int64_t)tl.s * p.M * p.W, (uint32_t)p.M * p.W * 2u);
    int l_row[2], l_col[2];
    uint32_t l_off[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      l_row[h] = 8 * h + (lane_e >> 3);
      l_col[h] = 8 * ((lane_e & 7) ^ ((l_row[h] >> 1) & 7));
      l_off[h] = ((uint32_t)(rw0 + l_row[h]) * (uint32_t)p.W + (uint32_t)(cw0 - col_lo + l_col[h])) * 2u;
    }
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      char *img = scr + (i & 1) * 2048;
#pragma unroll
      for (int j = 0; j < FN; ++j) *(u32x2 *)(img + w_off[j]) = pack_bf16(acc[i][j]);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const u32x4 v = *(const u32x4 *)(img + h * 1024 + lane_e * 16);
        if (full || (rw0 + 16 * i + l_row[h] < p.M && cw0 + l_col[h] < col_hi))
          __builtin_amdgcn_raw_buffer_store_b128(v, o16, (int)l_off[h],
                                                 (int)((uint32_t)(16 * i) * (uint32_t)p.W * 2u), kAuxSc1);
      }
      if (i % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
  } else {
  const __amdgpu_buffer_rsrc_t out_rsrc = make_rsrc(out_base, (uint32_t)p.M * ld_out * 4u);
  // Pair by pair through LDS (the stages are free now; each wavefront uses 4 KiB of its own):
  // written in the accumulator layout, read back linearly, stored as 8 rows x 128 bytes.
  {
  __syncthreads();
  char *scr = lds + wave * (kRingSlots * 1024);
  int lane_e = lane;                             // recomputed here rather than kept through the main loop
  asm volatile("" : "+v"(lane_e));
  const PairLane ue = pair_lane(lane_e);
  const int *u_row = ue.row, *u_col = ue.col, *u_acc = ue.acc;
  uint32_t out_u[2];
#pragma unroll
  for (int h = 0; h < 2; ++h)
    out_u[h] = ((uint32_t)(rw0 + u_row[h]) * ld_out + (uint32_t)(cw0 - col_org + u_col[h])) * 4u;
#pragma unroll
  for (int t = 0; t < NBLK / 2; ++t) {
    const int i = t / UJ, jj = t % UJ;
    char *slot = scr + ((2 * t) & (kRingSlots - 1)) * 1024;
    *(f32x4 *)(slot + u_acc[0]) = acc[i][2 * jj];
    *(f32x4 *)(slot + u_acc[1]) = acc[i][2 * jj + 1];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t blk_off = ((uint32_t)(16 * i) * ld_out + (uint32_t)(32 * jj)) * 4u;
      if (two_writers) {
        // op-and-store (Sec. 4.3): the other writer adds into the same words.  One word per lane
        // and instruction, so that an instruction covers two whole 128-byte rows of the pair.
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int rp = 2 * e + (lane_e >> 5);            // row position in the slot (see pair_lane)
          const int r = h ? (rp ^ 1) : rp;                 // the row it holds ...
          const int ar = 8 * h + r;
          const int ac = 4 * (((lane_e & 31) >> 2) ^ r) + (lane_e & 3);   // ... and the column
          const float v = *(const float *)(slot + h * 1024 + e * 256 + lane_e * 4);
          if (full || (rw0 + 16 * i + ar < p.M && cw0 + 32 * jj + ac < col_hi)) {
            float *dst = (float *)((char *)const_cast<float *>(out_base) + blk_off) +
                         (int64_t)(rw0 + ar) * ld_out + (cw0 - col_org + ac);
            __hip_atomic_fetch_add(dst, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
      } else {
        const f32x4 v = *(const f32x4 *)(slot + h * 1024 + lane * 16);
        if (full || (rw0 + 16 * i + u_row[h] < p.M && cw0 + 32 * jj + u_col[h] < col_hi))
          store_agent(out_rsrc, out_u[h], blk_off, v);
      }
    }
    // keep the scheduler from running many pairs ahead: it would park their values in registers
    if (t % 2 == 1) __builtin_amdgcn_sched_barrier(0);
  }
  }
  }

  stamp(it, 3);
  if (nkf == 0) flush_pending();                 // (no main loop ran: nothing was settled on the way)
  if (half0) {
    pending_half = tail_idx;                     // announced once the stores are acknowledged
  } else if (tracked) {
    pending_c = tl.c;
    pending_n = min(p.pair_m, p.Mt_t - tl.mi * p.pair_m);
  }
  }  // pieces of work
  flush_pending();
}

// ---------------------------------------------------------------------------------------------
// Unfused baseline, second kernel: the reduce-scatter's reduction (Sec. 2.3): out = C + incoming,
// tile by tile in the same issue order, driving the same tracker and release.
template <int BM, int BN>
__global__ __launch_bounds__(kThreads) void reduce_tile_kernel(const Plan p) {
  __shared__ uint32_t sh_word;
  Tile tl;
  int slot = 0, agent = 0;
  const int role = decode_block(p, blockIdx.x, tl, slot, agent);
  if (role == kRoleNone) return;
  if (role == kRoleRelease) {
    release_chunk(p, slot, agent, &sh_word);
    return;
  }
  const Trk trk = trk_open(p);
  const int tid = threadIdx.x;
  const int m0 = tl.mi * BM;
  const int col_lo = tl.c * p.W;
  const int n0 = col_lo + tl.nj * BN;
  const int rows = min(BM, p.M - m0);
  const int cols4 = min(BN, col_lo + p.W - n0) >> 2;
  const bool store_only = (p.flags & kFlagStep0StoreOnly) && tl.s == 0;
  const bool to_fwd = (p.flags & kFlagFwdDirect) && tl.c != p.own;
  float *out_base = to_fwd ? p.fwd + (int64_t)tl.s * p.M * p.W + (n0 - col_lo) : p.R + n0;
  const int64_t ld_out = to_fwd ? p.W : p.ldr;
  if (to_fwd && (p.flags & kFlagFwdBf16)) {
    // bfloat16 forward slot: eight sums = 16 bytes per lane
    const int cols8 = cols4 >> 1;
    uint16_t *out16 = (uint16_t *)p.fwd + (int64_t)tl.s * p.M * p.W + (n0 - col_lo);
    for (int e = tid; e < rows * cols8; e += kThreads) {
      const int rr = e / cols8, cc = e - rr * cols8;
      const int64_t row = m0 + rr;
      const f32x4 *c = (const f32x4 *)(p.C + row * p.ldc + n0) + 2 * cc;
      const f32x4 *r = (const f32x4 *)(p.R + row * p.ldr + n0) + 2 * cc;
      f32x4 lo = __builtin_nontemporal_load(c), hi = __builtin_nontemporal_load(c + 1);
      if (!store_only) {
        lo += __builtin_nontemporal_load(r);
        hi += __builtin_nontemporal_load(r + 1);
      }
      const u32x4 v = pack_bf16(lo, hi);
      asm volatile("global_store_dwordx4 %0, %1, off sc1"
                   : : "v"((u32x4 *)(out16 + row * p.W) + cc), "v"(v) : "memory");
    }
    track_tile(p, trk, tl.c);
    return;
  }
  const int total = rows * cols4;
  for (int e = tid; e < total; e += kThreads) {
    const int rr = e / cols4, cc = e - rr * cols4;
    const int64_t row = m0 + rr;
    f32x4 v = __builtin_nontemporal_load((const f32x4 *)(p.C + row * p.ldc + n0) + cc);
    if (!store_only)
      v += __builtin_nontemporal_load((const f32x4 *)(p.R + row * p.ldr + n0) + cc);
    store_agent((f32x4 *)(out_base + row * ld_out) + cc, v);
  }
  track_tile(p, trk, tl.c);
}

// The upstream neighbour's updates (the DMA updates of Sec. 4.1), stood in for on one GPU:
// `incoming` (p.C) is added into R tile by tile with the same op-and-store atomics as the local
// GEMM's tiles, in the same issue order, and every tile is counted in the same tracker.  With
// the first chunk stored only (Sec. 4.4) it has no upstream update: those tiles are skipped.
template <int BM, int BN>
__global__ __launch_bounds__(kThreads) void upstream_update_kernel(const Plan p) {
  const Trk trk = trk_open(p);
  // one workgroup per grid position, or fewer workgroups walking the positions in issue order
  for (int pos = blockIdx.x; pos < p.total_blocks; pos += gridDim.x) {
    Tile tl;
    int slot = 0, agent = 0;
    if (decode_block(p, pos, tl, slot, agent) != kRoleTile) continue;
    if ((p.flags & kFlagStep0StoreOnly) && tl.s == 0) continue;
    const int m0 = tl.mi * BM;
    const int col_lo = tl.c * p.W;
    const int n0 = col_lo + tl.nj * BN;
    const int rows = min(BM, p.M - m0);
    const int cols = min(BN, col_lo + p.W - n0);
    const int total = rows * cols;
    // One word per lane, so that an atomic instruction covers whole 128-byte lines; eight loads
    // in flight per lane before their adds go out (a workgroup would otherwise move one word per
    // lane per memory round trip).
    constexpr int kBatch = 8;
    for (int e0 = threadIdx.x; e0 < total; e0 += kBatch * kThreads) {
      float v[kBatch];
      int64_t at[kBatch];
#pragma unroll
      for (int k = 0; k < kBatch; ++k) {
        const int e = e0 + k * kThreads;
        const int rr = e / cols, cc = e - rr * cols;
        at[k] = (int64_t)(m0 + rr);
        v[k] = 0.f;
        if (e < total) v[k] = __builtin_nontemporal_load(p.C + at[k] * p.ldc + n0 + cc);
        at[k] = at[k] * p.ldr + n0 + cc;
      }
#pragma unroll
      for (int k = 0; k < kBatch; ++k)
        if (e0 + k * kThreads < total)
          __hip_atomic_fetch_add(p.R + at[k], v[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    track_tile(p, trk, tl.c);
  }
}

// The triggered transfers, as a launch of their own (two-writer mode, where no launch can wait
// for the other writer): workgroup (slot, agent) copies its rows of chunk order[slot] into the
// forward slot if the chunk's ready flag is set in the bank of the launch that last completed.
__global__ __launch_bounds__(kThreads) void release_ready_kernel(const Plan p) {
  const int slot = blockIdx.x / p.agents, agent = blockIdx.x % p.agents;
  if (slot > p.P - 2) return;
  const uint32_t g = __builtin_amdgcn_readfirstlane(__hip_atomic_load(
      p.track + 2 * trk_bank_words(p.P), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  const uint32_t *bank = p.track + ((g + 1u) & 1u) * trk_bank_words(p.P);   // bank (g - 1) & 1
  int c = p.rank + slot;
  if (c >= p.P) c -= p.P;
  if (__hip_atomic_load(bank + p.P + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
  copy_chunk_rows(p, slot, c, agent * p.rows_per_agent + (int)(threadIdx.x >> 6),
                  min(p.M, (agent + 1) * p.rows_per_agent), kThreads / 64);
}

// Clears tracker state: both banks (queue entries to empty, the rest to 0), gen, error and the
// flags of split tiles to 0.
__global__ void track_reset_kernel(uint32_t *track, int P) {
  const int bank = 3 * P + 2, n = 2 * bank + 2 + kTailSlots;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const int j = i < 2 * bank ? i % bank : -1;
    track[i] = (j >= 2 * P && j < 3 * P) ? kEmpty : 0u;
  }
}

// One step of the ring all-gather (Sec. 2.3): a chunk of M rows x W columns moves, unchanged,
// from the upstream neighbour's buffer into the same columns of this rank's.  One wavefront per
// row and pass, 16 bytes per lane, four accesses in flight per lane.
__global__ __launch_bounds__(kThreads) void ag_copy_kernel(const float *src, int64_t ld_src, float *dst,
                                                           int64_t ld_dst, int32_t M, int32_t W) {
  const int lane = threadIdx.x & 63;
  const int W4 = W >> 2;
  const int waves = (int)(gridDim.x * (blockDim.x >> 6));
  for (int r = (int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)); r < M; r += waves) {
    const f32x4 *s4 = (const f32x4 *)(src + (int64_t)r * ld_src);
    f32x4 *d4 = (f32x4 *)(dst + (int64_t)r * ld_dst);
    for (int c0 = lane; c0 < W4; c0 += 4 * 64) {
      f32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c0 + u * 64 < W4) v[u] = __builtin_nontemporal_load(s4 + c0 + u * 64);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c0 + u * 64 < W4) __builtin_nontemporal_store(v[u], d4 + c0 + u * 64);
    }
  }
}

// Copies n words of tracker state (for callers that want to read the state another array holds).
__global__ void track_copy_kernel(const uint32_t *src, uint32_t *dst, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x)
    dst[i] = __hip_atomic_load(&src[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace t3k
