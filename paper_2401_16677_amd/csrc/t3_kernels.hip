// Device code of the fused sliced-GEMM + reduce-scatter-reduction path for gfx950 (CDNA4).
//
// One workgroup (256 threads = 4 wavefronts of 64, arranged 2 x 2) produces one
// BM x BN output tile with v_mfma_f32_32x32x16_bf16.  A and B K-slabs of 64 bf16 are
// staged through LDS in an XOR-swizzled layout; the next slab is prefetched into
// registers while the current one is multiplied.  Two workgroups fit on a compute unit,
// so one workgroup's epilogue traffic (the reduction with the incoming partial, Sec. 4.3
// of the T3 paper) runs under the other's matrix work.
//
// Included by t3_api.hip only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace t3k {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kThreads = 256;
constexpr int kBK = 64;               // bf16 elements of K per slab: one 128-byte LDS row
constexpr int kChunksPerRow = 8;      // 16-byte chunks in an LDS row
constexpr uint32_t kEmpty = 0xFFFFFFFFu;

constexpr uint32_t kFlagStep0StoreOnly = 1u;
constexpr uint32_t kFlagFwdDirect = 2u;

enum Mode { kModeGemm = 0, kModeFused = 1 };

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
  int32_t M, N, K, P, rank, W, own;
  int32_t Mt, Wt, tpc;
  int32_t xcd_nbm, xcd_bmk, xcd_bnk;   // XCD grouping of a stage's tiles; xcd_nbm == 0: none
  int32_t unit_rows, units_per_chunk;  // release copy granularity
  uint32_t flags;
};

struct Tile {
  int s, c, mi, nj;
};

// blockIdx -> issue index -> tile.  Workgroups are dealt round-robin to the 8 XCDs, so
// inside a stage workgroup j lands on XCD j % 8; that XCD gets a compact block of
// xcd_bmk x xcd_bnk tiles which share A rows and B columns in its L2.
__device__ inline bool decode_tile(const Plan &p, Tile &tl) {
  const int b = blockIdx.x;
  const int s = b / p.tpc;
  const int j = b - s * p.tpc;
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
  const int64_t t = (int64_t)s * p.tpc + (int64_t)nj * p.Mt + mi;
  int c = p.rank + s;
  if (c >= p.P) c -= p.P;
  tl.s = s;
  tl.c = c;
  tl.mi = mi;
  tl.nj = nj;
  return t < p.limit;
}

// LDS row r keeps its 16-byte chunk k at position k ^ swz(r): 16 consecutive rows read
// at one k land in 16 different bank groups.
__device__ inline int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

// ---------------------------------------------------------------------------------------------
// Track & trigger (Sec. 4.2), then release of triggered chunks into their forward slots.
// Called by all threads of a workgroup after the tile's stores have been issued.
__device__ inline void track_and_release(const Plan &p, int c, uint32_t *sh) {
  const int tid = threadIdx.x;
  uint32_t *counter = p.track;
  uint32_t *ready = counter + p.P;
  uint32_t *queue = ready + p.P;
  uint32_t *queue_len = queue + p.P;
  uint32_t *claim = queue_len + 1;

  __threadfence();      // this thread's tile stores are visible device-wide ...
  __syncthreads();      // ... for every thread of the workgroup, before the tile is counted
  if (tid == 0) {
    const uint32_t old =
        __hip_atomic_fetch_add(&counter[c], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1u == (uint32_t)p.tpc) {   // the landing that reaches the threshold triggers
      if (c != p.own) {
        const uint32_t pos =
            __hip_atomic_fetch_add(queue_len, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&queue[pos], (uint32_t)c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __hip_atomic_store(&ready[c], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if ((p.flags & kFlagFwdDirect) || p.P == 1) return;

  // Release: every workgroup that finishes a tile hands out and copies pieces ("units" of
  // unit_rows rows) of the chunks that are ready, until none are left.  The workgroup that
  // triggered a chunk stays until all of its units are handed out, and a unit's claimer
  // finishes it before exiting, so every triggered chunk is in its slot when the grid ends.
  const int W4 = p.W >> 2;
  for (int s2 = 0; s2 < p.P - 1; ++s2) {
    int c2 = p.rank + s2;
    if (c2 >= p.P) c2 -= p.P;
    for (;;) {
      __syncthreads();
      if (tid == 0) {
        uint32_t u = kEmpty;
        if (__hip_atomic_load(&ready[c2], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) &&
            __hip_atomic_load(&claim[s2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <
                (uint32_t)p.units_per_chunk)
          u = __hip_atomic_fetch_add(&claim[s2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *sh = u;
      }
      __syncthreads();
      const uint32_t u = *sh;
      if (u >= (uint32_t)p.units_per_chunk) break;
      __threadfence();    // other workgroups' sums, published before ready[c2], are visible here
      const int r0 = (int)u * p.unit_rows;
      const int nr = min(p.unit_rows, p.M - r0);
      const float *src = p.R + (int64_t)r0 * p.ldr + (int64_t)c2 * p.W;
      float *dst = p.fwd + ((int64_t)s2 * p.M + r0) * p.W;
      const int total = nr * W4;
      for (int e = tid; e < total; e += kThreads) {
        const int rr = e / W4, cc = e - rr * W4;
        const f32x4 v = __builtin_nontemporal_load((const f32x4 *)(src + (int64_t)rr * p.ldr) + cc);
        __builtin_nontemporal_store(v, (f32x4 *)(dst + (int64_t)rr * p.W) + cc);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Global -> register loads of one K-slab: ROWS rows of 64 bf16, 16 bytes per thread per pass.
template <int ROWS>
__device__ inline void load_slab(uint4 (&regs)[ROWS * kChunksPerRow / kThreads],
                                 const uint16_t *base, const uint32_t (&off)[ROWS * kChunksPerRow / kThreads],
                                 int k0, int K, int kc_local) {
  constexpr int N = ROWS * kChunksPerRow / kThreads;
  if (k0 + kBK <= K) {
#pragma unroll
    for (int i = 0; i < N; ++i)
      regs[i] = *(const uint4 *)(base + k0 + off[i]);
  } else {   // ragged last slab: chunks past K are zeros (K is a multiple of 8)
    const bool in = k0 + kc_local < K;
#pragma unroll
    for (int i = 0; i < N; ++i)
      regs[i] = in ? *(const uint4 *)(base + k0 + off[i]) : make_uint4(0, 0, 0, 0);
  }
}

template <int BM, int BN, int MODE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void gemm_tile_kernel(const Plan p) {
  constexpr int WM = BM / 2, WN = BN / 2;       // wavefront tile
  constexpr int FM = WM / 32, FN = WN / 32;     // 32x32 MFMA blocks per wavefront
  constexpr int NA = BM * kChunksPerRow / kThreads;
  constexpr int NB = BN * kChunksPerRow / kThreads;

  __shared__ uint4 lds[(BM + BN) * kChunksPerRow];
  __shared__ uint32_t sh_word;

  Tile tl;
  if (!decode_tile(p, tl)) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const int m0 = tl.mi * BM;
  const int col_lo = tl.c * p.W;                 // chunk bounds in N
  const int col_hi = col_lo + p.W;
  const int n0 = col_lo + tl.nj * BN;

  // per-thread global offsets (in elements) of its 16-byte chunks; rows clamped into range
  const int ld_row = tid >> 3, ld_chunk = tid & 7;
  uint32_t offA[NA], offB[NB];
#pragma unroll
  for (int i = 0; i < NA; ++i)
    offA[i] = (uint32_t)(min(m0 + ld_row + i * 32, p.M - 1) * p.lda + ld_chunk * 8);
#pragma unroll
  for (int i = 0; i < NB; ++i)
    offB[i] = (uint32_t)(min(n0 + ld_row + i * 32, col_hi - 1) * p.ldb + ld_chunk * 8);
  const int st_slot = ld_row * kChunksPerRow + (ld_chunk ^ swz(ld_row));   // rows +32 keep swz

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 ra[NA], rb[NB];
  const int nk = (p.K + kBK - 1) / kBK;
  if (nk > 0) {
    load_slab<BM>(ra, p.A, offA, 0, p.K, ld_chunk * 8);
    load_slab<BN>(rb, p.B, offB, 0, p.K, ld_chunk * 8);
  }

  // fragment read addressing: lane reads row (lane & 31) of a 32-row block, chunk 2*kk + (lane>>5)
  const int fr = lane & 31, fh = lane >> 5, fs = swz(fr);
  const uint4 *ldsA = lds + (wm * WM + fr) * kChunksPerRow;
  const uint4 *ldsB = lds + (BM + wn * WN + fr) * kChunksPerRow;

  for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
    for (int i = 0; i < NA; ++i) lds[st_slot + i * 32 * kChunksPerRow] = ra[i];
#pragma unroll
    for (int i = 0; i < NB; ++i) lds[BM * kChunksPerRow + st_slot + i * 32 * kChunksPerRow] = rb[i];
    __syncthreads();
    if (kt + 1 < nk) {
      load_slab<BM>(ra, p.A, offA, (kt + 1) * kBK, p.K, ld_chunk * 8);
      load_slab<BN>(rb, p.B, offB, (kt + 1) * kBK, p.K, ld_chunk * 8);
    }
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      const int pos = (2 * kk + fh) ^ fs;
      bf16x8 af[FM], bf[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i)
        af[i] = __builtin_bit_cast(bf16x8, ldsA[i * 32 * kChunksPerRow + pos]);
#pragma unroll
      for (int j = 0; j < FN; ++j)
        bf[j] = __builtin_bit_cast(bf16x8, ldsB[j * 32 * kChunksPerRow + pos]);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator element 4*g + e of block (i, j) is row 8*g + 4*(lane>>5) + e,
  // column lane & 31 of the block: per register, 32 lanes cover 128 contiguous bytes of a row.
  const bool store_only = (MODE == kModeGemm) ||
                          ((p.flags & kFlagStep0StoreOnly) && tl.s == 0);
  const bool to_fwd = (MODE == kModeFused) && (p.flags & kFlagFwdDirect) && tl.c != p.own;
  const int64_t ld_in = (MODE == kModeGemm) ? p.ldc : p.ldr;
  float *out_base;
  int64_t ld_out;
  int col_shift;
  if (to_fwd) {
    out_base = p.fwd + (int64_t)tl.s * p.M * p.W;
    ld_out = p.W;
    col_shift = col_lo;
  } else {
    out_base = p.R;
    ld_out = ld_in;
    col_shift = 0;
  }
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int col = n0 + wn * WN + j * 32 + fr;
      const int row_b = m0 + wm * WM + i * 32 + 4 * fh;
      const bool col_ok = col < col_hi;
      float inc[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = row_b + 8 * (e >> 2) + (e & 3);
        inc[e] = 0.f;
        if (!store_only && col_ok && row < p.M)
          inc[e] = __builtin_nontemporal_load(p.R + (int64_t)row * ld_in + col);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = row_b + 8 * (e >> 2) + (e & 3);
        if (col_ok && row < p.M)
          __builtin_nontemporal_store(inc[e] + acc[i][j][e],
                                      out_base + (int64_t)row * ld_out + (col - col_shift));
      }
    }
  }

  if (MODE == kModeFused) track_and_release(p, tl.c, &sh_word);
}

// ---------------------------------------------------------------------------------------------
// Unfused baseline, second kernel: the reduce-scatter's reduction (Sec. 2.3): out = C + incoming,
// tile by tile in the same issue order, driving the same tracker.
template <int BM, int BN>
__global__ __launch_bounds__(kThreads) void reduce_tile_kernel(const Plan p) {
  __shared__ uint32_t sh_word;
  Tile tl;
  if (!decode_tile(p, tl)) return;
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
  const int total = rows * cols4;
  for (int e = tid; e < total; e += kThreads) {
    const int rr = e / cols4, cc = e - rr * cols4;
    const int64_t row = m0 + rr;
    f32x4 v = __builtin_nontemporal_load((const f32x4 *)(p.C + row * p.ldc + n0) + cc);
    if (!store_only)
      v += __builtin_nontemporal_load((const f32x4 *)(p.R + row * p.ldr + n0) + cc);
    __builtin_nontemporal_store(v, (f32x4 *)(out_base + row * ld_out) + cc);
  }
  track_and_release(p, tl.c, &sh_word);
}

// Clears tracker state: counters, flags, queue length and claims to 0, queue entries to empty.
__global__ void track_reset_kernel(uint32_t *track, int P) {
  const int n = 4 * P + 1;
  for (int i = threadIdx.x; i < n; i += blockDim.x)
    track[i] = (i >= 2 * P && i < 3 * P) ? kEmpty : 0u;
}

}  // namespace t3k
