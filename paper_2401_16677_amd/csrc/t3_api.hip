// Host side of the C ABI declared in include/t3.h: argument validation, the launch plan
// (ring order, tile grid, XCD grouping, release granularity) and the kernel launches.
#include "t3.h"

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <stdio.h>

#include <atomic>
#include <mutex>

#include "t3_kernels.hip"

namespace {

thread_local int32_t g_last_hip_error = 0;

struct TileShape {
  int32_t m, n;
};
// preference order of t3_default_tile
constexpr TileShape kTileShapes[] = {{256, 256}, {256, 128}, {128, 256}, {128, 128}};
constexpr int kNumTileShapes = sizeof(kTileShapes) / sizeof(kTileShapes[0]);
constexpr int kNumXcd = 8;            // the XCD grouping of decode_tile is written for 8 XCDs
constexpr int kDefaultCus = 256;       // compute units of an MI355X (host-only plan queries assume it)
constexpr int kMaxDevices = 64;
constexpr int kNtMinK = 3072;          // K from which result stores take the streaming hint
constexpr int64_t kMemorySideCacheBytes = 256ll << 20;
constexpr int kTailMinSlabs = 8;       // K-slabs of 64 a tile needs before a balanced tail splits it
// Matrix rate of one compute unit the start-up offsets are sized with: 4096 flop/clock at a
// sustained ~1.5 GHz under load, in flop per nanosecond.
constexpr double kCuFlopPerNs = 6.25e3;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// What the launch plan needs to know of the device it launches on, read from the runtime once
// per device (hardware attributes only; they never change while the process lives).
struct DeviceFacts {
  int cus;     // compute units: persistent workgroups are sized to them
  int xcds;    // accelerator dies the dispatcher deals workgroups to, round-robin
};
std::mutex g_facts_mutex;
DeviceFacts g_facts[kMaxDevices];
bool g_facts_known[kMaxDevices];

// Facts of the current device; T3_ERR_HIP if the runtime cannot tell.
t3_status device_facts(DeviceFacts *out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
  if (e == hipSuccess) {
    std::lock_guard<std::mutex> lock(g_facts_mutex);
    if (!g_facts_known[dev]) {
      DeviceFacts f{0, 0};
      e = hipDeviceGetAttribute(&f.cus, hipDeviceAttributeMultiprocessorCount, dev);
      if (e == hipSuccess && hipDeviceGetAttribute(&f.xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess) {
        (void)hipGetLastError();
        f.xcds = 1;                // unknown: plan without XCD grouping
      }
      if (e == hipSuccess && f.cus < 1) e = hipErrorInvalidDevice;
      if (e == hipSuccess) {
        g_facts[dev] = f;
        g_facts_known[dev] = true;
      }
    }
    if (e == hipSuccess) *out = g_facts[dev];
  }
  if (e != hipSuccess) {
    g_last_hip_error = (int32_t)e;
    return T3_ERR_HIP;
  }
  return T3_OK;
}

// Where tile kernels record their timelines (t3_timeline), for the launches of every thread.
std::atomic<uint64_t *> g_timeline{nullptr};
std::atomic<int64_t> g_timeline_wgs{0};

// Tracker state for t3_gemm_rs_fused_static, the entry point for callers that cannot allocate:
// one array per device (each GPU the library runs on holds its own copy at its own address
// until the process ends).  Host code never uses the array's name as an address: the device
// address is looked up once per device and kept.
constexpr int kStaticMaxTp = T3_STATIC_MAX_TP;
constexpr int kStaticTrackWords = 2 * (3 * kStaticMaxTp + 2) + 2 + t3k::kTailSlots;
static __device__ __align__(256) uint32_t scratch[kStaticTrackWords];
uint32_t *g_scratch_ptr[kMaxDevices];

// Device address of the current device's `scratch`; T3_ERR_HIP if the runtime cannot tell.
t3_status static_track(uint32_t **out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
  if (e == hipSuccess) {
    std::lock_guard<std::mutex> lock(g_facts_mutex);
    if (!g_scratch_ptr[dev]) {
      void *ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));   // the current device's copy
      if (e == hipSuccess && !ptr) e = hipErrorInvalidSymbol;
      if (e == hipSuccess) g_scratch_ptr[dev] = static_cast<uint32_t *>(ptr);
    }
    if (e == hipSuccess) *out = g_scratch_ptr[dev];
  }
  if (e != hipSuccess) {
    g_last_hip_error = (int32_t)e;
    return T3_ERR_HIP;
  }
  return T3_OK;
}

// Flags of the tiles a balanced tail splits, for t3_gemm, which is given no tracker state to
// keep them in: a few sets of flag words per device.  Two launches may share a set only one
// after the other (the second half of a tile clears the flag the first half raised), so behind
// every launch an event is recorded, and a launch that takes a set whose last user may still be
// running is made to wait for that event first: a launch on the same stream would have waited
// anyway, launches on more streams than there are sets get serialised.  A launch whose stream is
// being captured runs without a balanced tail (a replayed graph would use the set while this
// bookkeeping knows nothing of it).
constexpr int kGemmTailSets = 8;
static __device__ __align__(256) uint32_t gemm_tail_flags[kGemmTailSets * t3k::kTailSlots];
struct GemmTail {
  uint32_t *base = nullptr;              // device address of the current device's gemm_tail_flags
  hipEvent_t done[kGemmTailSets] = {};   // recorded behind the last launch that used the set
  hipStream_t stream[kGemmTailSets] = {};
  bool used[kGemmTailSets] = {};
  unsigned next = 0;
};
GemmTail g_gemm_tail[kMaxDevices];

// Launches the plain GEMM `q` (balanced tail wanted) on stream s with a set of flags, or without
// a balanced tail if no set can be had.  The whole sequence runs under the lock, so that the
// event of a set always belongs to its last launch.
template <typename LaunchFn>
t3_status launch_with_gemm_tail(t3k::Plan &q, hipStream_t s, LaunchFn launch_fn) {
  auto plain = [&]() {
    (void)hipGetLastError();
    q.tail_r = q.tail_q = 0;
    q.tail_flags = nullptr;
    return launch_fn(q);
  };
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  int dev = 0;
  if (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone ||
      hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return plain();
  std::lock_guard<std::mutex> lock(g_facts_mutex);
  GemmTail &g = g_gemm_tail[dev];
  if (!g.base) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(gemm_tail_flags)) != hipSuccess || !ptr) return plain();
    g.base = static_cast<uint32_t *>(ptr);
  }
  // the set this stream used last, else the next in turn
  int set = -1;
  for (int i = 0; i < kGemmTailSets; ++i)
    if (g.used[i] && g.stream[i] == s) set = i;
  if (set < 0) set = (int)(g.next++ % kGemmTailSets);
  if (!g.used[set]) {
    if (hipEventCreateWithFlags(&g.done[set], hipEventDisableTiming) != hipSuccess) return plain();
  } else if (hipStreamWaitEvent(s, g.done[set], 0) != hipSuccess) {
    return plain();
  }
  g.used[set] = true;
  g.stream[set] = s;
  q.tail_flags = g.base + set * t3k::kTailSlots;
  const t3_status st = launch_fn(q);
  // (a launch that failed used nothing; a record that fails leaves the older record in place)
  if (st == T3_OK && hipEventRecord(g.done[set], s) != hipSuccess) (void)hipGetLastError();
  return st;
}

// T3_STAGGER="groups,window_ns" from the environment, read once per process.
struct StaggerEnv {
  bool set = false, off = false;
  int groups = 0, window_ns = 0;
};
const StaggerEnv &stagger_env() {
  static const StaggerEnv env = [] {
    StaggerEnv v;
    if (const char *e = getenv("T3_STAGGER")) {
      int eg = 0, ens = 0;
      const int n = sscanf(e, "%d,%d", &eg, &ens);
      if (n == 2 && eg > 1 && ens > 0) {
        v.set = true;
        v.groups = eg;
        v.window_ns = ens;
      } else if (n >= 1 && eg == 0) {
        v.set = v.off = true;
      }
    }
    return v;
  }();
  return env;
}

t3_status check_shape(const t3_problem *p) {
  if (!p) return T3_ERR_NULL;
  if (p->M < 0 || p->N < 0 || p->K < 0 || p->tp < 1 || p->rank < 0 || p->rank >= p->tp)
    return T3_ERR_BAD_SHAPE;
  if (p->N % p->tp != 0) return T3_ERR_BAD_SHAPE;
  return T3_OK;
}

bool tile_supported(int32_t tm, int32_t tn) {
  for (int i = 0; i < kNumTileShapes; ++i)
    if (kTileShapes[i].m == tm && kTileShapes[i].n == tn) return true;
  return false;
}

void default_tile(const t3_problem *p, int cus, int32_t *tm, int32_t *tn) {
  // Cheapest shape by (work padded up to whole tiles) x (how much slower than the 256 x 256
  // tile the shape's main loop runs per product, measured) x (how far the tiles fall short of
  // filling the chip's `cus` compute units).  128 x 256 tiles are computed in pairs, as 256 x 256
  // workgroup tiles: they cost what those cost, padding of M to 256 rows included.
  static const double kSlower[kNumTileShapes] = {1.0, 1.21, 1.0, 1.28};
  const int64_t W = p->N / p->tp;
  double best = -1.0;
  *tm = 128;
  *tn = 128;
  for (int i = 0; i < kNumTileShapes; ++i) {
    const int64_t Mt = ceil_div(p->M, kTileShapes[i].m), Wt = ceil_div(W, kTileShapes[i].n);
    const int64_t T = Mt * Wt * p->tp;
    if (T == 0) continue;
    const bool paired = kTileShapes[i].m == 128 && kTileShapes[i].n == 256 && Mt > 1;
    const int64_t rows = paired ? ceil_div(p->M, 256) * 256 : Mt * kTileShapes[i].m;
    const int64_t groups = paired ? ceil_div(Mt, 2) * Wt * p->tp : T;     // workgroup tiles
    const double padded = (double)rows * (double)(Wt * kTileShapes[i].n) / ((double)p->M * (double)W);
    const double score = padded * kSlower[i] * (groups < cus ? (double)cus / (double)groups : 1.0);
    if (best < 0 || score < best) {
      best = score;
      *tm = kTileShapes[i].m;
      *tn = kTileShapes[i].n;
    }
  }
}

t3_status resolve_tile(const t3_problem *p, int32_t *tm, int32_t *tn) {
  if (p->tile_m == 0 && p->tile_n == 0) {
    default_tile(p, kDefaultCus, tm, tn);
    return T3_OK;
  }
  if (!tile_supported(p->tile_m, p->tile_n)) return T3_ERR_BAD_TILE;
  *tm = p->tile_m;
  *tn = p->tile_n;
  return T3_OK;
}

// the kernels test the same flag bits under their own names
static_assert(T3_FLAG_STEP0_STORE_ONLY == t3k::kFlagStep0StoreOnly &&
                  T3_FLAG_FWD_DIRECT == t3k::kFlagFwdDirect &&
                  T3_FLAG_TWO_WRITERS == t3k::kFlagTwoWriters && T3_FLAG_FWD_BF16 == t3k::kFlagFwdBf16,
              "flag bits of the header and of the kernels");
static_assert(sizeof(t3_problem) == 104, "layout documented in the header");
static_assert(T3_TIMELINE_ITEMS == t3k::kTimelineItems, "timeline layout of the header and of the kernels");

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

enum Need { kNeedAB = 1, kNeedR = 2, kNeedC = 4, kNeedFwd = 8, kNeedTrack = 16,
            kNeedTwoWriters = 32 /* the call exists only in two-writer mode */,
            kMayPair = 64 /* the call launches the tile kernel, which can compute 256 x 256
                             workgroup tiles under 128 x 256 tracked ones */ };

// The flag words of a balanced tail in tracker state: behind the two banks, gen and error.
inline uint32_t *tail_flags_in(uint32_t *track, int32_t tp) { return track + 2 * (3 * (int64_t)tp + 2) + 2; }

// Validates everything and fills the plan.  *empty is set when there is nothing to launch.
t3_status make_plan(const t3_problem *p, int need, const void *A, const void *B, const float *C,
                    float *R, void *fwd, uint32_t *track, t3k::Plan *plan, int32_t *tm,
                    int32_t *tn, bool *empty) {
  t3_status st = check_shape(p);
  if (st != T3_OK) return st;
  st = resolve_tile(p, tm, tn);
  if (st != T3_OK) return st;
  const bool fused_like = (need & kNeedTrack) != 0;
  const bool direct = fused_like && (p->flags & T3_FLAG_FWD_DIRECT);
  const bool two_writers = fused_like && (p->flags & T3_FLAG_TWO_WRITERS);
  if ((need & kNeedAB) && (!A || !B)) return T3_ERR_NULL;
  if ((need & kNeedR) && !R) return T3_ERR_NULL;
  if ((need & kNeedC) && !C) return T3_ERR_NULL;
  if ((need & kNeedTrack) && !track) return T3_ERR_NULL;
  if ((need & kNeedFwd) && p->tp > 1 && !fwd && !(two_writers && (need & kNeedAB)))
    return T3_ERR_NULL;                         // (the fused call releases nothing with two writers)
  if (p->flags & ~(T3_FLAG_STEP0_STORE_ONLY | T3_FLAG_FWD_DIRECT | T3_FLAG_TWO_WRITERS |
                   T3_FLAG_FWD_BF16))
    return T3_ERR_UNSUPPORTED;
  if (two_writers && direct) return T3_ERR_UNSUPPORTED;   // both writers must target R
  if ((need & kNeedTwoWriters) && !two_writers) return T3_ERR_UNSUPPORTED;
  // split-K: several workgroups add into one tile, so it needs the atomic updates of two-writer
  // mode, and every part needs at least one full K-slab of 64
  const int32_t split_k = p->split_k > 1 ? p->split_k : 1;
  if (p->split_k < 0) return T3_ERR_BAD_SHAPE;
  if (split_k > 1 && fused_like && (!two_writers || split_k > p->K / 64 || split_k > 64))
    return T3_ERR_UNSUPPORTED;
  // the unfused reduction kernel has no second writer to wait for
  if (two_writers && (need & kNeedC) && (need & kNeedFwd) && !(need & kNeedTwoWriters))
    return T3_ERR_UNSUPPORTED;

  const int64_t W = p->N / p->tp;
  if (need & kNeedAB) {
    if (p->b_layout != T3_B_NK && p->b_layout != T3_B_KN) return T3_ERR_BAD_SHAPE;
    if (p->a_layout != T3_A_MK && p->a_layout != T3_A_KM) return T3_ERR_BAD_SHAPE;
    if (p->reserved != 0) return T3_ERR_BAD_SHAPE;
    const bool kn = p->b_layout == T3_B_KN, km = p->a_layout == T3_A_KM;
    if (p->lda < (km ? p->M : p->K) || p->ldb < (kn ? p->N : p->K)) return T3_ERR_BAD_SHAPE;
    if (p->K % 8 || p->lda % 8 || p->ldb % 8 || !aligned16(A) || !aligned16(B)) return T3_ERR_ALIGN;
    // A stored K x M: 16-byte pieces run along M, and whole K-slabs of 64 only
    if (km && p->M % 8) return T3_ERR_ALIGN;
    if (km && p->K % 64) return T3_ERR_UNSUPPORTED;
    // B stored K x N: 16-byte pieces run along N, so chunks must be cut on multiples of 8
    // columns, and the transposed operand path takes whole K-slabs of 64 only
    if (kn && W % 8) return T3_ERR_ALIGN;
    if (kn && p->K % 64) return T3_ERR_UNSUPPORTED;
    // kernels address A and B with 32-bit element offsets
    if ((int64_t)(km ? p->K : p->M) * p->lda >= (1ll << 31) ||
        (int64_t)(kn ? p->K : p->N) * p->ldb >= (1ll << 31))
      return T3_ERR_UNSUPPORTED;
  }
  // kernels address R, C and a forward slot with 32-bit byte offsets
  if (need & kNeedR) {
    if (p->ldr < p->N) return T3_ERR_BAD_SHAPE;
    if (p->ldr % 4 || W % 4 || !aligned16(R)) return T3_ERR_ALIGN;
    if ((int64_t)p->M * p->ldr * 4 >= (1ll << 32)) return T3_ERR_UNSUPPORTED;
  }
  if (need & kNeedC) {
    if (p->ldc < p->N) return T3_ERR_BAD_SHAPE;
    if (p->ldc % 4 || W % 4 || !aligned16(C)) return T3_ERR_ALIGN;
    if ((int64_t)p->M * p->ldc * 4 >= (1ll << 32)) return T3_ERR_UNSUPPORTED;
  }
  if ((need & kNeedFwd) && fwd && !aligned16(fwd)) return T3_ERR_ALIGN;
  // bfloat16 forward slots move 8 elements per 16-byte access
  if ((need & kNeedFwd) && fused_like && (p->flags & T3_FLAG_FWD_BF16) && W % 8) return T3_ERR_ALIGN;

  // tracked tiles (the problem's tile shape): what the issue order, the tile range and the
  // tracker's thresholds are counted in
  const int64_t Mt_t = ceil_div(p->M, *tm), Wt = ceil_div(W, *tn);
  const int64_t tpc_t = Mt_t * Wt, T_t = tpc_t * p->tp;
  if (T_t >= (1ll << 31)) return T3_ERR_UNSUPPORTED;
  const int64_t limit_t = (p->tile_limit < 0 || p->tile_limit > T_t) ? T_t : p->tile_limit;
  const int64_t begin_t = p->tile_begin < 0 ? 0 : (p->tile_begin > limit_t ? limit_t : p->tile_begin);
  // Workgroup tiles.  128 x 256 tracked tiles are computed two at a time, as one 256 x 256
  // workgroup tile (tracked tiles 2 mi and 2 mi + 1 of a tile column are neighbours in the issue
  // order): the larger tile needs a third less operand traffic per product.  Only for ranges of
  // whole ring steps, so that no pair is cut by the range, and not with two writers.
  int64_t pair_m = 1;
  if ((need & kMayPair) && *tm == 128 && *tn == 256 && !two_writers && tpc_t > 0 && Mt_t > 1 &&
      begin_t % tpc_t == 0 && limit_t % tpc_t == 0) {
    pair_m = 2;
    *tm = 256;
  }
  const int64_t Mt = ceil_div(Mt_t, pair_m);
  const int64_t tpc = Mt * Wt, T = tpc * p->tp;
  *empty = (T == 0);

  // (the last refusals, before the device is asked anything: with release workgroups and with
  // split-K the grid still has to fit 31 bits)
  const int64_t n_agents = (fused_like && !direct && !two_writers && p->tp > 1) ? T3_AGENTS : 0;
  if (T + n_agents * (p->tp - 1) >= (1ll << 31)) return T3_ERR_UNSUPPORTED;
  if (two_writers && T * split_k >= (1ll << 31)) return T3_ERR_UNSUPPORTED;
  if ((need & kNeedTwoWriters) && (need & kNeedC) && p->upstream_agents < 0) return T3_ERR_BAD_SHAPE;

  DeviceFacts dev{kDefaultCus, kNumXcd};
  if (!*empty) {                                 // (nothing is launched otherwise: no device needed)
    st = device_facts(&dev);
    if (st != T3_OK) return st;
  }

  t3k::Plan &q = *plan;
  q.A = static_cast<const uint16_t *>(A);
  q.B = static_cast<const uint16_t *>(B);
  q.C = C;
  q.R = R;
  q.fwd = static_cast<float *>(fwd);     // (bfloat16 under T3_FLAG_FWD_BF16)
  q.track = track;
  q.lda = p->lda;
  q.ldb = p->ldb;
  q.ldr = p->ldr;
  q.ldc = p->ldc;
  q.limit = limit_t;
  q.begin = begin_t;
  if (q.begin >= q.limit) *empty = true;       // an empty tile range: nothing to launch
  q.M = p->M;
  q.N = p->N;
  q.K = p->K;
  q.P = p->tp;
  q.rank = p->rank;
  q.W = (int32_t)W;
  q.own = (p->rank + p->tp - 1) % p->tp;
  q.Mt = (int32_t)Mt;
  q.Wt = (int32_t)Wt;
  q.tpc = (int32_t)tpc;
  q.pair_m = (int32_t)pair_m;
  q.Mt_t = (int32_t)Mt_t;
  q.tpc_t = (int32_t)tpc_t;
  q.flags = fused_like ? p->flags : 0u;

  // XCD grouping: split a stage's Mt x Wt tiles into 8 equal blocks, one per XCD, choosing the
  // split whose block touches the fewest A rows + B columns.  (A device with another number of
  // XCDs runs without grouping: plain issue order inside a stage.)
  q.xcd_nbm = 0;
  q.xcd_bmk = q.xcd_bnk = 0;
  int64_t best = -1;
  for (int nbm = 1; nbm <= kNumXcd && dev.xcds == kNumXcd; nbm *= 2) {
    const int nbn = kNumXcd / nbm;
    if (Mt % nbm || Wt % nbn) continue;
    const int64_t foot = (Mt / nbm) * *tm + (Wt / nbn) * *tn;
    if (best < 0 || foot < best) {
      best = foot;
      q.xcd_nbm = nbm;
      q.xcd_bmk = (int32_t)(Mt / nbm);
      q.xcd_bnk = (int32_t)(Wt / nbn);
    }
  }

  // Release workgroups (default release mode only): `agents` per forwarded chunk, placed in
  // the grid `lag` stages after the chunk's own tiles, far enough that those tiles have been
  // dispatched and are mostly finished when the release workgroups start.
  q.agents = (int32_t)n_agents;
  // tile workgroups the device holds at once: one per compute unit, two of the smallest tile
  const int64_t resident = (int64_t)dev.cus * ((*tm == 128 && *tn == 128) ? 2 : 1);
  q.lag = (int32_t)(ceil_div(resident, tpc > 0 ? tpc : 1) + 1);
  if (q.lag > p->tp) q.lag = p->tp;
  q.rows_per_agent = q.agents ? (int32_t)ceil_div(p->M, q.agents) : 0;
  // Start-up phase offsets (see stagger_start): four groups over a 12 us window, or half an
  // estimated tile time if that is shorter, once there are tiles enough to fill the chip.
  // The environment variable T3_STAGGER="groups,window_ns" overrides this ("0" turns it off).
  q.stagger_blocks = q.stagger_groups = q.stagger_ticks = 0;
  {
    int g = 4;
    double window_ns = 12000.0;
    const double tile_ns = 2.0 * *tm * *tn * (double)p->K / kCuFlopPerNs;
    if (window_ns > tile_ns / 2) window_ns = tile_ns / 2;
    if (T < resident) g = 0;
    const StaggerEnv &env = stagger_env();
    if (env.set) {
      g = env.off ? 0 : env.groups;
      if (!env.off) window_ns = env.window_ns;
    }
    if (g > 1 && window_ns >= 100.0) {
      q.stagger_groups = g;
      q.stagger_ticks = (int32_t)(window_ns / 10.0 / g);   // 100 MHz ticks between consecutive groups
      q.stagger_blocks = (int32_t)resident;
    }
  }
  // workgroups that will do work: the tiles below the limit and the release workgroups of the
  // forwarded chunks those tiles complete
  // chunks all of whose tiles lie in [begin, limit); the forwarded ones among them get released
  int64_t released = 0;
  for (int64_t s = 0; s + 1 < p->tp; ++s)
    if (s * tpc_t >= q.begin && (s + 1) * tpc_t <= q.limit && tpc_t > 0) ++released;
  // (paired tiles: the range is whole ring steps, tpc workgroup tiles each)
  const int64_t wg_tiles = pair_m > 1 ? (q.limit - q.begin) / tpc_t * tpc : q.limit - q.begin;
  q.expected_done = (int32_t)(wg_tiles + q.agents * released);
  // updates expected per element (Sec. 4.2.1): with two writers the launches of both count in
  // one bank, which closes when the tiles of both have been counted
  q.upd_first = q.upd_rest = 1;
  q.split_k = 1;
  if (two_writers) {
    q.split_k = split_k;                        // local updates per element = parts of K (Sec. 7.7)
    const bool step0 = (p->flags & T3_FLAG_STEP0_STORE_ONLY) != 0;
    q.upd_rest = split_k + 1;
    q.upd_first = split_k + (step0 ? 0 : 1);
    const int64_t up_begin = (step0 && q.begin < tpc) ? (tpc < q.limit ? tpc : q.limit) : q.begin;
    q.expected_done = (int32_t)((q.limit - q.begin) * split_k + (q.limit - up_begin));
  }
  // K walks start at a different slab on every XCD (see the kernels' `koff`)
  q.k_groups = dev.xcds > 1 ? dev.xcds : 0;
  q.total_blocks = (int32_t)(T + (int64_t)q.agents * (p->tp - 1));
  q.resident = (int32_t)resident;
  // Results leave the XCD's L2 at once (streaming hint) where that L2 is better spent on slabs
  // of A and B: long K loops, or an output that the memory-side cache cannot hold anyway.
  // Measured: -3 % on gpt3_fc2 and hightp_outproj, -1 % on wide_fc2, but +6 % on gpt3_outproj
  // (short K loop, output within the memory-side cache), so not there; and not when release
  // workgroups read R back.
  q.nt_out = (q.agents == 0 && !two_writers &&
              (p->K >= kNtMinK || 4ll * p->M * p->N > kMemorySideCacheBytes)) ? 1 : 0;
  q.timeline = g_timeline.load();
  {
    const int64_t wgs = g_timeline_wgs.load();
    q.timeline_wgs = (int32_t)(wgs > (1ll << 30) ? (1ll << 30) : wgs);
  }
  // Balanced tail (see the kernels' work_item): persistent launches of the tile kernel over the
  // whole issue order whose last round of grid positions would fill at most half the chip; every
  // half needs a few K-slabs, and the partial sums pass through the fp32 destination (so not
  // through bfloat16 forward slots), each element with one writer at a time.
  q.tail_r = q.tail_q = 0;
  q.tail_flags = nullptr;
  const bool persistent = (need & kMayPair) && q.agents == 0 && !two_writers;
  const bool bf16_direct = direct && (p->flags & T3_FLAG_FWD_BF16);
  const bool default_layouts = p->b_layout == T3_B_NK && p->a_layout == T3_A_MK;
  const bool tail_kernel = !(*tm == 128 && *tn == 256);   // (128 x 256 tiles that are not paired: none)
  if (persistent && !bf16_direct && default_layouts && tail_kernel && T > resident && q.begin == 0 &&
      q.limit == T_t && p->K / 64 >= kTailMinSlabs) {
    const int64_t r = T % resident;
    if (r > 0 && 2 * r <= resident && r <= t3k::kTailSlots) {
      q.tail_r = (int32_t)r;
      q.tail_q = (int32_t)(T / resident);
      if (track) q.tail_flags = tail_flags_in(track, p->tp);   // (t3_gemm brings its own)
    }
  }
  return T3_OK;
}

// Launches `kernel` and returns what THIS launch returned: an error some earlier call left in
// the runtime is not taken for ours.
template <typename... KArgs>
t3_status launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s, KArgs... a) {
  void *args[] = {static_cast<void *>(&a)...};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, args, 0, s);
  if (e != hipSuccess) {
    g_last_hip_error = (int32_t)e;
    return T3_ERR_HIP;
  }
  return T3_OK;
}

inline unsigned grid_size(const t3k::Plan &q) { return (unsigned)q.total_blocks; }

template <int MODE, int BKN, int AKM>
t3_status launch_gemm_layout(const t3k::Plan &q, int32_t tm, int32_t tn, hipStream_t s) {
  // Persistent workgroups: as many as the chip holds at once, each walking the grid positions.
  // With release work in the grid (default release mode) every position gets a workgroup of
  // its own instead: a release position may have to wait for its chunk, and a persistent
  // workgroup would sit on its later tiles meanwhile.
  const bool persistent = q.agents == 0;
  const int64_t positions = (int64_t)q.total_blocks * (MODE == t3k::kModeFused ? q.split_k : 1);
  const dim3 grid((unsigned)(persistent && positions > q.resident ? q.resident : positions));
  // A balanced tail (make_plan decides; operands in their default layouts only) takes the
  // kernels' TAIL variants.  The 256 x 256 one of the plain GEMM is cut from the fused kernel
  // (TAIL = 2).
  if constexpr (!BKN && !AKM) {
    if (q.tail_r) {
      if (tm == 256 && tn == 256) {
        if (MODE == t3k::kModeGemm) {
          t3k::Plan g = q;
          g.flags = 0;
          g.ldr = q.ldc;                  // (R already is the output pointer)
          return launch(t3k::gemm_tile_kernel<256, 256, 2, 2, 2, t3k::kModeFused, 0, 0, 2>, grid, dim3(256), s, g);
        }
        return launch(t3k::gemm_tile_kernel<256, 256, 2, 2, 2, t3k::kModeFused, 0, 0, 1>, grid, dim3(256), s, q);
      }
      if (tm == 256 && tn == 128)
        return launch(t3k::gemm_tile_kernel<256, 128, 4, 2, 3, MODE, 0, 0, 1>, grid, dim3(512), s, q);
      if (tm == 128 && tn == 128)
        return launch(t3k::gemm_tile_kernel<128, 128, 2, 2, 2, MODE, 0, 0, 1>, grid, dim3(256), s, q);
    }
  }
  // K-slabs of 64 everywhere.  256 x 256: 4 wavefronts of 128 x 128 (or 8 of 128 x 64), two 64-KiB stages; the
  // 256 x 128 and 128 x 256 tiles: 8 wavefronts of 64 x 64, three 48-KiB stages; one workgroup
  // per compute unit.  128 x 128: 4 wavefronts of 64 x 64, two 32-KiB stages, two workgroups.
  if (tm == 256 && tn == 256) {
    // B stored N x K: four wavefronts of 128 x 128 with the hand-ordered main loop, which adds the
    // incoming partial on the way out.  It has no two-writer epilogue and does not write
    // bfloat16 forward slots itself: those, and B stored K x N, take the eight-wavefront kernel.
    const bool eight = BKN || AKM || (MODE == t3k::kModeFused &&
                               ((q.flags & t3k::kFlagTwoWriters) ||
                                ((q.flags & t3k::kFlagFwdDirect) && (q.flags & t3k::kFlagFwdBf16))));
    if constexpr (!BKN && !AKM) {
      if (!eight) return launch(t3k::gemm_tile_kernel<256, 256, 2, 2, 2, MODE, 0>, grid, dim3(256), s, q);
    }
    return launch(t3k::gemm_tile_kernel<256, 256, 2, 4, 2, MODE, BKN, AKM>, grid, dim3(512), s, q);
  }
  if (tm == 256 && tn == 128)
    return launch(t3k::gemm_tile_kernel<256, 128, 4, 2, 3, MODE, BKN, AKM>, grid, dim3(512), s, q);
  if (tm == 128 && tn == 256)
    return launch(t3k::gemm_tile_kernel<128, 256, 2, 4, 3, MODE, BKN, AKM>, grid, dim3(512), s, q);
  return launch(t3k::gemm_tile_kernel<128, 128, 2, 2, 2, MODE, BKN, AKM>, grid, dim3(256), s, q);
}

template <int MODE>
t3_status launch_gemm(const t3k::Plan &q, int32_t tm, int32_t tn, bool b_kn, bool a_km, hipStream_t s) {
  if (a_km) return b_kn ? launch_gemm_layout<MODE, 1, 1>(q, tm, tn, s) : launch_gemm_layout<MODE, 0, 1>(q, tm, tn, s);
  return b_kn ? launch_gemm_layout<MODE, 1, 0>(q, tm, tn, s) : launch_gemm_layout<MODE, 0, 0>(q, tm, tn, s);
}

}  // namespace

extern "C" {

const char *t3_status_string(t3_status s) {
  switch (s) {
    case T3_OK: return "ok";
    case T3_ERR_NULL: return "null pointer";
    case T3_ERR_BAD_SHAPE: return "bad shape";
    case T3_ERR_BAD_TILE: return "unsupported tile shape";
    case T3_ERR_ALIGN: return "misaligned pointer or leading dimension";
    case T3_ERR_UNSUPPORTED: return "unsupported request";
    case T3_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int32_t t3_last_hip_error(void) { return g_last_hip_error; }

t3_status t3_chunk_order(int32_t tp, int32_t rank, int32_t *order, int32_t *own) {
  if (!order || !own) return T3_ERR_NULL;
  if (tp < 1 || rank < 0 || rank >= tp) return T3_ERR_BAD_SHAPE;
  for (int32_t s = 0; s < tp; ++s) order[s] = (rank + s) % tp;
  *own = (rank + tp - 1) % tp;
  return T3_OK;
}

t3_status t3_default_tile(const t3_problem *p, int32_t *tile_m, int32_t *tile_n) {
  if (!tile_m || !tile_n) return T3_ERR_NULL;
  const t3_status st = check_shape(p);
  if (st != T3_OK) return st;
  default_tile(p, kDefaultCus, tile_m, tile_n);
  return T3_OK;
}

t3_status t3_tiles_per_chunk(const t3_problem *p, int64_t *tpc) {
  if (!tpc) return T3_ERR_NULL;
  t3_status st = check_shape(p);
  if (st != T3_OK) return st;
  int32_t tm, tn;
  st = resolve_tile(p, &tm, &tn);
  if (st != T3_OK) return st;
  *tpc = ceil_div(p->M, tm) * ceil_div(p->N / p->tp, tn);
  return T3_OK;
}

t3_status t3_tile_of(const t3_problem *p, int64_t t, int32_t *s, int32_t *c, int32_t *mi,
                     int32_t *nj) {
  if (!s || !c || !mi || !nj) return T3_ERR_NULL;
  int64_t tpc;
  const t3_status st = t3_tiles_per_chunk(p, &tpc);
  if (st != T3_OK) return st;
  if (t < 0 || t >= tpc * p->tp) return T3_ERR_BAD_SHAPE;
  int32_t tm, tn;
  resolve_tile(p, &tm, &tn);
  const int64_t Mt = ceil_div(p->M, tm);
  const int64_t q = t % tpc;
  *s = (int32_t)(t / tpc);
  *c = (p->rank + *s) % p->tp;
  *mi = (int32_t)(q % Mt);
  *nj = (int32_t)(q / Mt);
  return T3_OK;
}

int64_t t3_track_words(int32_t tp) { return tp < 1 ? 0 : 2 * (3ll * tp + 2) + 2 + t3k::kTailSlots; }

t3_status t3_track_reset(int32_t tp, uint32_t *track, void *stream) {
  if (!track) return T3_ERR_NULL;
  if (tp < 1 || tp > (1 << 20)) return T3_ERR_BAD_SHAPE;
  return launch(t3k::track_reset_kernel, dim3(1), dim3(256), static_cast<hipStream_t>(stream), track,
                (int)tp);
}

t3_status t3_gemm_rs_fused(const t3_problem *p, const void *A, const void *B, float *R,
                           void *fwd, uint32_t *track, void *stream) {
  t3k::Plan q;
  int32_t tm, tn;
  bool empty = false;
  const t3_status st = make_plan(p, kNeedAB | kNeedR | kNeedFwd | kNeedTrack | kMayPair, A, B, nullptr, R,
                                 fwd, track, &q, &tm, &tn, &empty);
  if (st != T3_OK) return st;
  if (empty) return T3_OK;
  return launch_gemm<t3k::kModeFused>(q, tm, tn, p->b_layout == T3_B_KN, p->a_layout == T3_A_KM,
                                      static_cast<hipStream_t>(stream));
}

t3_status t3_gemm_rs_fused_static(const t3_problem *p, const void *A, const void *B, float *R,
                                  void *fwd, uint32_t *track_copy, void *stream) {
  if (!p) return T3_ERR_NULL;
  if (p->tp > kStaticMaxTp) return T3_ERR_UNSUPPORTED;   // the static tracker state holds no more
  if (p->flags & T3_FLAG_TWO_WRITERS) return T3_ERR_UNSUPPORTED;   // needs a tracker that outlives the call
  // validate everything first (a non-null stand-in for the tracker pointer: nothing reads it)
  t3k::Plan q;
  int32_t tm, tn;
  bool empty = false;
  uint32_t stand_in = 0;
  t3_status st = make_plan(p, kNeedAB | kNeedR | kNeedFwd | kNeedTrack | kMayPair, A, B, nullptr, R, fwd,
                           &stand_in, &q, &tm, &tn, &empty);
  if (st != T3_OK) return st;
  uint32_t *track = nullptr;
  st = static_track(&track);
  if (st != T3_OK) return st;
  q.track = track;
  if (q.tail_r) q.tail_flags = tail_flags_in(track, p->tp);
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the array keeps the last call's contents: every call starts from a cleared tracker
  st = launch(t3k::track_reset_kernel, dim3(1), dim3(256), s, track, (int)p->tp);
  if (st != T3_OK) return st;
  if (!empty) {
    st = launch_gemm<t3k::kModeFused>(q, tm, tn, p->b_layout == T3_B_KN, p->a_layout == T3_A_KM, s);
    if (st != T3_OK) return st;
  }
  if (track_copy)
    st = launch(t3k::track_copy_kernel, dim3(1), dim3(256), s, (const uint32_t *)track, track_copy,
                (int)t3_track_words(p->tp));
  return st;
}

t3_status t3_gemm(const t3_problem *p, const void *A, const void *B, float *C, void *stream) {
  // (flags and split_k are ignored: make_plan sees no tracker for this call)
  t3k::Plan q;
  int32_t tm, tn;
  bool empty = false;
  const t3_status st = make_plan(p, kNeedAB | kNeedC | kMayPair, A, B, C, nullptr, nullptr, nullptr, &q,
                                 &tm, &tn, &empty);
  if (st != T3_OK) return st;
  if (empty) return T3_OK;
  q.R = C;   // the GEMM kernel's output pointer, addressed with ldc
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool b_kn = p->b_layout == T3_B_KN, a_km = p->a_layout == T3_A_KM;
  auto go = [&](const t3k::Plan &plan) { return launch_gemm<t3k::kModeGemm>(plan, tm, tn, b_kn, a_km, s); };
  return q.tail_r ? launch_with_gemm_tail(q, s, go) : go(q);
}

t3_status t3_rs_reduce(const t3_problem *p, const float *C, float *R, void *fwd,
                       uint32_t *track, void *stream) {
  t3k::Plan q;
  int32_t tm, tn;
  bool empty = false;
  const t3_status st = make_plan(p, kNeedC | kNeedR | kNeedFwd | kNeedTrack, nullptr, nullptr, C,
                                 R, fwd, track, &q, &tm, &tn, &empty);
  if (st != T3_OK) return st;
  if (empty) return T3_OK;
  const dim3 grid(grid_size(q)), block(t3k::kThreads);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (tm == 256 && tn == 256)
    return launch(t3k::reduce_tile_kernel<256, 256>, grid, block, s, q);
  else if (tm == 256 && tn == 128)
    return launch(t3k::reduce_tile_kernel<256, 128>, grid, block, s, q);
  else if (tm == 128 && tn == 256)
    return launch(t3k::reduce_tile_kernel<128, 256>, grid, block, s, q);
  return launch(t3k::reduce_tile_kernel<128, 128>, grid, block, s, q);
}

t3_status t3_upstream_update(const t3_problem *p, const float *incoming, float *R,
                             uint32_t *track, void *stream) {
  t3k::Plan q;
  int32_t tm, tn;
  bool empty = false;
  const t3_status st = make_plan(p, kNeedC | kNeedR | kNeedTrack | kNeedTwoWriters, nullptr, nullptr,
                                 incoming, R, nullptr, track, &q, &tm, &tn, &empty);
  if (st != T3_OK) return st;
  if (empty) return T3_OK;
  unsigned blocks = grid_size(q);
  if (p->upstream_agents > 0 && (unsigned)p->upstream_agents < blocks)
    blocks = (unsigned)p->upstream_agents;     // the rest of the positions are walked in a loop
  const dim3 grid(blocks), block(t3k::kThreads);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (tm == 256 && tn == 256)
    return launch(t3k::upstream_update_kernel<256, 256>, grid, block, s, q);
  else if (tm == 256 && tn == 128)
    return launch(t3k::upstream_update_kernel<256, 128>, grid, block, s, q);
  else if (tm == 128 && tn == 256)
    return launch(t3k::upstream_update_kernel<128, 256>, grid, block, s, q);
  return launch(t3k::upstream_update_kernel<128, 128>, grid, block, s, q);
}

t3_status t3_release_chunks(const t3_problem *p, const float *R, void *fwd,
                            const uint32_t *track, void *stream) {
  t3k::Plan q;
  int32_t tm, tn;
  bool empty = false;
  const t3_status st = make_plan(p, kNeedR | kNeedFwd | kNeedTrack | kNeedTwoWriters, nullptr,
                                 nullptr, nullptr, const_cast<float *>(R), fwd,
                                 const_cast<uint32_t *>(track), &q, &tm, &tn, &empty);
  if (st != T3_OK) return st;
  if (p->tp < 2 || p->M == 0 || p->N == 0) return T3_OK;
  q.agents = T3_AGENTS;
  q.rows_per_agent = (int32_t)ceil_div(p->M, q.agents);
  return launch(t3k::release_ready_kernel, dim3((unsigned)(q.agents * (p->tp - 1))),
                dim3(t3k::kThreads), static_cast<hipStream_t>(stream), q);
}

t3_status t3_timeline(uint64_t *stamps, int64_t words) {
  if (stamps && words < 0) return T3_ERR_BAD_SHAPE;
  if (stamps && (reinterpret_cast<uintptr_t>(stamps) & 7u)) return T3_ERR_ALIGN;
  // (the count first when switching off, the pointer first when switching on: a launch planned
  // in between records nothing rather than out of bounds)
  if (!stamps) {
    g_timeline.store(nullptr);
    g_timeline_wgs.store(0);
    return T3_OK;
  }
  g_timeline_wgs.store(0);
  g_timeline.store(stamps);
  g_timeline_wgs.store(words / (4 * T3_TIMELINE_ITEMS));
  return T3_OK;
}

t3_status t3_ag_step(const t3_problem *p, int32_t step, const float *upstream_R, int64_t ld_up,
                     float *R, void *stream) {
  const t3_status st = check_shape(p);
  if (st != T3_OK) return st;
  if (step < 0 || step >= p->tp - 1) return T3_ERR_BAD_SHAPE;
  if (!upstream_R || !R) return T3_ERR_NULL;
  const int64_t W = p->N / p->tp;
  if (p->ldr < p->N || ld_up < p->N) return T3_ERR_BAD_SHAPE;
  if (p->ldr % 4 || ld_up % 4 || W % 4 || !aligned16(R) || !aligned16(upstream_R)) return T3_ERR_ALIGN;
  if (p->M == 0 || W == 0) return T3_OK;
  const int64_t c = (p->rank + step) % p->tp;    // what the upstream neighbour owned, or got a step ago
  const unsigned rows_per_block = t3k::kThreads / 64;
  const unsigned blocks = (unsigned)(ceil_div(p->M, rows_per_block) < 4096 ? ceil_div(p->M, rows_per_block) : 4096);
  return launch(t3k::ag_copy_kernel, dim3(blocks), dim3(t3k::kThreads), static_cast<hipStream_t>(stream),
                upstream_R + c * W, ld_up, R + c * W, (int64_t)p->ldr, (int32_t)p->M, (int32_t)W);
}

}  // extern "C"
