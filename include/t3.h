/*
 * t3.h -- C ABI of the MI355X (gfx950) implementation of one tensor-parallel rank's
 * fused "sliced producer GEMM + ring reduce-scatter reduction + track & trigger" path
 * of T3 (arXiv 2401.16677).
 *
 * The problem, in the paper's terms: rank `rank` of a `tp`-way tensor-parallel group
 * holds a K-slice of a row-parallel layer (output projection or FC-2, Sec. 2.4) and
 * produces a full-size M x N *partial* output C = A.B.  The ring reduce-scatter that
 * follows cuts the output into `tp` column chunks of width W = N/tp (Sec. 2.3); a rank
 * produces the chunks in the staggered ring order order[s] = (rank + s) mod tp
 * (Sec. 4.1, Sec. 4.4), adds each to the partial received from its upstream
 * neighbour, hands every chunk but the last on to its downstream neighbour once all
 * of the chunk's updates have landed (the tracker and DMA trigger of Sec. 4.2), and
 * keeps the last one, own = (rank - 1) mod tp, fully reduced.
 *
 * On one GPU the upstream data is a caller-seeded "incoming" buffer R and the
 * downstream neighbour's memory is a forward buffer `fwd`.
 *
 * Conventions for every entry point
 *  - Pointers named A, B, C, R, fwd, track are DEVICE pointers owned by the caller.
 *    The library allocates and frees no device memory.  What it keeps: the compute-unit and XCD
 *    counts of each device it has launched on and T3_STAGGER (read-only after first use); two
 *    small arrays inside its own code object per device (the tracker state of
 *    t3_gemm_rs_fused_static; flag words for t3_gemm's balanced tail, with one HIP event per
 *    set of flags, created at first use); and the pointer given to t3_timeline.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *    asynchronous on that stream and never synchronise it.
 *  - Arguments are validated on the host before anything is enqueued; on any status
 *    other than T3_OK nothing was launched and no buffer was touched.
 *  - A and B are read only.  Buffers must not overlap each other.
 */
#ifndef T3_H
#define T3_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  T3_OK = 0,
  T3_ERR_NULL = 1,        /* a required pointer is NULL                                   */
  T3_ERR_BAD_SHAPE = 2,   /* M,N,K < 0; tp < 1; rank outside [0,tp); N % tp != 0; ld < width */
  T3_ERR_BAD_TILE = 3,    /* (tile_m, tile_n) is not one of the supported tile shapes     */
  T3_ERR_ALIGN = 4,       /* pointer, leading dimension or width breaks an alignment rule */
  T3_ERR_UNSUPPORTED = 5, /* valid request this build does not implement                  */
  T3_ERR_HIP = 6          /* the HIP runtime refused the launch; see t3_last_hip_error()  */
} t3_status;

typedef enum {
  T3_B_NK = 0, /* B stored N x K, K contiguous: element (k,n) at B[n*ldb + k] (forward-pass weight) */
  T3_B_KN = 1  /* B stored K x N, N contiguous: element (k,n) at B[k*ldb + n] (the non-transposed
                  operand of the backward-pass GEMMs, Sec. 5.2).  K must then be a multiple of 64
                  (T3_ERR_UNSUPPORTED otherwise) and N/tp a multiple of 8 (T3_ERR_ALIGN)            */
} t3_b_layout;

typedef enum {
  T3_A_MK = 0, /* A stored M x K, K contiguous: element (m,k) at A[m*lda + k]                        */
  T3_A_KM = 1  /* A stored K x M, M contiguous: element (m,k) at A[k*lda + m] (the transposed operand
                  of the backward-pass GEMMs, Sec. 5.2).  K must then be a multiple of 64
                  (T3_ERR_UNSUPPORTED otherwise) and M a multiple of 8 (T3_ERR_ALIGN)               */
} t3_a_layout;

/* flags */
#define T3_FLAG_STEP0_STORE_ONLY 1u /* the first chunk produced (order[0]) has no upstream data yet:
                                       it is stored, not added to R (Sec. 4.1, Sec. 4.4)             */
#define T3_FLAG_FWD_DIRECT 2u       /* sums of forwarded chunks are written straight into their
                                       forward slot (the remote-mapped store of Sec. 4.4, the
                                       direct reduce-scatter of Sec. 7.1); R keeps the incoming
                                       data there                                                    */

#define T3_FLAG_TWO_WRITERS 4u      /* the rank's buffer R receives TWO updates per element, as in the
                                       paper's ring reduce-scatter (Sec. 4.1, Sec. 4.2.1): the local
                                       GEMM's tile (t3_gemm_rs_fused) and the upstream neighbour's
                                       update (t3_upstream_update), each an atomic add (the
                                       op-and-store of Sec. 4.3) into R, in either order or at the
                                       same time; a chunk is ready after both.  With
                                       T3_FLAG_STEP0_STORE_ONLY chunk order[0] has no upstream update.
                                       Not combinable with T3_FLAG_FWD_DIRECT.                        */

#define T3_FLAG_FWD_BF16 8u         /* the forward slots hold bfloat16 instead of fp32: what is sent
                                       on is the fp32 sum rounded to nearest even, the 16-bit format
                                       activations travel in under mixed precision (Sec. 5.2).  With
                                       any release mode; R and the owned chunk stay fp32.  N/tp must
                                       be a multiple of 8 (T3_ERR_ALIGN)                             */

typedef struct {
  int32_t M, N, K;        /* tokens, hidden size, slice width of this rank                           */
  int32_t tp, rank;       /* ring size and this rank's position                                      */
  int32_t tile_m, tile_n; /* output tile = tracker granularity; 0,0 = t3_default_tile()              */
  int32_t b_layout;       /* t3_b_layout                                                             */
  int64_t lda, ldb;       /* leading dimensions of A (>= K for MK, >= M for KM) and B (>= K for NK,
                             >= N for KN), in bf16 elements, multiples of 8                          */
  int64_t ldr;            /* leading dimension of R (>= N), in floats, multiple of 4                 */
  int64_t ldc;            /* leading dimension of C (>= N) for t3_gemm / t3_rs_reduce, multiple of 4 */
  int64_t tile_limit;     /* < 0: run every tile.  Otherwise only tiles whose issue index is below
                             tile_limit run (a deterministic prefix of the issue order; debugging
                             and tests)                                                              */
  uint32_t flags;         /* T3_FLAG_*                                                               */
  int64_t tile_begin;     /* tiles whose issue index is below tile_begin do not run either: with
                             tile_limit, [tile_begin, tile_limit) is a range of the issue order,
                             e.g. one ring step s = [s*tpc, (s+1)*tpc) (Sec. 4.1).  0 = from the start  */
  int32_t split_k;        /* 0 or 1: one workgroup per tile.  S > 1 (two-writer mode only, S <= K/64,
                             S <= 64): S workgroups share a tile, each multiplying a part of K and
                             adding it into R, so the local GEMM makes S updates per element and
                             a chunk's threshold is (S + 1) * tpc (Sec. 7.7)                        */
  int32_t upstream_agents; /* t3_upstream_update only.  0: one workgroup per tile.  n > 0: at most n
                             workgroups walk the tiles in issue order, which caps the memory
                             traffic the upstream writer has in flight beside the GEMM: the
                             software stand-in for the arbitration policy of Sec. 4.5, which holds
                             communication accesses back while the producer is memory-bound.
                             < 0 is T3_ERR_BAD_SHAPE                                                */
  int32_t a_layout;       /* t3_a_layout; with T3_A_KM lda >= M                                      */
  int32_t reserved;       /* must be 0                                                               */
} t3_problem;

/*
 * Tiles and issue order.  A chunk is cut into Mt = ceil(M/tile_m) by Wt = ceil(W/tile_n)
 * tiles (tiles never straddle a chunk; the last row/column of tiles may be ragged),
 * tpc = Mt*Wt tiles per chunk, T = tp*tpc tiles in all.  Issue index t in [0,T) names
 * stage s = t / tpc (the GEMM "stage" of Sec. 2.5, one per ring step), chunk
 * c = order[s], and inside the chunk q = t % tpc, tile row mi = q % Mt, tile column
 * nj = q / Mt.  Workgroups are launched in issue order up to a permutation inside a
 * stage that groups tiles sharing operands on one XCD.
 *
 * Supported (tile_m, tile_n): (256,256), (256,128), (128,256), (128,128).
 *
 * Size limits (T3_ERR_UNSUPPORTED beyond them): A and B below 2^31 elements each, leading
 * dimension included (M*lda or K*lda, N*ldb or K*ldb);
 * M*ldr*4 and M*ldc*4 below 2^32 bytes (the kernels address R, C and a forward slot with
 * 32-bit byte offsets from a uniform base); fewer than 2^31 tiles.
 *
 * Launch shape.  In the direct release mode and for t3_gemm the tile kernel runs persistent
 * workgroups (as many as the device holds at once) that walk the grid positions in issue
 * order.  The first wave of workgroups starts in a few phase groups a few microseconds
 * apart, so that the compute units do not all reach their reduction traffic at the same
 * moment; the environment variable T3_STAGGER="groups,window_ns" (read once, at the first
 * launch of the process) overrides the default (4 groups over 12 us), T3_STAGGER=0 turns it
 * off.  Results do not depend on it.  The number of persistent workgroups follows the
 * device's compute-unit count; the XCD grouping is applied on devices with 8 XCDs.
 * Balanced tail: when the tiles of such a launch do not fill a whole number of rounds of the
 * persistent workgroups and the last round would occupy at most half of them, each tile of
 * that round is computed as two halves of K by two workgroups, the first at the start of the
 * launch and the second at its end, the partial sums passing through the place the result
 * goes to (R, C or the fp32 forward slot); the tile is counted when the second half has
 * stored it.  Tiles and counters are the same as without it, and so are the results up to
 * the order in which the K-slabs are added in fp32 (the partial sums are stored and reloaded
 * as they are; the order differs between workgroups anyway).  It applies to whole-problem
 * launches (no tile range) with A and B in their default layouts and K >= 512, not to
 * bfloat16 forward slots written directly, and for t3_gemm not while its stream is being
 * captured into a graph.
 *
 * Tracker state (Sec. 4.2): one caller-owned device array of t3_track_words(tp) uint32
 * words, cleared once by t3_track_reset().  It holds two banks of 3*tp + 2 words
 *   [0, tp)        counter[c]  tiles of chunk c that have landed
 *   [tp, 2tp)      ready[c]    1 once counter[c] == tpc
 *   [2tp, 3tp)     queue[i]    chunk ids in trigger order (forwarded chunks only, so at
 *                              most tp-1 entries are used); 0xFFFFFFFF = empty
 *   [3tp]          queue_len
 *   [3tp+1]        done        workgroups of the launch that have finished
 * followed by two global words
 *   [6tp+4]        gen         launches completed since the reset
 *   [6tp+5]        error       0, or 1 if a release workgroup gave up waiting for a chunk
 *                              (cannot happen in a launch that ran to completion)
 * and by 256 words the kernels use between the two halves of a split tile (balanced tail,
 * above); they are 0 whenever no launch is running.
 * A launch of t3_gemm_rs_fused / t3_rs_reduce works in bank gen & 1; its last workgroup
 * clears the other bank and increments gen.  So consecutive launches need no reset in
 * between, and after a launch has completed its results are in bank (gen - 1) & 1.  A
 * launch that executes no tile (empty problem, empty tile range) leaves the state untouched.
 * With a tile range, counters count the tiles of the range, and a chunk becomes ready (and
 * is released) only if all of its tiles lie in the range.
 * Counter, ready and queue-as-a-set are deterministic; the order of queue entries follows
 * the order in which chunks actually completed on the device.
 * Publication: ready[c] is THE flag.  A tile's results are written with device-scope
 * write-through stores and are acknowledged before the tile is counted; the count that
 * completes a chunk writes its queue entry and then sets ready[c] with a device-scope release
 * store.  A consumer on the same device that observes ready[c] == 1 with an acquiring load may
 * read chunk c and will find c in the queue.  queue_len by itself publishes nothing: it is
 * reserved before the entry is written and may run ahead of it.  (This is the ordering gfx950
 * gives agent-scope stores and atomics; it is not promised to other devices or to the host
 * before the launch has completed.)
 * A release workgroup that gives up waiting (see `error`) leaves its slot unfilled although
 * the call returned T3_OK: callers that use the default release mode check `error` (it stays 0
 * in any launch that runs to completion).
 */

/* Ring order of `rank` and the chunk it keeps: order[s] = (rank + s) mod tp is the chunk produced
   at ring step s (the staggered stage order of Sec. 4.4: GPU-0 runs stage 1 while GPU-1 runs stage
   2), own = (rank - 1) mod tp the one produced last and kept (Sec. 4.1, Sec. 4.4).
   Host pointers: order[tp], own[1].  T3_ERR_BAD_SHAPE unless 0 <= rank < tp. */
t3_status t3_chunk_order(int32_t tp, int32_t rank, int32_t *order, int32_t *own);

/* Tile shape the library would pick for this shape: the tracked region of Sec. 4.2.1 (there a
   wavefront's tile, here a workgroup's), chosen among the supported shapes for least padded
   work, fastest main loop and a full device (an MI355X's 256 compute units).  Host pointers. */
t3_status t3_default_tile(const t3_problem *p, int32_t *tile_m, int32_t *tile_n);

/* Tiles per chunk for the problem's (or the default) tile shape.  Host pointer. */
t3_status t3_tiles_per_chunk(const t3_problem *p, int64_t *tpc);

/* Issue index -> stage, chunk, tile row, tile column (host pointers).  T3_ERR_BAD_SHAPE
   if t is outside [0, T). */
t3_status t3_tile_of(const t3_problem *p, int64_t t, int32_t *s, int32_t *c, int32_t *mi,
                     int32_t *nj);

/* Number of uint32 words of tracker state for a ring of size tp (0 if tp < 1). */
int64_t t3_track_words(int32_t tp);

/* Clears the tracker state (a small fill kernel on `stream`): the set-up of the tracker's
   entries before a producer kernel runs (Sec. 4.2.1, Sec. 4.4).  Needed once before the first
   launch that uses `track`, not between launches.  track: device.  T3_ERR_BAD_SHAPE unless
   1 <= tp <= 2^20. */
t3_status t3_track_reset(int32_t tp, uint32_t *track, void *stream);

/*
 * The fused path (Sec. 4.1): C = A.B is produced tile by tile in issue order and never
 * stored on its own; each tile's epilogue forms incoming + C from R (Sec. 4.3's
 * op-and-store, done by the compute units), then bumps the chunk's counter; the tile
 * that completes a chunk marks it ready and, for forwarded chunks, appends it to the
 * trigger queue, which releases the chunk into its forward slot (Sec. 4.2.2).
 *
 *   A    bf16, see a_layout read
 *   B    bf16, see b_layout read
 *   R    fp32 [M][ldr]      in: incoming partials.  out: incoming + C on every executed
 *                           tile; with T3_FLAG_FWD_DIRECT only the own chunk is updated
 *   fwd  fp32 [tp-1][M][W]  out, dense: slot s holds chunk order[s] = incoming + C.
 *                           Default: a slot is filled once its chunk is complete (copied
 *                           from R by release workgroups of the same launch, which wait on
 *                           the chunk's ready flag) and left untouched otherwise.  T3_FLAG_FWD_DIRECT: executed tiles
 *                           are written as they finish.  May be NULL if tp == 1.
 *                           With T3_FLAG_FWD_BF16 (here and in t3_rs_reduce / t3_release_chunks)
 *                           the same array holds bfloat16: [tp-1][M][W] of 2 bytes.
 *   track                   tracker state (reset once; launches sharing it must be ordered
 *                           on one stream)
 * fp32 accumulation order is unspecified; integer outputs are exact.
 */
t3_status t3_gemm_rs_fused(const t3_problem *p, const void *A, const void *B, float *R,
                           void *fwd, uint32_t *track, void *stream);

/*
 * t3_gemm_rs_fused for callers that cannot allocate device memory at all -- code under HIP
 * graph capture, tight serving loops, harnesses that forbid it -- and so cannot supply the
 * tracker state either: the same kernels, the same results in R and fwd, with the tracker
 * state (the counters, flags and queue the kernels work in) held in a fixed array inside the
 * library instead of a caller's.  The call allocates and frees nothing.
 *
 *   A, B, R, fwd, stream    as for t3_gemm_rs_fused
 *   track_copy              NULL, or device memory of t3_track_words(tp) words that receives a
 *                           copy of the tracker state as the launch left it (same layout:
 *                           results in bank (gen - 1) & 1, gen == 1 after a launch that ran tiles)
 *
 * Limits: tp <= T3_STATIC_MAX_TP (T3_ERR_UNSUPPORTED beyond it); the array takes
 * t3_track_words(T3_STATIC_MAX_TP) words (under 3 KiB) on every device the library has run
 * on, until the process ends.  Every call clears it first (a small fill kernel on `stream`)
 * and all calls on one device share it: calls that overlap on one device -- different
 * streams, or graph replays in flight together -- race on it and must be serialised by the
 * caller.  Two-writer mode needs a caller's tracker (its second call must find the first
 * call's counts) and is refused here with T3_ERR_UNSUPPORTED.
 */
#define T3_STATIC_MAX_TP 64
t3_status t3_gemm_rs_fused_static(const t3_problem *p, const void *A, const void *B, float *R,
                                  void *fwd, uint32_t *track_copy, void *stream);

/* Unfused baseline, step 1: the plain sliced GEMM (Sec. 2.4).  C fp32 [M][ldc] out.
   tp/rank/tile_limit order the tiles exactly as in the fused call; flags are ignored. */
t3_status t3_gemm(const t3_problem *p, const void *A, const void *B, float *C, void *stream);

/* Unfused baseline, step 2: the reduce-scatter's reduction kernel (Sec. 2.3, the
   baseline of Sec. 4.3): reads C and R, writes what t3_gemm_rs_fused would have
   written to R / fwd, and drives the same tracker, tile by tile in the same order. */
t3_status t3_rs_reduce(const t3_problem *p, const float *C, float *R, void *fwd,
                       uint32_t *track, void *stream);

/*
 * Two-writer mode (T3_FLAG_TWO_WRITERS in p->flags for all three calls below).
 *
 *   R     fp32 [M][ldr]   in: what has been accumulated so far (zero before the first update of
 *                         a reduction).  out: + C on the tiles t3_gemm_rs_fused ran, + incoming
 *                         on the tiles t3_upstream_update ran.
 *
 * t3_gemm_rs_fused adds its tiles into R and counts them; it releases nothing (fwd is ignored and
 * may be NULL).  t3_upstream_update stands in for the upstream neighbour's DMA updates: it adds
 * `incoming` (fp32 [M][ldc]) into R tile by tile in the same issue order and counts every tile in
 * the same tracker; with T3_FLAG_STEP0_STORE_ONLY it skips chunk order[0].  The two calls must
 * use the same problem (tile range included) and tracker state and may run on different streams
 * at the same time; both must be enqueued after whatever used the tracker before has completed,
 * and BOTH must be made: the tracker closes its bank when the tiles of both have been counted.
 * A chunk's threshold is 2 * tpc (tpc for chunk order[0] under T3_FLAG_STEP0_STORE_ONLY).
 *
 * t3_release_chunks is the triggered transfer (Sec. 4.2.2) as a call of its own: ordered after
 * both updates, it copies every forwarded chunk whose ready flag the last completed launch left
 * set from R into its forward slot.  It changes no tracker state.
 */
t3_status t3_upstream_update(const t3_problem *p, const float *incoming, float *R,
                             uint32_t *track, void *stream);
t3_status t3_release_chunks(const t3_problem *p, const float *R, void *fwd,
                            const uint32_t *track, void *stream);

/*
 * One step of the ring all-gather that follows the reduce-scatter (Sec. 2.3: N-1 steps without
 * reductions until every device has all the reduced chunks; the "Sequential" all-gather of
 * Sec. 5.3).  Same ring as the reduce-scatter (Sec. 4.1): at step g = 0 .. tp-2 rank `rank`
 * takes chunk (rank + g) mod tp -- at step 0 the chunk its upstream neighbour rank+1 owns, later
 * what that neighbour took a step earlier -- unchanged, from the neighbour's buffer into the
 * same columns of its own.  After tp-1 steps R holds all tp reduced chunks.
 *
 *   upstream_R  fp32 [M][ld_up]  read: the upstream neighbour's buffer (on several GPUs: the
 *                                peer's memory; here the caller's stand-in), ld_up >= N
 *   R           fp32 [M][ldr]    columns [c W, (c+1) W) are overwritten, the rest is untouched
 *
 * T3_ERR_BAD_SHAPE if step is outside [0, tp-1); leading dimensions and W multiples of 4,
 * pointers 16-byte aligned (T3_ERR_ALIGN).  Tile shape, flags and tracker play no part.
 */
t3_status t3_ag_step(const t3_problem *p, int32_t step, const float *upstream_R, int64_t ld_up,
                     float *R, void *stream);

/*
 * Where a launch's time goes (a measuring aid for Sec. 4.1's overlap: how much of a tile's time
 * is reduction traffic and how much is matrix work).  While `stamps` is set, every launch of
 * the tile kernel (t3_gemm_rs_fused, t3_gemm_rs_fused_static, t3_gemm), from any thread,
 * records for workgroup w and its i-th piece of work (a tile, or half of one in a balanced
 * tail), i < T3_TIMELINE_ITEMS, four readings of the device's 100 MHz wall clock at
 * stamps[(w * T3_TIMELINE_ITEMS + i) * 4 + 0 .. 3]:
 *   0  the piece was taken
 *   1  the accumulators are set up: the incoming partial has arrived and is in place
 *   2  the main loop (and a ragged end of K) is done
 *   3  the results have been handed to the memory system (they are acknowledged later, while
 *      the next piece starts) and the next tile's incoming partial has been requested
 * Workgroups w >= words / (4 * T3_TIMELINE_ITEMS) record nothing, nor do the kernels that serve
 * 256 x 256 tiles with B stored K x N, A stored K x M, two writers or bfloat16 slots written
 * directly.  Entries a launch does not
 * write keep what they held.  stamps: device memory, 8-byte aligned, that stays valid until
 * the launches that were issued while it was set have finished; NULL switches recording off.
 * Later launches overwrite earlier ones.
 */
#define T3_TIMELINE_ITEMS 16
t3_status t3_timeline(uint64_t *stamps, int64_t words);

const char *t3_status_string(t3_status s);

/* hipError_t of the last T3_ERR_HIP on the calling thread (0 if none). */
int32_t t3_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* T3_H */
