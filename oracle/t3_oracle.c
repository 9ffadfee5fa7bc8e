/*
 * CPU oracle for one tensor-parallel rank's fused "sliced GEMM + ring
 * reduce-scatter reduction + track & trigger" path of T3 (arXiv 2401.16677).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, by-the-definition
 * implementation used only to check the GPU library and to be timed as a CPU
 * baseline.  It shares no code, header, table or helper with the HIP path and
 * must never be reached from the product path.
 *
 * Everything is written from the paper's prose:
 *   - sliced producer GEMM: each rank multiplies its K-slice and produces a
 *     full-size partial output (Sec. 2.4, Sec. 2.5);
 *   - ring reduce-scatter: the output is chunked P ways, a rank adds its local
 *     copy of a chunk to the copy received from upstream and forwards the sum;
 *     after P-1 steps it holds one fully reduced chunk (Sec. 2.3);
 *   - staggered chunk order across ranks and the "first chunk goes out, middle
 *     chunks are forwarded later, last chunk stays" map (Sec. 4.1, Sec. 4.4);
 *   - tracker: count updates per tracked region against a threshold, the write
 *     that reaches the threshold triggers the transfer; a per-transfer counter
 *     when a transfer block spans several tracked regions (Sec. 4.2.1, 4.2.2);
 *     the threshold scales with the updates expected per element, 2 where the
 *     upstream neighbour's update lands in the same memory (Sec. 4.2.1).
 *
 * Numerics: bf16 inputs are widened exactly, products are exact in fp64, sums
 * are accumulated in fp64 in ascending k, and the reduced value is rounded to
 * fp32 once.
 *
 * Parity pins (tests/test_oracle_pins.py): exact rational brute force on tiny
 * shapes, integer-exact cases, a library fp64 matmul, the zero-incoming /
 * slice-sum / linearity invariants, closure of the emulated P-rank ring onto
 * the unsliced GEMM, the paper's 4-GPU example map, and counter closed forms.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define T3O_OK 0
#define T3O_BAD_ARG 1
#define T3O_NOMEM 2

/* bf16 is the upper half of an IEEE binary32: widening is exact. */
static inline float widen_bf16(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

int t3o_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Ring order (Sec. 4.1 and the stagger of Sec. 4.4): data flows from rank
 * r+1 to r to r-1; rank r produces chunk r first, then r+1, ... so that the
 * chunk arriving from r+1 is the one being produced.  The chunk produced last
 * is never forwarded: it is the one the rank ends up owning.
 */
int t3o_chunk_order(int32_t P, int32_t r, int32_t *order, int32_t *own)
{
    if (P <= 0 || r < 0 || r >= P || !order || !own)
        return T3O_BAD_ARG;
    for (int32_t s = 0; s < P; ++s)
        order[s] = (r + s) % P;
    *own = order[P - 1];
    return T3O_OK;
}

/*
 * Sliced GEMM, selected rows (Sec. 2.4):  C[rows[i]][n] = sum_k A[m][k] * B[k][n].
 * A is M x K row-major (leading dimension lda, in elements).
 * B holds the K x N operand either as N x K with K contiguous (b_kn == 0,
 * element (k,n) at B[n*ldb + k]) or as K x N with N contiguous (b_kn == 1,
 * element (k,n) at B[k*ldb + n]).
 * rows == NULL means rows 0..nrows-1.  C is nrows x N, dense, fp64.
 */
int t3o_gemm_rows(int32_t M, int32_t N, int32_t K,
                  const uint16_t *A, int64_t lda,
                  const uint16_t *B, int64_t ldb, int32_t b_kn,
                  const int32_t *rows, int32_t nrows, double *C)
{
    if (M < 0 || N < 0 || K < 0 || nrows < 0 || (nrows && !C))
        return T3O_BAD_ARG;
    if ((M && K && !A) || (N && K && !B))
        return T3O_BAD_ARG;
    if (rows) {
        for (int32_t i = 0; i < nrows; ++i)
            if (rows[i] < 0 || rows[i] >= M)
                return T3O_BAD_ARG;
    } else if (nrows > M) {
        return T3O_BAD_ARG;
    }
    if (nrows == 0 || N == 0)
        return T3O_OK;

    /* b[k][n] widened once so the inner loop walks n contiguously */
    float *b = NULL;
    if (K > 0) {
        b = (float *)malloc((size_t)K * (size_t)N * sizeof(float));
        if (!b)
            return T3O_NOMEM;
#pragma omp parallel for schedule(static)
        for (int32_t k = 0; k < K; ++k)
            for (int32_t n = 0; n < N; ++n)
                b[(size_t)k * N + n] =
                    widen_bf16(b_kn ? B[(int64_t)k * ldb + n] : B[(int64_t)n * ldb + k]);
    }

#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < nrows; ++i) {
        const int32_t m = rows ? rows[i] : i;
        double *c = C + (size_t)i * N;
        for (int32_t n = 0; n < N; ++n)
            c[n] = 0.0;
        for (int32_t k = 0; k < K; ++k) {
            const double a = (double)widen_bf16(A[(int64_t)m * lda + k]);
            const float *bk = b + (size_t)k * N;
            for (int32_t n = 0; n < N; ++n)
                c[n] += a * (double)bk[n];
        }
    }
    free(b);
    return T3O_OK;
}

/*
 * Reduction of the local partial with the received partial (Sec. 2.3):
 * S = fl32( incoming + C ), the sum formed in fp64 and rounded once.
 * If skip_chunk >= 0, columns of that chunk (width N/P) take no incoming
 * contribution: the first chunk a rank produces has no upstream data yet and
 * is a pure store (Sec. 4.1, Sec. 4.4).
 * C is nrows x N dense; incoming/S rows are addressed through rows[] (or
 * 0..nrows-1) with their leading dimensions.
 */
int t3o_reduce_rows(int32_t N, int32_t P, int32_t skip_chunk,
                    const double *C, const float *incoming, int64_t ldi,
                    const int32_t *rows, int32_t nrows, float *S, int64_t lds)
{
    if (N < 0 || nrows < 0 || P <= 0 || N % P != 0 || skip_chunk >= P)
        return T3O_BAD_ARG;
    if (nrows && N && (!C || !incoming || !S))
        return T3O_BAD_ARG;
    const int32_t W = N / P;
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < nrows; ++i) {
        const int64_t m = rows ? rows[i] : i;
        for (int32_t n = 0; n < N; ++n) {
            const int drop = (skip_chunk >= 0 && n / W == skip_chunk);
            const double inc = drop ? 0.0 : (double)incoming[m * ldi + n];
            S[(int64_t)i * lds + n] = (float)(inc + C[(size_t)i * N + n]);
        }
    }
    return T3O_OK;
}

/*
 * Tile grid and issue order.  The output is cut into tile_m x tile_n tiles
 * that never straddle a chunk: per chunk Mt = ceil(M/tile_m) by
 * Wt = ceil(W/tile_n) tiles, tpc = Mt*Wt.  Issue index t walks the chunks in
 * ring order (stage s = t / tpc produces chunk order[s], Sec. 2.5 / Sec. 4.1)
 * and, inside a chunk, down the rows first: q = t % tpc, mi = q % Mt,
 * nj = q / Mt.
 */
int t3o_tile_of(int32_t M, int32_t N, int32_t P, int32_t r,
                int32_t tile_m, int32_t tile_n, int64_t t,
                int32_t *s, int32_t *c, int32_t *mi, int32_t *nj)
{
    if (M <= 0 || N <= 0 || P <= 0 || r < 0 || r >= P || N % P != 0 ||
        tile_m <= 0 || tile_n <= 0)
        return T3O_BAD_ARG;
    const int32_t W = N / P;
    const int64_t Mt = (M + tile_m - 1) / tile_m;
    const int64_t Wt = (W + tile_n - 1) / tile_n;
    const int64_t tpc = Mt * Wt;
    if (t < 0 || t >= tpc * P)
        return T3O_BAD_ARG;
    const int32_t stage = (int32_t)(t / tpc);
    const int64_t q = t % tpc;
    *s = stage;
    *c = (r + stage) % P;
    *mi = (int32_t)(q % Mt);
    *nj = (int32_t)(q / Mt);
    return T3O_OK;
}

/*
 * Track & trigger replay (Sec. 4.2.1, Sec. 4.2.2), at chunk granularity: each
 * landed tile update increments the counter of the chunk it belongs to; the
 * landing that brings a counter to the threshold marks the chunk ready and,
 * unless it is the chunk the rank keeps, appends it to the trigger queue.
 * The threshold is (tiles per chunk) x (updates expected per element of the
 * chunk): 1 where only the local GEMM writes, 2 where the upstream
 * neighbour's update lands in the same memory as well, which is the ring
 * reduce-scatter case of Sec. 4.2.1.  updates == NULL means 1 everywhere.
 * `landed` lists tile issue indices in the order their writes land (a tile
 * appears once per writer).  counter/ready/queue have P entries; queue is
 * filled in trigger order and unused entries are left at 0xFFFFFFFF.
 */
int t3o_track_upd(int32_t M, int32_t N, int32_t P, int32_t r,
                  int32_t tile_m, int32_t tile_n, const int32_t *updates,
                  const int64_t *landed, int64_t nlanded,
                  uint32_t *counter, uint32_t *ready, uint32_t *queue,
                  uint32_t *queue_len)
{
    if (M <= 0 || N <= 0 || P <= 0 || r < 0 || r >= P || N % P != 0 ||
        tile_m <= 0 || tile_n <= 0 || nlanded < 0 || (nlanded && !landed) ||
        !counter || !ready || !queue || !queue_len)
        return T3O_BAD_ARG;
    const int32_t W = N / P;
    const int64_t tpc = (int64_t)((M + tile_m - 1) / tile_m) * ((W + tile_n - 1) / tile_n);
    const int32_t own = (r + P - 1) % P;
    for (int32_t c = 0; c < P; ++c) {
        if (updates && updates[c] < 1)
            return T3O_BAD_ARG;
        counter[c] = 0;
        ready[c] = 0;
        queue[c] = 0xFFFFFFFFu;
    }
    *queue_len = 0;
    for (int64_t i = 0; i < nlanded; ++i) {
        const int64_t t = landed[i];
        if (t < 0 || t >= tpc * P)
            return T3O_BAD_ARG;
        const int32_t c = (int32_t)((r + t / tpc) % P);
        counter[c] += 1;
        if ((int64_t)counter[c] == tpc * (updates ? updates[c] : 1)) {
            ready[c] = 1;
            if (c != own) {
                queue[*queue_len] = (uint32_t)c;
                *queue_len += 1;
            }
        }
    }
    return T3O_OK;
}

int t3o_track(int32_t M, int32_t N, int32_t P, int32_t r,
              int32_t tile_m, int32_t tile_n,
              const int64_t *landed, int64_t nlanded,
              uint32_t *counter, uint32_t *ready, uint32_t *queue,
              uint32_t *queue_len)
{
    return t3o_track_upd(M, N, P, r, tile_m, tile_n, NULL, landed, nlanded, counter, ready,
                         queue, queue_len);
}
