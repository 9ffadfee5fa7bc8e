/*
 * A plain C program that uses the library through include/t3.h alone (no Python, no torch):
 * allocates device buffers with the HIP runtime, runs the fused path on small integer inputs,
 * and compares every output word with sums formed here by a triple loop (exact in fp32).
 * Built by __graft_entry__.build(); run by tests/test_gpu_parity.py.  Exit status 0 = all equal.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "t3.h"

#define CHECK_HIP(x)                                                              \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__);            \
      return 2;                                                                   \
    }                                                                             \
  } while (0)

static uint16_t bf16_of_small_int(int v) { /* exact: small integers fit 8 significant bits */
  float f = (float)v;
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

int main(int argc, char **argv) {
  const uint32_t flags = argc > 1 ? (uint32_t)strtoul(argv[1], NULL, 0) : T3_FLAG_FWD_DIRECT;
  enum { M = 300, N = 512, K = 72, TP = 4, RANK = 1, W = N / TP };
  static int a[M][K], b[N][K];
  static float inc[M][N], prod[M][N], R_host[M][N], fwd_host[TP - 1][M][W];
  static uint16_t a_bits[M][K], b_bits[N][K];
  for (int m = 0; m < M; ++m)
    for (int k = 0; k < K; ++k) a_bits[m][k] = bf16_of_small_int(a[m][k] = (m * 7 + k * 3) % 5 - 2);
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k) b_bits[n][k] = bf16_of_small_int(b[n][k] = (n * 5 + k) % 3 - 1);
  for (int m = 0; m < M; ++m)
    for (int n = 0; n < N; ++n) {
      int acc = 0;
      for (int k = 0; k < K; ++k) acc += a[m][k] * b[n][k];
      inc[m][n] = (float)((m + 3 * n) % 23 - 11);
      prod[m][n] = (float)acc;
    }

  t3_problem p;
  memset(&p, 0, sizeof p);
  p.M = M; p.N = N; p.K = K; p.tp = TP; p.rank = RANK;
  p.tile_m = 128; p.tile_n = 128; p.b_layout = T3_B_NK;
  p.lda = K; p.ldb = K; p.ldr = N; p.ldc = N; p.tile_limit = -1; p.flags = flags;

  int32_t order[TP], own = -1;
  if (t3_chunk_order(TP, RANK, order, &own) != T3_OK || own != (RANK + TP - 1) % TP) return 3;

  void *dA, *dB; float *dR, *dF; uint32_t *dT;
  const int64_t words = t3_track_words(TP);
  CHECK_HIP(hipMalloc(&dA, sizeof a_bits));
  CHECK_HIP(hipMalloc(&dB, sizeof b_bits));
  CHECK_HIP(hipMalloc((void **)&dR, sizeof inc));
  CHECK_HIP(hipMalloc((void **)&dF, sizeof fwd_host));
  CHECK_HIP(hipMalloc((void **)&dT, (size_t)words * 4));
  CHECK_HIP(hipMemcpy(dA, a_bits, sizeof a_bits, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dB, b_bits, sizeof b_bits, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dR, inc, sizeof inc, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemset(dF, 0xFF, sizeof fwd_host));

  t3_status st = t3_track_reset(TP, dT, NULL);
  if (st == T3_OK) st = t3_gemm_rs_fused(&p, dA, dB, dR, dF, dT, NULL);
  if (st != T3_OK) {
    fprintf(stderr, "t3 status %d (%s), hip error %d\n", (int)st, t3_status_string(st), (int)t3_last_hip_error());
    return 4;
  }
  CHECK_HIP(hipDeviceSynchronize());
  uint32_t *trk = (uint32_t *)malloc((size_t)words * 4);
  CHECK_HIP(hipMemcpy(R_host, dR, sizeof inc, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(fwd_host, dF, sizeof fwd_host, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(trk, dT, (size_t)words * 4, hipMemcpyDeviceToHost));

  /* tracker: two banks of 3*tp + 2 words, then gen and error; results in bank (gen - 1) & 1 */
  const int bank_words = 3 * TP + 2;
  const uint32_t gen = trk[2 * bank_words], err = trk[2 * bank_words + 1];
  const uint32_t *bank = trk + ((gen - 1) & 1) * bank_words;
  int64_t tpc = 0;
  if (t3_tiles_per_chunk(&p, &tpc) != T3_OK) return 3;
  long bad = 0;
  if (gen != 1 || err != 0 || bank[3 * TP] != TP - 1) ++bad;
  for (int c = 0; c < TP; ++c)
    if (bank[c] != (uint32_t)tpc || bank[TP + c] != 1) ++bad;

  const int direct = (flags & T3_FLAG_FWD_DIRECT) != 0;
  const int step0 = (flags & T3_FLAG_STEP0_STORE_ONLY) != 0;
  for (int s = 0; s < TP; ++s) {
    const int c = order[s];
    for (int m = 0; m < M; ++m)
      for (int j = 0; j < W; ++j) {
        /* the first chunk produced has no upstream data under T3_FLAG_STEP0_STORE_ONLY */
        const float w = prod[m][c * W + j] + ((step0 && s == 0) ? 0.0f : inc[m][c * W + j]);
        if (c == own) {
          bad += R_host[m][c * W + j] != w;
        } else {
          bad += fwd_host[s][m][j] != w;
          bad += R_host[m][c * W + j] != (direct ? inc[m][c * W + j] : w);
        }
      }
  }
  printf("c_abi_client flags=%u: %ld mismatches, gen=%u error=%u queue_len=%u\n", flags, bad, gen, err,
         bank[3 * TP]);
  free(trk);
  hipFree(dA); hipFree(dB); hipFree(dR); hipFree(dF); hipFree(dT);
  return bad ? 1 : 0;
}
