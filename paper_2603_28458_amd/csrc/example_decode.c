/*
 * example_decode.c -- the HISA indexer called from plain C, without Python or torch.
 *
 * A decode step for a small batch: n_seq sequences of different lengths, one query each at its last
 * position (Section 5.2 of the paper measures this regime).  The program
 *   1. builds keys, queries and gates on the host (a fixed linear congruential generator) and copies
 *      them to the GPU with the HIP runtime's C API,
 *   2. pools the keys (hisa_pool_blocks), keeps m blocks per query (hisa_block_score_topk) and k tokens
 *      inside them (hisa_token_refine_topk),
 *   3. copies the indices back and checks what must hold for ANY correct result (Section 4.1): block
 *      ids ascending, unique, visible, first and own block kept; token ids ascending, unique, visible,
 *      inside the kept blocks; min(k, candidates) of them.
 * Exit status 0 and a line "example ok" when everything holds.
 *
 * Build (the package's build step does this):
 *   gcc -std=c11 -O1 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -I<repo>/include example_decode.c \
 *       -L<repo>/paper_2603_28458_amd/lib -lhisa -L/opt/rocm/lib -lamdhip64 -lm -o example_decode
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hisa.h"

#define CHECK_HIP(x)                                                              \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "%s:%d: HIP error %d (%s)\n", __FILE__, __LINE__, (int)e_, hipGetErrorString(e_)); \
      return 2;                                                                   \
    }                                                                             \
  } while (0)

#define CHECK_HISA(x)                                                             \
  do {                                                                            \
    int s_ = (x);                                                                 \
    if (s_ != HISA_OK) {                                                          \
      fprintf(stderr, "%s:%d: hisa status %d (%s)\n", __FILE__, __LINE__, s_, hisa_status_string(s_)); \
      return 3;                                                                   \
    }                                                                             \
  } while (0)

static uint32_t lcg_state = 20260328u;
static float lcg_uniform(void) { /* in (-1, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return ((float)(lcg_state >> 8) / 8388608.0f) - 1.0f;
}

static uint16_t to_bf16(float x) { /* round to nearest even; finite inputs */
  uint32_t b;
  memcpy(&b, &x, 4);
  return (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}

enum { N_SEQ = 6, S_MAX = 4096, D = 128, H = 64, B = 128, M_KEEP = 6, K_KEEP = 512 };

int main(void) {
  static const int32_t seq_len[N_SEQ] = {4096, 3333, 1500, 129, 128, 7};
  const int T = N_SEQ, n_blocks = S_MAX / B;
  int32_t q_seq[N_SEQ], q_pos[N_SEQ];
  for (int n = 0; n < N_SEQ; ++n) {
    q_seq[n] = n;
    q_pos[n] = seq_len[n] - 1;
  }

  /* host data */
  const size_t n_keys = (size_t)N_SEQ * S_MAX * D, n_q = (size_t)T * H * D;
  uint16_t* h_k = (uint16_t*)calloc(n_keys, 2);
  uint16_t* h_q = (uint16_t*)malloc(n_q * 2);
  float* h_w = (float*)malloc((size_t)T * H * 4);
  if (!h_k || !h_q || !h_w) return 1;
  for (int n = 0; n < N_SEQ; ++n)
    for (int s = 0; s < seq_len[n]; ++s)
      for (int i = 0; i < D; ++i) h_k[((size_t)n * S_MAX + s) * D + i] = to_bf16(lcg_uniform());
  for (size_t i = 0; i < n_q; ++i) h_q[i] = to_bf16(lcg_uniform());
  for (int i = 0; i < T * H; ++i) h_w[i] = 0.5f * (lcg_uniform() + 1.0f);

  /* device buffers */
  void *d_k, *d_q, *d_w, *d_len, *d_qseq, *d_qpos, *d_pooled, *d_blk, *d_top, *d_ws;
  CHECK_HIP(hipMalloc(&d_k, n_keys * 2));
  CHECK_HIP(hipMalloc(&d_q, n_q * 2));
  CHECK_HIP(hipMalloc(&d_w, (size_t)T * H * 4));
  CHECK_HIP(hipMalloc(&d_len, N_SEQ * 4));
  CHECK_HIP(hipMalloc(&d_qseq, T * 4));
  CHECK_HIP(hipMalloc(&d_qpos, T * 4));
  CHECK_HIP(hipMalloc(&d_pooled, (size_t)N_SEQ * n_blocks * D * 2));
  CHECK_HIP(hipMalloc(&d_blk, (size_t)T * M_KEEP * 4));
  CHECK_HIP(hipMalloc(&d_top, (size_t)T * K_KEEP * 4));
  CHECK_HIP(hipMemcpy(d_k, h_k, n_keys * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_q, h_q, n_q * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_w, h_w, (size_t)T * H * 4, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_len, seq_len, N_SEQ * 4, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_qseq, q_seq, T * 4, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(d_qpos, q_pos, T * 4, hipMemcpyHostToDevice));

  hisa_keys keys = {d_k, NULL, (const int32_t*)d_len, N_SEQ, S_MAX, D, HISA_BF16};
  hisa_queries queries = {d_q, (const float*)d_w, (const int32_t*)d_qseq, (const int32_t*)d_qpos, NULL, T, H, 0,
                          HISA_BF16};

  /* one workspace for both stages: the larger of the two recommendations */
  size_t ws1 = hisa_workspace_bytes(HISA_OP_BLOCK_SCORE_TOPK, &queries, &keys, B, M_KEEP, K_KEEP, 0);
  size_t ws2 = hisa_workspace_bytes(HISA_OP_TOKEN_REFINE_TOPK, &queries, &keys, B, M_KEEP, K_KEEP, 0);
  size_t ws_bytes = ws1 > ws2 ? ws1 : ws2;
  if (ws_bytes < 256) ws_bytes = 256;
  CHECK_HIP(hipMalloc(&d_ws, ws_bytes));

  printf("libhisa %s: %d sequences, s_max %d, H %d, d %d, B %d, m %d, k %d, workspace %zu bytes\n", hisa_version(),
         N_SEQ, S_MAX, H, D, B, M_KEEP, K_KEEP, ws_bytes);
  CHECK_HISA(hisa_pool_blocks(&keys, B, 0, n_blocks, d_pooled, HISA_BF16, NULL));
  CHECK_HISA(hisa_block_score_topk(&queries, &keys, d_pooled, HISA_BF16, B, M_KEEP, (int32_t*)d_blk, NULL, d_ws,
                                   ws_bytes, NULL));
  CHECK_HISA(hisa_token_refine_topk(&queries, &keys, B, M_KEEP, (const int32_t*)d_blk, K_KEEP, (int32_t*)d_top, NULL,
                                    NULL, d_ws, ws_bytes, NULL));
  CHECK_HIP(hipDeviceSynchronize());

  int32_t h_blk[N_SEQ * M_KEEP];
  int32_t* h_top = (int32_t*)malloc((size_t)T * K_KEEP * 4);
  if (!h_top) return 1;
  CHECK_HIP(hipMemcpy(h_blk, d_blk, sizeof(h_blk), hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(h_top, d_top, (size_t)T * K_KEEP * 4, hipMemcpyDeviceToHost));

  int bad = 0;
  for (int t = 0; t < T; ++t) {
    const int pos = q_pos[t], own = pos / B, visible_blocks = own + 1;
    const int want_blocks = visible_blocks < M_KEEP ? visible_blocks : M_KEEP;
    const int32_t* bl = h_blk + t * M_KEEP;
    int nb = 0, has_first = 0, has_own = 0;
    long n_cand = 0;
    for (int i = 0; i < M_KEEP; ++i) {
      if (bl[i] < 0) {
        for (int j = i; j < M_KEEP; ++j) bad += bl[j] != -1; /* padding stays at the end */
        break;
      }
      bad += bl[i] > own;                  /* visible */
      bad += i > 0 && bl[i] <= bl[i - 1];  /* ascending, unique */
      has_first |= bl[i] == 0;
      has_own |= bl[i] == own;
      const int first_tok = bl[i] * B, last_tok = (bl[i] + 1) * B - 1 < pos ? (bl[i] + 1) * B - 1 : pos;
      n_cand += last_tok - first_tok + 1;
      ++nb;
    }
    bad += nb != want_blocks || !has_first || !has_own;
    const long want_tok = n_cand < K_KEEP ? n_cand : K_KEEP;
    const int32_t* tk = h_top + (size_t)t * K_KEEP;
    long nt = 0;
    for (int i = 0; i < K_KEEP; ++i) {
      if (tk[i] < 0) {
        for (int j = i; j < K_KEEP; ++j) bad += tk[j] != -1;
        break;
      }
      bad += tk[i] > pos;
      bad += i > 0 && tk[i] <= tk[i - 1];
      int in_kept = 0;
      for (int j = 0; j < nb; ++j) in_kept |= tk[i] / B == bl[j];
      bad += !in_kept;
      ++nt;
    }
    bad += nt != want_tok;
    printf("query %d: position %d, kept blocks %d of %d visible, tokens %ld of %ld candidates\n", t, pos, nb,
           visible_blocks, nt, n_cand);
  }
  if (bad) {
    fprintf(stderr, "example FAILED: %d violations\n", bad);
    return 4;
  }
  printf("example ok\n");
  hipFree(d_ws);
  hipFree(d_top);
  hipFree(d_blk);
  hipFree(d_pooled);
  hipFree(d_qpos);
  hipFree(d_qseq);
  hipFree(d_len);
  hipFree(d_w);
  hipFree(d_q);
  hipFree(d_k);
  free(h_top);
  free(h_w);
  free(h_q);
  free(h_k);
  return 0;
}
