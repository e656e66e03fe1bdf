/*
 * Pure-C user of the library: no Python, no torch.  Allocates with the HIP runtime, runs one tiny
 * gate-selection + sparse-decode step through the C ABI of include/seer.h and checks it against the
 * CPU oracle (oracle/seer_oracle.c, linked in as the checker).  Exit code 0 = parity.
 *
 * Workload: batch 2, 8 query / 2 kv heads, head dim 128, block 64, sequence lengths 1000 and 333
 * (both end in a partial block), token budget 512; inputs from a fixed linear congruential generator.
 * Then the training-side forward on the first 200 tokens of the same tensors (queries drawn afresh),
 * second sequence cut to 77 tokens.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/seer.h"

/* oracle entry points (see oracle/seer_oracle.c) */
typedef struct {
  const uint16_t* k; const uint16_t* v;
  int64_t stride_seq, stride_head, stride_token;
  const int32_t* page_table; int32_t max_pages, page_size;
} oracle_kv_t;
int oracle_gate_select(const uint16_t*, const uint16_t*, int64_t, int64_t, int64_t, const int32_t*, int, int, int, int,
                       int, int, int32_t, const int32_t*, double, int32_t*, int32_t*, int, double*);
int oracle_sparse_decode(const uint16_t*, const oracle_kv_t*, const int32_t*, const int32_t*, const int32_t*, int, int,
                         int, int, int, int, float, double*, double*, const uint8_t*);
int oracle_attn_ground_truth(const uint16_t*, const oracle_kv_t*, const int32_t*, int, int, int, int, int, int, float,
                             double*, double*, double*);

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_SEER(x) do { seer_status s_ = (x); if (s_ != SEER_OK) { fprintf(stderr, "%s -> %s\n", #x, seer_status_string(s_)); return 3; } } while (0)

static uint32_t lcg_state = 12345u;
static float uniform_pm1(void) {             /* uniform in (-1, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return ((lcg_state >> 8) / 8388608.0f) - 1.0f;
}
static uint16_t to_bf16(float f) {           /* round to nearest even */
  uint32_t u; memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
static float from_bf16(uint16_t h) { uint32_t u = (uint32_t)h << 16; float f; memcpy(&f, &u, 4); return f; }
static void fill(uint16_t* p, size_t n, float scale) { for (size_t i = 0; i < n; ++i) p[i] = to_bf16(scale * 1.7f * uniform_pm1()); }

int main(void) {
  enum { B = 2, Hq = 8, Hkv = 2, D = 128, BS = 64, SMAX = 1024, NB = SMAX / BS, BUDGET = 512, MAXSEL = BUDGET / BS };
  const int32_t seqlens[B] = {1000, 333};
  const float scale = 1.0f / sqrtf((float)D);
  const size_t nq = (size_t)B * Hq * D, nkv = (size_t)B * Hkv * SMAX * D, nqg = (size_t)B * Hkv * D, nkc = (size_t)B * Hkv * NB * D;
  uint16_t *q = malloc(nq * 2), *k = malloc(nkv * 2), *v = malloc(nkv * 2), *qg = malloc(nqg * 2), *kc = malloc(nkc * 2);
  fill(q, nq, 1.f); fill(k, nkv, 1.f); fill(v, nkv, 1.f); fill(qg, nqg, 1.f); fill(kc, nkc, 1.f);

  /* ---- oracle ---- */
  int32_t ref_idx[B * Hkv * MAXSEL], ref_cnt[B * Hkv];
  if (oracle_gate_select(qg, kc, (int64_t)Hkv * NB * D, (int64_t)NB * D, D, seqlens, B, Hkv, D, NB, BS, 0, BUDGET, NULL, 0.0,
                         ref_idx, ref_cnt, MAXSEL, NULL)) return 4;
  oracle_kv_t okv = {k, v, (int64_t)Hkv * SMAX * D, (int64_t)SMAX * D, D, NULL, 0, 0};
  double* ref_out = malloc(nq * sizeof(double));
  double ref_lse[B * Hq];
  if (oracle_sparse_decode(q, &okv, seqlens, ref_idx, ref_cnt, MAXSEL, B, Hq, Hkv, D, BS, scale, ref_out, ref_lse, NULL)) return 4;

  /* ---- device ---- */
  void *dq, *dk, *dv, *dqg, *dkc, *dsl, *didx, *dcnt, *dout, *dlse, *ws_g, *ws_d;
  size_t wsg = 0, wsd = 0;
  CHECK_SEER(seer_gate_workspace_bytes(B, Hkv, NB, &wsg));
  CHECK_SEER(seer_decode_workspace_bytes(B, Hq, Hkv, D, MAXSEL, &wsd));
  CHECK_HIP(hipMalloc(&dq, nq * 2)); CHECK_HIP(hipMalloc(&dk, nkv * 2)); CHECK_HIP(hipMalloc(&dv, nkv * 2));
  CHECK_HIP(hipMalloc(&dqg, nqg * 2)); CHECK_HIP(hipMalloc(&dkc, nkc * 2)); CHECK_HIP(hipMalloc(&dsl, sizeof seqlens));
  CHECK_HIP(hipMalloc(&didx, sizeof ref_idx)); CHECK_HIP(hipMalloc(&dcnt, sizeof ref_cnt));
  CHECK_HIP(hipMalloc(&dout, nq * 4)); CHECK_HIP(hipMalloc(&dlse, B * Hq * 4));
  CHECK_HIP(hipMalloc(&ws_g, wsg)); CHECK_HIP(hipMalloc(&ws_d, wsd));
  CHECK_HIP(hipMemcpy(dq, q, nq * 2, hipMemcpyHostToDevice)); CHECK_HIP(hipMemcpy(dk, k, nkv * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dv, v, nkv * 2, hipMemcpyHostToDevice)); CHECK_HIP(hipMemcpy(dqg, qg, nqg * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dkc, kc, nkc * 2, hipMemcpyHostToDevice)); CHECK_HIP(hipMemcpy(dsl, seqlens, sizeof seqlens, hipMemcpyHostToDevice));
  hipStream_t stream;
  CHECK_HIP(hipStreamCreate(&stream));

  CHECK_SEER(seer_gate_select(dqg, dkc, (int64_t)Hkv * NB * D, (int64_t)NB * D, D, dsl, B, Hkv, D, NB, BS, SEER_SELECT_TOPK,
                              BUDGET, NULL, 0.0, didx, dcnt, MAXSEL, ws_g, wsg, SEER_HINT_NONE, stream));
  seer_kv_layout kv = {dk, dv, (int64_t)Hkv * SMAX * D, (int64_t)SMAX * D, D, NULL, 0, 0};
  CHECK_SEER(seer_sparse_decode(dq, &kv, dsl, didx, dcnt, MAXSEL, B, Hq, Hkv, D, BS, scale, dout, SEER_F32, dlse, ws_d, wsd, SEER_HINT_NONE, stream));
  CHECK_HIP(hipStreamSynchronize(stream));

  int32_t idx[B * Hkv * MAXSEL], cnt[B * Hkv];
  float* out = malloc(nq * 4);
  float lse[B * Hq];
  CHECK_HIP(hipMemcpy(idx, didx, sizeof idx, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(cnt, dcnt, sizeof cnt, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(out, dout, nq * 4, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(lse, dlse, sizeof lse, hipMemcpyDeviceToHost));

  if (memcmp(idx, ref_idx, sizeof idx) || memcmp(cnt, ref_cnt, sizeof cnt)) { fprintf(stderr, "block indices differ from the oracle\n"); return 5; }
  double max_err = 0.0, max_lse = 0.0;
  for (size_t i = 0; i < nq; ++i) { double e = fabs((double)out[i] - ref_out[i]); if (e > max_err) max_err = e; }
  for (int i = 0; i < B * Hq; ++i) { double e = fabs((double)lse[i] - ref_lse[i]); if (e > max_lse) max_lse = e; }
  printf("c_abi_check: indices bit-exact (%d + %d blocks), max |out - oracle| = %.3e, max |lse - oracle| = %.3e\n",
         cnt[0], cnt[Hkv], max_err, max_lse);
  (void)from_bf16;
  if (!(max_err <= 2e-4) || !(max_lse <= 1e-4)) { fprintf(stderr, "outside tolerance\n"); return 6; }

  /* ---- training-side forward: causal attention + ground truth over T tokens of the same K/V ---- */
  {
    enum { T = 200, NBT = (T + BS - 1) / BS };
    const int32_t tlens[B] = {T, 77};
    const size_t ntq = (size_t)B * T * Hq * D, ngt = (size_t)B * Hkv * T * NBT;
    uint16_t* tq = malloc(ntq * 2);
    fill(tq, ntq, 1.f);
    double *r_out = malloc(ntq * sizeof(double)), *r_lse = malloc((size_t)B * T * Hq * sizeof(double)),
           *r_gt = malloc(ngt * sizeof(double));
    if (oracle_attn_ground_truth(tq, &okv, tlens, B, T, Hq, Hkv, D, BS, scale, r_out, r_lse, r_gt)) return 4;
    void *dtq, *dtl, *dto, *dtlse, *dgt, *ws_t;
    size_t wst = 0;
    CHECK_SEER(seer_attn_ground_truth_workspace_bytes(B, T, Hq, Hkv, D, BS, &wst));
    CHECK_HIP(hipMalloc(&dtq, ntq * 2)); CHECK_HIP(hipMalloc(&dtl, sizeof tlens)); CHECK_HIP(hipMalloc(&dto, ntq * 4));
    CHECK_HIP(hipMalloc(&dtlse, (size_t)B * T * Hq * 4)); CHECK_HIP(hipMalloc(&dgt, ngt * 4)); CHECK_HIP(hipMalloc(&ws_t, wst));
    CHECK_HIP(hipMemcpy(dtq, tq, ntq * 2, hipMemcpyHostToDevice)); CHECK_HIP(hipMemcpy(dtl, tlens, sizeof tlens, hipMemcpyHostToDevice));
    CHECK_SEER(seer_attn_ground_truth(dtq, &kv, dtl, B, T, Hq, Hkv, D, BS, scale, dto, SEER_F32, dtlse, dgt, ws_t, wst, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    float *t_out = malloc(ntq * 4), *t_lse = malloc((size_t)B * T * Hq * 4), *t_gt = malloc(ngt * 4);
    CHECK_HIP(hipMemcpy(t_out, dto, ntq * 4, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(t_lse, dtlse, (size_t)B * T * Hq * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(t_gt, dgt, ngt * 4, hipMemcpyDeviceToHost));
    double e_out = 0.0, e_lse = 0.0, e_gt = 0.0;
    for (size_t i = 0; i < ntq; ++i) { double e = fabs((double)t_out[i] - r_out[i]); if (e > e_out) e_out = e; }
    for (size_t i = 0; i < (size_t)B * T * Hq; ++i) {
      if (isinf(r_lse[i])) { if (!(isinf(t_lse[i]) && t_lse[i] < 0)) return 8; continue; }
      double e = fabs((double)t_lse[i] - r_lse[i]); if (e > e_lse) e_lse = e;
    }
    for (size_t i = 0; i < ngt; ++i) {
      double e = fabs((double)t_gt[i] - r_gt[i]) / (fabs(r_gt[i]) + 1e-3);
      if (e > e_gt) e_gt = e;
    }
    printf("c_abi_check: training forward max |out - oracle| = %.3e, |lse| = %.3e, ground truth rel = %.3e\n", e_out, e_lse, e_gt);
    if (!(e_out <= 6e-3) || !(e_lse <= 1e-4) || !(e_gt <= 2e-4)) { fprintf(stderr, "training forward outside tolerance\n"); return 8; }
    if (seer_attn_ground_truth(dtq, &kv, dtl, B, T, Hq, Hkv, D, 48, scale, dto, SEER_F32, dtlse, dgt, ws_t, wst, stream) != SEER_ERR_UNSUPPORTED) return 7;
  }

  /* error paths need no device work */
  if (seer_sparse_decode(NULL, &kv, dsl, didx, dcnt, MAXSEL, B, Hq, Hkv, D, BS, scale, dout, SEER_F32, dlse, ws_d, wsd, SEER_HINT_NONE, stream) != SEER_ERR_NULL) return 7;
  if (seer_sparse_decode(dq, &kv, dsl, didx, dcnt, MAXSEL, B, Hq, Hkv, D, BS, scale, dout, SEER_F32, dlse, ws_d, 16, SEER_HINT_NONE, stream) != SEER_ERR_WORKSPACE) return 7;
  return 0;
}
