/*
 * Runs every entry point of the C oracle (oracle/seer_oracle.c) on small inputs sized exactly - every
 * buffer is a heap allocation of precisely the bytes the call may touch - so that a build with
 * -fsanitize=address,undefined reports any read or write outside them and any undefined behaviour.
 * CPU only.  Built and run by tests/test_abi.py; exit code 0 = clean run with sane outputs.
 *
 * Shapes: batch 3, 6 query / 2 kv heads (group 3), head dim 128, block 32; sequence lengths 100 (partial
 * last block), 64 (exact) and 0 (empty); contiguous and paged (page = 2 blocks, shuffled) caches.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  const uint16_t* k; const uint16_t* v;
  int64_t stride_seq, stride_head, stride_token;
  const int32_t* page_table; int32_t max_pages, page_size;
} oracle_kv_t;
int oracle_gate_select(const uint16_t*, const uint16_t*, int64_t, int64_t, int64_t, const int32_t*, int, int, int, int,
                       int, int, int32_t, const int32_t*, double, int32_t*, int32_t*, int, double*);
int oracle_sparse_decode(const uint16_t*, const oracle_kv_t*, const int32_t*, const int32_t*, const int32_t*, int, int,
                         int, int, int, int, float, double*, double*, const uint8_t*);
int oracle_sparse_decode_multi(const uint16_t*, const oracle_kv_t*, const int32_t*, const int32_t*, const int32_t*, int,
                               int, int, int, int, int, int, float, double*, double*, const uint8_t*);
int oracle_gate_q(const uint16_t*, const uint16_t*, const float*, const float*, int, const int32_t*, int, int, int, int, int,
                  double*, uint16_t*);
int oracle_kc_update(const oracle_kv_t*, const uint16_t*, const float*, const float*, int, const int32_t*, const int32_t*,
                     const int32_t*, int, int, int, int, int, int, double*, uint16_t*);
int oracle_attn_ground_truth(const uint16_t*, const oracle_kv_t*, const int32_t*, int, int, int, int, int, int, float,
                             double*, double*, double*);

static uint32_t lcg = 2463534242u;
static float unif(void) { lcg = lcg * 1664525u + 1013904223u; return ((lcg >> 8) / 8388608.0f) - 1.0f; }
static uint16_t bf16(float f) { uint32_t u; memcpy(&u, &f, 4); u += 0x7fffu + ((u >> 16) & 1u); return (uint16_t)(u >> 16); }
static uint16_t* rand_bf16(size_t n) { uint16_t* p = malloc(n * 2); for (size_t i = 0; i < n; ++i) p[i] = bf16(1.5f * unif()); return p; }
static int finite_all(const double* x, size_t n) { for (size_t i = 0; i < n; ++i) if (!isfinite(x[i])) return 0; return 1; }

int main(void) {
  enum { B = 3, Hq = 6, Hkv = 2, D = 128, BS = 32, SMAX = 128, NB = SMAX / BS, T = 3 };
  const int32_t seqlens_h[B] = {100, 64, 0};
  int32_t* seqlens = malloc(sizeof seqlens_h); memcpy(seqlens, seqlens_h, sizeof seqlens_h);
  uint16_t* q = rand_bf16((size_t)B * Hq * D);
  uint16_t* k = rand_bf16((size_t)B * Hkv * SMAX * D);
  uint16_t* v = rand_bf16((size_t)B * Hkv * SMAX * D);
  uint16_t* qg = rand_bf16((size_t)B * Hkv * D);
  uint16_t* kc = rand_bf16((size_t)B * Hkv * NB * D);
  oracle_kv_t kv = {k, v, (int64_t)Hkv * SMAX * D, (int64_t)SMAX * D, D, NULL, 0, 0};

  /* ---- gate: three modes, exact-size outputs ---- */
  int32_t* idx = malloc(sizeof(int32_t) * B * Hkv * NB);
  int32_t* cnt = malloc(sizeof(int32_t) * B * Hkv);
  double* scores = malloc(sizeof(double) * B * Hkv * NB);
  if (oracle_gate_select(qg, kc, (int64_t)Hkv * NB * D, (int64_t)NB * D, D, seqlens, B, Hkv, D, NB, BS, 0, 2 * BS, NULL, 0.0,
                         idx, cnt, 2, scores)) return 10;                       /* top-k into a list of exactly 2 */
  int32_t bb[B] = {3, 0, 9};
  int32_t* bbp = malloc(sizeof bb); memcpy(bbp, bb, sizeof bb);
  if (oracle_gate_select(qg, kc, (int64_t)Hkv * NB * D, (int64_t)NB * D, D, seqlens, B, Hkv, D, NB, BS, 0, 0, bbp, 0.0,
                         idx, cnt, NB, NULL)) return 11;
  if (oracle_gate_select(qg, kc, (int64_t)Hkv * NB * D, (int64_t)NB * D, D, seqlens, B, Hkv, D, NB, BS, 1, 0, NULL, 0.3,
                         idx, cnt, NB, NULL)) return 12;
  if (oracle_gate_select(qg, kc, (int64_t)Hkv * NB * D, (int64_t)NB * D, D, seqlens, B, Hkv, D, NB, BS, 2, 0, NULL, 0.7,
                         idx, cnt, NB, NULL)) return 13;
  if (cnt[0] < 1 || cnt[0] > NB || cnt[2 * Hkv] != 0) return 14;                /* sequence 2 is empty */

  /* ---- decode on the top-p lists (contiguous), then dense, then paged ---- */
  double* out = malloc(sizeof(double) * B * Hq * D);
  double* lse = malloc(sizeof(double) * B * Hq);
  const float scale = 1.0f / sqrtf((float)D);
  if (oracle_sparse_decode(q, &kv, seqlens, idx, cnt, NB, B, Hq, Hkv, D, BS, scale, out, lse, NULL)) return 20;
  if (!finite_all(out, (size_t)B * Hq * D) || !isinf(lse[2 * Hq])) return 21;
  if (oracle_sparse_decode(q, &kv, seqlens, NULL, NULL, 0, B, Hq, Hkv, D, BS, scale, out, lse, NULL)) return 22;
  enum { PAGE = 2 * BS, NPG = SMAX / PAGE };
  uint16_t* pk = malloc((size_t)(B * NPG + 1) * Hkv * PAGE * D * 2);
  uint16_t* pv = malloc((size_t)(B * NPG + 1) * Hkv * PAGE * D * 2);
  int32_t* pt = malloc(sizeof(int32_t) * B * NPG);
  for (int i = 0; i < B; ++i)
    for (int pg = 0; pg < NPG; ++pg) {
      const int phys = B * NPG - (i * NPG + pg);          /* reversed order, page 0 unused */
      pt[i * NPG + pg] = phys;
      for (int h = 0; h < Hkv; ++h) {
        memcpy(pk + (((size_t)phys * Hkv + h) * PAGE) * D, k + (((size_t)i * Hkv + h) * SMAX + (size_t)pg * PAGE) * D, (size_t)PAGE * D * 2);
        memcpy(pv + (((size_t)phys * Hkv + h) * PAGE) * D, v + (((size_t)i * Hkv + h) * SMAX + (size_t)pg * PAGE) * D, (size_t)PAGE * D * 2);
      }
    }
  memset(pk, 0, (size_t)Hkv * PAGE * D * 2); memset(pv, 0, (size_t)Hkv * PAGE * D * 2);
  oracle_kv_t pkv = {pk, pv, (int64_t)Hkv * PAGE * D, (int64_t)PAGE * D, D, pt, NPG, PAGE};
  double* out2 = malloc(sizeof(double) * B * Hq * D);
  double* lse2 = malloc(sizeof(double) * B * Hq);
  if (oracle_sparse_decode(q, &pkv, seqlens, NULL, NULL, 0, B, Hq, Hkv, D, BS, scale, out2, lse2, NULL)) return 23;
  for (size_t i = 0; i < (size_t)B * Hq * D; ++i) if (out[i] != out2[i]) return 24;   /* paged == contiguous, bit for bit */

  /* ---- several new tokens ---- */
  uint16_t* qm = rand_bf16((size_t)B * T * Hq * D);
  double* outm = malloc(sizeof(double) * B * T * Hq * D);
  double* lsem = malloc(sizeof(double) * B * T * Hq);
  if (oracle_sparse_decode_multi(qm, &kv, seqlens, idx, cnt, NB, B, T, Hq, Hkv, D, BS, scale, outm, lsem, NULL)) return 30;

  /* ---- front-end ---- */
  const int n_pos = SMAX + 1;
  float* co = malloc(sizeof(float) * n_pos * D / 2);
  float* si = malloc(sizeof(float) * n_pos * D / 2);
  for (int p = 0; p < n_pos; ++p)
    for (int c = 0; c < D / 2; ++c) { const double a = p * pow(1.0e6, -2.0 * c / D); co[p * D / 2 + c] = (float)cos(a); si[p * D / 2 + c] = (float)sin(a); }
  uint16_t* wq = rand_bf16((size_t)Hkv * D * (Hq / Hkv) * D);
  uint16_t* wk = rand_bf16((size_t)Hkv * D * 3 * D);
  double* qg64 = malloc(sizeof(double) * B * Hkv * D);
  uint16_t* qg16 = malloc(2 * (size_t)B * Hkv * D);
  if (oracle_gate_q(q, wq, co, si, n_pos, seqlens, B, Hq, Hkv, D, D, qg64, qg16)) return 40;
  double* kc64 = malloc(sizeof(double) * B * Hkv * NB * D);
  uint16_t* kc16 = malloc(2 * (size_t)B * Hkv * NB * D);
  for (size_t i = 0; i < (size_t)B * Hkv * NB * D; ++i) { kc64[i] = NAN; kc16[i] = 0; }
  if (oracle_kc_update(&kv, wk, co, si, n_pos, seqlens, NULL, NULL, B, Hkv, D, D, NB, BS, kc64, kc16)) return 41;
  if (oracle_kc_update(&pkv, wk, co, si, n_pos, seqlens, NULL, NULL, B, Hkv, D, D, NB, BS, kc64, kc16)) return 42;
  if (!isfinite(kc64[0]) || !isnan(kc64[3 * D])) return 43;        /* sequence 0: blocks 0..2 full, block 3 partial */

  /* ---- training-side ground truth on the first 100 / 64 / 0 tokens ---- */
  enum { TT = 100, NBT = (TT + BS - 1) / BS };
  uint16_t* qt = rand_bf16((size_t)B * TT * Hq * D);
  double* outt = malloc(sizeof(double) * B * TT * Hq * D);
  double* lset = malloc(sizeof(double) * B * TT * Hq);
  double* gt = malloc(sizeof(double) * B * Hkv * TT * NBT);
  if (oracle_attn_ground_truth(qt, &kv, seqlens, B, TT, Hq, Hkv, D, BS, scale, outt, lset, gt)) return 50;
  double rs = 0.0;
  for (int j = 0; j < NBT; ++j) rs += gt[(size_t)(0 * Hkv + 1) * TT * NBT + (size_t)77 * NBT + j];
  if (fabs(rs - 1.0) > 1e-12) return 51;

  free(seqlens); free(q); free(k); free(v); free(qg); free(kc); free(idx); free(cnt); free(scores); free(bbp); free(out);
  free(lse); free(pk); free(pv); free(pt); free(out2); free(lse2); free(qm); free(outm); free(lsem); free(co); free(si);
  free(wq); free(wk); free(qg64); free(qg16); free(kc64); free(kc16); free(qt); free(outt); free(lset); free(gt);
  printf("oracle sanitizer run clean\n");
  return 0;
}
