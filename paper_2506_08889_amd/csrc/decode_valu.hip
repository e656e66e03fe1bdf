// Block-sparse flash-decoding, split-K main kernel, vector-ALU formulation (Sec. 3.3).
//
// Grid (Hkv, B, num_splits): a work-group owns one (sequence, kv head) query group and one
// contiguous slice of its selected-block list.  A K or V row is 256 bytes = 16 lanes x one
// 128-bit load, so a wavefront reads 4 token rows per load instruction, fully coalesced; the
// 4 waves x 4 row slots form 16 independent online-softmax streams that are merged once at
// the end of the slice (first inside each wave by shuffles, then across waves through LDS).
// q.k is reduced over the 16 lanes of a row with xor-shuffles.  fp32 accumulation; logits
// are kept in the base-2 domain (scale*log2(e) folded in) so the exponentials are exp2.
//
// This is the formulation the MFMA kernel is measured against (selected with SEER_KNOB_DECODE_IMPL);
// every supported block size runs on either kernel, one new token per call only.
#include "seer_internal.h"

namespace seer {

template <int G>
__global__ __launch_bounds__(256) void seer_decode_split_valu_kernel(DecodeParams p) {
  __shared__ float sm_acc[4][G][kHeadDim];
  __shared__ float sm_ml[4][G][2];

  int split, hk, i;
  decode_wg_coords(p, &split, &hk, &i);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int slot = lane >> 4, c = lane & 15;

  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  const int bs = p.block_size;
  const int nb = (S + bs - 1) / bs;
  const int64_t grp = (int64_t)i * p.Hkv + hk;
  const int32_t* list;
  const int n = group_list(p, grp, nb, &list);
  const int begin = split * p.blocks_per_split;
  if (begin >= n) {
    emit_empty_if_single_split(p, i, hk);
    return;
  }
  const int end = (begin + p.blocks_per_split < n) ? begin + p.blocks_per_split : n;

  float qf[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const uint4 r = *reinterpret_cast<const uint4*>(
        p.q + ((int64_t)i * p.Hq + (int64_t)hk * G + h) * kHeadDim + c * 8);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      qf[h][2 * e] = bf16_lo(w[e]) * p.scale_log2e;
      qf[h][2 * e + 1] = bf16_hi(w[e]) * p.scale_log2e;
    }
  }

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = -INFINITY;
    l[h] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
  }

  for (int blk = begin; blk < end; ++blk) {
    const int j = list ? list[blk] : blk;
    if (j < 0 || j >= nb) continue;
    if (p.page_table && ((int64_t)j * bs) / p.page_size >= p.max_pages) continue;
    const int64_t off = block_offset(p, i, hk, j);
    const int ntok = (S - j * bs < bs) ? S - j * bs : bs;
    const uint16_t* kb = p.k + off + c * 8;
    const uint16_t* vb = p.v + off + c * 8;
    for (int tt = wave * 4 + slot; tt < ntok; tt += 16) {
      const uint4 kr = load_stream16(kb + (int64_t)tt * p.stride_token);
      const uint4 vr = load_stream16(vb + (int64_t)tt * p.stride_token);
      const uint32_t kw[4] = {kr.x, kr.y, kr.z, kr.w};
      const uint32_t vw[4] = {vr.x, vr.y, vr.z, vr.w};
      float kf[8], vf[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        kf[2 * e] = bf16_lo(kw[e]);
        kf[2 * e + 1] = bf16_hi(kw[e]);
        vf[2 * e] = bf16_lo(vw[e]);
        vf[2 * e + 1] = bf16_hi(vw[e]);
      }
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float x = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) x = fmaf(qf[h][e], kf[e], x);
        // The 16 lanes of this row are all active or all inactive, so the shuffles below
        // only ever read active lanes.
        x += __shfl_xor(x, 1);
        x += __shfl_xor(x, 2);
        x += __shfl_xor(x, 4);
        x += __shfl_xor(x, 8);
        const float mn = fmaxf(m[h], x);
        const float alpha = exp2f(m[h] - mn);   // m = -inf on the first token: exp2(-inf) = 0
        const float pr = exp2f(x - mn);
        l[h] = l[h] * alpha + pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(pr, vf[e], acc[h][e] * alpha);
        m[h] = mn;
      }
    }
  }

  // ---- merge the 4 row slots of the wave (all lanes take part) ---------------------------
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float ma = fmaxf(m[h], __shfl_xor(m[h], 16));
    ma = fmaxf(ma, __shfl_xor(ma, 32));
    const float f = (m[h] == -INFINITY) ? 0.f : exp2f(m[h] - ma);
    float ls = l[h] * f;
    ls += __shfl_xor(ls, 16);
    ls += __shfl_xor(ls, 32);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float a = acc[h][e] * f;
      a += __shfl_xor(a, 16);
      a += __shfl_xor(a, 32);
      acc[h][e] = a;
    }
    m[h] = ma;
    l[h] = ls;
  }
  if (slot == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sm_acc[wave][h][c * 8 + e] = acc[h][e];
      if (c == 0) { sm_ml[wave][h][0] = m[h]; sm_ml[wave][h][1] = l[h]; }
    }
  }
  __syncthreads();

  // ---- merge the 4 waves and write the partial of this split --------------------------------
  for (int o = tid; o < G * kHeadDim; o += 256) {
    const int h = o / kHeadDim, dd = o % kHeadDim;
    float ma = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) ma = fmaxf(ma, sm_ml[w][h][0]);
    float ls = 0.f, a = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = sm_ml[w][h][0];
      const float f = (mw == -INFINITY) ? 0.f : exp2f(mw - ma);
      ls += sm_ml[w][h][1] * f;
      a += sm_acc[w][h][dd] * f;
    }
    emit_slice(p, i, hk, split, h, dd, ma, ls, a);
  }
}

hipError_t launch_decode_split_valu(const DecodeParams& p, hipStream_t s) {
  const dim3 grid = decode_grid(p);
  dim3 block(256);
  switch (p.g) {
#define SEER_CASE(G) \
  case G: hipLaunchKernelGGL(seer_decode_split_valu_kernel<G>, grid, block, 0, s, p); break;
    SEER_CASE(1) SEER_CASE(2) SEER_CASE(3) SEER_CASE(4)
    SEER_CASE(5) SEER_CASE(6) SEER_CASE(7) SEER_CASE(8)
#undef SEER_CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace seer
