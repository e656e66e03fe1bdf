// Log-sum-exp merge of the split-K partials of the flash-decoding kernels (Sec. 3.3: the
// block list is partitioned along num_split; each part leaves a running max m, a sum l and an
// unnormalised output, combined here into out and lse).
//
// One work-group of 128 threads per query row (head, or new token x head).  The first wave reads the (m, l) pairs of all
// slices in parallel (one slice per lane), reduces the max and turns them into weights in LDS;
// then thread dd accumulates feature dd over the slices with independent, unrolled loads.
#include "seer_internal.h"

namespace seer {

constexpr int kMergeMaxSplits = 256;   // == the planner's cap on num_splits

__global__ __launch_bounds__(128) void seer_decode_merge_kernel(DecodeParams p) {
  __shared__ float wgt[kMergeMaxSplits];
  __shared__ float tot[2];

  const int g = p.rows;            // rows of a group's tile (new tokens x heads)
  const int h = blockIdx.x % g, hk = blockIdx.x / g, i = blockIdx.y;
  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  const int nb = (S + p.block_size - 1) / p.block_size;
  const int64_t grp = (int64_t)i * p.Hkv + hk;
  const int32_t* list;
  const int n = group_list(p, grp, nb, &list);
  int nsv = (n + p.blocks_per_split - 1) / p.blocks_per_split;   // slices that wrote a partial
  nsv = nsv < p.num_splits ? nsv : p.num_splits;
  const float* ml = p.part_ml + (grp * p.num_splits * g + h) * 2;          // slice stride g*2
  const float* pa = p.part_acc + (grp * p.num_splits * g + h) * kHeadDim;  // slice stride g*128
  const int tid = threadIdx.x;

  if (tid < 64) {
    float m_loc[kMergeMaxSplits / 64], l_loc[kMergeMaxSplits / 64];
    float ma = -INFINITY;
#pragma unroll
    for (int r = 0; r < kMergeMaxSplits / 64; ++r) {
      const int s = r * 64 + tid;
      m_loc[r] = -INFINITY;
      l_loc[r] = 0.f;
      if (s < nsv) {
        m_loc[r] = ml[(int64_t)s * g * 2];
        l_loc[r] = ml[(int64_t)s * g * 2 + 1];
      }
      ma = fmaxf(ma, m_loc[r]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ma = fmaxf(ma, __shfl_xor(ma, o));
    float L = 0.f;
#pragma unroll
    for (int r = 0; r < kMergeMaxSplits / 64; ++r) {
      const int s = r * 64 + tid;
      const float f = (m_loc[r] == -INFINITY) ? 0.f : exp2f(m_loc[r] - ma);
      if (s < nsv) wgt[s] = f;
      L += l_loc[r] * f;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) L += __shfl_xor(L, o);
    if (tid == 0) { tot[0] = ma; tot[1] = L; }
  }
  __syncthreads();

  float a = 0.f;
  int s = 0;
  for (; s + 4 <= nsv; s += 4) {
    const float a0 = pa[(int64_t)(s + 0) * g * kHeadDim + tid];
    const float a1 = pa[(int64_t)(s + 1) * g * kHeadDim + tid];
    const float a2 = pa[(int64_t)(s + 2) * g * kHeadDim + tid];
    const float a3 = pa[(int64_t)(s + 3) * g * kHeadDim + tid];
    a += a0 * wgt[s] + a1 * wgt[s + 1] + a2 * wgt[s + 2] + a3 * wgt[s + 3];
  }
  for (; s < nsv; ++s) a += pa[(int64_t)s * g * kHeadDim + tid] * wgt[s];
  store_output(p, output_row(p, i, hk, h), tid, tot[0], tot[1], a);
  // every unit of the split kernel has been handed out: leave its hand-out word valid and at zero
  if (p.sched && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *p.sched = (unsigned long long)kSchedMagic << 32;
}

hipError_t launch_decode_merge(const DecodeParams& p, hipStream_t s) {
  if (p.num_splits > kMergeMaxSplits) return hipErrorInvalidValue;
  dim3 grid(p.Hkv * p.rows, p.B);
  hipLaunchKernelGGL(seer_decode_merge_kernel, grid, dim3(128), 0, s, p);
  return hipGetLastError();
}

}  // namespace seer
