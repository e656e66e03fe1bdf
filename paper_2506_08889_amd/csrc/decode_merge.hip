// Log-sum-exp merge of the split-K partials of the flash-decoding kernels (Sec. 3.3: the
// block list is partitioned along num_split; each part leaves a running max m, a sum l and an
// unnormalised output, combined here into out and lse).
#include "seer_internal.h"

namespace seer {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__global__ __launch_bounds__(256) void seer_decode_merge_kernel(DecodeParams p) {
  const int hk = blockIdx.x, i = blockIdx.y;
  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  const int nb = (S + p.block_size - 1) / p.block_size;
  const int64_t grp = (int64_t)i * p.Hkv + hk;
  const int32_t* list;
  const int n = group_list(p, grp, nb, &list);
  int nsv = (n + p.blocks_per_split - 1) / p.blocks_per_split;   // splits that wrote a partial
  nsv = nsv < p.num_splits ? nsv : p.num_splits;
  const int g = p.g;
  const float* ml = p.part_ml + grp * p.num_splits * g * 2;
  const float* pa = p.part_acc + grp * p.num_splits * g * kHeadDim;

  for (int o = threadIdx.x; o < g * kHeadDim; o += 256) {
    const int h = o / kHeadDim, dd = o % kHeadDim;
    float ma = -INFINITY;
    for (int s = 0; s < nsv; ++s) ma = fmaxf(ma, ml[(s * g + h) * 2]);
    float L = 0.f, a = 0.f;
    if (ma != -INFINITY) {
      for (int s = 0; s < nsv; ++s) {
        const float ms = ml[(s * g + h) * 2];
        const float f = (ms == -INFINITY) ? 0.f : exp2f(ms - ma);
        L += ml[(s * g + h) * 2 + 1] * f;
        a += pa[(s * g + h) * kHeadDim + dd] * f;
      }
    }
    const float r = (L > 0.f) ? a / L : 0.f;
    const int64_t row = (int64_t)i * p.Hq + (int64_t)hk * g + h;
    if (p.out_is_f32) reinterpret_cast<float*>(p.out)[row * kHeadDim + dd] = r;
    else reinterpret_cast<uint16_t*>(p.out)[row * kHeadDim + dd] = f32_to_bf16_rne(r);
    if (dd == 0 && p.lse)
      p.lse[row] = (L > 0.f) ? (ma + log2f(L)) * 0.6931471805599453f : -INFINITY;
  }
}

hipError_t launch_decode_merge(const DecodeParams& p, hipStream_t s) {
  dim3 grid(p.Hkv, p.B);
  hipLaunchKernelGGL(seer_decode_merge_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace seer
