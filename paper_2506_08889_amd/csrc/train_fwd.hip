// Training-side forward (Sec. 2.3): dense causal attention that also leaves what the AttnGate's
// distillation target is made of, in the manner the section describes - the block-level row maxima
// that the online softmax computes anyway are kept per (query row, key block) and turned into
// probabilities once the row's log-sum-exp is known.
//
// Kernel 1, seer_attn_fwd_kernel: grid (query tiles of 128 rows, longest first; query head; sequence),
// 256 threads.  A wave owns 32 query rows as two 16-row tiles and walks the keys 64 at a time (two
// 32-key chunks).  The matrix-core formulation is the one of the decode kernel, with query rows in
// the place of the heads of a group (lane = 16*q + n):
//   S^T = K Q^T   A = 16 keys x 32 features from the work-group's K tile in LDS (XOR-swizzled rows,
//                 double-buffered: the next tile is fetched into registers during the current one
//                 and stored before the single barrier of the iteration); B = Q^T in registers.
//   softmax       lane holds 4 keys x 2 tiles of one query row; causal mask on the diagonal chunks;
//                 the chunk maximum doubles as the block maximum (running over the chunks of a block).
//   O^T = V^T P^T B = P^T rounded to bf16, already in operand layout; A = V^T built in registers
//                 from coalesced row loads (8 rows x 16 bytes per lane, 16-bit interleaves).
// Kernel 2, seer_gt_finalize_kernel: per (sequence, kv head, 64 query rows): block probabilities
// exp2(raw - lse2), maximum over the g heads, row sums, normalised rows written through an LDS
// transpose so that both the reads (along rows) and the writes (along blocks) are coalesced.
#include "seer_internal.h"

namespace seer {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ uint32_t tf_pack_lo(uint32_t x, uint32_t y) { return (x & 0xffffu) | (y << 16); }
__device__ __forceinline__ uint32_t tf_pack_hi(uint32_t x, uint32_t y) { return (x >> 16) | (y & 0xffff0000u); }
__device__ __forceinline__ uint32_t tf_dword(const uint4& v, int i) {
  return i == 0 ? v.x : (i == 1 ? v.y : (i == 2 ? v.z : v.w));
}
__device__ __forceinline__ uint32_t tf_pack_bf16(float a, float b) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, r);
}

constexpr int kQTile = 128;   // query rows per work-group
constexpr int kKTile = 64;    // keys per iteration

}  // namespace

__global__ __launch_bounds__(256, 2) void seer_attn_fwd_kernel(TrainFwdParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char kbuf[2][kKTile * 256];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, q4 = lane >> 4;
  const int qt = (int)gridDim.x - 1 - (int)blockIdx.x;      // the tiles with the most keys first
  const int h = blockIdx.y, i = blockIdx.z, hk = h / p.g;
  int S = p.T;
  if (p.seqlens) {
    S = p.seqlens[i];
    S = S < 0 ? 0 : (S > p.T ? p.T : S);
  }
  const int r0 = qt * kQTile;
  const int wrow0 = r0 + 32 * wave;

  // ---- rows of this lane and their Q^T operands -------------------------------------------------
  int qrow[2];
  uint4 qb[2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    qrow[a] = wrow0 + 16 * a + n16;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      qb[a][kk] = make_uint4(0, 0, 0, 0);
      if (qrow[a] < p.T)
        qb[a][kk] = *reinterpret_cast<const uint4*>(p.q + (((int64_t)i * p.T + qrow[a]) * p.Hq + h) * kHeadDim +
                                                    kk * 32 + q4 * 8);
    }
  }

  const uint16_t* kbase = p.k + (int64_t)i * p.stride_seq + (int64_t)hk * p.stride_head;
  const uint16_t* vbase = p.v + (int64_t)i * p.stride_seq + (int64_t)hk * p.stride_head;
  const int64_t st = p.stride_token;
  int kend = r0 + kQTile;                    // keys [0, kend) matter to this work-group
  kend = kend < S ? kend : S;
  int wave_end = wrow0 + 32;                 // keys [0, wave_end) matter to this wave
  wave_end = wave_end < S ? wave_end : S;
  if (r0 >= S) {                             // a tile of padding rows: nothing to read
    kend = 0;
    wave_end = 0;
  }
  const int ntiles = (kend + kKTile - 1) / kKTile;

  // K tile staging: thread covers rows 16*u + tid/16, 16-byte chunk tid%16
  const int srow = tid >> 4, schunk = tid & 15;
  uint4 kreg[4];
  auto load_ktile = [&](int kt0) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int key = kt0 + 16 * u + srow;
      kreg[u] = make_uint4(0, 0, 0, 0);
      if (key < p.T) kreg[u] = *reinterpret_cast<const uint4*>(kbase + (int64_t)key * st + schunk * 8);
    }
  };
  auto store_ktile = [&](int buf) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = 16 * u + srow;
      *reinterpret_cast<uint4*>(kbuf[buf] + row * 256 + ((schunk ^ (row & 15)) << 4)) = kreg[u];
    }
  };
  // V rows of a 32-key chunk: load j covers key tau(q4, j) = j < 4 ? 4*q4 + j : 16 + 4*q4 + (j - 4)
  uint4 vr[8];
  auto load_v = [&](int key0) {
    const uint16_t* base = vbase + n16 * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int key = key0 + ((j < 4) ? 4 * q4 + j : 16 + 4 * q4 + (j - 4));
      vr[j] = make_uint4(0, 0, 0, 0);
      if (key < p.T) vr[j] = *reinterpret_cast<const uint4*>(base + (int64_t)key * st);
    }
  };

  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f}, bmax[2] = {-INFINITY, -INFINITY};
  f32x4_t oacc[2][8];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 8; ++e) oacc[a][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  if (ntiles > 0) {
    load_ktile(0);
    store_ktile(0);
    if (wave_end > 0) load_v(0);
  }
  __syncthreads();

  float* rawbase = p.raw + ((int64_t)i * p.Hq + h) * p.nb * (int64_t)p.Tp;

  for (int it = 0; it < ntiles; ++it) {
    const int kt0 = it * kKTile;
    const bool more = it + 1 < ntiles;
    if (more) load_ktile(kt0 + kKTile);
    const unsigned char* kt = kbuf[it & 1];

#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int key0 = kt0 + 32 * c;
      if (key0 < wave_end) {                 // wave-uniform: some row of this wave sees the chunk
        // ---- S^T = K Q^T -----------------------------------------------------------------------
        f32x4_t sacc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int t = 0; t < 2; ++t) sacc[a][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int row = 32 * c + 16 * t + n16;
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            const uint4 ka = *reinterpret_cast<const uint4*>(kt + row * 256 + (((kk * 4 + q4) ^ n16) << 4));
#pragma unroll
            for (int a = 0; a < 2; ++a)
              sacc[a][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka),
                                                                   __builtin_bit_cast(bf16x8_t, qb[a][kk]),
                                                                   sacc[a][t], 0, 0, 0);
          }
        }

        // ---- online softmax per query tile; lane holds keys key0 + 16t + 4*q4 + r of row qrow[a] ---
        uint4 pb[2];
        const int jblk = key0 / p.block_size;
        const bool blk_start = (key0 % p.block_size) == 0;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          float x[8];
#pragma unroll
          for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) x[4 * t + r] = sacc[a][t][r] * p.scale_log2e;
          if (key0 + 31 > wrow0 + 16 * a) {  // the diagonal passes through this chunk for some row
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (key0 + 16 * t + 4 * q4 + r > qrow[a]) x[4 * t + r] = -INFINITY;
          }
          float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          // block maximum of the logits of this row (Sec. 2.3: the row maxima are reused)
          bmax[a] = blk_start ? mx : fmaxf(bmax[a], mx);
          if (q4 == 0 && qrow[a] < p.T) rawbase[(int64_t)jblk * p.Tp + qrow[a]] = bmax[a];

          const float m_new = fmaxf(m_run[a], mx);
          const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
          const float alpha = __builtin_amdgcn_exp2f(m_run[a] - m_ref);
          float pr[8], psum = 0.f;
#pragma unroll
          for (int cc = 0; cc < 8; ++cc) {
            pr[cc] = __builtin_amdgcn_exp2f(x[cc] - m_ref);
            psum += pr[cc];
          }
          l_run[a] = l_run[a] * alpha + psum;
          m_run[a] = m_new;
          if (__ballot(alpha != 1.0f)) {
#pragma unroll
            for (int e = 0; e < 8; ++e) oacc[a][e] *= alpha;
          }
          pb[a] = make_uint4(tf_pack_bf16(pr[0], pr[1]), tf_pack_bf16(pr[2], pr[3]), tf_pack_bf16(pr[4], pr[5]),
                             tf_pack_bf16(pr[6], pr[7]));
        }

        // ---- O^T += V^T P^T ---------------------------------------------------------------------
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          uint32_t o[4];
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const uint32_t x0 = tf_dword(vr[2 * jj], e >> 1), x1 = tf_dword(vr[2 * jj + 1], e >> 1);
            o[jj] = (e & 1) ? tf_pack_hi(x0, x1) : tf_pack_lo(x0, x1);
          }
          const uint4 va = make_uint4(o[0], o[1], o[2], o[3]);
#pragma unroll
          for (int a = 0; a < 2; ++a)
            oacc[a][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, va),
                                                                 __builtin_bit_cast(bf16x8_t, pb[a]), oacc[a][e],
                                                                 0, 0, 0);
        }
        if (key0 + 32 < wave_end) load_v(key0 + 32);
      }
    }

    if (more) store_ktile((it + 1) & 1);
    __syncthreads();
  }

  // ---- results: lane (n16, q4) holds O[row n16 of tile a][32*q4 + 8*r + e] in oacc[a][e][r] ---------
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    float l = l_run[a];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const int row = qrow[a];
    if (row >= p.T) continue;
    const bool real = row < S;
    const float inv = (real && l > 0.f) ? 1.0f / l : 0.f;
    const int64_t orow = ((int64_t)i * p.T + row) * p.Hq + h;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int c0 = 32 * q4 + 8 * r;
      if (p.out_is_f32) {
        float* dst = reinterpret_cast<float*>(p.out) + orow * kHeadDim + c0;
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e] = oacc[a][e][r] * inv;
      } else {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2)
          w[e >> 1] = (uint32_t)f32_to_bf16_rne(oacc[a][e][r] * inv) |
                      ((uint32_t)f32_to_bf16_rne(oacc[a][e + 1][r] * inv) << 16);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(p.out) + orow * kHeadDim + c0) =
            make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
    if (q4 == 0) {
      const float l2 = (real && l > 0.f) ? m_run[a] + log2f(l) : -INFINITY;
      p.lse2[((int64_t)i * p.Hq + h) * p.T + row] = l2;
      if (p.lse) p.lse[orow] = l2 * 0.6931471805599453f;
    }
  }
}

// Grid (ceil(T/64), Hkv, B), 256 threads: thread (tq = tid % 64, part = tid / 64).
__global__ __launch_bounds__(256) void seer_gt_finalize_kernel(TrainFwdParams p) {
  __shared__ float part_sum[4][64];
  __shared__ float tile[64][65];

  const int tid = threadIdx.x, tq = tid & 63, part = tid >> 6;
  const int t0 = blockIdx.x * 64, hk = blockIdx.y, i = blockIdx.z;
  int S = p.T;
  if (p.seqlens) {
    S = p.seqlens[i];
    S = S < 0 ? 0 : (S > p.T ? p.T : S);
  }
  const int t = t0 + tq;
  const bool real = t < S;
  const int nvis = real ? t / p.block_size + 1 : 0;        // blocks with a key s <= t
  int tile_last = t0 + 63;
  tile_last = tile_last < S - 1 ? tile_last : S - 1;
  const int nvis_tile = tile_last >= t0 ? tile_last / p.block_size + 1 : 0;

  const int g = p.g;
  float l2[kMaxGroup];
#pragma unroll
  for (int hh = 0; hh < kMaxGroup; ++hh)
    l2[hh] = (hh < g && real) ? p.lse2[((int64_t)i * p.Hq + hk * g + hh) * p.T + t] : 0.f;
  const float* raw0 = p.raw + ((int64_t)i * p.Hq + (int64_t)hk * g) * p.nb * (int64_t)p.Tp;
  auto block_prob = [&](int j) -> float {   // max over the heads of the block's largest probability
    float r = 0.f;
    for (int hh = 0; hh < g; ++hh) {
      const float x = raw0[((int64_t)hh * p.nb + j) * p.Tp + t];
      r = fmaxf(r, exp2f(x - l2[hh]));
    }
    return r;
  };

  float sum = 0.f;
  for (int j = part; j < nvis; j += 4) sum += block_prob(j);
  part_sum[part][tq] = sum;
  __syncthreads();
  const float total = part_sum[0][tq] + part_sum[1][tq] + part_sum[2][tq] + part_sum[3][tq];
  const float inv = total > 0.f ? 1.0f / total : 0.f;

  float* gbase = p.gt + (((int64_t)i * p.Hkv + hk) * p.T) * (int64_t)p.nb;
  for (int j0 = 0; j0 < p.nb; j0 += 64) {
    if (j0 < nvis_tile) {
      // rows of the tile in parallel, 16 blocks per thread; then transposed out
      for (int u = 0; u < 16; ++u) {
        const int jj = part * 16 + u, j = j0 + jj;
        tile[tq][jj] = (j < nvis) ? block_prob(j) * inv : 0.f;
      }
      __syncthreads();
      for (int u = 0; u < 16; ++u) {
        const int row = part * 16 + u, j = j0 + tq;
        if (t0 + row < p.T && j < p.nb) gbase[(int64_t)(t0 + row) * p.nb + j] = tile[row][tq];
      }
      __syncthreads();
    } else {
      for (int u = 0; u < 16; ++u) {
        const int row = part * 16 + u, j = j0 + tq;
        if (t0 + row < p.T && j < p.nb) gbase[(int64_t)(t0 + row) * p.nb + j] = 0.f;
      }
    }
  }
}

hipError_t launch_attn_fwd(const TrainFwdParams& p, hipStream_t s) {
  const dim3 grid((p.T + kQTile - 1) / kQTile, p.Hq, p.B);
  hipLaunchKernelGGL(seer_attn_fwd_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_gt_finalize(const TrainFwdParams& p, hipStream_t s) {
  const dim3 grid((p.T + 63) / 64, p.Hkv, p.B);
  hipLaunchKernelGGL(seer_gt_finalize_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace seer
