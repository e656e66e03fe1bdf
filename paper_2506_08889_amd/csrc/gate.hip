// AttnGate block selection on gfx950: gate scores against the K Compression Cache (Eq. 1c,
// Sec. 3.2) and token-budget top-k / threshold selection (Sec. 3.1).
//
// Scores are accumulated in fp64 from exactly converted bf16 inputs: a bf16 x bf16 product
// has a 16-bit significand, so each fp64 FMA adds an exact product and the sum is the exact
// dot product unless the exponents of the 128 terms spread over more than ~30 bits.  That
// makes the order of equal-looking scores independent of summation order, which is what a
// bit-exact index list needs.
#include "seer_internal.h"

namespace seer {

// ---------------------------------------------------------------------------------------
// Score kernel.  One kc row is 256 bytes: 16 lanes x one 128-bit load, so a wavefront
// reads 4 rows per load instruction, fully coalesced.  Work-group = 4 waves x 4 loads in
// flight x 4 rows = 64 rows.  Memory-bound: 256 B per score.
// ---------------------------------------------------------------------------------------
constexpr int kScoreRowsPerWg = 64;

__global__ __launch_bounds__(256) void seer_gate_score_kernel(GateParams p) {
  const int i = blockIdx.z, h = blockIdx.y;
  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  int nfull = S / p.block_size;
  nfull = nfull < p.nb_max ? nfull : p.nb_max;
  const int j0 = blockIdx.x * kScoreRowsPerWg;
  if (j0 >= nfull) return;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int slot = lane >> 4, c = lane & 15;
  const int64_t grp = (int64_t)i * p.Hkv + h;

  const uint4 qr = *reinterpret_cast<const uint4*>(p.q_gate + grp * kHeadDim + c * 8);
  double qd[8];
  {
    const uint32_t w[4] = {qr.x, qr.y, qr.z, qr.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      qd[2 * e] = (double)bf16_lo(w[e]);
      qd[2 * e + 1] = (double)bf16_hi(w[e]);
    }
  }

  const uint16_t* base = p.kc + (int64_t)i * p.kc_stride_batch + (int64_t)h * p.kc_stride_head;
  uint4 kr[4];
  int jj[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    jj[it] = j0 + wave * 16 + it * 4 + slot;
    kr[it] = make_uint4(0, 0, 0, 0);
    if (jj[it] < nfull)
      kr[it] = *reinterpret_cast<const uint4*>(base + (int64_t)jj[it] * p.kc_stride_block + c * 8);
  }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const uint32_t w[4] = {kr[it].x, kr[it].y, kr[it].z, kr[it].w};
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc = fma((double)bf16_lo(w[e]), qd[2 * e], acc);
      acc = fma((double)bf16_hi(w[e]), qd[2 * e + 1], acc);
    }
    // sum over the 16 lanes that share a row
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    acc += __shfl_xor(acc, 8);
    if (c == 0 && jj[it] < nfull) p.scores[grp * p.nb_max + jj[it]] = acc + 0.0;  // -0 -> +0
  }
}

// ---------------------------------------------------------------------------------------
// Select kernel: one work-group per (sequence, kv head).
//   top-k:     radix select (8 passes of 8 bits over order-preserving 64-bit keys) finds the
//              k-th largest score and how many blocks equal to it are still needed; an
//              ordered compaction then emits, in ascending block order, every block above
//              it plus the first `need` blocks equal to it (lowest index wins a tie).
//   threshold: fp64 softmax over the full blocks (max, sum of exp, divide) and the same
//              ordered compaction on S_j > tau.
// The scores of one group are at most a few thousand doubles and stay in L2 across passes.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t score_key(double s) {
  const uint64_t b = (uint64_t)__double_as_longlong(s);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

__device__ __forceinline__ double wg_reduce_max(double x, double* sm) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmax(x, __shfl_xor(x, o));
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[wave] = x;
  __syncthreads();
  return fmax(fmax(sm[0], sm[1]), fmax(sm[2], sm[3]));
}

__device__ __forceinline__ double wg_reduce_sum(double x, double* sm) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[wave] = x;
  __syncthreads();
  return (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

__global__ __launch_bounds__(256) void seer_gate_select_kernel(GateParams p) {
  __shared__ int hist[256];
  __shared__ int scan[256];
  __shared__ int wcnt[2][4];
  __shared__ int digit_sel[2];
  __shared__ double red[4];

  const int i = blockIdx.y, h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t grp = (int64_t)i * p.Hkv + h;
  int32_t* out = p.block_idx + grp * p.max_sel;
  const double* sc = p.scores + grp * p.nb_max;

  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  int nfull = S / p.block_size;
  int nb = (S + p.block_size - 1) / p.block_size;
  if (nb > p.nb_max) { nb = p.nb_max; nfull = nfull < nb ? nfull : nb; }
  const bool partial = nb > nfull;

  // ---- decide what "selected" means -----------------------------------------------------
  uint64_t T = ~0ull;      // top-k: key of the k-th largest score
  int need_eq = 0;         // top-k: how many blocks equal to T are taken
  int from_full = 0;
  bool force_last = partial;
  double m = 0.0, Z = 1.0;

  if (p.mode == 0) {
    long long k = p.budget_blocks ? (long long)p.budget_blocks[i]
                                  : ((long long)p.budget_tokens + p.block_size - 1) / p.block_size;
    k = k < 0 ? 0 : k;
    k = k > nb ? nb : k;
    k = k > p.max_sel ? p.max_sel : k;
    from_full = (int)k;
    if (partial && k > 0) from_full = (int)k - 1;
    from_full = from_full > nfull ? nfull : from_full;
    force_last = partial && k > 0;

    if (from_full > 0) {
      uint64_t prefix = 0, mask = 0;
      int remaining = from_full;
      for (int pass = 7; pass >= 0; --pass) {
        const int shift = pass * 8;
        hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < nfull; j += 256) {
          const uint64_t key = score_key(sc[j]);
          if ((key & mask) == prefix) atomicAdd(&hist[(int)((key >> shift) & 0xff)], 1);
        }
        __syncthreads();
        // suffix sums over digits: scan[d] = number of candidates with digit >= d
        scan[tid] = hist[tid];
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {
          int add = (tid + o < 256) ? scan[tid + o] : 0;
          __syncthreads();
          scan[tid] += add;
          __syncthreads();
        }
        const int above = (tid < 255) ? scan[tid + 1] : 0;
        if (above < remaining && remaining <= scan[tid]) {   // exactly one digit satisfies this
          digit_sel[0] = tid;
          digit_sel[1] = remaining - above;
        }
        __syncthreads();
        prefix |= (uint64_t)digit_sel[0] << shift;
        mask |= 0xffull << shift;
        remaining = digit_sel[1];
        __syncthreads();
      }
      T = prefix;
      need_eq = remaining;
    }
  } else {
    if (nfull > 0) {
      double mx = -INFINITY;
      for (int j = tid; j < nfull; j += 256) mx = fmax(mx, __dmul_rn(sc[j], p.inv_sqrt_dg));
      m = wg_reduce_max(mx, red);
      double z = 0.0;
      for (int j = tid; j < nfull; j += 256) z += exp(__dsub_rn(__dmul_rn(sc[j], p.inv_sqrt_dg), m));
      Z = wg_reduce_sum(z, red);
    }
  }

  // ---- ordered compaction -----------------------------------------------------------------
  int run_gt = 0, run_eq = 0;
  const bool any_full = (p.mode == 0) ? (from_full > 0) : (nfull > 0);
  if (any_full) {
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    for (int base = 0; base < nfull; base += 256) {
      const int j = base + tid;
      bool gt = false, eq = false;
      if (j < nfull) {
        const double s = sc[j];
        if (p.mode == 0) {
          const uint64_t key = score_key(s);
          gt = key > T;
          eq = key == T;
        } else {
          const double Sj = __ddiv_rn(exp(__dsub_rn(__dmul_rn(s, p.inv_sqrt_dg), m)), Z);
          gt = Sj > p.threshold;
        }
      }
      const uint64_t bg = __ballot(gt), be = __ballot(eq);
      const int pg = __popcll(bg & lt_mask), pe = __popcll(be & lt_mask);
      __syncthreads();
      if (lane == 0) { wcnt[0][wave] = __popcll(bg); wcnt[1][wave] = __popcll(be); }
      __syncthreads();
      int og = 0, oe = 0, tg = 0, te = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int a = wcnt[0][w], b = wcnt[1][w];
        if (w < wave) { og += a; oe += b; }
        tg += a; te += b;
      }
      const int eq_before = run_eq + oe + pe;
      const bool take = gt || (eq && eq_before < need_eq);
      const int pos = run_gt + og + pg + (eq_before < need_eq ? eq_before : need_eq);
      if (take && pos < p.max_sel) out[pos] = j;
      run_gt += tg;
      run_eq += te;
    }
  }
  int n = run_gt + (run_eq < need_eq ? run_eq : need_eq);
  n = n < p.max_sel ? n : p.max_sel;
  if (force_last && n < p.max_sel) {
    if (tid == 0) out[n] = nb - 1;
    n += 1;
  }
  for (int q = n + tid; q < p.max_sel; q += 256) out[q] = -1;
  if (tid == 0) p.nblk[grp] = n;
}

hipError_t launch_gate_score(const GateParams& p, hipStream_t s) {
  dim3 grid((p.nb_max + kScoreRowsPerWg - 1) / kScoreRowsPerWg, p.Hkv, p.B);
  hipLaunchKernelGGL(seer_gate_score_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_gate_select(const GateParams& p, hipStream_t s) {
  dim3 grid(p.Hkv, p.B);
  hipLaunchKernelGGL(seer_gate_select_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace seer
