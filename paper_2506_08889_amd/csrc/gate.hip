// AttnGate block selection on gfx950: gate scores against the K Compression Cache (Eq. 1c,
// Sec. 3.2) and token-budget top-k / threshold selection (Sec. 3.1), plus top-p (Sec. 6.2).
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

// ---------------------------------------------------------------------------------------
// Cross-lane steps on the VALU's data-parallel lane moves (no trip through the LDS crossbar, so a
// chain of them costs tens of cycles instead of many hundreds).  Controls: quad_perm [1,0,3,2] = 0xB1,
// quad_perm [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140, row_shr:n = 0x110 + n.
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ int lane_move_i32(int x) {     // lanes without a source lane receive 0
  return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ double lane_move_f64(double x) {
  return __hiloint2double(lane_move_i32<CTRL>(__double2hiint(x)), lane_move_i32<CTRL>(__double2loint(x)));
}
__device__ __forceinline__ double readlane_f64(double x, int l) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l), __builtin_amdgcn_readlane(__double2loint(x), l));
}
// Sum / maximum over each row of 16 lanes, delivered to all 16 (pairs, quads, halves, row: the same tree
// in every lane, so all 16 hold the same bits).
__device__ __forceinline__ double row16_sum_f64(double x) {
  x += lane_move_f64<0xB1>(x);
  x += lane_move_f64<0x4E>(x);
  x += lane_move_f64<0x141>(x);
  x += lane_move_f64<0x140>(x);
  return x;
}
__device__ __forceinline__ double row16_max_f64(double x) {
  x = fmax(x, lane_move_f64<0xB1>(x));
  x = fmax(x, lane_move_f64<0x4E>(x));
  x = fmax(x, lane_move_f64<0x141>(x));
  x = fmax(x, lane_move_f64<0x140>(x));
  return x;
}
// ... and over the 64 lanes of a wave (uniform result).
__device__ __forceinline__ double wave_sum_f64(double x) {
  x = row16_sum_f64(x);
  return (readlane_f64(x, 0) + readlane_f64(x, 16)) + (readlane_f64(x, 32) + readlane_f64(x, 48));
}
__device__ __forceinline__ double wave_max_f64(double x) {
  x = row16_max_f64(x);
  return fmax(fmax(readlane_f64(x, 0), readlane_f64(x, 16)), fmax(readlane_f64(x, 32), readlane_f64(x, 48)));
}
// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ int wave_inclusive_scan_i32(int x) {
  x += lane_move_i32<0x111>(x);
  x += lane_move_i32<0x112>(x);
  x += lane_move_i32<0x114>(x);
  x += lane_move_i32<0x118>(x);
  const int r0 = __builtin_amdgcn_readlane(x, 15), r1 = __builtin_amdgcn_readlane(x, 31), r2 = __builtin_amdgcn_readlane(x, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return x + (row >= 1 ? r0 : 0) + (row >= 2 ? r1 : 0) + (row >= 3 ? r2 : 0);
}

// The query of a group as 8 fp64 values per lane (lane c of 16 holds features 8c .. 8c+7).
__device__ __forceinline__ void load_gate_query(const uint16_t* q_row, int c, double (&qd)[8]) {
  const uint4 qr = *reinterpret_cast<const uint4*>(q_row + c * 8);
  const uint32_t w[4] = {qr.x, qr.y, qr.z, qr.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    qd[2 * e] = (double)bf16_lo(w[e]);
    qd[2 * e + 1] = (double)bf16_hi(w[e]);
  }
}

// Score of one cache row: each of the 16 lanes that share the row holds 8 of its features in `kr`;
// exact bf16 products accumulated by fp64 FMAs, then summed over the 16 lanes.  Every lane of the 16
// returns the score (-0 folded into +0 so that equal scores have equal bit patterns).
__device__ __forceinline__ double gate_row_score(const uint4& kr, const double (&qd)[8]) {
  const uint32_t w[4] = {kr.x, kr.y, kr.z, kr.w};
  double acc = 0.0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    acc = fma((double)bf16_lo(w[e]), qd[2 * e], acc);
    acc = fma((double)bf16_hi(w[e]), qd[2 * e + 1], acc);
  }
  return row16_sum_f64(acc) + 0.0;
}

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

  double qd[8];
  load_gate_query(p.q_gate + grp * kHeadDim, c, qd);

  const uint16_t* base = p.kc + (int64_t)i * p.kc_stride_batch + (int64_t)h * p.kc_stride_head;
  uint4 kr[4];
  int jj[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    jj[it] = j0 + wave * 16 + it * 4 + slot;
    kr[it] = make_uint4(0, 0, 0, 0);
    if (jj[it] < nfull)
      kr[it] = load_stream16(base + (int64_t)jj[it] * p.kc_stride_block + c * 8);
  }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const double sc = gate_row_score(kr[it], qd);
    if (c == 0 && jj[it] < nfull) p.scores[grp * p.nb_max + jj[it]] = sc;
  }
}

// The same scores for batches whose sequences differ widely in length: at most 8 work-groups per
// (sequence, kv head), each walking every 8th tile of 64 cache rows with the next tile requested before
// the current one is reduced.  With one work-group per tile of the longest sequence most of them would
// start past the end of their own cache (c5: 23 of 33 thousand) and only hold a slot while they find
// that out; equal-length batches are faster with the one-tile work-groups above.
__global__ __launch_bounds__(256) void seer_gate_score_walk_kernel(GateParams p) {
  const int i = blockIdx.z, h = blockIdx.y;
  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  int nfull = S / p.block_size;
  nfull = nfull < p.nb_max ? nfull : p.nb_max;
  const int j_first = blockIdx.x * kScoreRowsPerWg;
  if (j_first >= nfull) return;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int slot = lane >> 4, c = lane & 15;
  const int64_t grp = (int64_t)i * p.Hkv + h;

  double qd[8];
  load_gate_query(p.q_gate + grp * kHeadDim, c, qd);

  const uint16_t* base = p.kc + (int64_t)i * p.kc_stride_batch + (int64_t)h * p.kc_stride_head;
  const int step = gridDim.x * kScoreRowsPerWg;       // the work-groups of a group interleave their tiles
  const int r = wave * 16 + slot;                     // this lane's row within a tile, + 4 * it
  uint4 kr[4], kn[4];
  auto load_tile = [&](int j0, uint4 (&dst)[4]) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int j = j0 + r + it * 4;
      dst[it] = make_uint4(0, 0, 0, 0);
      if (j < nfull) dst[it] = load_stream16(base + (int64_t)j * p.kc_stride_block + c * 8);
    }
  };
  load_tile(j_first, kr);
  for (int j0 = j_first; j0 < nfull; j0 += step) {
    const bool more = j0 + step < nfull;
    if (more) load_tile(j0 + step, kn);               // the next tile is in flight during the reduction
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const double sc = gate_row_score(kr[it], qd);
      const int j = j0 + r + it * 4;
      if (c == 0 && j < nfull) p.scores[grp * p.nb_max + j] = sc;
    }
    if (more) {
#pragma unroll
      for (int it = 0; it < 4; ++it) kr[it] = kn[it];
    }
  }
}

// ---------------------------------------------------------------------------------------
// Select kernel: one work-group per (sequence, kv head).  The scores of the group are first
// brought into LDS (up to kSelectLdsBlocks of them; longer caches are re-read from L2).
//   top-k:     fast path - scores binned linearly between their minimum and maximum (monotone,
//              and evenly filled, so LDS atomics do not pile up), one scan finds the bin holding
//              the k-th largest score, blocks in higher bins are taken and the few blocks of the
//              boundary bin are ranked exactly against each other (key, then lower index).
//              Fallback (crowded boundary bin, i.e. many equal scores; or scores left in global
//              memory) - radix select over order-preserving 64-bit keys, 8 bits per pass from the
//              top: LDS histogram of the still-undecided candidates, the first wave scans the 256
//              bins (4 per lane, descending) and picks the digit that holds the k-th largest key;
//              it stops as soon as every candidate left in that bin is needed; after all 8 passes
//              the k-th key is known exactly and `need_eq` of its duplicates are taken, lowest
//              index first.
//   threshold: fp64 softmax over the full blocks (max, sum of exp, divide), S_j > tau.
//   top-p:     the radix walk steered by probability mass (2^-62 fixed point, exact sums).
//   Either way an ordered compaction emits the ascending list: thread t owns blocks t, t + 256, ...;
//   per row of 256 blocks a wave ballot ranks the hits inside the wave and the four waves' counts, laid
//   out in LDS, give the offset of every (row, wave) - one barrier, every score classified once.
// A work-group has two waves per SIMD at most, so nothing hides instruction latency here: reductions
// and scans inside a wave run on lane moves in the VALU (see the helpers above), every work-group step
// costs one barrier, and state is cleared while the scores are still on their way.
// ---------------------------------------------------------------------------------------
constexpr int kSelectLdsBlocks = 8192;
constexpr int kLinBins = 1024;    // top-k fast path: bins over [min score, max score]
constexpr int kMaxCand = 256;     // ... and the most blocks its boundary bin may hold
constexpr int kMaxOwn = kSelectLdsBlocks / 256;   // blocks per thread and pass of the ordered compaction

__device__ __forceinline__ uint64_t score_key(double s) {
  const uint64_t b = (uint64_t)__double_as_longlong(s);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

// Linear bin of a score between the group's minimum and maximum: monotone non-decreasing in s.
__device__ __forceinline__ int lin_bin_of(double s, double lo, double scale) {
  const int b = (int)__dmul_rn(__dsub_rn(s, lo), scale);
  return b < 0 ? 0 : (b > kLinBins - 1 ? kLinBins - 1 : b);
}

// f(j, score) for the blocks j = t, t + 256, ... < n of thread t, four scores requested at a time
// (a loop with one LDS or L2 read per trip would wait out the read's latency on every trip).
template <typename F>
__device__ __forceinline__ void for_own_scores(const double* sc, int first, int n, F f) {
  for (int j0 = first + (int)threadIdx.x; j0 < n; j0 += 4 * 256) {
    double v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 256;
      v[u] = j < n ? sc[j] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 256;
      if (j < n) f(j, v[u]);
    }
  }
}

// Work-group (4 waves) reductions: one barrier each; every call gets LDS slots of its own (`sm`, 4
// doubles per value) so that no barrier is needed before the slots are written.
__device__ __forceinline__ void wg_reduce_max2(double& a, double& b, double* sm /* [8] */) {
  a = wave_max_f64(a);
  b = wave_max_f64(b);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sm[wave] = a; sm[4 + wave] = b; }
  __syncthreads();
  a = fmax(fmax(sm[0], sm[1]), fmax(sm[2], sm[3]));
  b = fmax(fmax(sm[4], sm[5]), fmax(sm[6], sm[7]));
}

__device__ __forceinline__ double wg_reduce_max(double x, double* sm /* [4] */) {
  x = wave_max_f64(x);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = x;
  __syncthreads();
  return fmax(fmax(sm[0], sm[1]), fmax(sm[2], sm[3]));
}

__device__ __forceinline__ double wg_reduce_sum(double x, double* sm /* [4] */) {
  x = wave_sum_f64(x);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = x;
  __syncthreads();
  return (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

// Exclusive prefix over the 256 threads of a per-thread count (one barrier; `sm` = 4 ints of its own).
__device__ __forceinline__ int wg_exclusive_scan(int a, int* sm /* [4] */) {
  const int wave = threadIdx.x >> 6;
  const int incl = wave_inclusive_scan_i32(a);
  if ((threadIdx.x & 63) == 63) sm[wave] = incl;
  __syncthreads();
  int before = 0;
#pragma unroll
  for (int w = 0; w < 3; ++w) before += (w < wave) ? sm[w] : 0;
  return before + incl - a;
}

// Ranks, in block order, of the blocks whose bit is set: thread t holds bit u for block c0 + 256 u + t
// (u < rows <= 32).  Calls f(u, rank) for every set bit of the calling thread and returns the number of
// set bits of the whole work-group.  One barrier; `rowcnt` = 128 ints, not in use by anyone else until
// the next barrier after the call.
template <typename F>
__device__ __forceinline__ int ordered_ranks(uint32_t bits, int rows, int* rowcnt, F f) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int u = 0; u < rows; ++u) {
    const unsigned long long b = __ballot((bits >> u) & 1u);
    if (lane == 0) rowcnt[u * 4 + wave] = __popcll(b);
  }
  __syncthreads();
  int run = 0;
  for (int u0 = 0; u0 < rows; u0 += 4) {      // four rows' counts requested at a time
    int4 c[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) c[k] = reinterpret_cast<const int4*>(rowcnt)[(u0 + k) & (kMaxOwn - 1)];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int u = u0 + k;
      if (u < rows) {                         // uniform
        const int off = run + (wave > 0 ? c[k].x : 0) + (wave > 1 ? c[k].y : 0) + (wave > 2 ? c[k].z : 0);
        run += (c[k].x + c[k].y) + (c[k].z + c[k].w);
        const unsigned long long b = __ballot((bits >> u) & 1u);
        if ((bits >> u) & 1u)
          f(u, off + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0u)));
      }
    }
  }
  return run;
}

// SRC: 0 = scores stay in global memory (cache longer than the LDS budget), 1 = scores of the
// score kernel are copied into LDS, 2 = fused: this kernel computes the scores itself, straight
// into LDS (one launch, no score workspace traffic).
// NT: threads per work-group while the fused form streams the cache rows (256 or 1024; the waves beyond
// the first four end before the selection starts, which runs on 256 threads in every form).
template <int SRC, int NT = 256>
__global__ __launch_bounds__(NT) void seer_gate_select_kernel(GateParams p) {
  static_assert(SRC == 2 || NT == 256, "only the fused form streams with more than four waves");
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
  __shared__ int hist[256];
  __shared__ unsigned long long mass[256];   // top-p: fixed-point probability mass per digit
  __shared__ unsigned long long mass_sel[2];
  __shared__ int wcnt[4];
  __shared__ __attribute__((aligned(16))) int rowcnt[4 * kMaxOwn];
  __shared__ int digit_sel[3];
  __shared__ double red[16];
  __shared__ int lin_hist[kLinBins];           // top-k fast path: linear-bin histogram
  __shared__ unsigned long long cand_key[kMaxCand];
  __shared__ int cand_idx[kMaxCand];
  __shared__ int cand_n;

  const int i = blockIdx.y, h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t grp = (int64_t)i * p.Hkv + h;
  int32_t* out = p.block_idx + grp * p.max_sel;
  const double* sc_g = p.scores + grp * p.nb_max;

  int S = p.seqlens[i];
  long long k_blocks = (p.mode == 0 && p.budget_blocks) ? (long long)p.budget_blocks[i] : 0;
  if (SRC != 0 && p.mode == 0) {        // top-k fast path state, cleared while the scores are on their way
    for (int b = tid; b < kLinBins; b += NT) lin_hist[b] = 0;
    if (tid == 0) cand_n = 0;
  }
  const double* sc = sc_g;
  if (SRC == 1) {
    // every score slot of the group is requested before the sequence length has arrived (one memory
    // round trip instead of two); slots past the last full block hold whatever the workspace held and
    // are never looked at
    double* sl = reinterpret_cast<double*>(dyn_smem);
    for_own_scores(sc_g, 0, p.nb_max, [&](int j, double v) { sl[j] = v; });
    sc = sl;
  }
  S = S < 0 ? 0 : S;
  int nfull = S / p.block_size;
  int nb = (S + p.block_size - 1) / p.block_size;
  if (nb > p.nb_max) { nb = p.nb_max; nfull = nfull < nb ? nfull : nb; }
  const bool partial = nb > nfull;
  if (SRC == 1) __syncthreads();
  if (SRC == 2) {
    // Stream the group's cache rows: 16 lanes per 256-byte row, 4 rows per wave and load, 8 loads
    // (32 KiB per work-group) per step, the next step's loads issued before the current reduction.
    double* sl = reinterpret_cast<double*>(dyn_smem);
    const int slot = lane >> 4, c = lane & 15;
    double qd[8];
    load_gate_query(p.q_gate + grp * kHeadDim, c, qd);
    const uint16_t* base = p.kc + (int64_t)i * p.kc_stride_batch + (int64_t)h * p.kc_stride_head + c * 8;
    constexpr int kU = NT == 1024 ? 4 : 8;       // loads in flight per lane and step
    constexpr int kRowsPerLoad = NT / 16;        // 4 rows per wave
    constexpr int kRowsPerStep = kU * kRowsPerLoad;
    uint4 kr[kU], kn[kU];
    auto load_rows = [&](int j0, uint4 (&dst)[kU]) {
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int jl = j0 + u * kRowsPerLoad + wave * 4 + slot;
        dst[u] = make_uint4(0, 0, 0, 0);
        if (jl < nfull) dst[u] = load_stream16(base + (int64_t)jl * p.kc_stride_block);
      }
    };
    load_rows(0, kr);
    for (int j0 = 0; j0 < nfull; j0 += kRowsPerStep) {
      const bool more = j0 + kRowsPerStep < nfull;
      if (more) load_rows(j0 + kRowsPerStep, kn);   // the next rows are in flight during the reduction
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int jl = j0 + u * kRowsPerLoad + wave * 4 + slot;
        const double sc = gate_row_score(kr[u], qd);
        if (c == 0 && jl < nfull) sl[jl] = sc;
      }
      if (more) {
#pragma unroll
        for (int u = 0; u < kU; ++u) kr[u] = kn[u];
      }
    }
    __syncthreads();
    if (NT > 256 && tid >= 256) return;          // a barrier waits only for the waves that still run
    sc = sl;
  }

  // ---- decide what "selected" means -----------------------------------------------------
  uint64_t T = ~0ull;      // top-k: selected if key > T, or key == T among the first need_eq
  int need_eq = 0;
  bool take_ge = false;    // top-k, early exit: selected if key >= T
  int from_full = 0;
  bool force_last = partial;
  double m = 0.0, Z = 1.0;
  bool lin_fast = false;   // top-k fast path taken: selected = bin above lin_sel, or flagged inside it
  int lin_sel = 0;
  double lin_lo = 0.0, lin_scale = 0.0;

  if (p.mode == 0) {
    long long k = p.budget_blocks ? k_blocks : ((long long)p.budget_tokens + p.block_size - 1) / p.block_size;
    k = k < 0 ? 0 : k;
    k = k > nb ? nb : k;
    k = k > p.max_sel ? p.max_sel : k;
    from_full = (int)k;
    if (partial && k > 0) from_full = (int)k - 1;
    from_full = from_full > nfull ? nfull : from_full;
    force_last = partial && k > 0;

    if (from_full >= nfull) {
      T = 0;               // every full block is taken
      take_ge = true;
    } else if (from_full > 0 && SRC != 0) {
      // Fast path.  Scores are binned linearly between their minimum and maximum (monotone in
      // the score, and unlike the leading bits of a float it spreads the blocks evenly, so the
      // LDS atomics do not pile up); one scan finds the bin that holds the k-th largest score;
      // every block in a higher bin is selected, and the few blocks inside the boundary bin are
      // ranked exactly (key, then lower index) against each other.  Falls through to the radix
      // walk when that bin is crowded (many equal or nearly equal scores).
      double hi = -INFINITY, nlo = -INFINITY;
      for_own_scores(sc, 0, nfull, [&](int, double v) { hi = fmax(hi, v); nlo = fmax(nlo, -v); });
      wg_reduce_max2(hi, nlo, red + 8);     // (lin_hist and cand_n were cleared before the scores arrived)
      const double lo = -nlo;
      const double scale = __ddiv_rn((double)kLinBins, __dsub_rn(hi, lo));
      if (hi > lo && scale > 0.0 && scale < 1.0e300) {
        unsigned char* flags = dyn_smem + (size_t)p.nb_max * sizeof(double);
        for_own_scores(sc, 0, nfull, [&](int, double v) { atomicAdd(&lin_hist[lin_bin_of(v, lo, scale)], 1); });
        __syncthreads();
        // thread t owns bins 1023-4t .. 1020-4t (descending); exclusive scan of the counts from the top
        const int b0 = kLinBins - 1 - 4 * tid;
        const int c0 = lin_hist[b0], c1 = lin_hist[b0 - 1], c2 = lin_hist[b0 - 2], c3 = lin_hist[b0 - 3];
        int above = wg_exclusive_scan(c0 + c1 + c2 + c3, wcnt);
        if (above < from_full && from_full <= above + c0 + c1 + c2 + c3) {   // exactly one thread
          int bsel = b0, cnt = c0;
          if (from_full > above + c0) {
            above += c0; bsel = b0 - 1; cnt = c1;
            if (from_full > above + c1) {
              above += c1; bsel = b0 - 2; cnt = c2;
              if (from_full > above + c2) { above += c2; bsel = b0 - 3; cnt = c3; }
            }
          }
          digit_sel[0] = bsel;
          digit_sel[1] = from_full - above;     // blocks still needed from the boundary bin
          digit_sel[2] = cnt;                   // blocks in the boundary bin
        }
        __syncthreads();
        lin_sel = digit_sel[0];
        const int need = digit_sel[1], cnt = digit_sel[2];
        if (cnt <= kMaxCand) {
          for_own_scores(sc, 0, nfull, [&](int j, double v) {
            if (lin_bin_of(v, lo, scale) == lin_sel) {
              const int at = atomicAdd(&cand_n, 1);
              cand_key[at] = score_key(v);
              cand_idx[at] = j;
            }
          });
          __syncthreads();
          if (tid < cnt) {        // every block of the boundary bin gets its flag written: taken or not
            const unsigned long long mk = cand_key[tid];
            const int mi = cand_idx[tid];
            int rank = 0;
            for (int u = 0; u < cnt; ++u) {
              const unsigned long long uk = cand_key[u];
              rank += (uk > mk) || (uk == mk && cand_idx[u] < mi);
            }
            flags[mi] = rank < need ? 1 : 0;
          }
          __syncthreads();
          lin_lo = lo;
          lin_scale = scale;
          lin_fast = true;
        }
      }
    }
    if (from_full > 0 && from_full < nfull && !lin_fast) {
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
        if (wave == 0) {
          // lane owns digits d0, d0-1, d0-2, d0-3 (descending); scan candidates from the top digit
          const int d0 = 255 - 4 * lane;
          const int c0 = hist[d0], c1 = hist[d0 - 1], c2 = hist[d0 - 2], c3 = hist[d0 - 3];
          const int own = c0 + c1 + c2 + c3;
          const int incl = wave_inclusive_scan_i32(own);
          int above = incl - own;                     // candidates with a digit above d0
          if (above < remaining && remaining <= incl) {   // true for exactly one lane
            int dsel = d0, cnt = c0;
            if (remaining > above + c0) {
              above += c0; dsel = d0 - 1; cnt = c1;
              if (remaining > above + c1) {
                above += c1; dsel = d0 - 2; cnt = c2;
                if (remaining > above + c2) { above += c2; dsel = d0 - 3; cnt = c3; }
              }
            }
            digit_sel[0] = dsel;
            digit_sel[1] = remaining - above;   // still needed from that digit's bin
            digit_sel[2] = cnt;                 // candidates in that bin
          }
        }
        __syncthreads();
        prefix |= (uint64_t)digit_sel[0] << shift;
        mask |= 0xffull << shift;
        remaining = digit_sel[1];
        const bool all_of_bin = remaining == digit_sel[2];
        __syncthreads();
        if (all_of_bin) { take_ge = true; break; }   // key >= prefix (low bits zero) is the selection
      }
      T = prefix;
      need_eq = take_ge ? 0 : remaining;
    }
  } else {
    if (nfull > 0) {
      double mx = -INFINITY;
      for_own_scores(sc, 0, nfull, [&](int, double v) { mx = fmax(mx, __dmul_rn(v, p.inv_sqrt_dg)); });
      m = wg_reduce_max(mx, red);
      double z = 0.0;
      for_own_scores(sc, 0, nfull, [&](int, double v) { z += exp(__dsub_rn(__dmul_rn(v, p.inv_sqrt_dg), m)); });
      Z = wg_reduce_sum(z, red + 4);
    }
    if (p.mode == 2 && nfull > 0) {
      // Top-p: the same radix walk as top-k, but steered by probability mass instead of counts.
      // Masses are accumulated as 2^-62 fixed point, so the sums are exact integers and do not
      // depend on the order in which the work-group adds them.
      const double kFix = 4611686018427387904.0;   // 2^62
      auto fixed_mass = [&](double s) -> unsigned long long {
        const double Sj = __ddiv_rn(exp(__dsub_rn(__dmul_rn(s, p.inv_sqrt_dg), m)), Z);
        return (unsigned long long)(Sj * kFix);
      };
      unsigned long long want = p.threshold >= 1.0 ? (unsigned long long)kFix
                                : (p.threshold > 0.0 ? (unsigned long long)(p.threshold * kFix) : 0ull);
      if (want == 0) want = 1;                       // at least the best block
      uint64_t prefix = 0, kmask = 0;
      // p >= 1 asks for the whole mass; every softmax probability is positive, so only the set of all
      // full blocks has it (decided here, not left to how the rounded masses happen to add up)
      bool done = p.threshold >= 1.0;
      if (done) { T = 0; take_ge = true; }
      for (int pass = 7; pass >= 0 && !done; --pass) {
        const int shift = pass * 8;
        hist[tid] = 0;
        mass[tid] = 0;
        __syncthreads();
        for (int j = tid; j < nfull; j += 256) {
          const double s = sc[j];
          const uint64_t key = score_key(s);
          if ((key & kmask) == prefix) {
            const int dgt = (int)((key >> shift) & 0xff);
            atomicAdd(&hist[dgt], 1);
            atomicAdd(&mass[dgt], fixed_mass(s));
          }
        }
        __syncthreads();
        if (wave == 0) {
          const int d0 = 255 - 4 * lane;
          const unsigned long long m0 = mass[d0], m1 = mass[d0 - 1], m2 = mass[d0 - 2], m3 = mass[d0 - 3];
          const unsigned long long own = m0 + m1 + m2 + m3;
          unsigned long long incl = own;
#pragma unroll
          for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long x = __shfl_up(incl, o);
            if (lane >= o) incl += x;
          }
          unsigned long long above = incl - own;
          if (lane == 63 && incl < want) {           // p exceeds the mass that is there: keep everything
            digit_sel[0] = -1;
          }
          if (above < want && want <= incl) {
            int dsel = d0;
            unsigned long long bm = m0;
            if (want > above + m0) {
              above += m0; dsel = d0 - 1; bm = m1;
              if (want > above + m1) {
                above += m1; dsel = d0 - 2; bm = m2;
                if (want > above + m2) { above += m2; dsel = d0 - 3; bm = m3; }
              }
            }
            digit_sel[0] = dsel;
            digit_sel[2] = hist[dsel];
            mass_sel[0] = want - above;              // mass still needed from that bin
            mass_sel[1] = bm;
          }
        }
        __syncthreads();
        const int dsel = digit_sel[0];
        if (dsel < 0) {                              // keep every full block
          T = 0; take_ge = true; done = true;
        } else {
          prefix |= (uint64_t)dsel << shift;
          kmask |= 0xffull << shift;
          want = mass_sel[0];
          if (digit_sel[2] == 1) { T = prefix; take_ge = true; done = true; }   // that block completes the nucleus
          else if (pass == 0) {
            // several blocks with exactly this score: equal masses, take as many as are needed
            const unsigned long long each = mass_sel[1] / (unsigned long long)digit_sel[2];
            long long c = each ? (long long)((want + each - 1) / each) : digit_sel[2];
            c = c < 1 ? 1 : (c > digit_sel[2] ? digit_sel[2] : c);
            T = prefix; need_eq = (int)c; done = true;
          }
        }
        __syncthreads();
      }
    }
  }

  // ---- ordered compaction: thread t owns blocks t, t + 256, ... (8192 blocks per pass) -------------
  const bool any_full = (p.mode == 0) ? (from_full > 0) : (nfull > 0);
  int n = 0;
  if (any_full) {
    auto classify = [&](int j, double s, bool* gt, bool* eq) {
      if (lin_fast) {
        const int b = lin_bin_of(s, lin_lo, lin_scale);
        const unsigned char* flags = dyn_smem + (size_t)p.nb_max * sizeof(double);
        *gt = b > lin_sel || (b == lin_sel && flags[j] != 0);
        *eq = false;
      } else if (p.mode != 1) {
        const uint64_t key = score_key(s);
        *gt = take_ge ? key >= T : key > T;
        *eq = !take_ge && key == T;
      } else {
        const double Sj = __ddiv_rn(exp(__dsub_rn(__dmul_rn(s, p.inv_sqrt_dg), m)), Z);
        *gt = Sj > p.threshold;
        *eq = false;
      }
    };
    int eq_before = 0;
    for (int c0 = 0; c0 < nfull; c0 += 256 * kMaxOwn) {
      const int left = nfull - c0;
      const int rows = left >= 256 * kMaxOwn ? kMaxOwn : (left + 255) >> 8;
      uint32_t take = 0, ties = 0;
      const int c1 = c0 + rows * 256 < nfull ? c0 + rows * 256 : nfull;
      for_own_scores(sc, c0, c1, [&](int j, double v) {
        bool gt, eq;
        classify(j, v, &gt, &eq);
        const int u = (j - c0) >> 8;
        take |= (uint32_t)gt << u;
        ties |= (uint32_t)eq << u;
      });
      if (need_eq > 0) {      // blocks that tie with the k-th score: the first need_eq of them in block order
        uint32_t add = 0;
        const int tot = ordered_ranks(ties, rows, rowcnt, [&](int u, int r) { if (eq_before + r < need_eq) add |= 1u << u; });
        eq_before += tot;
        take |= add;
        __syncthreads();      // rowcnt is written again below
      }
      const int base = n;
      n += ordered_ranks(take, rows, rowcnt, [&](int u, int r) {
        const int pos = base + r;
        if (pos < p.max_sel) out[pos] = c0 + u * 256 + tid;
      });
      if (c0 + 256 * kMaxOwn < nfull) __syncthreads();   // the next pass rewrites rowcnt
    }
  }
  n = n < p.max_sel ? n : p.max_sel;
  if (force_last && n < p.max_sel) {
    if (tid == 0) out[n] = nb - 1;
    n += 1;
  }
  for (int q = n + tid; q < p.max_sel; q += 256) out[q] = -1;
  if (tid == 0) p.nblk[grp] = n;
}

hipError_t launch_gate_score(const GateParams& p, bool ragged, hipStream_t s) {
  const int tiles = (p.nb_max + kScoreRowsPerWg - 1) / kScoreRowsPerWg;
  if (ragged && tiles > 8) {
    hipLaunchKernelGGL(seer_gate_score_walk_kernel, dim3(8, p.Hkv, p.B), dim3(256), 0, s, p);
  } else {
    hipLaunchKernelGGL(seer_gate_score_kernel, dim3(tiles, p.Hkv, p.B), dim3(256), 0, s, p);
  }
  return hipGetLastError();
}

// Dynamic LDS of the select kernel for `nb` blocks held in LDS: fp64 scores + one flag byte each.
static size_t select_dyn_lds(int nb) { return (size_t)nb * (sizeof(double) + 1); }

// Can a work-group of `kernel` get `dyn` bytes of dynamic LDS on top of its static arrays on the
// current device?  Requests beyond the 64 KiB every device grants need the function's limit raised
// first; a device that cannot hold the sum is answered with false (the caller takes another path).
template <typename K>
static bool reserve_dyn_lds(K kernel, size_t dyn) {
  hipFuncAttributes fa;
  if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kernel)) != hipSuccess) { (void)hipGetLastError(); return false; }
  if (fa.sharedSizeBytes + dyn <= 64 * 1024) return true;
  int dev = 0, max_lds = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  if (fa.sharedSizeBytes + dyn > (size_t)max_lds) return false;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn) !=
      hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

hipError_t launch_gate_select(const GateParams& p, hipStream_t s) {
  dim3 grid(p.Hkv, p.B);
  const size_t dyn = select_dyn_lds(p.nb_max);
  if (p.nb_max <= kSelectLdsBlocks && reserve_dyn_lds(seer_gate_select_kernel<1>, dyn))
    hipLaunchKernelGGL(seer_gate_select_kernel<1>, grid, dim3(256), dyn, s, p);
  else      // scores stay in global memory (L2): a cache longer than the LDS the device grants
    hipLaunchKernelGGL(seer_gate_select_kernel<0>, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

bool gate_fused_possible(const GateParams& p) {
  const size_t dyn = select_dyn_lds(p.nb_max);
  return p.nb_max <= kSelectLdsBlocks && reserve_dyn_lds(seer_gate_select_kernel<2, 256>, dyn) &&
         reserve_dyn_lds(seer_gate_select_kernel<2, 1024>, dyn);
}

// Caches of 512 blocks and more are streamed by 16 waves per group (one wave reads 4 rows per load, so
// shorter caches would leave most of them without rows), the rest by 4.
hipError_t launch_gate_fused(const GateParams& p, hipStream_t s) {
  dim3 grid(p.Hkv, p.B);
  const size_t dyn = select_dyn_lds(p.nb_max);
  if (p.nb_max >= 512)
    hipLaunchKernelGGL((seer_gate_select_kernel<2, 1024>), grid, dim3(1024), dyn, s, p);
  else
    hipLaunchKernelGGL((seer_gate_select_kernel<2, 256>), grid, dim3(256), dyn, s, p);
  return hipGetLastError();
}

}  // namespace seer
