// Training-side forward (Sec. 2.3): dense causal attention that also leaves what the AttnGate's
// distillation target is made of, in the manner the section describes - the block-level row maxima
// that the online softmax computes anyway are kept per (query row, key block) and turned into
// probabilities once the row's log-sum-exp is known.
//
// Kernel 1, seer_attn_fwd_kernel: one work-group of 256 threads per (sequence, query head, tile of 128
// query rows), ordered so that the heads of a GQA group share an XCD's L2.  A wave owns 32 query rows
// as two 16-row tiles and walks the keys 64 at a time (one softmax step per 64 keys, two 32-key halves
// for the PV product).  The matrix-core formulation is the one of the decode kernel, with query rows
// in the place of the heads of a group (lane = 16*q + n):
//   S^T = K Q^T   A = 16 keys x 32 features from the work-group's K tile in LDS (XOR-swizzled rows,
//                 double-buffered: the next tile is fetched into registers during the current one
//                 and stored before the single barrier of the iteration); B = Q^T in registers.
//   softmax       lane holds 4 keys x 2 tiles of one query row; causal mask on the diagonal chunks;
//                 the chunk maximum doubles as the block maximum (running over the chunks of a block).
//   O^T = V^T P^T B = P^T rounded to bf16, already in operand layout; A = V^T straight from the
//                 work-group's V tile in LDS through the transposing LDS read (ds_read_b64_tr_b16):
//                 two reads of 4 keys each give a lane its 8 keys of one feature, no permutes.
// K and V tiles are fetched by all 256 threads one iteration ahead, directly into the other LDS stage,
// so a row crosses the memory system once per work-group and its latency is covered by a whole
// iteration of arithmetic.
// Kernel 2, seer_gt_finalize_kernel: per (sequence, kv head, 64 query rows): block probabilities
// exp2(raw - lse2), maximum over the g heads, row sums, normalised rows written through an LDS
// transpose so that both the reads (along rows) and the writes (along blocks) are coalesced.
#include "seer_internal.h"

#include <type_traits>

namespace seer {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ uint32_t tf_pack_bf16(float a, float b) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, r);
}

#define SEER_LDS_PTR(ptr) ((__attribute__((address_space(3))) void*)(ptr))
#define SEER_LDS_PTR_T(type, ptr) ((__attribute__((address_space(3))) type*)(ptr))
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

constexpr int kQTile = 128;   // query rows per work-group
constexpr int kKTile = 64;    // keys per iteration

}  // namespace

// ROWS128: stride_token == 128 elements (rows back to back), so row offsets are immediates.
template <bool ROWS128>
__global__ __launch_bounds__(256, 2) void seer_attn_fwd_kernel(TrainFwdParams p) {
  // Two stages of the K and V tiles, as four separate arrays: the compiler then knows that the
  // asynchronous fills of one stage cannot touch the stage being read.
  __shared__ __attribute__((aligned(16))) unsigned char kbuf_a[kKTile * 256];
  __shared__ __attribute__((aligned(16))) unsigned char kbuf_b[kKTile * 256];
  __shared__ __attribute__((aligned(16))) unsigned char vbuf_a[kKTile * 256];
  __shared__ __attribute__((aligned(16))) unsigned char vbuf_b[kKTile * 256];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, q4 = lane >> 4;
  // Work-group id -> (sequence, kv head, query tile, head of the group).  Work-groups are dealt to the 8
  // XCDs round-robin by id, and each XCD has its own L2.  Work-groups that read the same K/V stream
  // are therefore given ids that are equal mod 8: always the g heads of a group on the same query
  // tile, and - when the (sequence, kv head) groups divide evenly over the XCDs - all query tiles of a
  // group, so that its K/V is filled into one L2 only.  Query tiles with the most keys come first.
  const int nqt = (p.T + kQTile - 1) / kQTile;
  const int G = p.B * p.Hkv;
  const int id = blockIdx.x, x8 = id & 7, t8 = id >> 3;
  const int hh = t8 % p.g;
  int grp, qt;
  if ((G & 7) == 0) {                          // group = 8 * (slot / nqt) + XCD, tile = slot % nqt
    const int slot = t8 / p.g;
    grp = (slot / nqt) * 8 + x8;
    qt = nqt - 1 - slot % nqt;
  } else {                                     // (group, tile) pairs round-robin over the XCDs
    const int pair = (t8 / p.g) * 8 + x8;
    if (pair >= G * nqt) return;               // padding of the last set of 8
    grp = pair / nqt;
    qt = nqt - 1 - pair % nqt;
  }
  const int hk = grp % p.Hkv, i = grp / p.Hkv, h = hk * p.g + hh;
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
      if (qrow[a] < S)                         // padding rows (>= S) compute on zeros: whatever they hold stays out
        qb[a][kk] = *reinterpret_cast<const uint4*>(p.q + (((int64_t)i * p.T + qrow[a]) * p.Hq + h) * kHeadDim +
                                                    kk * 32 + q4 * 8);
    }
  }

  const uint16_t* kbase = p.k + (int64_t)i * p.stride_seq + (int64_t)hk * p.stride_head;
  const uint16_t* vbase = p.v + (int64_t)i * p.stride_seq + (int64_t)hk * p.stride_head;
  const int64_t st = ROWS128 ? (int64_t)kHeadDim : p.stride_token;
  int kend = r0 + kQTile;                    // keys [0, kend) matter to this work-group
  kend = kend < S ? kend : S;
  int wave_end = wrow0 + 32;                 // keys [0, wave_end) matter to this wave
  wave_end = wave_end < S ? wave_end : S;
  if (r0 >= S) {                             // a tile of padding rows: nothing to read
    kend = 0;
    wave_end = 0;
  }
  const int ntiles = (kend + kKTile - 1) / kKTile;

  // K / V tile staging.  Thread (srow = tid/16, schunk = tid%16) owns the 16-byte slot `schunk` of rows
  // 16*u + srow of a tile.  K rows are kept XOR-swizzled (slot s of row r holds chunk s ^ (r & 15):
  // operand reads walk 16 rows at one chunk), V rows swizzled in 32-byte units (slot s of row r holds
  // chunk s ^ 2*(r & 7): the transposing operand reads walk 16 rows at one 32-byte column).  Whole tiles are
  // fetched straight into LDS (global_load_lds: a wave fills 1 KiB = its 4 rows, lane l at +16*l, so
  // the swizzle is applied to the global address); no staging registers, no LDS store instructions.
  // The last tile of a sequence whose length is not a multiple of 64 goes through registers with the
  // rows at and beyond the sequence's length zeroed: those keys are masked (P = 0), but 0 x NaN or
  // 0 x Inf from whatever the padding holds would still poison the PV product of the real rows.
  const int srow = tid >> 4, schunk = tid & 15;
  const int wave_rows = __builtin_amdgcn_readfirstlane(wave) * 4;
  const uint16_t* kptr = kbase + (int64_t)srow * st + ((schunk ^ (srow & 15)) * 8);
  const uint16_t* vptr = vbase + (int64_t)srow * st + ((schunk ^ ((srow & 7) << 1)) * 8);
  auto fetch_tile = [&](int kt0, unsigned char* kdst, unsigned char* vdst) {
    const uint16_t* kp = kptr + (int64_t)kt0 * st;
    const uint16_t* vp = vptr + (int64_t)kt0 * st;
    if (kt0 + kKTile <= S) {                 // work-group-uniform: every row of the tile is a real key
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        __builtin_amdgcn_global_load_lds(kp + (int64_t)(16 * u) * st, SEER_LDS_PTR(kdst + (16 * u + wave_rows) * 256),
                                         16, 0, 0);
        __builtin_amdgcn_global_load_lds(vp + (int64_t)(16 * u) * st, SEER_LDS_PTR(vdst + (16 * u + wave_rows) * 256),
                                         16, 0, 0);
      }
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        uint4 kr = make_uint4(0, 0, 0, 0), vr = make_uint4(0, 0, 0, 0);
        if (kt0 + 16 * u + srow < S) {
          kr = *reinterpret_cast<const uint4*>(kp + (int64_t)(16 * u) * st);
          vr = *reinterpret_cast<const uint4*>(vp + (int64_t)(16 * u) * st);
        }
        const int row = 16 * u + srow;
        *reinterpret_cast<uint4*>(kdst + row * 256 + (schunk << 4)) = kr;     // kr already is the swizzled chunk
        *reinterpret_cast<uint4*>(vdst + row * 256 + (schunk << 4)) = vr;     // likewise
      }
    }
  };

  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f}, bmax[2] = {-INFINITY, -INFINITY};
  f32x4_t oacc[2][8];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 8; ++e) oacc[a][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  if (ntiles > 0) fetch_tile(0, kbuf_a, vbuf_a);
  __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): the fills have landed
  __syncthreads();

  float* rawbase = p.raw + ((int64_t)i * p.Hq + h) * raw_head_elems(p.nb, p.Tp, p.block_size);

  // One 64-key tile for this wave.  MASKED: the tile may hold keys beyond some row of the wave (only
  // the last tile or two of a wave's range); interior tiles carry no masking code at all.
  auto tile_body = [&](auto masked_tag, const int kt0, const unsigned char* kt, const unsigned char* vt) {
    constexpr bool MASKED = decltype(masked_tag)::value;
      // ---- S^T = K Q^T for the four 16-key tiles; all issued before the softmax so that the
      //      matrix core works on the later tiles while the vector units start on the first --------
      f32x4_t sacc[2][4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int row = 16 * t + n16;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const uint4 ka = *reinterpret_cast<const uint4*>(kt + row * 256 + (((kk * 4 + q4) ^ n16) << 4));
#pragma unroll
          for (int a = 0; a < 2; ++a)
            sacc[a][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8_t, ka), __builtin_bit_cast(bf16x8_t, qb[a][kk]),
                kk == 0 ? f32x4_t{0.f, 0.f, 0.f, 0.f} : sacc[a][t], 0, 0, 0);
        }
      }

      // ---- online softmax over the 64 keys per query tile; lane holds keys kt0 + 16t + 4*q4 + r ------
      uint4 pb[2][2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        // x holds the unscaled logits; scale_log2e > 0, so maxima commute with the scaling, and the
        // scaling itself is folded into the exponent: exp2(x * s - m)
        float x[16];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int r = 0; r < 4; ++r) x[4 * t + r] = sacc[a][t][r];
        if (MASKED && kt0 + 63 > wrow0 + 16 * a) {     // the diagonal passes through this tile for some row
#pragma unroll
          for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (kt0 + 16 * t + 4 * q4 + r > qrow[a]) x[4 * t + r] = -INFINITY;
        }
        // maxima of the two 32-key halves (a block may be one half), then of the tile
        float mh[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const float* y = x + 8 * c;
          float mx = fmaxf(fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])), fmaxf(fmaxf(y[4], y[5]), fmaxf(y[6], y[7])));
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          mh[c] = mx * p.scale_log2e;
        }
        // block maxima of the logits of this row (Sec. 2.3: the row maxima are reused)
        if (p.block_size == 16) {              // one block per 16-key tile: four maxima of 4 values + rows
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            float mx = fmaxf(fmaxf(x[4 * t], x[4 * t + 1]), fmaxf(x[4 * t + 2], x[4 * t + 3]));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const int j = (kt0 >> 4) + t;
            if (q4 == 0 && qrow[a] < p.T && j < p.nb && j * 16 <= qrow[a])     // only blocks the row can see have a slot
              rawbase[raw_index(j, qrow[a], p.Tp, 16)] = mx * p.scale_log2e;
          }
        } else if (p.block_size == 32) {
          if (q4 == 0 && qrow[a] < p.T) {
            const int j0 = kt0 >> 5;
            if (j0 * 32 <= qrow[a]) rawbase[raw_index(j0, qrow[a], p.Tp, 32)] = mh[0];
            if (j0 + 1 < p.nb && (j0 + 1) * 32 <= qrow[a]) rawbase[raw_index(j0 + 1, qrow[a], p.Tp, 32)] = mh[1];
          }
        } else {
          const float mt = fmaxf(mh[0], mh[1]);
          bmax[a] = (kt0 % p.block_size) == 0 ? mt : fmaxf(bmax[a], mt);
          // (a wave only works on tiles that start at or before its rows, so the row sees this block)
          if (q4 == 0 && qrow[a] < p.T) rawbase[raw_index(kt0 / p.block_size, qrow[a], p.Tp, p.block_size)] = bmax[a];
        }

        const float m_new = fmaxf(m_run[a], fmaxf(mh[0], mh[1]));
        const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run[a] - m_ref);
        float pr[16], psum = 0.f;
#pragma unroll
        for (int cc = 0; cc < 16; ++cc) {
          pr[cc] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[cc], p.scale_log2e, -m_ref));
          psum += pr[cc];
        }
        l_run[a] = l_run[a] * alpha + psum;
        m_run[a] = m_new;
        if (__ballot(alpha != 1.0f)) {
#pragma unroll
          for (int e = 0; e < 8; ++e) oacc[a][e] *= alpha;
        }
#pragma unroll
        for (int c = 0; c < 2; ++c)
          pb[a][c] = make_uint4(tf_pack_bf16(pr[8 * c + 0], pr[8 * c + 1]), tf_pack_bf16(pr[8 * c + 2], pr[8 * c + 3]),
                                tf_pack_bf16(pr[8 * c + 4], pr[8 * c + 5]), tf_pack_bf16(pr[8 * c + 6], pr[8 * c + 7]));
      }

      // ---- O^T += V^T P^T per 32-key half and 16-feature tile e.  The A operand of lane (n16, q4) is
      //      V[key tau(q4, j)][feature 16e + n16], j = 0..7, tau(q4, j) = j < 4 ? 4*q4 + j : 16 + 4*q4 + (j - 4)
      //      (the order the probabilities sit in).  A transposing read hands lane n16 of a 16-lane group
      //      element n16 % 4 of the 8-byte pieces addressed by lanes n16/4, n16/4 + 4, + 8, + 12 of the
      //      group; so lane n16 addresses key 4*q4 + n16/4 (and that key + 16), features 16e + 4*(n16 % 4)
      //      .. + 3, and receives four consecutive keys of feature 16e + n16 per read. -------------------
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int row0 = 32 * c + 4 * q4 + (n16 >> 2);                   // the key this lane addresses (and row0 + 16)
        const int sw = (row0 & 7) << 1;                                  // (row0 + 16) & 7 == row0 & 7
        const unsigned char* vrow = vt + row0 * 256 + ((n16 & 1) << 3);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int slot = (2 * e + ((n16 & 3) >> 1)) ^ sw;              // 16-byte slot that holds the piece
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SEER_LDS_PTR_T(s16x4_t, vrow + (slot << 4)));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(SEER_LDS_PTR_T(s16x4_t, vrow + 16 * 256 + (slot << 4)));
          const s16x8_t va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
          for (int a = 0; a < 2; ++a)
            oacc[a][e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, va),
                                                                 __builtin_bit_cast(bf16x8_t, pb[a][c]), oacc[a][e],
                                                                 0, 0, 0);
        }
      }
  };

  // One iteration: start the fill of the other stage, work on this one, wait for the fill, barrier.
  auto iteration = [&](const int it, const unsigned char* kt, const unsigned char* vt, unsigned char* knext,
                       unsigned char* vnext) {
    const int kt0 = it * kKTile;
    if (it + 1 < ntiles) fetch_tile(kt0 + kKTile, knext, vnext);
    if (kt0 < wave_end) {                     // wave-uniform: some row of this wave sees the tile
      if (kt0 + 63 > wrow0) tile_body(std::true_type{}, kt0, kt, vt);
      else tile_body(std::false_type{}, kt0, kt, vt);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
    __syncthreads();
  };
  for (int it = 0; it < ntiles; it += 2) {
    iteration(it, kbuf_a, vbuf_a, kbuf_b, vbuf_b);
    if (it + 1 < ntiles) iteration(it + 1, kbuf_b, vbuf_b, kbuf_a, vbuf_a);
  }

  // ---- results: lane (n16, q4) holds O[row n16 of tile a][16*e + 4*q4 + r] in oacc[a][e][r] ---------
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
    for (int e = 0; e < 8; ++e) {
      const int c0 = 16 * e + 4 * q4;
      if (p.out_is_f32) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.out) + orow * kHeadDim + c0) =
            make_float4(oacc[a][e][0] * inv, oacc[a][e][1] * inv, oacc[a][e][2] * inv, oacc[a][e][3] * inv);
      } else {
        const uint32_t w0 = (uint32_t)f32_to_bf16_rne(oacc[a][e][0] * inv) | ((uint32_t)f32_to_bf16_rne(oacc[a][e][1] * inv) << 16);
        const uint32_t w1 = (uint32_t)f32_to_bf16_rne(oacc[a][e][2] * inv) | ((uint32_t)f32_to_bf16_rne(oacc[a][e][3] * inv) << 16);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(p.out) + orow * kHeadDim + c0) = make_uint2(w0, w1);
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
  const int64_t head_elems = raw_head_elems(p.nb, p.Tp, p.block_size);
  const float* raw0 = p.raw + ((int64_t)i * p.Hq + (int64_t)hk * g) * head_elems;
  // N blocks at once for this row: every load is issued (index clamped) before the first exponential,
  // so a thread keeps N * g reads in flight; blocks the row cannot see give 0.
  auto block_probs = [&](auto n_tag, const int (&js)[decltype(n_tag)::value], float (&out)[decltype(n_tag)::value]) {
    constexpr int N = decltype(n_tag)::value;
    float x[N][kMaxGroup];
#pragma unroll
    for (int u = 0; u < N; ++u) {
      const int j = js[u] < nvis ? js[u] : 0;
      // 32-bit arithmetic: one head's slice holds fewer than 2^31 floats (checked on the host)
      const int at = j * p.Tp - p.block_size * (j * (j - 1) / 2) + (t - j * p.block_size);
#pragma unroll
      for (int hh = 0; hh < kMaxGroup; ++hh)
        x[u][hh] = (hh < g && real) ? raw0[hh * head_elems + at] : -INFINITY;
    }
#pragma unroll
    for (int u = 0; u < N; ++u) {
      float r = 0.f;
#pragma unroll
      for (int hh = 0; hh < kMaxGroup; ++hh)
        if (hh < g) r = fmaxf(r, exp2f(x[u][hh] - l2[hh]));
      out[u] = js[u] < nvis ? r : 0.f;
    }
  };

  float sum = 0.f;
  for (int j = part; j < nvis_tile; j += 16) {      // blocks j, j+4, j+8, j+12 (the four parts interleave)
    const int js[4] = {j, j + 4, j + 8, j + 12};
    float v[4];
    block_probs(std::integral_constant<int, 4>{}, js, v);
    sum += (v[0] + v[1]) + (v[2] + v[3]);
  }
  part_sum[part][tq] = sum;
  __syncthreads();
  const float total = part_sum[0][tq] + part_sum[1][tq] + part_sum[2][tq] + part_sum[3][tq];
  const float inv = total > 0.f ? 1.0f / total : 0.f;

  float* gbase = p.gt + (((int64_t)i * p.Hkv + hk) * p.T) * (int64_t)p.nb;
  for (int j0 = 0; j0 < p.nb; j0 += 64) {
    if (j0 < nvis_tile) {
      // rows of the tile in parallel, 16 blocks per thread; then transposed out
#pragma unroll
      for (int u0 = 0; u0 < 16; u0 += 8) {
        int js[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) js[u] = j0 + part * 16 + u0 + u;
        float v[8];
        block_probs(std::integral_constant<int, 8>{}, js, v);
#pragma unroll
        for (int u = 0; u < 8; ++u) tile[tq][part * 16 + u0 + u] = v[u] * inv;
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
  const long pairs = (long)p.B * p.Hkv * ((p.T + kQTile - 1) / kQTile);
  const dim3 grid((unsigned)(((pairs + 7) / 8) * 8 * p.g));
  if (p.stride_token == kHeadDim)
    hipLaunchKernelGGL(seer_attn_fwd_kernel<true>, grid, dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL(seer_attn_fwd_kernel<false>, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_gt_finalize(const TrainFwdParams& p, hipStream_t s) {
  const dim3 grid((p.T + 63) / 64, p.Hkv, p.B);
  hipLaunchKernelGGL(seer_gt_finalize_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace seer
