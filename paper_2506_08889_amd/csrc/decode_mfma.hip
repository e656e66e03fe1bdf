// Block-sparse flash-decoding, split-K main kernel, MFMA formulation for gfx950 (Sec. 3.3).
//
// Grid (Hkv, B, num_splits): a work-group owns one (sequence, kv head) query group and one
// contiguous slice of its selected-block list (the list is partitioned over its capacity,
// not over the blocks of the sequence).  Inside the work-group the 4 wavefronts are fully
// independent: wave w takes the 32-token half-blocks w, w+4, ... of the slice, keeps its own
// running max / sum / output, and the four are merged once at the end through LDS.  There is
// no barrier in the main loop.
//
// The g query heads of the group are padded to the 16-wide side of v_mfma_f32_16x16x32_bf16.
// Written for the MFMA operand layout (lane = 16*q + n):
//   A[i][k]: lane holds row i = n, k = 8q..8q+7      B[k][j]: lane holds column j = n, k = 8q..8q+7
//   D[i][j]: lane holds column j = n, rows i = 4q..4q+3
//
//   S^T = K Q^T   A = 16 tokens x 32 features of K, B = Q^T (head = column).  K rows arrive by
//                 coalesced 128-bit loads (16 lanes = one 256-byte row), are written to a
//                 wave-private, XOR-swizzled LDS tile and read back in operand layout.
//   softmax       D gives each lane 4 tokens of one head (x2 tiles): max over the lane's 8
//                 values and across q (2 shuffles); exponentials in the base-2 domain.
//   O^T = V^T P^T B = P^T (as hi + lo bf16 terms) is exactly the layout D left the probabilities in (tile 0 -> k slots
//                 0..3, tile 1 -> k slots 4..7 of each lane), so P never moves.  A = V^T needs,
//                 per lane, 8 tokens of one feature: each lane loads 8 rows x 16 bytes (again
//                 fully coalesced), and 32 in-lane 16-bit interleaves build the 8 operands;
//                 operand e covers features {8n+e}.  D then leaves lane (n,q) with
//                 O[head n][32q .. 32q+31], contiguous.
//
// With 16-token blocks a 32-row step is fed by two list entries (rows 0-15 and 16-31), each with its
// own address, valid count and position.
//
// Loads for the next half-block are issued as soon as the registers of the current one have
// been consumed (K after its copy to LDS, V after the interleave), so each wave keeps 8-16 KiB
// in flight.
#include "seer_internal.h"

namespace seer {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

namespace {

struct HalfBlock {
  int64_t off;   // element offset of the first token of the half-block
  int ntok;      // valid tokens (1..32); 0 = no more work
  int tok0;      // position of its first token in the sequence
  // 16-token blocks only: a step takes two list entries; rows 0..15 come from the first (fields above,
  // ntok <= 16) and rows 16..31 from the second (fields below; ntok2 = 0 when the list has run out)
  int64_t off2;
  int ntok2;
  int tok2;
};

__device__ __forceinline__ uint32_t pack_lo(uint32_t x, uint32_t y) { return (x & 0xffffu) | (y << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t x, uint32_t y) { return (x >> 16) | (y & 0xffff0000u); }

__device__ __forceinline__ uint32_t dword_of(const uint4& v, int i) {
  return i == 0 ? v.x : (i == 1 ? v.y : (i == 2 ? v.z : v.w));
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, r);
}

}  // namespace

// 4 waves x (32 rows x 256 B) K staging; reused for the final cross-wave merge.
constexpr int kSliceLdsBytes = 4 * 32 * 256 + 4 * kMaxRows * 2 * 4;

// One slice of one group's list, by one work-group of 4 waves: slice `split` of (sequence i, kv head hk).
// ROWS128: stride_token == 128 elements (rows back to back), so every row offset is an immediate.
// B16: 16-token blocks, two list entries per 32-row step.
template <bool ROWS128, bool B16>
__device__ __forceinline__ void decode_slice(const DecodeParams& p, unsigned char* smem, const int i, const int hk,
                                             const int split) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n16 = lane & 15, q4 = lane >> 4;
  const int g = p.g, rows = p.rows;

  const int bs = p.block_size;
  const int64_t grp = (int64_t)i * p.Hkv + hk;
  const int begin = split * p.blocks_per_split;
  const int32_t* list = p.block_idx ? p.block_idx + grp * p.max_blocks : nullptr;
  // Entries of this slice that exist in memory whatever the group's count turns out to be.
  const int slice_cap = (begin + p.blocks_per_split < p.max_blocks) ? begin + p.blocks_per_split : p.max_blocks;

  // ---- block descriptors ---------------------------------------------------------------------
  // Lane e of a 64-entry chunk holds list entry begin + 64*chunk + e.  A chunk is fetched in two
  // stages ahead of its use (list entry, then its page id), each issued one loop iteration apart,
  // so neither the index -> address dependency nor the page-table lookup is ever waited for in the
  // main loop; the first chunk's list entries are requested before the group's count is known.
  int pf_chunk = -1, pf_stage = 0, j_pf = -1, pg_pf = 0;
  auto pf_stage1 = [&](int chunk) {
    pf_chunk = chunk;
    pf_stage = 1;
    const int pe = begin + chunk * 64 + lane;
    j_pf = -1;
    if (pe < slice_cap) j_pf = list ? list[pe] : pe;
  };
  auto pf_stage2 = [&]() {
    pf_stage = 2;
    pg_pf = 0;
    if (p.page_table) {
      int64_t pi = ((int64_t)j_pf * bs) / p.page_size;
      pi = pi < 0 ? 0 : (pi >= p.max_pages ? p.max_pages - 1 : pi);    // always a valid table slot
      pg_pf = p.page_table[(int64_t)i * p.max_pages + pi];
    }
  };
  pf_stage1(0);

  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  const int nb = (S + bs - 1) / bs;
  int n;
  if (p.block_idx) {
    n = p.nblk[grp];
    n = n < 0 ? 0 : (n < p.max_blocks ? n : p.max_blocks);
  } else {
    n = nb < p.max_blocks ? nb : p.max_blocks;
  }
  if (begin >= n) {
    emit_empty_if_single_split(p, i, hk);
    return;
  }
  const int end = (begin + p.blocks_per_split < n) ? begin + p.blocks_per_split : n;
  const int hpb = bs >> 5;                 // half-blocks (32 tokens) per block
  const int nh = B16 ? (end - begin + 1) >> 1 : (end - begin) * hpb;      // 32-row steps in this slice
  const int64_t st = ROWS128 ? (int64_t)kHeadDim : p.stride_token;
  pf_stage2();

  // ---- Q^T operand: row n16 = (new token t, head h); zero rows for the padding ------------------
  const int row_t = n16 / g, row_h = n16 - row_t * g;
  uint4 qb[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    qb[kk] = make_uint4(0, 0, 0, 0);
    if (n16 < rows)
      qb[kk] = *reinterpret_cast<const uint4*>(
          p.q + (((int64_t)i * p.q_len + row_t) * p.Hq + (int64_t)hk * g + row_h) * kHeadDim + kk * 32 + q4 * 8);
  }
  // Query t of q_len sees the tokens before position S - (q_len - 1 - t); with one new token that is S.
  const int row_limit = (n16 < rows) ? S - (p.q_len - 1 - row_t) : S;
  const int causal_from = S - p.q_len + 1;     // first position that is masked for some row

  int loaded_chunk = -1;
  int64_t d_off = 0;
  int d_ntok = 0, d_tok = 0;
  auto finalize_chunk = [&](int chunk) {
    if (pf_chunk != chunk) pf_stage1(chunk);
    if (pf_stage < 2) pf_stage2();
    const int pe = begin + chunk * 64 + lane;
    const int j = j_pf;
    bool ok = pe < end && j >= 0 && j < nb;
    if (ok && p.page_table) ok = ((int64_t)j * bs) / p.page_size < p.max_pages;
    d_off = 0;
    d_ntok = 0;
    d_tok = 0;
    if (ok) {
      const int64_t t0 = (int64_t)j * bs;
      d_tok = j * bs;
      d_off = p.page_table ? (int64_t)pg_pf * p.stride_seq + (int64_t)hk * p.stride_head + (t0 % p.page_size) * p.stride_token
                           : (int64_t)i * p.stride_seq + (int64_t)hk * p.stride_head + t0 * p.stride_token;
      d_ntok = (S - j * bs < bs) ? S - j * bs : bs;
    }
    loaded_chunk = chunk;
  };

  int hb = wave;
  auto advance = [&]() -> HalfBlock {
    HalfBlock r;
    r.off = 0;
    r.ntok = 0;
    r.tok0 = 0;
    r.off2 = 0;
    r.ntok2 = 0;
    r.tok2 = 0;
    while (hb < nh) {
      const int e = B16 ? 2 * hb : hb / hpb, half = B16 ? 0 : hb - e * hpb;
      const int chunk = e >> 6;
      if (chunk != loaded_chunk) {
        finalize_chunk(chunk);
        if (begin + (chunk + 1) * 64 < end) pf_stage1(chunk + 1);
      } else if (pf_chunk > loaded_chunk && pf_stage == 1) {
        pf_stage2();
      }
      const int src = e & 63;
      const int nt_blk = __shfl(d_ntok, src);
      const int lo = __shfl((int)(uint32_t)(uint64_t)d_off, src);
      const int hi = __shfl((int)(uint32_t)((uint64_t)d_off >> 32), src);
      const int tk = __shfl(d_tok, src);
      hb += 4;
      if (B16) {                               // the entry's partner sits in the next lane (e is even)
        const int nt2 = __shfl(d_ntok, src + 1);
        const int lo2 = __shfl((int)(uint32_t)(uint64_t)d_off, src + 1);
        const int hi2 = __shfl((int)(uint32_t)((uint64_t)d_off >> 32), src + 1);
        const int tk2 = __shfl(d_tok, src + 1);
        if (nt_blk > 0 || nt2 > 0) {
          r.off = (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
          r.ntok = nt_blk;
          r.tok0 = tk;
          r.off2 = (int64_t)(((uint64_t)(uint32_t)hi2 << 32) | (uint32_t)lo2);
          r.ntok2 = nt2;
          r.tok2 = tk2;
          if (r.ntok == 0) {                   // keep "ntok > 0 means work": an invalid first entry swaps out
            r.off = r.off2; r.ntok = r.ntok2; r.tok0 = r.tok2;
            r.ntok2 = 0;
          }
          return r;
        }
        continue;
      }
      int nt = nt_blk - half * 32;
      nt = nt > 32 ? 32 : nt;
      if (nt > 0) {
        r.off = (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo) + (int64_t)half * 32 * st;
        r.ntok = nt;
        r.tok0 = tk + half * 32;
        return r;
      }
    }
    return r;
  };

  // K rows: load u covers rows 4u + q4 (16 lanes = one row).  V rows: load j covers the token of
  // k-slot j of this lane's q: tau(q, j) = j < 4 ? 4q + j : 16 + 4q + (j - 4).
  uint4 kr[8], vr[8];
  auto load_k = [&](const HalfBlock& b) {
    if (B16) {                                 // rows 0..15 from the first block, 16..31 from the second
      const uint16_t* b0 = p.k + b.off + n16 * 8;
      const uint16_t* b1 = p.k + b.off2 + n16 * 8;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int rr = 4 * (u & 3) + q4;
        kr[u] = make_uint4(0, 0, 0, 0);
        if (rr < (u < 4 ? b.ntok : b.ntok2)) kr[u] = load_stream16((u < 4 ? b0 : b1) + (int64_t)rr * st);
      }
      return;
    }
    const uint16_t* base = p.k + b.off + n16 * 8;
    if (b.ntok == 32) {
#pragma unroll
      for (int u = 0; u < 8; ++u) kr[u] = load_stream16(base + (int64_t)(4 * u + q4) * st);
    } else {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        kr[u] = make_uint4(0, 0, 0, 0);
        if (4 * u + q4 < b.ntok) kr[u] = load_stream16(base + (int64_t)(4 * u + q4) * st);
      }
    }
  };
  auto load_v = [&](const HalfBlock& b) {
    if (B16) {
      const uint16_t* b0 = p.v + b.off + n16 * 8;
      const uint16_t* b1 = p.v + b.off2 + n16 * 8;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int rr = 4 * q4 + (j & 3);       // slot j < 4: row 4*q4 + j of the first block, else of the second
        vr[j] = make_uint4(0, 0, 0, 0);
        if (rr < (j < 4 ? b.ntok : b.ntok2)) vr[j] = load_stream16((j < 4 ? b0 : b1) + (int64_t)rr * st);
      }
      return;
    }
    const uint16_t* base = p.v + b.off + n16 * 8;
    if (b.ntok == 32) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = (j < 4) ? 4 * q4 + j : 16 + 4 * q4 + (j - 4);
        vr[j] = load_stream16(base + (int64_t)row * st);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = (j < 4) ? 4 * q4 + j : 16 + 4 * q4 + (j - 4);
        vr[j] = make_uint4(0, 0, 0, 0);
        if (row < b.ntok) vr[j] = load_stream16(base + (int64_t)row * st);
      }
    }
  };

  unsigned char* kt = smem + wave * (32 * 256);   // this wave's K tile

  float m_run = -INFINITY, l_run = 0.f;
  f32x4_t oacc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) oacc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  HalfBlock cur = advance();
  if (cur.ntok > 0) {
    load_k(cur);
    load_v(cur);
  }

  while (cur.ntok > 0) {
    const HalfBlock nxt = advance();

    // ---- 1. K tile -> LDS (swizzled: 16-byte chunk c of row r lands at chunk c ^ (r & 15)) ---
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = 4 * u + q4;
      *reinterpret_cast<uint4*>(kt + row * 256 + ((n16 ^ (row & 15)) << 4)) = kr[u];
    }
    if (nxt.ntok > 0) load_k(nxt);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- 2. S^T = K Q^T for the two 16-token tiles -------------------------------------------
    f32x4_t sacc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      sacc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      const int row = 16 * t + n16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const uint4 a = *reinterpret_cast<const uint4*>(kt + row * 256 + (((kk * 4 + q4) ^ n16) << 4));
        sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                          __builtin_bit_cast(bf16x8_t, qb[kk]), sacc[t], 0, 0, 0);
      }
    }
    __builtin_amdgcn_wave_barrier();

    // ---- 3. online softmax (base-2 domain); lane holds tokens 16t + 4q + r of head n16 -------
    float x[8];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) x[4 * t + r] = sacc[t][r] * p.scale_log2e;
    if (B16) {
      if (cur.ntok < 16 || cur.ntok2 < 16 || cur.tok0 + 16 > causal_from || cur.tok2 + 16 > causal_from) {
        // tile t is block t of the pair: its own valid count and its own place in the sequence
        const int lim0 = (cur.ntok < row_limit - cur.tok0) ? cur.ntok : row_limit - cur.tok0;
        const int lim1 = (cur.ntok2 < row_limit - cur.tok2) ? cur.ntok2 : row_limit - cur.tok2;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (4 * q4 + r >= (t == 0 ? lim0 : lim1)) x[4 * t + r] = -INFINITY;
      }
    } else if (cur.ntok < 32 || cur.tok0 + 32 > causal_from) {
      // ragged tail of the sequence and / or the causal limit of this row among the new tokens
      const int lim = (cur.ntok < row_limit - cur.tok0) ? cur.ntok : row_limit - cur.tok0;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (16 * t + 4 * q4 + r >= lim) x[4 * t + r] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    // A row may have seen nothing yet (every token so far beyond its causal limit): keep the
    // exponent arguments finite-or-minus-infinity, never inf - inf.
    const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);
    float pr[8], psum = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      pr[c] = __builtin_amdgcn_exp2f(x[c] - m_ref);
      psum += pr[c];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__ballot(alpha != 1.0f)) {
#pragma unroll
      for (int e = 0; e < 8; ++e) oacc[e] *= alpha;
    }
    // Probabilities enter the bf16 MFMA as two terms, p = hi + lo (hi = bf16(p), lo = bf16(p - hi)),
    // so the PV product carries ~16 mantissa bits instead of 8; the second MFMA per operand is free
    // at this arithmetic intensity.
    uint4 pb, pl;
    {
      uint32_t h[4], l[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        h[c] = pack_bf16(pr[2 * c], pr[2 * c + 1]);
        l[c] = pack_bf16(pr[2 * c] - __uint_as_float(h[c] << 16), pr[2 * c + 1] - __uint_as_float(h[c] & 0xffff0000u));
      }
      pb = make_uint4(h[0], h[1], h[2], h[3]);
      pl = make_uint4(l[0], l[1], l[2], l[3]);
    }

    // ---- 4. O^T += V^T P^T ----------------------------------------------------------------------
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t o[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const uint32_t a = dword_of(vr[2 * jj], e >> 1), b = dword_of(vr[2 * jj + 1], e >> 1);
        o[jj] = (e & 1) ? pack_hi(a, b) : pack_lo(a, b);
      }
      const uint4 va = make_uint4(o[0], o[1], o[2], o[3]);
      oacc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, va),
                                                        __builtin_bit_cast(bf16x8_t, pb), oacc[e], 0, 0, 0);
      oacc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, va),
                                                        __builtin_bit_cast(bf16x8_t, pl), oacc[e], 0, 0, 0);
    }
    if (nxt.ntok > 0) load_v(nxt);
    cur = nxt;
  }

  // ---- merge the four waves; lane (n16,q4) holds O[head n16][32*q4 + 8*r + e] in oacc[e][r] -------
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  __syncthreads();                                    // K tiles are dead from here on
  float* sm_acc = reinterpret_cast<float*>(smem);     // [4][16][128] = the 32 KiB of the K tiles
  float* sm_ml = sm_acc + 4 * kMaxRows * kHeadDim;    // [4][16][2]
  if (n16 < rows) {
    float* dst = sm_acc + ((wave * kMaxRows + n16) * kHeadDim) + 32 * q4;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[8 * r + e] = oacc[e][r];
    if (q4 == 0) {
      sm_ml[(wave * kMaxRows + n16) * 2 + 0] = m_run;
      sm_ml[(wave * kMaxRows + n16) * 2 + 1] = l_run;
    }
  }
  __syncthreads();

  for (int o = tid; o < rows * kHeadDim; o += 256) {
    const int h = o / kHeadDim, dd = o % kHeadDim;
    float ma = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) ma = fmaxf(ma, sm_ml[(w * kMaxRows + h) * 2]);
    float ls = 0.f, a = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = sm_ml[(w * kMaxRows + h) * 2];
      const float f = (mw == -INFINITY) ? 0.f : exp2f(mw - ma);
      ls += sm_ml[(w * kMaxRows + h) * 2 + 1] * f;
      a += sm_acc[(w * kMaxRows + h) * kHeadDim + dd] * f;
    }
    emit_slice(p, i, hk, split, h, dd, ma, ls, a);
  }
}

// Grid (Hkv, B, num_splits): one work-group per (group, slice).
template <bool ROWS128, bool B16>
__global__ __launch_bounds__(256, 2) void seer_decode_split_mfma_kernel(DecodeParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[kSliceLdsBytes];
  int split, hk, i;
  decode_wg_coords(p, &split, &hk, &i);
  decode_slice<ROWS128, B16>(p, smem, i, hk, split);
}

// ---------------------------------------------------------------------------------------------------
// Lists of very different lengths: a fixed set of W work-groups (two per compute unit) walks the slices
// that exist instead of one work-group per (group, slice of the list capacity), most of which would
// find nothing to do and only hold a slot while they find out (a threshold selection may list every
// block, so the capacity is the whole sequence).
//   First pass: work-group w takes the first slice of group w straight away, like the grid kernel would.
//   Then every work-group derives the same table of the remaining units from the groups' counts:
//     [0, G - W)   first slices of the groups W .. G-1 (when there are more groups than work-groups),
//     then         the further slices of full length of all groups, in group order,
//     then         the shorter last slices in four classes by length (at least 3/4, 1/2, 1/4 of a full
//                  slice, then the rest) - so the launch ends on its shortest units.
//   Units are handed out through a counter in the workspace - whichever work-group is free takes the
//   next one, so compute units that get less of the memory system take fewer - or, when the counter
//   does not hold a valid state (first use of a workspace), round-robin.  The partial result of a unit
//   does not depend on who computes it, so results stay bit-identical from run to run.
// ---------------------------------------------------------------------------------------------------
constexpr int kMaxPersistGroups = 2048;

template <bool ROWS128, bool B16>
__global__ __launch_bounds__(256, 2) void seer_decode_persist_mfma_kernel(DecodeParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[kSliceLdsBytes];
  __shared__ int pfx_full[kMaxPersistGroups + 1];   // exclusive prefix of the groups' full-length slices after the first
  // ... and of their shorter last slices after the first, by length class c = floor(4 * entries / L)
  // (0 or 1 per group and class, so 16 bits hold any prefix)
  __shared__ unsigned short pfx_rem[4][kMaxPersistGroups + 1];
  __shared__ int wsum[5][4];
  __shared__ int s_next, s_dynamic;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int G = p.B * p.Hkv, L = p.blocks_per_split, W = gridDim.x, w = blockIdx.x;

  if (w < G) decode_slice<ROWS128, B16>(p, smem, w / p.Hkv, w % p.Hkv, 0);
  if (p.num_splits == 1) {                    // the list capacity fits one slice: nothing but first slices
    for (int grp = w + W; grp < G; grp += W) {
      __syncthreads();
      decode_slice<ROWS128, B16>(p, smem, grp / p.Hkv, grp % p.Hkv, 0);
    }
    return;
  }

  // ---- hand-out word [kSchedMagic - taken : 32 | taken : 32]: one add moves one from the high half to
  // the low half, so high + low == kSchedMagic holds for every state that started valid and all
  // work-groups reach the same verdict.  The merge kernel of the call leaves it reset.
  constexpr unsigned long long kTake = 0xFFFFFFFF00000001ull;
  unsigned long long took = 0;
  if (tid == 0 && p.sched) took = __hip_atomic_fetch_add(p.sched, kTake, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // ---- unit table: thread t owns groups [t*per, (t+1)*per) ---------------------------------------
  {
    const int per = (G + 255) / 256;
    const int g0 = tid * per;
    int f_sum = 0, r_sum[4] = {0, 0, 0, 0};
    for (int u = 0; u < per; ++u) {
      const int grp = g0 + u;
      if (grp >= G) break;
      int n;
      if (p.block_idx) {
        n = p.nblk[grp];
        n = n < 0 ? 0 : (n < p.max_blocks ? n : p.max_blocks);
      } else {
        int S = p.seqlens[grp / p.Hkv];
        S = S < 0 ? 0 : S;
        const int nb = (S + p.block_size - 1) / p.block_size;
        n = nb < p.max_blocks ? nb : p.max_blocks;
      }
      const int full = n / L, rest = n % L;
      const int cls = (full > 0 && rest != 0) ? (4 * rest) / L : -1;
      pfx_full[grp] = f_sum;                  // local exclusive prefix, made global below
      f_sum += full > 0 ? full - 1 : 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        pfx_rem[c][grp] = (unsigned short)r_sum[c];
        r_sum[c] += cls == c ? 1 : 0;
      }
    }
    int fi = f_sum, ri[4] = {r_sum[0], r_sum[1], r_sum[2], r_sum[3]};   // inclusive scan over the threads
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int xf = __shfl_up(fi, o);
      int xr[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) xr[c] = __shfl_up(ri[c], o);
      if (lane >= o) {
        fi += xf;
#pragma unroll
        for (int c = 0; c < 4; ++c) ri[c] += xr[c];
      }
    }
    __syncthreads();                          // the first pass is done with its LDS; wsum is free
    if (lane == 63) {
      wsum[0][wave] = fi;
#pragma unroll
      for (int c = 0; c < 4; ++c) wsum[1 + c][wave] = ri[c];
    }
    __syncthreads();
    int fo = fi - f_sum, ro[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) ro[c] = ri[c] - r_sum[c];
    for (int ww = 0; ww < wave; ++ww) {
      fo += wsum[0][ww];
#pragma unroll
      for (int c = 0; c < 4; ++c) ro[c] += wsum[1 + c][ww];
    }
    for (int u = 0; u < per; ++u) {
      const int grp = g0 + u;
      if (grp >= G) break;
      pfx_full[grp] += fo;
#pragma unroll
      for (int c = 0; c < 4; ++c) pfx_rem[c][grp] = (unsigned short)(pfx_rem[c][grp] + ro[c]);
    }
    if (tid == 255) {
      pfx_full[G] = wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
#pragma unroll
      for (int c = 0; c < 4; ++c) pfx_rem[c][G] = (unsigned short)(wsum[1 + c][0] + wsum[1 + c][1] + wsum[1 + c][2] + wsum[1 + c][3]);
    }
    if (tid == 0) {
      const bool valid = p.sched && (uint32_t)(took >> 32) + (uint32_t)took == kSchedMagic;
      s_next = valid ? (int)(uint32_t)took : w;
      s_dynamic = valid ? 1 : 0;
    }
    __syncthreads();
  }
  const int first_more = G > W ? G - W : 0;   // first slices that the first pass did not cover
  const int UF = pfx_full[G];
  const int UR3 = pfx_rem[3][G], UR2 = pfx_rem[2][G], UR1 = pfx_rem[1][G], UR0 = pfx_rem[0][G];
  const int D = first_more + UF + UR3 + UR2 + UR1 + UR0;
  const bool dynamic = s_dynamic != 0;
  int d = s_next;
  __syncthreads();

  while (d < D) {
    int grp, split;
    if (d < first_more) {
      grp = W + d;
      split = 0;
    } else {
      int key = d - first_more;
      int lo = 0, hi = G;                     // invariant: pfx[lo] <= key < pfx[hi]
      if (key < UF) {
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (pfx_full[mid] <= key) lo = mid; else hi = mid;
        }
        split = 1 + key - pfx_full[lo];
      } else {
        key -= UF;
        int c = 3;                            // longest class first
        if (key >= UR3) { key -= UR3; c = 2; if (key >= UR2) { key -= UR2; c = 1; if (key >= UR1) { key -= UR1; c = 0; } } }
        const unsigned short* pfx = pfx_rem[c];
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if ((int)pfx[mid] <= key) lo = mid; else hi = mid;
        }
        split = 1 + pfx_full[lo + 1] - pfx_full[lo];
      }
      // pfx[lo] <= key < pfx[lo + 1]: group lo owns the unit (groups without a unit of this kind repeat
      // their successor's prefix value and are never landed on)
      grp = lo;
    }
    decode_slice<ROWS128, B16>(p, smem, grp / p.Hkv, grp % p.Hkv, split);
    if (tid == 0)
      s_next = dynamic ? (int)(uint32_t)__hip_atomic_fetch_add(p.sched, kTake, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                       : d + W;
    __syncthreads();                          // next unit known; the slice's LDS (K tiles / merge arrays) is free again
    d = s_next;
    __syncthreads();
  }
}

hipError_t launch_decode_split_mfma(const DecodeParams& p, hipStream_t s) {
  const bool rows128 = p.stride_token == kHeadDim;
  if (p.persist_wgs > 0) {
    const dim3 grid(p.persist_wgs);
    if (p.block_size == 16) {
      if (rows128) hipLaunchKernelGGL((seer_decode_persist_mfma_kernel<true, true>), grid, dim3(256), 0, s, p);
      else hipLaunchKernelGGL((seer_decode_persist_mfma_kernel<false, true>), grid, dim3(256), 0, s, p);
    } else {
      if (rows128) hipLaunchKernelGGL((seer_decode_persist_mfma_kernel<true, false>), grid, dim3(256), 0, s, p);
      else hipLaunchKernelGGL((seer_decode_persist_mfma_kernel<false, false>), grid, dim3(256), 0, s, p);
    }
    return hipGetLastError();
  }
  const dim3 grid = decode_grid(p);
  if (p.block_size == 16) {
    if (rows128) hipLaunchKernelGGL((seer_decode_split_mfma_kernel<true, true>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((seer_decode_split_mfma_kernel<false, true>), grid, dim3(256), 0, s, p);
  } else {
    if (rows128) hipLaunchKernelGGL((seer_decode_split_mfma_kernel<true, false>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((seer_decode_split_mfma_kernel<false, false>), grid, dim3(256), 0, s, p);
  }
  return hipGetLastError();
}

bool decode_persist_possible(int groups) { return groups <= kMaxPersistGroups; }

}  // namespace seer
