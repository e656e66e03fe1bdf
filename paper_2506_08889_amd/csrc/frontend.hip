// AttnGate front-end on gfx950: the Q branch (Eq. 1a) that turns the g pre-RoPE query heads of a
// kv head into one gate query, and the K branch (Eq. 1b) that turns a block of b pre-RoPE keys
// into one entry of the K Compression Cache (Sec. 3.2): max / min / average pooling over the
// tokens, concatenation, a per-kv-head linear layer and RoPE at the block's first position.
//
// Both are a batch of matrix-vector products against one weight matrix per kv head, so 16 vectors
// are processed together as the N side of v_mfma_f32_16x16x32_bf16 (operand layout as in
// decode_mfma.hip: lane = 16*q + n; A row n, B column n, k = 8q..8q+7; D column n, rows 4q..4q+3).
// The 128 output features are 8 M-tiles; a wave (K branch) or a work-group (Q branch) owns tiles t and
// t + 4, i.e. features [16t, 16t+16) and their rotate-half partners [64+16t, 64+16t+16), so RoPE is
// lane-local.
#include "seer_internal.h"

namespace seer {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef short s16x2_t __attribute__((ext_vector_type(2)));

namespace {

__device__ __forceinline__ uint32_t pack2_bf16_rne(float a, float b) {
  return (uint32_t)f32_to_bf16_rne(a) | ((uint32_t)f32_to_bf16_rne(b) << 16);
}

// Rotate-half RoPE on the two accumulators of a lane (features c = c0..c0+3 and c + 64) and store.
__device__ __forceinline__ void rope_store(const f32x4_t& lo, const f32x4_t& hi, const float* rope_cos,
                                           const float* rope_sin, int64_t pos, int c0, uint16_t* dst) {
  const float4 co = *reinterpret_cast<const float4*>(rope_cos + pos * (kHeadDim / 2) + c0);
  const float4 si = *reinterpret_cast<const float4*>(rope_sin + pos * (kHeadDim / 2) + c0);
  const float cv[4] = {co.x, co.y, co.z, co.w}, sv[4] = {si.x, si.y, si.z, si.w};
  float zl[4], zh[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    zl[r] = lo[r] * cv[r] - hi[r] * sv[r];
    zh[r] = hi[r] * cv[r] + lo[r] * sv[r];
  }
  *reinterpret_cast<uint2*>(dst + c0) = make_uint2(pack2_bf16_rne(zl[0], zl[1]), pack2_bf16_rne(zl[2], zl[3]));
  *reinterpret_cast<uint2*>(dst + kHeadDim / 2 + c0) =
      make_uint2(pack2_bf16_rne(zh[0], zh[1]), pack2_bf16_rne(zh[2], zh[3]));
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Q branch.  Grid (ceil(B/16), Hkv, 4); a work-group computes, for 16 sequences of one kv head, the
// 16 output features [16z, 16z+16) and their rotate-half partners (+64).  The g*128 input features
// are cut into 4g steps of 32; wave v takes steps [v*g, (v+1)*g) and issues all of its loads at once
// (B operand straight from q_nope - the g heads of a group are contiguous - and two weight rows per
// lane), so the kernel is one memory round trip deep; the four partial tiles are added in wave order
// through LDS and wave 0 applies RoPE and stores.  (The first form walked the whole input per wave in
// g dependent rounds: 13.9 us at batch 64 against the launch floor this one sits on.)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void seer_gate_q_kernel(FrontQParams p) {
  __shared__ float part[3][2][64][4];                // partial tiles of waves 1..3

  const int h = blockIdx.y, i0 = blockIdx.x * 16, z = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n16 = lane & 15, q4 = lane >> 4;
  const int g = p.g, gd = g * kHeadDim;
  const int i = i0 + n16;
  const bool valid = i < p.B;

  int64_t pos = 0;
  if (wave == 0 && valid) pos = (int64_t)p.seqlens[i] - 1;          // requested first: the rotation angles depend on it

  const uint16_t* x = p.q_nope + ((int64_t)(valid ? i : 0) * p.Hq + (int64_t)h * g) * kHeadDim + wave * g * 32 + q4 * 8;
  const uint16_t* w0 = p.wq + ((int64_t)h * kHeadDim + 16 * z + n16) * gd + wave * g * 32 + q4 * 8;
  const uint16_t* w1 = w0 + (int64_t)64 * gd;
  uint4 b[kMaxGroup], a0[kMaxGroup], a1[kMaxGroup];
#pragma unroll
  for (int u = 0; u < kMaxGroup; ++u) {
    if (u < g) {
      b[u] = make_uint4(0, 0, 0, 0);
      if (valid) b[u] = *reinterpret_cast<const uint4*>(x + u * 32);
      a0[u] = *reinterpret_cast<const uint4*>(w0 + u * 32);
      a1[u] = *reinterpret_cast<const uint4*>(w1 + u * 32);
    }
  }
  const int c0 = 16 * z + 4 * q4;                     // this lane's features c0..c0+3 (and +64)
  float4 co = make_float4(1.f, 1.f, 1.f, 1.f), si = make_float4(0.f, 0.f, 0.f, 0.f);
  if (wave == 0 && valid) {
    pos = pos < 0 ? 0 : (pos >= p.n_pos ? p.n_pos - 1 : pos);
    co = *reinterpret_cast<const float4*>(p.rope_cos + pos * (kHeadDim / 2) + c0);
    si = *reinterpret_cast<const float4*>(p.rope_sin + pos * (kHeadDim / 2) + c0);
  }
  f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < kMaxGroup; ++u) {
    if (u < g) {
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a0[u]), __builtin_bit_cast(bf16x8_t, b[u]), acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a1[u]), __builtin_bit_cast(bf16x8_t, b[u]), acc1, 0, 0, 0);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      part[wave - 1][0][lane][r] = acc0[r];
      part[wave - 1][1][lane][r] = acc1[r];
    }
  }
  __syncthreads();
  if (wave != 0 || !valid) return;
#pragma unroll
  for (int v = 0; v < 3; ++v)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      acc0[r] += part[v][0][lane][r];
      acc1[r] += part[v][1][lane][r];
    }
  // rotate-half RoPE on the lane's two accumulators (features c and c + 64) and store
  const float cv[4] = {co.x, co.y, co.z, co.w}, sv[4] = {si.x, si.y, si.z, si.w};
  float zl[4], zh[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    zl[r] = acc0[r] * cv[r] - acc1[r] * sv[r];
    zh[r] = acc1[r] * cv[r] + acc0[r] * sv[r];
  }
  uint16_t* dst = p.q_gate + ((int64_t)i * p.Hkv + h) * kHeadDim;
  *reinterpret_cast<uint2*>(dst + c0) = make_uint2(pack2_bf16_rne(zl[0], zl[1]), pack2_bf16_rne(zl[2], zl[3]));
  *reinterpret_cast<uint2*>(dst + kHeadDim / 2 + c0) = make_uint2(pack2_bf16_rne(zh[0], zh[1]), pack2_bf16_rne(zh[2], zh[3]));
}

// ---------------------------------------------------------------------------------------------
// K branch.  Grid (ceil(max_blocks/16), Hkv, B); a work-group handles 16 consecutive blocks of one
// (sequence, kv head): each wave pools 4 of them (16 lanes per 256-byte key row, coalesced,
// non-temporal), the pooled vectors go to a swizzled LDS tile as the B operand
// [max | min | avg_hi | avg_lo] (the fp32 average is carried as two bf16 terms so the bf16 MFMA
// loses nothing; the weight columns of the average are simply used twice), then
// Y[128 x 16] = W U^T, RoPE, store.  Memory-bound on the key read: 256 B per (token, kv head).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void seer_kc_update_kernel(FrontKParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char u_lds[16 * 1024];   // 16 blocks x 512 bf16

  const int h = blockIdx.y, i = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n16 = lane & 15, q4 = lane >> 4;
  const int bs = p.block_size;

  int S = p.seqlens[i];
  S = S < 0 ? 0 : S;
  int nfull = S / bs;
  nfull = nfull < p.nb_max ? nfull : p.nb_max;
  int j0 = p.block_begin ? p.block_begin[i] : 0;
  int j1 = p.block_end ? p.block_end[i] : nfull;
  j0 = j0 < 0 ? 0 : j0;
  j1 = j1 > nfull ? nfull : j1;
  if (j0 + (int)blockIdx.x * p.tiles_per_wg * 16 >= j1) return;

  // The weight rows of this wave (2 M-tiles x 512 input features) stay in registers for all tiles
  // of the work-group: re-reading them per tile cost as many (poorly coalesced) load instructions
  // as the keys themselves.
  const int d3 = 3 * kHeadDim;
  uint4 wa0[16], wa1[16];
  {
    const uint16_t* w0 = p.wk + ((int64_t)h * kHeadDim + 16 * wave + n16) * d3 + q4 * 8;
    const uint16_t* w1 = w0 + (int64_t)64 * d3;
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      const int wcol = (kk < 12 ? kk : kk - 4) * 32;        // avg_lo reuses the average's weight columns
      wa0[kk] = *reinterpret_cast<const uint4*>(w0 + wcol);
      wa1[kk] = *reinterpret_cast<const uint4*>(w1 + wcol);
    }
  }

  for (int tile = 0; tile < p.tiles_per_wg; ++tile) {
  const int jt = j0 + ((int)blockIdx.x * p.tiles_per_wg + tile) * 16;   // first block of this tile
  if (jt >= j1) break;
  if (tile > 0) __syncthreads();                 // the previous tile's pooled vectors have been consumed

  // ---- pooling: wave w handles blocks jt + 4w .. jt + 4w + 3 --------------------------------
  // The rows of a lane (q4, q4 + 4, ...) are taken 8 at a time ("chunk"); the loads of the next
  // chunk - possibly of the next block - are issued before the current chunk is reduced.
  const int trips = (bs + 31) >> 5;              // chunks per block
  const int nchunks = 4 * trips;
  auto block_base = [&](int j) -> const uint16_t* {
    const int64_t t0 = (int64_t)j * bs;
    int64_t off;
    if (p.page_table) {
      int64_t pi = t0 / p.page_size;
      pi = pi >= p.max_pages ? p.max_pages - 1 : pi;
      off = (int64_t)p.page_table[(int64_t)i * p.max_pages + pi] * p.stride_seq + (int64_t)h * p.stride_head +
            (t0 % p.page_size) * p.stride_token;
    } else {
      off = (int64_t)i * p.stride_seq + (int64_t)h * p.stride_head + t0 * p.stride_token;
    }
    return p.k_nope + off + n16 * 8;
  };
  auto load_chunk = [&](uint4 (&r)[8], int ch) {
    const int bb = ch / trips, trip = ch - bb * trips;
    const int j = jt + 4 * wave + bb;
    const int t = q4 + 32 * trip;
#pragma unroll
    for (int u = 0; u < 8; ++u) r[u] = make_uint4(0, 0, 0, 0);
    if (j < j1) {
      const uint16_t* base = block_base(j);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (t + 4 * u < bs) r[u] = load_stream16(base + (int64_t)(t + 4 * u) * p.stride_token);
    }
  };

  // Running statistics of the current block, per lane 8 features (4 words of 2 bf16):
  //   max / min on the raw 16-bit patterns made order-preserving (magnitude bits flipped for
  //   negative values) with packed int16 max / min - no unpacking, no NaN canonicalisation;
  //   sum by v_dot2_f32_bf16 against (1, 1) on row pairs interleaved with one byte permute.
  uint32_t smax[4], smin[4];
  float sm[8];
  auto reset_stats = [&]() {
#pragma unroll
    for (int e = 0; e < 4; ++e) { smax[e] = 0x80008000u; smin[e] = 0x7fff7fffu; }
#pragma unroll
    for (int e = 0; e < 8; ++e) sm[e] = 0.f;
  };
  auto sortable = [](uint32_t w) -> uint32_t {       // involution: also maps back
    const s16x2_t v = __builtin_bit_cast(s16x2_t, w);
    return __builtin_bit_cast(uint32_t, (s16x2_t)(v ^ ((v >> 15) & (short)0x7fff)));
  };
  const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3f803f80u);
  auto reduce_rows = [&](const uint4 (&r)[8], int nrow) {     // nrow = 4 or 8 valid rows (uniform)
#pragma unroll
    for (int u = 0; u < 8; u += 2) {
      if (u < nrow) {
        const uint32_t a[4] = {r[u].x, r[u].y, r[u].z, r[u].w};
        const uint32_t b[4] = {r[u + 1].x, r[u + 1].y, r[u + 1].z, r[u + 1].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const s16x2_t ta = __builtin_bit_cast(s16x2_t, sortable(a[e])), tb = __builtin_bit_cast(s16x2_t, sortable(b[e]));
          const s16x2_t hi = __builtin_elementwise_max(ta, tb), lo = __builtin_elementwise_min(ta, tb);
          smax[e] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2_t, smax[e]), hi));
          smin[e] = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(s16x2_t, smin[e]), lo));
          const uint32_t f0 = __builtin_amdgcn_perm(b[e], a[e], 0x05040100u);   // feature 2e of both rows
          const uint32_t f1 = __builtin_amdgcn_perm(b[e], a[e], 0x07060302u);   // feature 2e+1 of both rows
          sm[2 * e] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f0), ones, sm[2 * e], false);
          sm[2 * e + 1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f1), ones, sm[2 * e + 1], false);
        }
      }
    }
  };
  auto finish_block = [&](int n, int j) {
    // combine the 4 row groups of the wave, write the block's pooled vector, reset
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s16x2_t x = __builtin_bit_cast(s16x2_t, smax[e]), y = __builtin_bit_cast(s16x2_t, smin[e]);
      x = __builtin_elementwise_max(x, __builtin_bit_cast(s16x2_t, (uint32_t)__shfl_xor((int)__builtin_bit_cast(uint32_t, x), 16)));
      x = __builtin_elementwise_max(x, __builtin_bit_cast(s16x2_t, (uint32_t)__shfl_xor((int)__builtin_bit_cast(uint32_t, x), 32)));
      y = __builtin_elementwise_min(y, __builtin_bit_cast(s16x2_t, (uint32_t)__shfl_xor((int)__builtin_bit_cast(uint32_t, y), 16)));
      y = __builtin_elementwise_min(y, __builtin_bit_cast(s16x2_t, (uint32_t)__shfl_xor((int)__builtin_bit_cast(uint32_t, y), 32)));
      smax[e] = __builtin_bit_cast(uint32_t, x);
      smin[e] = __builtin_bit_cast(uint32_t, y);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) { sm[e] += __shfl_xor(sm[e], 16); sm[e] += __shfl_xor(sm[e], 32); }
    if (q4 == 0) {
      uint32_t pmx[4], pmn[4], phi[4], plo[4];
      const float inv = 1.0f / (float)bs;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pmx[e] = (j < j1) ? sortable(smax[e]) : 0u;             // back to bf16 patterns (exact values)
        pmn[e] = (j < j1) ? sortable(smin[e]) : 0u;
        const float v0 = sm[2 * e] * inv, v1 = sm[2 * e + 1] * inv;
        const uint16_t h0 = f32_to_bf16_rne(v0), h1 = f32_to_bf16_rne(v1);
        const float r0 = v0 - __uint_as_float((uint32_t)h0 << 16), r1 = v1 - __uint_as_float((uint32_t)h1 << 16);
        phi[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        plo[e] = pack2_bf16_rne(r0, r1);
      }
      // U[n][part*128 + 8*n16 .. +8]: 16-byte chunk index part*16 + n16, swizzled with n
      unsigned char* row = u_lds + n * 1024;
      *reinterpret_cast<uint4*>(row + (((0 * 16 + n16) ^ n) << 4)) = make_uint4(pmx[0], pmx[1], pmx[2], pmx[3]);
      *reinterpret_cast<uint4*>(row + (((1 * 16 + n16) ^ n) << 4)) = make_uint4(pmn[0], pmn[1], pmn[2], pmn[3]);
      *reinterpret_cast<uint4*>(row + (((2 * 16 + n16) ^ n) << 4)) = make_uint4(phi[0], phi[1], phi[2], phi[3]);
      *reinterpret_cast<uint4*>(row + (((3 * 16 + n16) ^ n) << 4)) = make_uint4(plo[0], plo[1], plo[2], plo[3]);
    }
    reset_stats();
  };
  auto process_chunk = [&](const uint4 (&r)[8], int ch) {
    const int bb = ch / trips, trip = ch - bb * trips;
    const int rows_left = (bs - 32 * trip + 3 - q4) >> 2;        // rows of this lane still in the block
    reduce_rows(r, rows_left >= 8 ? 8 : 4);                       // block sizes are multiples of 16
    if (trip == trips - 1) finish_block(4 * wave + bb, jt + 4 * wave + bb);
  };

  reset_stats();
  uint4 bufa[8], bufb[8];                      // ping-pong: the next chunk is in flight while one is reduced
  load_chunk(bufa, 0);
  for (int ch = 0; ch < nchunks; ch += 2) {    // nchunks = 4 * trips is even
    load_chunk(bufb, ch + 1);
    process_chunk(bufa, ch);
    if (ch + 2 < nchunks) load_chunk(bufa, ch + 2);
    process_chunk(bufb, ch + 1);
  }
  __syncthreads();

  // ---- Y = W U^T for this wave's two M-tiles --------------------------------------------------
  f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < 16; ++kk) {
    const uint4 b = *reinterpret_cast<const uint4*>(u_lds + n16 * 1024 + (((kk * 4 + q4) ^ n16) << 4));
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wa0[kk]), __builtin_bit_cast(bf16x8_t, b), acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wa1[kk]), __builtin_bit_cast(bf16x8_t, b), acc1, 0, 0, 0);
  }
  const int j = jt + n16;
  if (j < j1) {
    int64_t pos = (int64_t)j * bs;
    pos = pos >= p.n_pos ? p.n_pos - 1 : pos;
    rope_store(acc0, acc1, p.rope_cos, p.rope_sin, pos, 16 * wave + 4 * q4,
               p.kc + (int64_t)i * p.kc_stride_batch + (int64_t)h * p.kc_stride_head + (int64_t)j * p.kc_stride_block);
  }
  }   // tile loop
}

hipError_t launch_gate_q(const FrontQParams& p, hipStream_t s) {
  dim3 grid((p.B + 15) / 16, p.Hkv, 4);
  hipLaunchKernelGGL(seer_gate_q_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_kc_update(const FrontKParams& p0, int max_blocks, int cus, hipStream_t s) {
  FrontKParams p = p0;
  const long tiles = (max_blocks + 15) / 16;
  // enough work-groups for ~8 per CU, at most 16 tiles (256 blocks) per work-group
  long per = tiles * p.Hkv * p.B / ((long)cus * 8);
  per = per < 1 ? 1 : (per > 16 ? 16 : per);
  p.tiles_per_wg = (int)per;
  dim3 grid((unsigned)((tiles + per - 1) / per), p.Hkv, p.B);
  hipLaunchKernelGGL(seer_kc_update_kernel, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace seer
