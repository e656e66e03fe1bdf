// Internal declarations shared by the host ABI layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace seer {

constexpr int kHeadDim = 128;   // d and d_gate; one row is 256 bytes = 16 lanes x 16 B
constexpr int kMaxGroup = 8;    // query heads per kv head
constexpr int kMaxRows = 16;    // query rows (new tokens x heads of a group) per kv head = one MFMA tile side
constexpr uint32_t kSchedMagic = 0x5EE7C0DEu;   // high half + low half of a valid unit hand-out word
constexpr size_t kDecodeWsHeader = 256;         // bytes in front of the partials: the hand-out word

struct DecodeParams {
  const uint16_t* q;            // bf16 [B,q_len,Hq,128]
  const uint16_t* k;
  const uint16_t* v;
  int64_t stride_seq, stride_head, stride_token;
  const int32_t* page_table;    // or nullptr
  int32_t max_pages, page_size;
  const int32_t* seqlens;       // [B]
  const int32_t* block_idx;     // [B,Hkv,max_sel] or nullptr (dense)
  const int32_t* nblk;          // [B,Hkv]
  int32_t max_blocks;           // max_sel (sparse) or block cap (dense)
  int32_t B, Hq, Hkv, g, block_size;
  int32_t q_len, rows;          // new tokens per sequence (1 = plain decode), rows = q_len * g
  float scale_log2e;            // scale * log2(e): logits are kept in the base-2 domain
  int32_t num_splits, blocks_per_split;
  int32_t persist_wgs;          // > 0: that many work-groups walk the slices that exist (ragged lists), else one per (group, slice)
  unsigned long long* sched;    // workspace word handing out units to them, or nullptr (round-robin)
  float* part_acc;              // [B*Hkv, num_splits, rows, 128] unnormalised partial outputs
  float* part_ml;               // [B*Hkv, num_splits, rows, 2]   running max (base-2 domain), sum
  void* out;                    // [B,q_len,Hq,128] bf16 or fp32
  float* lse;                   // [B,q_len,Hq] or nullptr
  int32_t out_is_f32;
};

struct GateParams {
  const uint16_t* q_gate;       // bf16 [B,Hkv,128]
  const uint16_t* kc;
  int64_t kc_stride_batch, kc_stride_head, kc_stride_block;
  const int32_t* seqlens;
  int32_t B, Hkv, nb_max, block_size;
  int32_t mode;                 // seer_select_mode: 0 top-k, 1 threshold, 2 top-p
  int32_t budget_tokens;
  const int32_t* budget_blocks; // [B] or nullptr
  double threshold;             // tau (mode 1) or p (mode 2)
  double inv_sqrt_dg;
  int32_t* block_idx;           // [B,Hkv,max_sel]
  int32_t* nblk;                // [B,Hkv]
  int32_t max_sel;
  double* scores;               // workspace [B,Hkv,nb_max]
};

struct FrontQParams {
  const uint16_t* q_nope;       // bf16 [B,Hq,128] pre-RoPE queries of the current token
  const uint16_t* wq;           // bf16 [Hkv,128,g*128]
  const float* rope_cos;        // [n_pos,64]
  const float* rope_sin;
  int32_t n_pos;
  const int32_t* seqlens;
  int32_t B, Hq, Hkv, g;
  uint16_t* q_gate;             // bf16 [B,Hkv,128]
};

struct FrontKParams {
  const uint16_t* k_nope;       // pre-RoPE keys, KV-cache addressing
  int64_t stride_seq, stride_head, stride_token;
  const int32_t* page_table;
  int32_t max_pages, page_size;
  const uint16_t* wk;           // bf16 [Hkv,128,384]
  const float* rope_cos;
  const float* rope_sin;
  int32_t n_pos;
  const int32_t* seqlens;
  const int32_t* block_begin;   // [B] or nullptr
  const int32_t* block_end;     // [B] or nullptr
  int32_t B, Hkv, nb_max, block_size;
  int32_t tiles_per_wg;         // 16-block tiles handled by one work-group (set by the launcher)
  uint16_t* kc;
  int64_t kc_stride_batch, kc_stride_head, kc_stride_block;
};

struct TrainFwdParams {
  const uint16_t* q;            // bf16 [B,T,Hq,128]
  const uint16_t* k;            // contiguous KV addressing
  const uint16_t* v;
  int64_t stride_seq, stride_head, stride_token;
  const int32_t* seqlens;       // [B] or nullptr
  int32_t B, T, Hq, Hkv, g, block_size, nb;
  int32_t Tp;                   // T rounded up to a multiple of 16
  float scale_log2e;
  float* raw;                   // per (sequence, head): block maxima of the base-2 logits, block-major and
                                // triangular - block j holds rows j*block_size .. Tp-1 (see raw_block_offset)
  float* lse2;                  // [B,Hq,T] base-2 log-sum-exp of every query row
  void* out;                    // [B,T,Hq,128]
  float* lse;                   // [B,T,Hq] or nullptr
  float* gt;                    // [B,Hkv,T,nb]
  int32_t out_is_f32;
};

// Layout of TrainFwdParams::raw for one (sequence, head).  A query row sees block j only from row
// j*block_size on, so block j stores rows j*bs .. Tp-1 (Tp - j*bs floats, a multiple of 16) and the
// blocks follow each other: half the footprint of a full [nb][Tp] rectangle.
__host__ __device__ inline int64_t raw_block_offset(int64_t j, int64_t Tp, int64_t bs) {
  return j * Tp - bs * (j * (j - 1) / 2);
}
__host__ __device__ inline int64_t raw_head_elems(int64_t nb, int64_t Tp, int64_t bs) { return raw_block_offset(nb, Tp, bs); }
// element of (block j, row q), q >= j*bs
__host__ __device__ inline int64_t raw_index(int64_t j, int64_t q, int64_t Tp, int64_t bs) {
  return raw_block_offset(j, Tp, bs) + (q - j * bs);
}

// Launchers (each returns the hipError_t of the launch).
hipError_t launch_attn_fwd(const TrainFwdParams& p, hipStream_t s);
hipError_t launch_gt_finalize(const TrainFwdParams& p, hipStream_t s);
hipError_t launch_gate_q(const FrontQParams& p, hipStream_t s);
hipError_t launch_kc_update(const FrontKParams& p, int max_blocks, int cus, hipStream_t s);
hipError_t launch_gate_score(const GateParams& p, bool ragged, hipStream_t s);
hipError_t launch_gate_select(const GateParams& p, hipStream_t s);
bool gate_fused_possible(const GateParams& p);
hipError_t launch_gate_fused(const GateParams& p, hipStream_t s);
hipError_t launch_decode_split_valu(const DecodeParams& p, hipStream_t s);
hipError_t launch_decode_split_mfma(const DecodeParams& p, hipStream_t s);
hipError_t launch_decode_merge(const DecodeParams& p, hipStream_t s);
bool decode_persist_possible(int groups);
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int wgs, hipStream_t s);

// ---- device helpers -------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// 16-byte load of data that is read exactly once per call (K/V rows, compression-cache rows).
// Marked non-temporal: on MI355X this raised the sparse decode kernel from 6.0 to 6.8 TB/s, the
// streamed rows no longer displace each other through the cache hierarchy on their way in.
#ifndef SEER_NT_LOADS
#define SEER_NT_LOADS 1
#endif
__device__ __forceinline__ uint4 load_stream16(const uint16_t* ptr) {
#if SEER_NT_LOADS
  typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(ptr));
  return make_uint4(r[0], r[1], r[2], r[3]);
#else
  return *reinterpret_cast<const uint4*>(ptr);
#endif
}

// Work-group -> (split, kv head, sequence).  Grid (Hkv, B, num_splits): the split index is the
// slowest dimension, so consecutive work-group ids are consecutive (sequence, kv-head) groups of
// the same split.  Work-groups are handed to the 8 XCDs round-robin by linear id, so every XCD
// gets an equal share of every split; with the split fastest, XCD k would receive only split k
// of every group, and the later splits are empty for all but the longest lists (measured on the
// variable-length workloads: 1.75x slower).
__device__ __forceinline__ void decode_wg_coords(const DecodeParams& p, int* split, int* hk, int* i) {
  *hk = blockIdx.x;
  *i = blockIdx.y;
  *split = blockIdx.z;
}
inline dim3 decode_grid(const DecodeParams& p) { return dim3(p.Hkv, p.B, p.num_splits); }

// Number of list entries of a group and the list itself (nullptr: dense, entry p is block p).
__device__ __forceinline__ int group_list(const DecodeParams& p, int64_t grp, int nb,
                                          const int32_t** list) {
  if (p.block_idx) {
    int n = p.nblk[grp];
    n = n < 0 ? 0 : n;
    *list = p.block_idx + grp * p.max_blocks;
    return n < p.max_blocks ? n : p.max_blocks;
  }
  *list = nullptr;
  return nb < p.max_blocks ? nb : p.max_blocks;
}

// Element offset of the first token of block j of (sequence i, kv head hk).
__device__ __forceinline__ int64_t block_offset(const DecodeParams& p, int i, int hk, int j) {
  const int64_t t0 = (int64_t)j * p.block_size;
  if (p.page_table) {
    const int64_t page = p.page_table[(int64_t)i * p.max_pages + t0 / p.page_size];
    return page * p.stride_seq + (int64_t)hk * p.stride_head + (t0 % p.page_size) * p.stride_token;
  }
  return (int64_t)i * p.stride_seq + (int64_t)hk * p.stride_head + t0 * p.stride_token;
}

// fp32 -> bf16, round to nearest even.
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Final value of one output element from a (max, sum, unnormalised accumulator) triple in the
// base-2 domain; also writes lse (natural log) from the thread that owns feature 0.
__device__ __forceinline__ void store_output(const DecodeParams& p, int64_t row, int dd, float ma,
                                             float l, float a) {
  const float r = (l > 0.f) ? a / l : 0.f;
  if (p.out_is_f32) reinterpret_cast<float*>(p.out)[row * kHeadDim + dd] = r;
  else reinterpret_cast<uint16_t*>(p.out)[row * kHeadDim + dd] = f32_to_bf16_rne(r);
  if (dd == 0 && p.lse) p.lse[row] = (l > 0.f) ? (ma + log2f(l)) * 0.6931471805599453f : -INFINITY;
}

// Row r of a group's tile is (new token t = r / g, head h = r % g); its place in out / lse.
__device__ __forceinline__ int64_t output_row(const DecodeParams& p, int i, int hk, int r) {
  const int t = r / p.g, h = r - t * p.g;
  return ((int64_t)i * p.q_len + t) * p.Hq + (int64_t)hk * p.g + h;
}

// What a split kernel does with the merged (ma, l, a) of its slice for (row r, feature dd):
// with a single split it is the final result, otherwise a partial for the merge kernel.
__device__ __forceinline__ void emit_slice(const DecodeParams& p, int i, int hk, int split, int r,
                                           int dd, float ma, float l, float a) {
  const int64_t grp = (int64_t)i * p.Hkv + hk;
  if (p.num_splits == 1) {
    store_output(p, output_row(p, i, hk, r), dd, ma, l, a);
  } else {
    const int64_t pidx = (grp * p.num_splits + split) * p.rows + r;
    p.part_acc[pidx * kHeadDim + dd] = a;
    if (dd == 0) {
      p.part_ml[pidx * 2 + 0] = ma;
      p.part_ml[pidx * 2 + 1] = l;
    }
  }
}

// A work-group whose slice starts past the end of the list has nothing to do, except that with a
// single split it owns the (empty) result of the group.
__device__ __forceinline__ void emit_empty_if_single_split(const DecodeParams& p, int i, int hk) {
  if (p.num_splits != 1) return;
  for (int o = threadIdx.x; o < p.rows * kHeadDim; o += blockDim.x)
    store_output(p, output_row(p, i, hk, o / kHeadDim), o % kHeadDim, -INFINITY, 0.f, 0.f);
}

}  // namespace seer
