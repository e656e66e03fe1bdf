// Internal declarations shared by the host ABI layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace seer {

constexpr int kHeadDim = 128;   // d and d_gate; one row is 256 bytes = 16 lanes x 16 B
constexpr int kMaxGroup = 8;    // query heads per kv head

struct DecodeParams {
  const uint16_t* q;            // bf16 [B,Hq,128]
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
  float scale_log2e;            // scale * log2(e): logits are kept in the base-2 domain
  int32_t num_splits, blocks_per_split;
  float* part_acc;              // [B*Hkv, num_splits, g, 128] unnormalised partial outputs
  float* part_ml;               // [B*Hkv, num_splits, g, 2]   running max (base-2 domain), sum
  void* out;                    // [B,Hq,128] bf16 or fp32
  float* lse;                   // [B,Hq] or nullptr
  int32_t out_is_f32;
};

struct GateParams {
  const uint16_t* q_gate;       // bf16 [B,Hkv,128]
  const uint16_t* kc;
  int64_t kc_stride_batch, kc_stride_head, kc_stride_block;
  const int32_t* seqlens;
  int32_t B, Hkv, nb_max, block_size;
  int32_t mode;                 // 0 top-k, 1 threshold
  int32_t budget_tokens;
  const int32_t* budget_blocks; // [B] or nullptr
  double threshold;
  double inv_sqrt_dg;
  int32_t* block_idx;           // [B,Hkv,max_sel]
  int32_t* nblk;                // [B,Hkv]
  int32_t max_sel;
  double* scores;               // workspace [B,Hkv,nb_max]
};

// Launchers (each returns the hipError_t of the launch).
hipError_t launch_gate_score(const GateParams& p, hipStream_t s);
hipError_t launch_gate_select(const GateParams& p, hipStream_t s);
hipError_t launch_decode_split_valu(const DecodeParams& p, hipStream_t s);
hipError_t launch_decode_split_mfma(const DecodeParams& p, hipStream_t s);
hipError_t launch_decode_merge(const DecodeParams& p, hipStream_t s);

// ---- device helpers -------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

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

}  // namespace seer
