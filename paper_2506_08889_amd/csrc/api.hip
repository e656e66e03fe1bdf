// Host side of the C ABI declared in include/seer.h: argument validation, split planning,
// workspace carving and kernel launches.  Nothing here allocates device memory or
// synchronises the stream (the optional profiling path creates HIP events).
#include "../../include/seer.h"

#include <math.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "seer_internal.h"

// Scratch memory of seer_sparse_decode_noalloc: part of the library's code object, one copy per GPU.
static __device__ __align__(256) unsigned char scratch[SEER_NOALLOC_SCRATCH_BYTES];

namespace {

// Measurement / test knobs (seer_set_knob).  Atomic so that a setter on one thread never tears a
// reader on another; a call reads each knob once.  What a caller knows about its own lists travels
// with the call (the `hints` argument), not through these.
std::atomic<int> g_knob_impl{0};
std::atomic<int> g_knob_splits{0};
std::atomic<int> g_knob_gate{0};

struct ProfEvent { int cls; hipEvent_t a, b; };
bool g_prof_on = false;
std::vector<ProfEvent> g_prof;
std::mutex g_prof_mu;

int cu_count() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
      cus = prop.multiProcessorCount;
    else
      cus = 256;   // MI355X
    (void)hipGetLastError();
  }
  return cus;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// How the block list is cut: num_splits slices of blocks_per_split list entries each (the
// partition runs over the list capacity, not over the blocks of the sequence, Sec. 3.3).
// Measured on MI355X for lists of equal length: about one work-group per CU is enough to reach
// the HBM rate, more slices only add partials for the merge kernel; and a merge launch costs
// about 6.5 us, which a work-group needs to read about 8 blocks of 64 tokens by itself
// (~0.8 us each), so short lists are only cut when the slices save more than the merge costs.
// A slice has at least 4 list entries.
// Lists of very different lengths (SEER_HINT_RAGGED_LISTS) get slices of about 2048 tokens so
// that the longest list is spread over many work-groups (about 1000 when the batch is small: batch 32
// with 8 k-64 k-token sequences at block 128 runs its split kernel in 88 us with 7-block slices against
// 92 us with 13-block ones, while batch 128 gets slower below 2048); equal-length lists lose ~5 % to
// slicing, hence the opt-in.  (Measured on batch 128 with mixed lengths, a work-group pays about 3 us for every
// slice it starts: slices of 512 / 1024 / 2048 / 4096 tokens give 73 / 77 / 80 / 82 % of the HBM peak
// at 50 % sparsity and 67 / 70 / 70-73 / 67-68 % at 95 %, where long slices no longer balance.)
constexpr long kMinSliceBlocks = 4;    // at least one block per wave of a work-group
constexpr long kMaxSplits = 256;

long max_splits_for(int max_blocks) {
  long m = (max_blocks + kMinSliceBlocks - 1) / kMinSliceBlocks;
  return m < 1 ? 1 : (m > kMaxSplits ? kMaxSplits : m);
}

void plan_splits(int B, int Hkv, int max_blocks, int block_size, bool ragged, int* num_splits,
                 int* blocks_per_split) {
  const long groups = (long)B * Hkv;
  const long slots = (long)cu_count();
  const long cap = max_splits_for(max_blocks);
  const int forced = g_knob_splits.load(std::memory_order_relaxed);
  long ns;
  if (forced > 0) {
    ns = forced;
  } else {
    ns = groups >= slots ? 1 : (slots + groups / 2) / groups;
    if (ns > cap) ns = cap;
    if (ns > 1) {
      // microseconds a lone work-group saves by reading max_blocks / ns blocks instead of all
      const double saved = 0.8 * (block_size / 64.0) * max_blocks * (1.0 - 1.0 / (double)ns);
      if (saved < 6.5) ns = 1;
    }
    if (ragged) {
      // about 2048 tokens per slice; shorter (down to 768) when the whole batch holds only a few slices
      // per resident work-group, so that a launch of two or three units per slot still ends evenly
      const double per_slot = (double)groups * max_blocks * block_size / (2.0 * (double)slots);   // upper bound
      long tok = (long)(per_slot / 3.0);
      tok = tok < 768 ? 768 : (tok > 2048 ? 2048 : tok);
      long len_r = tok / block_size;
      if (len_r < kMinSliceBlocks) len_r = kMinSliceBlocks;
      const long ns_r = (max_blocks + len_r - 1) / len_r;
      if (ns_r > ns) ns = ns_r;
    }
  }
  if (ns > cap) ns = cap;
  if (ns < 1) ns = 1;
  long len = (max_blocks + ns - 1) / ns;
  if (len < 1) len = 1;
  ns = (max_blocks + len - 1) / len;
  if (ns < 1) ns = 1;
  *num_splits = (int)ns;
  *blocks_per_split = (int)len;
}

// Workspace for the largest plan any knob setting can produce, so a size queried once stays valid.
size_t decode_ws_bytes(int B, int Hkv, int g, long num_splits) {
  const size_t parts = (size_t)B * Hkv * num_splits * g;
  return seer::kDecodeWsHeader + align_up(parts * seer::kHeadDim * sizeof(float), 256) +
         align_up(parts * 2 * sizeof(float), 256);
}

struct Timed {
  int cls;
  hipStream_t s;
  hipEvent_t a = nullptr, b = nullptr;
  bool on;
  Timed(int c, hipStream_t st) : cls(c), s(st), on(g_prof_on) {
    if (on) {
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
      (void)hipEventRecord(a, s);
    }
  }
  ~Timed() {
    if (on) {
      (void)hipEventRecord(b, s);
      std::lock_guard<std::mutex> lk(g_prof_mu);
      g_prof.push_back({cls, a, b});
    }
  }
};

bool block_size_ok(int bs) { return bs == 16 || bs == 32 || bs == 64 || bs == 128; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- built-in scratch of the entry point that allocates nothing --------------------------------
// Device memory that lives in the library's code object: every GPU that loads the library holds its
// own copy at its own address until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; the address it returns (per device) is what kernels receive.
constexpr size_t kNoAllocScratchBytes = SEER_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// Address of `scratch` on the current device; looked up once per device, with that device current.
seer_status scratch_of_current_device(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return SEER_ERR_HIP; }
  if (dev < 0 || dev >= kMaxDevices) return SEER_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return SEER_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return SEER_OK;
}

// builtin_scratch: the split-K partials go to the library's own `scratch` array instead of a caller
// workspace (workspace / workspace_bytes are ignored).
seer_status decode_common(const void* q, const seer_kv_layout* kv, const int32_t* seqlens,
                          const int32_t* block_idx, const int32_t* nblk, int max_blocks, bool sparse,
                          int B, int q_len, int Hq, int Hkv, int d, int block_size, float scale, void* out,
                          seer_dtype out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                          bool builtin_scratch, uint32_t hints, void* stream) {
  if (!q || !kv || !seqlens || !out) return SEER_ERR_NULL;
  if (!kv->k || !kv->v) return SEER_ERR_NULL;
  if (sparse && (!block_idx || !nblk)) return SEER_ERR_NULL;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || max_blocks <= 0 || d <= 0 || block_size <= 0 || q_len <= 0)
    return SEER_ERR_SHAPE;
  if (Hq % Hkv != 0) return SEER_ERR_SHAPE;
  if (B > 65535 || Hkv > 65535) return SEER_ERR_UNSUPPORTED;
  if (hints & ~(uint32_t)SEER_HINT_RAGGED_LISTS) return SEER_ERR_UNSUPPORTED;
  const int g = Hq / Hkv;
  const int rows = g * q_len;
  const int impl = g_knob_impl.load(std::memory_order_relaxed);
  if (d != seer::kHeadDim || g > seer::kMaxGroup || !block_size_ok(block_size)) return SEER_ERR_UNSUPPORTED;
  // several new tokens share the MFMA tile with the heads of the group: 16 rows, MFMA kernel only
  if (q_len > 1 && (rows > seer::kMaxRows || impl == 1)) return SEER_ERR_UNSUPPORTED;
  if (out_dtype != SEER_BF16 && out_dtype != SEER_F32) return SEER_ERR_UNSUPPORTED;
  if (kv->stride_token < d || (kv->stride_token % 8) || (kv->stride_head % 8) || (kv->stride_seq % 8))
    return SEER_ERR_SHAPE;
  if (!aligned16(kv->k) || !aligned16(kv->v) || !aligned16(q)) return SEER_ERR_SHAPE;
  if (kv->page_table) {
    if (kv->page_size <= 0 || kv->max_pages <= 0 || kv->page_size % block_size != 0) return SEER_ERR_SHAPE;
  }
  int ns, len;
  plan_splits(B, Hkv, max_blocks, block_size, (hints & SEER_HINT_RAGGED_LISTS) != 0, &ns, &len);
  if (builtin_scratch) {
    // the plan of this very call must fit the array; checked on the host, before the device is touched
    if (decode_ws_bytes(B, Hkv, rows, ns) > kNoAllocScratchBytes) return SEER_ERR_SCRATCH;
    const seer_status st = scratch_of_current_device(&workspace);
    if (st != SEER_OK) return st;
  } else {
    const size_t need = decode_ws_bytes(B, Hkv, rows, max_splits_for(max_blocks));
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
      return SEER_ERR_WORKSPACE;
  }

  seer::DecodeParams p{};
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(kv->k);
  p.v = static_cast<const uint16_t*>(kv->v);
  p.stride_seq = kv->stride_seq;
  p.stride_head = kv->stride_head;
  p.stride_token = kv->stride_token;
  p.page_table = kv->page_table;
  p.max_pages = kv->max_pages;
  p.page_size = kv->page_size;
  p.seqlens = seqlens;
  p.block_idx = sparse ? block_idx : nullptr;
  p.nblk = sparse ? nblk : nullptr;
  p.max_blocks = max_blocks;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.g = g; p.block_size = block_size;
  p.q_len = q_len;
  p.rows = rows;
  p.scale_log2e = (float)((double)scale * 1.4426950408889634);
  p.num_splits = ns;
  p.blocks_per_split = len;
  const size_t parts = (size_t)B * Hkv * ns * rows;
  char* ws = static_cast<char*>(workspace);
  p.part_acc = reinterpret_cast<float*>(ws + seer::kDecodeWsHeader);
  p.part_ml = reinterpret_cast<float*>(ws + seer::kDecodeWsHeader + align_up(parts * seer::kHeadDim * sizeof(float), 256));
  // Lists of very different lengths on the MFMA kernel: two work-groups per compute unit walk the slices
  // that exist, handed out through a word in front of the partials (kept valid by the merge kernel).
  const bool ragged = (hints & SEER_HINT_RAGGED_LISTS) != 0;
  if (ragged && impl != 1 && seer::decode_persist_possible(B * Hkv)) {
    const long units = (long)B * Hkv * ns, slots = 2L * cu_count();
    p.persist_wgs = (int)(units < slots ? units : slots);
    p.sched = ns > 1 ? reinterpret_cast<unsigned long long*>(ws) : nullptr;
  }
  p.out = out;
  p.lse = lse;
  p.out_is_f32 = out_dtype == SEER_F32;

  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool use_mfma = impl != 1;
  hipError_t e;
  {
    Timed t(SEER_KERNEL_DECODE_SPLIT, s);
    e = use_mfma ? seer::launch_decode_split_mfma(p, s) : seer::launch_decode_split_valu(p, s);
  }
  if (e != hipSuccess) return SEER_ERR_HIP;
  if (ns > 1) {   // a single slice wrote out and lse itself
    Timed t(SEER_KERNEL_DECODE_MERGE, s);
    e = seer::launch_decode_merge(p, s);
  }
  return e == hipSuccess ? SEER_OK : SEER_ERR_HIP;
}

}  // namespace

extern "C" {

int seer_version(void) { return 100; }

const char* seer_status_string(int status) {
  switch (status) {
    case SEER_OK: return "ok";
    case SEER_ERR_NULL: return "a required pointer is NULL";
    case SEER_ERR_SHAPE: return "bad or inconsistent sizes, strides or alignment";
    case SEER_ERR_UNSUPPORTED: return "unsupported configuration";
    case SEER_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SEER_ERR_CAPACITY: return "max_sel cannot hold the requested selection";
    case SEER_ERR_HIP: return "HIP runtime error";
    case SEER_ERR_SCRATCH: return "the call needs more than the built-in scratch buffer of the no-allocation entry point";
    default: return "unknown status";
  }
}

// Gate workspace: fp64 scores of every block, then the gate queries of seer_gate_select_q.
static size_t gate_scores_bytes(int B, int Hkv, int nb_max) { return align_up((size_t)B * Hkv * nb_max * sizeof(double), 256); }

seer_status seer_gate_workspace_bytes(int B, int Hkv, int nb_max, size_t* bytes) {
  if (!bytes) return SEER_ERR_NULL;
  if (B <= 0 || Hkv <= 0 || nb_max <= 0) return SEER_ERR_SHAPE;
  *bytes = gate_scores_bytes(B, Hkv, nb_max) + align_up((size_t)B * Hkv * seer::kHeadDim * sizeof(uint16_t), 256);
  return SEER_OK;
}

seer_status seer_decode_workspace_bytes(int B, int Hq, int Hkv, int d, int max_blocks, size_t* bytes) {
  if (!bytes) return SEER_ERR_NULL;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || max_blocks <= 0 || Hq % Hkv) return SEER_ERR_SHAPE;
  // Hq may be q_len * (query heads) for seer_sparse_decode_multi: up to 16 rows per kv head
  if (d != seer::kHeadDim || Hq / Hkv > seer::kMaxRows) return SEER_ERR_UNSUPPORTED;
  *bytes = decode_ws_bytes(B, Hkv, Hq / Hkv, max_splits_for(max_blocks));
  return SEER_OK;
}

seer_status seer_decode_plan(int B, int Hkv, int max_blocks, int block_size, uint32_t hints, int* num_splits,
                             int* blocks_per_split) {
  if (!num_splits || !blocks_per_split) return SEER_ERR_NULL;
  if (B <= 0 || Hkv <= 0 || max_blocks <= 0) return SEER_ERR_SHAPE;
  if (!block_size_ok(block_size) || (hints & ~(uint32_t)SEER_HINT_RAGGED_LISTS)) return SEER_ERR_UNSUPPORTED;
  plan_splits(B, Hkv, max_blocks, block_size, (hints & SEER_HINT_RAGGED_LISTS) != 0, num_splits, blocks_per_split);
  return SEER_OK;
}

seer_status seer_gate_select(const void* q_gate, const void* kc_cache, int64_t kc_stride_batch,
                             int64_t kc_stride_head, int64_t kc_stride_block, const int32_t* seqlens,
                             int B, int Hkv, int Dg, int nb_max, int block_size, seer_select_mode mode,
                             int32_t budget_tokens, const int32_t* budget_blocks, double threshold,
                             int32_t* block_idx, int32_t* nblk, int max_sel, void* workspace,
                             size_t workspace_bytes, uint32_t hints, void* stream) {
  if (!q_gate || !kc_cache || !seqlens || !block_idx || !nblk) return SEER_ERR_NULL;
  if (B <= 0 || Hkv <= 0 || Dg <= 0 || nb_max <= 0 || block_size <= 0 || max_sel <= 0) return SEER_ERR_SHAPE;
  if (B > 65535 || Hkv > 65535) return SEER_ERR_UNSUPPORTED;
  if (Dg != seer::kHeadDim || !block_size_ok(block_size)) return SEER_ERR_UNSUPPORTED;
  if (mode != SEER_SELECT_TOPK && mode != SEER_SELECT_THRESHOLD && mode != SEER_SELECT_TOPP) return SEER_ERR_UNSUPPORTED;
  if (hints & ~(uint32_t)SEER_HINT_RAGGED_LISTS) return SEER_ERR_UNSUPPORTED;
  if ((kc_stride_batch % 8) || (kc_stride_head % 8) || (kc_stride_block % 8) || kc_stride_block < Dg)
    return SEER_ERR_SHAPE;
  if (!aligned16(q_gate) || !aligned16(kc_cache)) return SEER_ERR_SHAPE;
  if (mode == SEER_SELECT_THRESHOLD || mode == SEER_SELECT_TOPP) {
    if (!(threshold == threshold)) return SEER_ERR_SHAPE;   // NaN
    if (max_sel < nb_max) return SEER_ERR_CAPACITY;
  } else if (!budget_blocks) {
    if (budget_tokens < 0) return SEER_ERR_SHAPE;
    long k = ((long)budget_tokens + block_size - 1) / block_size;
    if (k > nb_max) k = nb_max;
    if (max_sel < k) return SEER_ERR_CAPACITY;
  }
  size_t need = 0;
  seer_gate_workspace_bytes(B, Hkv, nb_max, &need);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SEER_ERR_WORKSPACE;

  seer::GateParams p{};
  p.q_gate = static_cast<const uint16_t*>(q_gate);
  p.kc = static_cast<const uint16_t*>(kc_cache);
  p.kc_stride_batch = kc_stride_batch;
  p.kc_stride_head = kc_stride_head;
  p.kc_stride_block = kc_stride_block;
  p.seqlens = seqlens;
  p.B = B; p.Hkv = Hkv; p.nb_max = nb_max; p.block_size = block_size;
  p.mode = (int)mode;
  p.budget_tokens = budget_tokens;
  p.budget_blocks = budget_blocks;
  p.threshold = threshold;
  p.inv_sqrt_dg = 1.0 / sqrt((double)Dg);
  p.block_idx = block_idx;
  p.nblk = nblk;
  p.max_sel = max_sel;
  p.scores = static_cast<double*>(workspace);

  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  // The fused kernel (one work-group per group computes its scores straight into LDS, then selects)
  // saves a launch and the score workspace and is the faster form wherever a group's scores fit into
  // LDS (measured in one process, step of gate + decode, fused vs score kernel + select kernel: batch
  // 16 x 32k tokens 59.0 vs 60.6 us; batch 32 x 8k-64k tokens at block 128 105.8 vs 109.0 us; batch
  // 128 x 4k-128k tokens 376 vs 382 us; batch 64 x 128k tokens 560.4 vs 562.2 us).  Longer caches take
  // the wide score kernel (every CU streams cache rows) followed by the select kernel.
  bool fused = seer::gate_fused_possible(p);
  const int gate_impl = g_knob_gate.load(std::memory_order_relaxed);
  if (gate_impl == 1) fused = false;
  if (fused) {
    Timed t(SEER_KERNEL_GATE_SELECT, s);
    e = seer::launch_gate_fused(p, s);
    return e == hipSuccess ? SEER_OK : SEER_ERR_HIP;
  }
  {
    Timed t(SEER_KERNEL_GATE_SCORE, s);
    e = seer::launch_gate_score(p, (hints & SEER_HINT_RAGGED_LISTS) != 0, s);
  }
  if (e != hipSuccess) return SEER_ERR_HIP;
  {
    Timed t(SEER_KERNEL_GATE_SELECT, s);
    e = seer::launch_gate_select(p, s);
  }
  return e == hipSuccess ? SEER_OK : SEER_ERR_HIP;
}

seer_status seer_sparse_decode(const void* q, const seer_kv_layout* kv, const int32_t* seqlens,
                               const int32_t* block_idx, const int32_t* nblk, int max_sel, int B, int Hq,
                               int Hkv, int d, int block_size, float scale, void* out,
                               seer_dtype out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                               uint32_t hints, void* stream) {
  return decode_common(q, kv, seqlens, block_idx, nblk, max_sel, true, B, 1, Hq, Hkv, d, block_size, scale,
                       out, out_dtype, lse, workspace, workspace_bytes, false, hints, stream);
}

seer_status seer_sparse_decode_noalloc(const void* q, const seer_kv_layout* kv, const int32_t* seqlens,
                                       const int32_t* block_idx, const int32_t* nblk, int max_sel, int B, int Hq,
                                       int Hkv, int d, int block_size, float scale, void* out,
                                       seer_dtype out_dtype, float* lse, uint32_t hints, void* stream) {
  return decode_common(q, kv, seqlens, block_idx, nblk, max_sel, true, B, 1, Hq, Hkv, d, block_size, scale,
                       out, out_dtype, lse, nullptr, 0, true, hints, stream);
}

seer_status seer_sparse_decode_multi(const void* q, const seer_kv_layout* kv, const int32_t* seqlens,
                                     const int32_t* block_idx, const int32_t* nblk, int max_sel, int B, int q_len,
                                     int Hq, int Hkv, int d, int block_size, float scale, void* out,
                                     seer_dtype out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                                     uint32_t hints, void* stream) {
  return decode_common(q, kv, seqlens, block_idx, nblk, max_sel, true, B, q_len, Hq, Hkv, d, block_size, scale,
                       out, out_dtype, lse, workspace, workspace_bytes, false, hints, stream);
}

seer_status seer_dense_decode(const void* q, const seer_kv_layout* kv, const int32_t* seqlens, int max_blocks,
                              int B, int Hq, int Hkv, int d, int block_size, float scale, void* out,
                              seer_dtype out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                              uint32_t hints, void* stream) {
  return decode_common(q, kv, seqlens, nullptr, nullptr, max_blocks, false, B, 1, Hq, Hkv, d, block_size,
                       scale, out, out_dtype, lse, workspace, workspace_bytes, false, hints, stream);
}

seer_status seer_gate_q(const void* q_nope, const void* wq, const float* rope_cos, const float* rope_sin,
                        int n_pos, const int32_t* seqlens, int B, int Hq, int Hkv, int d, int Dg, void* q_gate,
                        void* stream) {
  if (!q_nope || !wq || !rope_cos || !rope_sin || !seqlens || !q_gate) return SEER_ERR_NULL;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || n_pos <= 0 || Hq % Hkv) return SEER_ERR_SHAPE;
  if (Hkv > 65535) return SEER_ERR_UNSUPPORTED;
  if (d != seer::kHeadDim || Dg != seer::kHeadDim || Hq / Hkv > seer::kMaxGroup) return SEER_ERR_UNSUPPORTED;
  if (!aligned16(q_nope) || !aligned16(wq) || !aligned16(rope_cos) || !aligned16(rope_sin) || !aligned16(q_gate))
    return SEER_ERR_SHAPE;
  seer::FrontQParams p{};
  p.q_nope = static_cast<const uint16_t*>(q_nope);
  p.wq = static_cast<const uint16_t*>(wq);
  p.rope_cos = rope_cos;
  p.rope_sin = rope_sin;
  p.n_pos = n_pos;
  p.seqlens = seqlens;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.g = Hq / Hkv;
  p.q_gate = static_cast<uint16_t*>(q_gate);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  {
    Timed t(SEER_KERNEL_GATE_Q, s);
    e = seer::launch_gate_q(p, s);
  }
  return e == hipSuccess ? SEER_OK : SEER_ERR_HIP;
}

seer_status seer_gate_select_q(const void* q_nope, const void* wq, const float* rope_cos, const float* rope_sin,
                               int n_pos, const void* kc_cache, int64_t kc_stride_batch, int64_t kc_stride_head,
                               int64_t kc_stride_block, const int32_t* seqlens, int B, int Hq, int Hkv, int d, int Dg,
                               int nb_max, int block_size, seer_select_mode mode, int32_t budget_tokens,
                               const int32_t* budget_blocks, double threshold, int32_t* block_idx, int32_t* nblk,
                               int max_sel, void* q_gate_out, void* workspace, size_t workspace_bytes, uint32_t hints,
                               void* stream) {
  // The gate query of every group is made once, by a small kernel in front of the score kernel (the
  // 128 x g*128 matrix-vector product is far too much to repeat in each of the score kernel's
  // work-groups), into the tail of the workspace unless the caller wants to see it.
  if (!workspace || B <= 0 || Hkv <= 0 || nb_max <= 0) return !workspace ? SEER_ERR_WORKSPACE : SEER_ERR_SHAPE;
  size_t need = 0;
  seer_gate_workspace_bytes(B, Hkv, nb_max, &need);
  if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return SEER_ERR_WORKSPACE;
  void* q_gate = q_gate_out ? q_gate_out : static_cast<char*>(workspace) + gate_scores_bytes(B, Hkv, nb_max);
  // validate the selection's arguments before the first launch (NULL kc_cache etc. must not leave a
  // half-done call behind): the checks of seer_gate_select that do not depend on q_gate
  if (!kc_cache || !seqlens || !block_idx || !nblk) return SEER_ERR_NULL;
  if (block_size <= 0 || max_sel <= 0) return SEER_ERR_SHAPE;
  if (B > 65535 || Hkv > 65535 || !block_size_ok(block_size)) return SEER_ERR_UNSUPPORTED;
  if (mode != SEER_SELECT_TOPK && mode != SEER_SELECT_THRESHOLD && mode != SEER_SELECT_TOPP) return SEER_ERR_UNSUPPORTED;
  if (hints & ~(uint32_t)SEER_HINT_RAGGED_LISTS) return SEER_ERR_UNSUPPORTED;
  if ((kc_stride_batch % 8) || (kc_stride_head % 8) || (kc_stride_block % 8) || kc_stride_block < Dg) return SEER_ERR_SHAPE;
  if (!aligned16(kc_cache)) return SEER_ERR_SHAPE;
  if (mode == SEER_SELECT_THRESHOLD || mode == SEER_SELECT_TOPP) {
    if (!(threshold == threshold)) return SEER_ERR_SHAPE;
    if (max_sel < nb_max) return SEER_ERR_CAPACITY;
  } else if (!budget_blocks) {
    if (budget_tokens < 0) return SEER_ERR_SHAPE;
    long k = ((long)budget_tokens + block_size - 1) / block_size;
    if (k > nb_max) k = nb_max;
    if (max_sel < k) return SEER_ERR_CAPACITY;
  }
  seer_status st = seer_gate_q(q_nope, wq, rope_cos, rope_sin, n_pos, seqlens, B, Hq, Hkv, d, Dg, q_gate, stream);
  if (st != SEER_OK) return st;
  return seer_gate_select(q_gate, kc_cache, kc_stride_batch, kc_stride_head, kc_stride_block, seqlens, B, Hkv, Dg, nb_max,
                          block_size, mode, budget_tokens, budget_blocks, threshold, block_idx, nblk, max_sel, workspace,
                          workspace_bytes, hints, stream);
}

seer_status seer_kc_update(const seer_kv_layout* k_nope, const void* wk, const float* rope_cos,
                           const float* rope_sin, int n_pos, const int32_t* seqlens, const int32_t* block_begin,
                           const int32_t* block_end, int max_blocks, int B, int Hkv, int d, int Dg, int nb_max,
                           int block_size, void* kc_cache, int64_t kc_stride_batch, int64_t kc_stride_head,
                           int64_t kc_stride_block, void* stream) {
  if (!k_nope || !k_nope->k || !wk || !rope_cos || !rope_sin || !seqlens || !kc_cache) return SEER_ERR_NULL;
  if (B <= 0 || Hkv <= 0 || n_pos <= 0 || nb_max <= 0 || max_blocks <= 0 || block_size <= 0) return SEER_ERR_SHAPE;
  if (B > 65535 || Hkv > 65535) return SEER_ERR_UNSUPPORTED;
  if (d != seer::kHeadDim || Dg != seer::kHeadDim || !block_size_ok(block_size)) return SEER_ERR_UNSUPPORTED;
  if (k_nope->stride_token < d || (k_nope->stride_token % 8) || (k_nope->stride_head % 8) || (k_nope->stride_seq % 8))
    return SEER_ERR_SHAPE;
  if ((kc_stride_batch % 8) || (kc_stride_head % 8) || (kc_stride_block % 8) || kc_stride_block < Dg)
    return SEER_ERR_SHAPE;
  if (!aligned16(k_nope->k) || !aligned16(wk) || !aligned16(rope_cos) || !aligned16(rope_sin) || !aligned16(kc_cache))
    return SEER_ERR_SHAPE;
  if (k_nope->page_table &&
      (k_nope->page_size <= 0 || k_nope->max_pages <= 0 || k_nope->page_size % block_size != 0))
    return SEER_ERR_SHAPE;
  seer::FrontKParams p{};
  p.k_nope = static_cast<const uint16_t*>(k_nope->k);
  p.stride_seq = k_nope->stride_seq;
  p.stride_head = k_nope->stride_head;
  p.stride_token = k_nope->stride_token;
  p.page_table = k_nope->page_table;
  p.max_pages = k_nope->max_pages;
  p.page_size = k_nope->page_size;
  p.wk = static_cast<const uint16_t*>(wk);
  p.rope_cos = rope_cos;
  p.rope_sin = rope_sin;
  p.n_pos = n_pos;
  p.seqlens = seqlens;
  p.block_begin = block_begin;
  p.block_end = block_end;
  p.B = B; p.Hkv = Hkv; p.nb_max = nb_max; p.block_size = block_size;
  p.kc = static_cast<uint16_t*>(kc_cache);
  p.kc_stride_batch = kc_stride_batch;
  p.kc_stride_head = kc_stride_head;
  p.kc_stride_block = kc_stride_block;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  {
    Timed t(SEER_KERNEL_KC_UPDATE, s);
    e = seer::launch_kc_update(p, max_blocks < nb_max ? max_blocks : nb_max, cu_count(), s);
  }
  return e == hipSuccess ? SEER_OK : SEER_ERR_HIP;
}

static size_t attn_gt_ws_bytes(int B, int T, int Hq, int block_size) {
  const int64_t nb = ((int64_t)T + block_size - 1) / block_size, Tp = ((int64_t)T + 15) / 16 * 16;
  return align_up((size_t)B * Hq * (size_t)seer::raw_head_elems(nb, Tp, block_size) * sizeof(float), 256) +
         align_up((size_t)B * Hq * T * sizeof(float), 256);
}
// The finalize kernel addresses one head's block maxima with 32-bit offsets.
static bool attn_gt_rows_fit(int T, int block_size) {
  const double nb = ((double)T + block_size - 1) / block_size;
  return nb * ((double)T + 16) < 2147483648.0;
}
static bool attn_gt_sizes_ok(int B, int T, int Hq, int Hkv, seer_status* why) {
  if (B <= 0 || T <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv) { *why = SEER_ERR_SHAPE; return false; }
  if (B > 65535 || Hq > 65535) { *why = SEER_ERR_UNSUPPORTED; return false; }
  // one work-group per (sequence, query head, 128-row tile) in a 1-D grid
  if ((double)B * Hq * ((T + 127) / 128) > 2.0e9) { *why = SEER_ERR_UNSUPPORTED; return false; }
  return true;
}

seer_status seer_attn_ground_truth_workspace_bytes(int B, int T, int Hq, int Hkv, int d, int block_size,
                                                   size_t* bytes) {
  if (!bytes) return SEER_ERR_NULL;
  seer_status why;
  if (!attn_gt_sizes_ok(B, T, Hq, Hkv, &why)) return why;
  if (d != seer::kHeadDim || Hq / Hkv > seer::kMaxGroup ||
      !block_size_ok(block_size) || !attn_gt_rows_fit(T, block_size))
    return SEER_ERR_UNSUPPORTED;
  *bytes = attn_gt_ws_bytes(B, T, Hq, block_size);
  return SEER_OK;
}

seer_status seer_attn_ground_truth(const void* q, const seer_kv_layout* kv, const int32_t* seqlens, int B, int T,
                                   int Hq, int Hkv, int d, int block_size, float scale, void* out,
                                   seer_dtype out_dtype, float* lse, float* gt, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  if (!q || !kv || !out || !gt) return SEER_ERR_NULL;
  if (!kv->k || !kv->v) return SEER_ERR_NULL;
  seer_status why;
  if (!attn_gt_sizes_ok(B, T, Hq, Hkv, &why)) return why;
  if (d != seer::kHeadDim || Hq / Hkv > seer::kMaxGroup ||
      !block_size_ok(block_size) || !attn_gt_rows_fit(T, block_size))
    return SEER_ERR_UNSUPPORTED;
  if (kv->page_table) return SEER_ERR_UNSUPPORTED;      // whole-sequence training batches are contiguous
  if (!(scale > 0.f) || scale > 3.0e38f) return SEER_ERR_UNSUPPORTED;   // row maxima are taken before scaling
  if (out_dtype != SEER_BF16 && out_dtype != SEER_F32) return SEER_ERR_UNSUPPORTED;
  if (kv->stride_token < d || (kv->stride_token % 8) || (kv->stride_head % 8) || (kv->stride_seq % 8))
    return SEER_ERR_SHAPE;
  if (!aligned16(kv->k) || !aligned16(kv->v) || !aligned16(q) || !aligned16(out)) return SEER_ERR_SHAPE;
  const size_t need = attn_gt_ws_bytes(B, T, Hq, block_size);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SEER_ERR_WORKSPACE;

  seer::TrainFwdParams p{};
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(kv->k);
  p.v = static_cast<const uint16_t*>(kv->v);
  p.stride_seq = kv->stride_seq;
  p.stride_head = kv->stride_head;
  p.stride_token = kv->stride_token;
  p.seqlens = seqlens;
  p.B = B; p.T = T; p.Hq = Hq; p.Hkv = Hkv; p.g = Hq / Hkv; p.block_size = block_size;
  p.nb = (T + block_size - 1) / block_size;
  p.Tp = (T + 15) / 16 * 16;
  p.scale_log2e = (float)((double)scale * 1.4426950408889634);
  p.raw = static_cast<float*>(workspace);
  p.lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                    align_up((size_t)B * Hq * (size_t)seer::raw_head_elems(p.nb, p.Tp, block_size) * sizeof(float), 256));
  p.out = out;
  p.lse = lse;
  p.gt = gt;
  p.out_is_f32 = out_dtype == SEER_F32;

  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  {
    Timed t(SEER_KERNEL_ATTN_FWD, s);
    e = seer::launch_attn_fwd(p, s);
  }
  if (e != hipSuccess) return SEER_ERR_HIP;
  {
    Timed t(SEER_KERNEL_GT_FINALIZE, s);
    e = seer::launch_gt_finalize(p, s);
  }
  return e == hipSuccess ? SEER_OK : SEER_ERR_HIP;
}

seer_status seer_hbm_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return SEER_ERR_NULL;
  if (bytes < 16 || !aligned16(src) || !aligned16(sink)) return SEER_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  {
    Timed t(SEER_KERNEL_STREAM_READ, s);
    e = seer::launch_stream_read(src, bytes, sink, cu_count() * 8, s);
  }
  return e == hipSuccess ? SEER_OK : SEER_ERR_HIP;
}

seer_status seer_set_knob(int knob, int value) {
  switch (knob) {
    case SEER_KNOB_DECODE_IMPL:
      if (value < 0 || value > 2) return SEER_ERR_SHAPE;
      g_knob_impl = value;
      return SEER_OK;
    case SEER_KNOB_DECODE_SPLITS:
      if (value < 0) return SEER_ERR_SHAPE;
      g_knob_splits = value;
      return SEER_OK;
    case SEER_KNOB_GATE_IMPL:
      if (value < 0 || value > 2) return SEER_ERR_SHAPE;
      g_knob_gate = value;
      return SEER_OK;
    default: return SEER_ERR_UNSUPPORTED;
  }
}

seer_status seer_get_knob(int knob, int* value) {
  if (!value) return SEER_ERR_NULL;
  switch (knob) {
    case SEER_KNOB_DECODE_IMPL: *value = g_knob_impl; return SEER_OK;
    case SEER_KNOB_DECODE_SPLITS: *value = g_knob_splits; return SEER_OK;
    case SEER_KNOB_GATE_IMPL: *value = g_knob_gate; return SEER_OK;
    default: return SEER_ERR_UNSUPPORTED;
  }
}

seer_status seer_profile_enable(int on) {
  g_prof_on = on != 0;
  return SEER_OK;
}

seer_status seer_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (auto& e : g_prof) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  g_prof.clear();
  return SEER_OK;
}

seer_status seer_profile_durations(int which, double* ms, int capacity, int* launches) {
  if (!launches || (capacity > 0 && !ms)) return SEER_ERR_NULL;
  if (which < 0 || which >= SEER_KERNEL_CLASSES || capacity < 0) return SEER_ERR_SHAPE;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int n = 0;
  for (auto& e : g_prof) {
    if (e.cls != which) continue;
    if (n < capacity) {
      if (hipEventSynchronize(e.b) != hipSuccess) return SEER_ERR_HIP;
      float t = 0.f;
      if (hipEventElapsedTime(&t, e.a, e.b) != hipSuccess) return SEER_ERR_HIP;
      ms[n] = t;
    }
    ++n;
  }
  *launches = n;
  return SEER_OK;
}

}  // extern "C"
