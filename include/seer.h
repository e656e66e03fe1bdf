/*
 * seer.h - C ABI of the SeerAttention-R decode hot path for AMD MI355X (gfx950).
 *
 * Two operations, both shared by all query heads of a kv head (GQA-shared sparsity,
 * Sec. 2.2 "Aggregation of Query Heads"):
 *
 *   seer_gate_select    AttnGate block selection: score of every cached block against the
 *                       K Compression Cache (Eq. 1c, Sec. 3.2), then token-budget top-k or
 *                       threshold selection (Sec. 3.1), last block forced while it is
 *                       partial (Sec. 3.2, Fig. 3).
 *   seer_sparse_decode  block-sparse flash-decoding: attention of the new token over the
 *                       selected KV blocks only, split over the selected-block list and
 *                       merged by log-sum-exp (Sec. 3.3).
 *   seer_dense_decode   the same kernels walking every block (the dense flash-decode the
 *                       sparse kernel is compared with, Sec. 4.4).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless marked "host".  The caller owns all
 *     buffers; the library never allocates, frees or synchronises.  Scratch memory is a
 *     caller-supplied workspace sized by the *_workspace_bytes queries.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default
 *     stream) and the calls return immediately.
 *   - bf16 data is the upper half of an IEEE fp32.  K/V/q/kc base pointers are 16-byte
 *     aligned and all strides are multiples of 8 elements; the innermost (feature)
 *     dimension is contiguous.
 *   - Return value: SEER_OK or a negative seer_status.  Argument errors that the host can
 *     see (NULL pointers, unsupported sizes, short workspace) are reported before anything
 *     is launched.  Data-dependent conditions on the device are defined behaviour, not
 *     errors (see each call).
 *   - Supported sizes: head dim d = 128, gate dim Dg = 128, block_size in {16, 32, 64, 128}
 *     (64 and 128 are the tuned ones), group size Hq/Hkv
 *     in 1..8, at most 65535 sequences and kv heads.
 */
#ifndef SEER_H
#define SEER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum seer_status {
  SEER_OK = 0,
  SEER_ERR_NULL = -1,        /* a required pointer is NULL                          */
  SEER_ERR_SHAPE = -2,       /* a size is non-positive or sizes are inconsistent    */
  SEER_ERR_UNSUPPORTED = -3, /* valid but not implemented (d, Dg, block size, g)    */
  SEER_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or too small          */
  SEER_ERR_CAPACITY = -5,    /* max_sel cannot hold the selection that was asked for */
  SEER_ERR_HIP = -6,         /* a HIP runtime call failed (launch error)            */
  SEER_ERR_SCRATCH = -7      /* seer_sparse_decode_noalloc: the call needs more than the built-in scratch */
} seer_status;

typedef enum seer_select_mode {
  SEER_SELECT_TOPK = 0,      /* token budget -> block budget -> top-k (Sec. 3.1)    */
  SEER_SELECT_THRESHOLD = 1, /* softmaxed gate score > threshold (Sec. 3.1)         */
  SEER_SELECT_TOPP = 2       /* smallest set of best blocks with gate mass >= p (Sec. 6.2) */
} seer_select_mode;

typedef enum seer_dtype { SEER_BF16 = 0, SEER_F32 = 1 } seer_dtype;

/*
 * What the caller knows about the block lists of ONE call (bit set, passed as `hints`; 0 = nothing).
 * A hint never changes a result, only the launch plan.
 *   SEER_HINT_RAGGED_LISTS  the lists of this call differ widely in length (per-sequence budgets,
 *                           threshold or top-p selection, mixed sequence lengths): the decode calls
 *                           cut the lists into slices of about 2048 tokens so that the longest list
 *                           spreads over many work-groups, and seer_gate_select walks long caches
 *                           with few work-groups per sequence.  Lists of about equal length (one
 *                           token budget on long sequences) are ~5 % faster without it.
 * Unknown bits are refused (SEER_ERR_UNSUPPORTED).
 */
typedef enum seer_hint { SEER_HINT_NONE = 0, SEER_HINT_RAGGED_LISTS = 1 } seer_hint;

/*
 * Addressing of the bf16 KV cache.  Element (sequence i, kv head h, token t, feature c):
 *   contiguous (page_table == NULL):  i*stride_seq + h*stride_head + t*stride_token + c
 *   paged:  page = page_table[i*max_pages + t/page_size];
 *           page*stride_seq + h*stride_head + (t%page_size)*stride_token + c
 * page_size must be a multiple of block_size, so a block never straddles two pages.
 * k and v use the same strides.  Tensors larger than 4 GiB are fine (64-bit addressing).
 */
typedef struct seer_kv_layout {
  const void* k;             /* device, bf16 */
  const void* v;             /* device, bf16 */
  int64_t stride_seq;        /* elements between sequences (contiguous) or pages (paged) */
  int64_t stride_head;       /* elements between kv heads   */
  int64_t stride_token;      /* elements between tokens, >= d */
  const int32_t* page_table; /* device [B, max_pages] physical page ids, or NULL */
  int32_t max_pages;
  int32_t page_size;
} seer_kv_layout;

/* Library version (major*10000 + minor*100 + patch). */
int seer_version(void);

/* Static, never-NULL description of a status code. */
const char* seer_status_string(int status);

/* Bytes of workspace seer_gate_select needs for these sizes (host call, no device work). */
seer_status seer_gate_workspace_bytes(int B, int Hkv, int nb_max, size_t* bytes /* host, out */);

/*
 * Bytes of workspace seer_sparse_decode / seer_dense_decode need.  max_blocks is max_sel for
 * the sparse call and the largest number of blocks of any sequence for the dense call.  The size
 * covers every split plan the knobs can produce, so it stays valid when a knob changes.
 */
seer_status seer_decode_workspace_bytes(int B, int Hq, int Hkv, int d, int max_blocks,
                                        size_t* bytes /* host, out */);

/*
 * How the decode calls will cut the block lists for these sizes and hints (host call, no device
 * work): num_splits slices of blocks_per_split list entries each, the partition along num_split of
 * Sec. 3.3.  num_splits * blocks_per_split >= max_blocks; num_splits == 1 means no merge kernel is
 * launched.
 */
seer_status seer_decode_plan(int B, int Hkv, int max_blocks, int block_size, uint32_t hints,
                             int* num_splits /* host, out */, int* blocks_per_split /* host, out */);

/*
 * AttnGate block selection (Eq. 1c; Sec. 3.1; Sec. 3.2).
 *
 * For every (sequence i, kv head h), with S = seqlens[i], nfull = S / block_size full blocks,
 * nb = ceil(S / block_size) blocks (both capped at nb_max):
 *   score s_j = sum_c q_gate[i,h,c] * kc_cache[i,h,j,c] for j < nfull, accumulated in fp64 (the
 *   bf16 products are exact, so the score is the exact dot product for all practical inputs);
 *   entries j >= nfull are never read (a partial block's entry is stale, Sec. 3.2).
 *   TOPK:      k = budget_blocks ? budget_blocks[i] : ceil(budget_tokens / block_size), clamped
 *              to [0, min(nb, max_sel)].  If the last block is partial it is selected and uses
 *              one of the k slots; the remaining slots go to the highest-scoring full blocks,
 *              equal scores resolved towards the lower block index.  k = 0 selects nothing.
 *   THRESHOLD: S_j = softmax_j(s_j / sqrt(Dg)) over the full blocks, in fp64; blocks with
 *              S_j > threshold (strict) are selected, plus the last block if it is partial.
 *   TOPP:      nucleus selection, the adaptive-sparsity direction named in Sec. 6.2: walking the
 *              full blocks from the highest score down (equal scores: lower index first), blocks
 *              are kept until their accumulated S_j reaches p (passed in `threshold`); at least one
 *              block is kept; p beyond the total mass keeps all; plus the partial last block.
 *              (Masses are summed in 2^-62 fixed point, so a prefix whose mass lies within ~1e-15
 *              of p may be cut one block earlier or later than a sequential fp64 sum would.)
 * Output: block_idx[i,h,0..n) ascending block ids, block_idx[i,h,n..max_sel) = -1, nblk[i,h] = n.
 *
 * q_gate   bf16 [B,Hkv,Dg] contiguous.
 * kc_cache bf16, element (i,h,j,c) at i*kc_stride_batch + h*kc_stride_head + j*kc_stride_block + c.
 * seqlens  int32 [B]: tokens in the cache including the current one.
 * budget_blocks int32 [B] or NULL.  threshold is only read in THRESHOLD mode.
 * Errors: THRESHOLD and TOPP modes need max_sel >= nb_max (SEER_ERR_CAPACITY); TOPK mode with a token
 * budget needs max_sel >= min(ceil(budget_tokens/block_size), nb_max) (SEER_ERR_CAPACITY).
 */
seer_status seer_gate_select(const void* q_gate, const void* kc_cache, int64_t kc_stride_batch,
                             int64_t kc_stride_head, int64_t kc_stride_block,
                             const int32_t* seqlens, int B, int Hkv, int Dg, int nb_max,
                             int block_size, seer_select_mode mode, int32_t budget_tokens,
                             const int32_t* budget_blocks, double threshold,
                             int32_t* block_idx /* out [B,Hkv,max_sel] */,
                             int32_t* nblk /* out [B,Hkv] */, int max_sel, void* workspace,
                             size_t workspace_bytes, uint32_t hints, void* stream);

/*
 * Block-sparse flash-decoding (Sec. 3.3).
 *
 * For every (sequence i, kv head h) and each of its g = Hq/Hkv query heads (query head hq
 * belongs to kv head hq / g):  T = tokens of the blocks listed in
 * block_idx[i,h,0..min(nblk[i,h],max_sel)), a block j covering [j*block_size,
 * min((j+1)*block_size, seqlens[i]));  x_t = scale * q.K_t;  lse = log sum_T exp(x_t);
 * out = sum_T exp(x_t - lse) V_t.  Entries < 0 or >= ceil(seqlens[i]/block_size) are skipped;
 * the list need not be sorted; duplicate entries are a caller error (the block would count
 * twice).  An empty T gives out = 0 and lse = -inf.  Accumulation is fp32.
 *
 * q bf16 [B,Hq,d]; out [B,Hq,d] of out_dtype; lse fp32 [B,Hq] (natural log; may be NULL).
 */
seer_status seer_sparse_decode(const void* q, const seer_kv_layout* kv /* host struct */,
                               const int32_t* seqlens, const int32_t* block_idx,
                               const int32_t* nblk, int max_sel, int B, int Hq, int Hkv, int d,
                               int block_size, float scale, void* out, seer_dtype out_dtype,
                               float* lse, void* workspace, size_t workspace_bytes, uint32_t hints,
                               void* stream);

/*
 * seer_sparse_decode for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation,
 * same kernels and same results as seer_sparse_decode; the split-K partials go to a scratch array of
 * SEER_NOALLOC_SCRATCH_BYTES that is part of the library image (each GPU the library runs on holds
 * its own copy until the process ends).  The call allocates and frees nothing.
 *   - Limit: the plan of the call (seer_decode_plan) must fit the array:
 *       2 * align256(B * Hkv * num_splits * (Hq/Hkv) * 4 * {128, 2} bytes)  <=  SEER_NOALLOC_SCRATCH_BYTES,
 *     about B * Hkv * num_splits * (Hq/Hkv) <= 64 000 partial rows; with a single slice (num_splits
 *     == 1) nothing is stored there at all.  Larger calls return SEER_ERR_SCRATCH before anything is
 *     launched.
 *   - All calls on one GPU share that GPU's array.  Nothing in it has to be cleared between calls
 *     (every partial a merge reads was written by the split kernel of the same call), but two calls
 *     that overlap on one GPU (different streams or threads) race on it: keep them on one stream.
 *   - The first call on each device looks up the array's device address (once per device, host work
 *     only); make that first call outside stream capture.
 */
#define SEER_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
seer_status seer_sparse_decode_noalloc(const void* q, const seer_kv_layout* kv /* host struct */,
                                       const int32_t* seqlens, const int32_t* block_idx,
                                       const int32_t* nblk, int max_sel, int B, int Hq, int Hkv, int d,
                                       int block_size, float scale, void* out, seer_dtype out_dtype,
                                       float* lse, uint32_t hints, void* stream);

/*
 * Several new tokens per sequence in one call - the multi-token / speculative decoding direction of
 * Sec. 6.3, where the q_len x g query rows of a kv head fill the matrix-core tile that a single
 * token leaves mostly empty.  The q_len queries of sequence i are its last q_len tokens (positions
 * seqlens[i]-q_len .. seqlens[i]-1; seqlens counts them, their K/V are already in the cache); query t
 * attends the cached tokens up to and including its own position, restricted to the listed blocks;
 * one list per (sequence, kv head) is shared by the q_len queries (how a gate combines the
 * selections of several queries is left to the caller).  Query t alone equals seer_sparse_decode on a
 * sequence of length seqlens[i]-q_len+1+t.
 * q bf16 [B,q_len,Hq,d]; out [B,q_len,Hq,d]; lse fp32 [B,q_len,Hq].  q_len * (Hq/Hkv) <= 16 and
 * the matrix-core kernel (SEER_ERR_UNSUPPORTED otherwise).  Workspace:
 * seer_decode_workspace_bytes(B, q_len*Hq, Hkv, d, max_sel).
 */
seer_status seer_sparse_decode_multi(const void* q, const seer_kv_layout* kv /* host struct */,
                                     const int32_t* seqlens, const int32_t* block_idx, const int32_t* nblk,
                                     int max_sel, int B, int q_len, int Hq, int Hkv, int d, int block_size,
                                     float scale, void* out, seer_dtype out_dtype, float* lse,
                                     void* workspace, size_t workspace_bytes, uint32_t hints, void* stream);

/*
 * Dense flash-decode over all ceil(seqlens[i]/block_size) blocks of every sequence: the
 * baseline the sparse kernel's speed-up is measured against (Sec. 4.4).  max_blocks >= the
 * largest block count of any sequence (blocks beyond it are not visited).
 */
seer_status seer_dense_decode(const void* q, const seer_kv_layout* kv /* host struct */,
                              const int32_t* seqlens, int max_blocks, int B, int Hq, int Hkv, int d,
                              int block_size, float scale, void* out, seer_dtype out_dtype,
                              float* lse, void* workspace, size_t workspace_bytes, uint32_t hints,
                              void* stream);

/*
 * AttnGate front-end, Q branch (Eq. 1a): per (sequence i, kv head h) the g pre-RoPE query heads
 * of the group are concatenated head-major into g*d features, multiplied by that head's weight
 * matrix wq[h] (Dg x g*d, row-major) and rotated (RoPE, rotate-half pairing: feature c with
 * c + Dg/2) at the position of the current token, seqlens[i] - 1.  fp32 accumulation, output
 * rounded to bf16: q_gate is what seer_gate_select consumes.
 *
 * q_nope bf16 [B,Hq,d]; wq bf16 [Hkv,Dg,g*d]; rope_cos / rope_sin fp32 [n_pos, Dg/2] (16-byte
 * aligned; row p holds cos / sin of p * theta_c; positions >= n_pos use the last row);
 * q_gate out bf16 [B,Hkv,Dg].
 */
seer_status seer_gate_q(const void* q_nope, const void* wq, const float* rope_cos, const float* rope_sin,
                        int n_pos, const int32_t* seqlens, int B, int Hq, int Hkv, int d, int Dg,
                        void* q_gate, void* stream);

/*
 * AttnGate from the raw query (Eq. 1a followed by Eq. 1c and the selection of Sec. 3.1): what
 * seer_gate_q followed by seer_gate_select computes, as one call of a decode step.  The gate query of
 * every (sequence, kv head) is made once by a small kernel in front of the gate kernel(s) and kept in
 * the workspace; pass q_gate_out (bf16 [B,Hkv,Dg], device) to receive it, or NULL.  Arguments as in
 * the two calls; the workspace is the one of seer_gate_select (seer_gate_workspace_bytes covers both).
 * All host-visible argument errors of both calls are reported before anything is launched.
 */
seer_status seer_gate_select_q(const void* q_nope, const void* wq, const float* rope_cos, const float* rope_sin,
                               int n_pos, const void* kc_cache, int64_t kc_stride_batch, int64_t kc_stride_head,
                               int64_t kc_stride_block, const int32_t* seqlens, int B, int Hq, int Hkv, int d, int Dg,
                               int nb_max, int block_size, seer_select_mode mode, int32_t budget_tokens,
                               const int32_t* budget_blocks, double threshold,
                               int32_t* block_idx /* out [B,Hkv,max_sel] */, int32_t* nblk /* out [B,Hkv] */,
                               int max_sel, void* q_gate_out /* out or NULL */, void* workspace,
                               size_t workspace_bytes, uint32_t hints, void* stream);

/*
 * AttnGate front-end, K branch = K Compression Cache update (Eq. 1b, Sec. 3.2): for every
 * sequence i, kv head h and block j in [block_begin[i], block_end[i]) (defaults 0 and
 * seqlens[i]/block_size; always clamped to the full blocks of the sequence and to nb_max): the
 * block's b pre-RoPE keys are max-, min- and average-pooled over the tokens, concatenated
 * [max | min | avg] (3d features), multiplied by wk[h] (Dg x 3d, row-major) and rotated at the
 * position of the block's first token, j*block_size.  The entry is written as bf16 to
 * kc_cache[i,h,j,:]; other entries are not touched.  Call it for the newest block whenever
 * seqlens[i] reaches a multiple of block_size (Sec. 3.2), or for all blocks after a prefill.
 *
 * k_nope: pre-RoPE keys in KV-cache addressing (k_nope->k is read, ->v ignored).
 * max_blocks >= the largest block_end[i] - block_begin[i] of the call (it sizes the launch).
 */
seer_status seer_kc_update(const seer_kv_layout* k_nope /* host struct */, const void* wk,
                           const float* rope_cos, const float* rope_sin, int n_pos, const int32_t* seqlens,
                           const int32_t* block_begin, const int32_t* block_end, int max_blocks, int B,
                           int Hkv, int d, int Dg, int nb_max, int block_size, void* kc_cache,
                           int64_t kc_stride_batch, int64_t kc_stride_head, int64_t kc_stride_block,
                           void* stream);

/*
 * Training-side forward pass (Sec. 2.3, ground truth for the self-distillation of the gate, and
 * its efficient generation inside a flash-attention forward): dense causal attention over whole
 * sequences that also emits the target distribution the AttnGate is trained against.
 *
 * For sequence i (S = seqlens ? min(seqlens[i], T) : T), query position t < S, query head hq
 * (kv head h = hq / g):  x_s = scale * q[i,t,hq].K[i,h,s] for s = 0..t;  P_s = softmax_s(x);
 *   out[i,t,hq] = sum_s P_s V[i,h,s];  lse[i,t,hq] = log sum_s exp(x_s);
 *   c[hq][j]  = max of P_s over the keys s <= t of block j = [j*block_size, (j+1)*block_size)
 *               (column-wise 1-D max pooling of the attention row);
 *   r[h][j]   = max of c[hq][j] over the g query heads of kv head h;
 *   gt[i,h,t,j] = r[h][j] / sum_j' r[h][j']  (sums to 1 over the blocks; 0 for blocks after t).
 * Rows t >= S are padding: out = 0, lse = -inf, gt = 0.
 * The block maxima are taken from the block-level row maxima of the logits that the online
 * softmax computes anyway and are turned into probabilities once the row's lse is known.
 * fp32 accumulation; probabilities enter the PV product rounded to bf16.
 *
 * q bf16 [B,T,Hq,d] contiguous; kv: contiguous addressing only (page_table must be NULL), at least
 * T tokens per sequence; out [B,T,Hq,d] of out_dtype; lse fp32 [B,T,Hq] (may be NULL);
 * gt fp32 [B,Hkv,T,ceil(T/block_size)].  block_size in {16, 32, 64, 128}, d = 128, g in 1..8, scale > 0
 * (SEER_ERR_UNSUPPORTED otherwise).
 * Workspace: seer_attn_ground_truth_workspace_bytes (the block maxima of the rows that can see a block,
 * i.e. about half of B*Hq*ceil(T/block_size)*T floats, plus one log-sum-exp per row and head).
 */
seer_status seer_attn_ground_truth_workspace_bytes(int B, int T, int Hq, int Hkv, int d, int block_size,
                                                   size_t* bytes /* host, out */);
seer_status seer_attn_ground_truth(const void* q, const seer_kv_layout* kv /* host struct */,
                                   const int32_t* seqlens /* [B] or NULL */, int B, int T, int Hq, int Hkv,
                                   int d, int block_size, float scale, void* out, seer_dtype out_dtype,
                                   float* lse, float* gt, void* workspace, size_t workspace_bytes,
                                   void* stream);

/*
 * Measurement aid, not part of the method: a plain streaming read of `bytes` bytes (multiple of
 * 16) from device memory `src`, no gather and no arithmetic.  Its rate is the practical HBM read
 * ceiling the decode kernels are compared with.  `sink` is 16 bytes of device memory that the
 * kernel may write (it practically never does).
 */
seer_status seer_hbm_read_probe(const void* src, size_t bytes, void* sink, void* stream);

/*
 * Measurement and test knobs (process-wide, host call; each is one atomic integer that a call reads
 * once, so setting one while calls run on other threads is safe but affects whichever calls read it
 * afterwards).  They force a kernel variant or a split count so that every variant can be measured
 * and tested; production callers leave them at 0 and describe their lists through `hints`.
 * Unknown knobs return SEER_ERR_UNSUPPORTED.
 *   SEER_KNOB_DECODE_IMPL    0 = auto, 1 = VALU kernel, 2 = MFMA kernel
 *   SEER_KNOB_DECODE_SPLITS  0 = auto, n > 0 = force n splits of the block list
 *   SEER_KNOB_GATE_IMPL      0 = auto (one fused kernel when the cache has at most 8192 blocks per
 *                            sequence, else score kernel + select kernel), 1 = score kernel + select
 *                            kernel, 2 = same as 0
 */
typedef enum seer_knob {
  SEER_KNOB_DECODE_IMPL = 0,
  SEER_KNOB_DECODE_SPLITS = 1,
  SEER_KNOB_GATE_IMPL = 3
} seer_knob;
seer_status seer_set_knob(int knob, int value);
seer_status seer_get_knob(int knob, int* value /* host, out */);

/*
 * Per-kernel timing for the bench.  While enabled, each kernel launch of the calls above is
 * bracketed by HIP events on the caller's stream.  seer_profile_durations synchronises on the
 * recorded events and returns, for the kernel class `which`, the number of launches seen since the
 * last reset and, in launch order, the duration in milliseconds of the first `capacity` of them
 * (ms may be NULL when capacity is 0); the caller forms the mean, median and minimum.
 */
typedef enum seer_kernel_class {
  SEER_KERNEL_GATE_SCORE = 0,
  SEER_KERNEL_GATE_SELECT = 1,
  SEER_KERNEL_DECODE_SPLIT = 2,
  SEER_KERNEL_DECODE_MERGE = 3,
  SEER_KERNEL_STREAM_READ = 4,
  SEER_KERNEL_GATE_Q = 5,
  SEER_KERNEL_KC_UPDATE = 6,
  SEER_KERNEL_ATTN_FWD = 7,
  SEER_KERNEL_GT_FINALIZE = 8,
  SEER_KERNEL_CLASSES = 9
} seer_kernel_class;
seer_status seer_profile_enable(int on);
seer_status seer_profile_reset(void);
seer_status seer_profile_durations(int which, double* ms /* host, out [capacity] */, int capacity,
                                   int* launches /* host, out */);

#ifdef __cplusplus
}
#endif
#endif /* SEER_H */
