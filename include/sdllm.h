/*
 * sdllm.h -- C ABI of the MI355X (gfx950) hot path of one Streaming-dLLM
 * block-wise diffusion decode step.
 *
 * The operations, one call each:
 *   sdllm_block_attention    bidirectional attention of (active block + kept suffix)
 *                            queries over (prefix cache + active block + kept suffix) K/V
 *   sdllm_confidence_unmask  vocab softmax -> max-probability / argmax -> dynamic-threshold
 *                            commit -> block-done / EOS early-exit flags
 *   sdllm_lm_head_unmask     the same unmask fed by the vocabulary projection of the hidden
 *                            states instead of stored logits (the logits never reach memory)
 *   sdllm_kv_append          copy the finished block's K/V into the prefix cache
 *   sdllm_rope_gathered      rotary embedding of the pruned rows with their original position ids
 *   sdllm_suffix_keep_indices  (host) which suffix rows the attenuation-guided rule keeps
 *   sdllm_init               (optional) one-time set-up on the current device, so that later calls only launch
 * Diagnostics that are not part of the decode step (device ceilings) are declared in sdllm_diag.h.
 *
 * Conventions common to all calls
 *   - Every buffer is CALLER-ALLOCATED DEVICE memory unless said otherwise; the library
 *     never allocates, frees or keeps a pointer.  Scratch memory comes from a caller-provided
 *     device workspace whose size the *_workspace_bytes query returns (0 = none needed).
 *     A workspace needs no initialisation and holds nothing between calls; two calls that
 *     may run at the same time need different workspaces.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: they never synchronise and never read device data on the host.  Results,
 *     including counters and flags, land in device memory.
 *   - Layouts are row-major with the last dimension contiguous: [B, H, T, D].  All base
 *     pointers must be 16-byte aligned.
 *   - dtype is SDLLM_FP32 (float) or SDLLM_BF16 (bfloat16 bit patterns, uint16_t).
 *   - Return value: SDLLM_OK or an SDLLM_ERR_* code.  Argument validation happens on the
 *     host before any HIP call, so it works on a machine without a GPU.  A human-readable
 *     message for the calling thread's last failure is available from sdllm_last_error().
 *   - Concurrent calls are allowed when they use different workspaces and outputs.
 *   - A call's launch plan is a pure function of its parameter struct: nothing is read from the process
 *     environment.
 *   - Every call except sdllm_validate_keep_idx may be recorded into a HIP graph (stream capture): after
 *     sdllm_init() on the device a call consists of kernel launches only (no memset, no copy, no attribute call).
 */
#ifndef SDLLM_H
#define SDLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SDLLM_VERSION 200

enum {
  SDLLM_OK = 0,
  SDLLM_ERR_INVALID_ARG = 1, /* NULL pointer, negative size, inconsistent shape, misalignment */
  SDLLM_ERR_UNSUPPORTED = 2, /* dtype / head_dim / size outside the compiled set              */
  SDLLM_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than *_workspace_bytes()            */
  SDLLM_ERR_HIP = 4          /* a HIP launch failed; text in sdllm_last_error()               */
};

enum { SDLLM_FP32 = 0, SDLLM_BF16 = 1 };

/* One-time set-up on the CURRENT device (optional; every call does what it needs on first use).  Opts every kernel
 * of the library in to its LDS size and looks up the library's device-resident scratch array, so that the calls
 * that follow consist of kernel launches only -- what a caller recording them into a HIP graph needs.  Idempotent,
 * thread-safe, once per device.  Errors: HIP. */
int sdllm_init(void);

/* ---------------------------------------------------------------------------------------
 * Attention over the pruned sequence  x~ = prefix U current U kept-suffix  (paper Eq. 8).
 * The queries are the current block and the kept suffix; they attend, without any mask
 * (bidirectional), to the K/V of the whole pruned sequence (paper section 3.3, paragraph
 * after Eq. 8; bidirectionality: sections 1 and 3.2).  The kept suffix rows are selected
 * on the device through keep_idx; nothing is materialised.
 *
 *   B, Hq, Hkv, D   batch, query heads, KV heads (Hq % Hkv == 0; query head h reads KV head
 *                   h / (Hq/Hkv)), head dim.  bf16: D in {64, 128}; fp32: D % 4 == 0, D <= 256.
 *   prefix_len      P: valid rows of the caches (prompt + committed blocks), >= 0
 *   prefix_cap      row capacity of the caches (row stride of the cache's T axis), >= P
 *   K               block length (>= 1);  S: full suffix length (>= 0)
 *   n_keep          s: number of kept suffix rows, 0 <= s <= S
 *   scale           softmax scale; <= 0 selects 1/sqrt(D)
 *   kv_splits       0 = choose automatically; n >= 1 forces n key-range splits (bf16 only)
 * ------------------------------------------------------------------------------------- */
typedef struct sdllm_attn_params {
  int32_t dtype;
  int32_t B, Hq, Hkv, D;
  int32_t prefix_len, prefix_cap;
  int32_t K, S, n_keep;
  float scale;
  int32_t kv_splits;
} sdllm_attn_params;

/* Bytes of device workspace sdllm_block_attention needs for these parameters (0 if none);
 * (size_t)-1 if the parameters are invalid. */
size_t sdllm_attention_workspace_bytes(const sdllm_attn_params* p);

/*
 *   q_block  [B,Hq,K,D]        q_suffix [B,Hq,S,D]      (q_suffix may be NULL iff n_keep == 0)
 *   k_cache, v_cache [B,Hkv,prefix_cap,D]  rows 0..P-1 are read  (may be NULL iff P == 0)
 *   k_block, v_block [B,Hkv,K,D]
 *   k_suffix, v_suffix [B,Hkv,S,D]                         (may be NULL iff n_keep == 0)
 *   keep_idx [n_keep] int32 on the device, shared by the batch; PRECONDITION (not checked,
 *            it would need a sync): strictly increasing, every value in [0, S).
 *   out      [B,Hq,K+n_keep,D], same dtype: block rows first, then the kept suffix rows in
 *            keep_idx order.  Written entirely.
 * Inputs are only read.  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP.
 */
int sdllm_block_attention(const sdllm_attn_params* p,
                          const void* q_block, const void* q_suffix,
                          const void* k_cache, const void* v_cache,
                          const void* k_block, const void* v_block,
                          const void* k_suffix, const void* v_suffix,
                          const int32_t* keep_idx,
                          void* out,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Debug check of sdllm_block_attention's precondition on keep_idx (the index set of Eq. 7 as the device sees it):
 * copies the n_keep entries to the host, SYNCHRONISES `stream`, and verifies that they are strictly increasing and
 * lie in [0, S).  Not for the decode loop and not capturable.  keep_idx may be NULL iff n_keep == 0.
 * Returns SDLLM_OK, or INVALID_ARG with the first offending entry in sdllm_last_error(), or HIP. */
int sdllm_validate_keep_idx(const int32_t* keep_idx, int32_t n_keep, int32_t S, void* stream);

/* ---------------------------------------------------------------------------------------
 * Confidence-aware unmasking of the active block.
 *   For every masked position i (paper Eq. 4):  xhat_i = argmax_j z_ij (lowest id on ties),
 *   c_i = max softmax(z_i) = 1 / sum_j exp(z_ij - max_j z_ij).
 *   Threshold (paper Eq. 10):  tau = tau0 * (1 - alpha * (1 - r_mask)),
 *   r_mask = (m + r_extra_masked) / (K + r_extra_total), m = masked positions of this
 *   sequence's block before the call (r_extra_* = 0: ratio over the block; = n_keep: ratio over
 *   the whole query).
 *   Selection (paper Eq. 9 and the sentence before it): commit every masked i with
 *   c_i >= tau; if there is none, commit the single masked position of highest confidence
 *   (lowest position on ties).  Update (paper Eq. 5): committed positions get tokens = xhat,
 *   masked = 0; every other element of tokens / masked is left untouched.
 *   block_done[b] = 1 iff no masked position is left (end of paper section 3.1), else 0.
 *   eos_seen[b] is OR-ed with (a token committed by this call equals eos_id and its
 *   confidence >= tau_eos) -- the early-exit test of paper section 3.3; skipped if eos_id < 0.
 *   Sequences are independent (per-sequence m, tau, fallback, flags).
 *
 *   dtype of logits, B, K (1..4096), V (>= 1), ld = row stride of logits in elements (>= V;
 *   ld * sizeof(element) must be a multiple of 16).
 * ------------------------------------------------------------------------------------- */
typedef struct sdllm_unmask_params {
  int32_t dtype;
  int32_t B, K, V;
  int64_t ld;
  float tau0, alpha;
  int32_t r_extra_masked, r_extra_total;
  int32_t eos_id;
  float tau_eos;
} sdllm_unmask_params;

size_t sdllm_unmask_workspace_bytes(const sdllm_unmask_params* p);

/*
 *   logits      [B,K,ld]  read only; only rows of masked positions are read
 *   tokens      [B,K] int32   in/out        masked [B,K] uint8 (0 / non-zero)  in/out (the kernels read the
 *               aligned 4-byte words that hold its bytes: up to 3 bytes on either side of the array are read,
 *               never used, and lie in the same page as an array byte)
 *   confidence  [B,K] float   out, optional (NULL ok): c_i for positions masked on entry,
 *               other entries untouched
 *   n_committed [B] int32 out      block_done [B] uint8 out
 *   eos_seen    [B] uint8 in/out, optional (NULL ok)
 * Logits outside the method's domain (NaN, +inf): the position's confidence is NaN, it never passes the threshold
 * and ranks last for the fallback; a row without any finite logit has xhat = 0.  Every store stays in bounds.
 */
int sdllm_confidence_unmask(const sdllm_unmask_params* p,
                            const void* logits,
                            int32_t* tokens, uint8_t* masked,
                            float* confidence,
                            int32_t* n_committed, uint8_t* block_done,
                            uint8_t* eos_seen,
                            void* workspace, size_t workspace_bytes, void* stream);

/* sdllm_confidence_unmask for callers that cannot allocate device memory or carry a workspace around: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels, same
 * results bit for bit; the per-row partial results live in a device-resident array of the library itself
 * (SDLLM_NOALLOC_SCRATCH_BYTES, present once on every GPU the library runs on until the process ends) instead of
 * a caller workspace.  The call allocates nothing and frees nothing.
 *   Limit: sdllm_unmask_workspace_bytes(p) <= SDLLM_NOALLOC_SCRATCH_BYTES, else SDLLM_ERR_UNSUPPORTED (nothing is
 *   launched).  1 MiB holds 87381 partial triples: e.g. 512 rows x 64 vocabulary splits.
 *   All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams,
 *   different threads) race on it and must be serialised by the caller.  Nothing needs clearing between calls
 *   (every slot that is read was written by the same call), so a smaller call after a larger one is fine.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP. */
#define SDLLM_NOALLOC_SCRATCH_BYTES (1u << 20)
int sdllm_confidence_unmask_noalloc(const sdllm_unmask_params* p,
                                    const void* logits,
                                    int32_t* tokens, uint8_t* masked,
                                    float* confidence,
                                    int32_t* n_committed, uint8_t* block_done,
                                    uint8_t* eos_seen,
                                    void* stream);

/* ---------------------------------------------------------------------------------------
 * Vocabulary projection fused into the unmask.  Paper Eq. 3 produces the logits z = f_theta(x); the
 * last map of f_theta is the projection of the final hidden state onto the vocabulary,
 * z_i = W h_i, and Eq. 4 reads z_i for the masked positions of the active block only.  This call
 * forms those logits on the matrix cores (bf16 operands, fp32 accumulation) and reduces them to
 * (max, sum of exp, argmax) on the fly: they are never stored.  Everything after that -- Eq. 4's
 * confidence, Eq. 10, Eq. 9 with its fallback, Eq. 5, the block-done and EOS flags -- is exactly
 * sdllm_confidence_unmask (same tie rules, same outputs).  Hidden rows of unmasked positions are
 * not read.
 *
 *   B, K (1..4096; B*K <= 65536), V >= 1, Hd = model width (multiple of 32)
 *   ld_h, ld_w  row strides of hidden / weight in elements (>= Hd, multiples of 8; B*K*ld_h < 2^31)
 *   tau0 ... tau_eos as in sdllm_unmask_params.  bf16 only.
 *   weight_packed  0: weight is [V, ld_w] row-major.  1: weight is the image that
 *                  sdllm_lm_head_pack_weight writes (ld_w is ignored).  W is a model weight: packed once,
 *                  it lets every kernel read its matrix-core operands as contiguous kilobytes.
 * ------------------------------------------------------------------------------------- */
typedef struct sdllm_lm_head_params {
  int32_t B, K, V, Hd;
  int64_t ld_h, ld_w;
  float tau0, alpha;
  int32_t r_extra_masked, r_extra_total;
  int32_t eos_id;
  float tau_eos;
  int32_t weight_packed;
} sdllm_lm_head_params;

/* The packed image of a projection matrix: [ceil(V/16)][Hd/32][64][8] bf16, where entry [nb][ks][lane][e]
 * is W[min(16 nb + lane % 16, V - 1)][32 ks + 8 (lane / 16) + e] -- the A operand of one
 * v_mfma_f32_16x16x32_bf16 for vocabulary rows 16 nb .. 16 nb + 15 and k-step ks, one kilobyte, lane by lane
 * (rows past V repeat the last row; their logits are discarded).  Hd must be a multiple of 32, ld_w >= Hd a
 * multiple of 8; weight and packed are device pointers, 16-byte aligned, and must not overlap.
 * sdllm_lm_head_packed_weight_bytes returns the size of the image ((size_t)-1 for invalid V / Hd). */
size_t sdllm_lm_head_packed_weight_bytes(int32_t V, int32_t Hd);
int sdllm_lm_head_pack_weight(int32_t V, int32_t Hd, int64_t ld_w, const void* weight, void* packed, void* stream);

size_t sdllm_lm_head_unmask_workspace_bytes(const sdllm_lm_head_params* p);

/*
 *   hidden  [B,K,ld_h] bf16, read only (rows of masked positions)
 *   weight  [V,ld_w]   bf16, read only: row v is the projection vector of token id v (no bias)
 *   tokens, masked, confidence, n_committed, block_done, eos_seen: as for sdllm_confidence_unmask
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP.
 */
int sdllm_lm_head_unmask(const sdllm_lm_head_params* p,
                         const void* hidden, const void* weight,
                         int32_t* tokens, uint8_t* masked,
                         float* confidence,
                         int32_t* n_committed, uint8_t* block_done,
                         uint8_t* eos_seen,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Launch plan the library would use for these parameters (host only, no HIP call).  The masked count is
 * device data, so a call launches every kernel shape that B*K admits and the masked count found on the
 * device decides which of them does the work (the others exit at once): up to 32, 33..64 and 65..128 masked
 * positions take three kernels that stream W once with every position resident, more take 256-position row
 * chunks.  The plan describes the shape that serves B*K masked positions: rows of hidden per row chunk,
 * rows of W per vocabulary tile, number of tiles, row chunks in the grid, workgroups launched, LDS bytes
 * per workgroup; triples_per_position is the workspace's row length (the largest tile count among the
 * shapes launched).  Returns SDLLM_OK or the validation error. */
typedef struct sdllm_lm_head_plan {
  int32_t rows_per_chunk;
  int32_t vocab_rows_per_tile;
  int32_t vocab_tiles;
  int32_t row_chunks;
  int32_t workgroups;
  int32_t lds_bytes;
  int32_t triples_per_position;
} sdllm_lm_head_plan;

int sdllm_plan_lm_head(const sdllm_lm_head_params* p, sdllm_lm_head_plan* plan);

/* ---------------------------------------------------------------------------------------
 * KV append: the prefix K/V is kept and reused instead of recomputed (paper section 3.3,
 * first paragraph on decoding).  When a block is finished its K/V rows become rows
 * P..P+K-1 of every layer's cache:
 *     cache[l][b,h,P+r,:] <- block[l][b,h,r,:]   for all layers, K and V, bit for bit.
 * Nothing else in the caches is written.  The caller then advances prefix_len by K.
 *
 *   n_layers >= 1; B, Hkv, D, K >= 1; prefix_len + K <= prefix_cap; D * sizeof(element) % 16 == 0
 *   cache_layer_stride / block_layer_stride: distance between layers in ELEMENTS
 *   (0 = densely packed: B*Hkv*prefix_cap*D resp. B*Hkv*K*D).
 * ------------------------------------------------------------------------------------- */
typedef struct sdllm_append_params {
  int32_t dtype;
  int32_t n_layers, B, Hkv, D, K;
  int32_t prefix_len, prefix_cap;
  int64_t cache_layer_stride, block_layer_stride;
} sdllm_append_params;

/*
 *   k_caches, v_caches [n_layers][B,Hkv,prefix_cap,D]  in/out
 *   k_blocks, v_blocks [n_layers][B,Hkv,K,D]           read only
 *   do_append [B] uint8 on the device, or NULL = every sequence; sequences with 0 are skipped
 */
int sdllm_kv_append(const sdllm_append_params* p,
                    void* k_caches, void* v_caches,
                    const void* k_blocks, const void* v_blocks,
                    const uint8_t* do_append,
                    void* stream);

/* ---------------------------------------------------------------------------------------
 * Attenuation-guided suffix rule (paper Eq. 7 and Fig. 4): of the S mask positions after the
 * active block keep the w nearest blocks (a sliding window of w_blocks * K positions) and, when
 * keep_trailing != 0, the trailing position S-1, which carries the final length through its
 * position id.  HOST helper (integer only, no HIP call): writes the kept positions, relative to
 * the start of the suffix and strictly increasing, to the HOST array out_idx (capacity `cap`
 * entries) and their number to *n_keep.  n_keep = min(w_blocks*K, S) (+1 if the trailing position
 * is kept and lies outside the window).  The list is what sdllm_block_attention takes as
 * keep_idx after a copy to the device.
 * Errors: INVALID_ARG (NULL pointer, negative S / w_blocks, K < 1, cap too small).
 * ------------------------------------------------------------------------------------- */
int sdllm_suffix_keep_indices(int32_t S, int32_t K, int32_t w_blocks, int32_t keep_trailing,
                              int32_t* out_idx, int32_t cap, int32_t* n_keep);

/* ---------------------------------------------------------------------------------------
 * Rotary position embedding of the pruned rows with their ORIGINAL position ids (paper section
 * 3.3, the sentence before Eq. 7: the kept suffix tokens keep the logical order of the sequence
 * through their RoPE position ids; the ablation on trailing positional information is about this
 * id).  Applied to a query or a key tensor before sdllm_block_attention (once per tensor):
 *     block row r           -> position pos0 + r
 *     kept suffix row j     -> position pos0 + K + keep_idx[j]      (not pos0 + K + j)
 * Rotation of each pair (x_a, x_b) by the angle position * theta_base^(-2i/D), i = 0..D/2-1:
 *     x_a' = x_a cos - x_b sin,   x_b' = x_b cos + x_a sin,
 * (a, b) = (i, i + D/2) when interleaved == 0, (2i, 2i + 1) otherwise.  cos / sin are evaluated
 * in double precision, the products in fp32; bf16 results are rounded to nearest even.
 *
 *   dtype, B, H (heads of this tensor), D (multiple of 16, <= 512), K >= 1, S >= 0,
 *   0 <= n_keep <= S, pos0 >= 0 (pos0 + K + S must fit int32), theta_base > 1.
 * ------------------------------------------------------------------------------------- */
typedef struct sdllm_rope_params {
  int32_t dtype;
  int32_t B, H, D;
  int32_t K, S, n_keep;
  int32_t pos0;
  float theta_base;
  int32_t interleaved;
} sdllm_rope_params;

/*
 *   x_block  [B,H,K,D] read     out_block  [B,H,K,D] written entirely (may be x_block: in place)
 *   x_suffix [B,H,S,D] read     out_suffix [B,H,S,D]: ONLY the kept rows are written, at their own
 *            index keep_idx[j] (so the tensor is used with the same keep_idx afterwards); may be
 *            x_suffix.  Both may be NULL iff n_keep == 0.
 *   keep_idx [n_keep] int32 on the device; precondition as for sdllm_block_attention.
 * Apart from exact in-place use the outputs must not overlap the inputs.  No workspace.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP.
 */
int sdllm_rope_gathered(const sdllm_rope_params* p,
                        const void* x_block, const void* x_suffix,
                        const int32_t* keep_idx,
                        void* out_block, void* out_suffix,
                        void* stream);

/* ---------------------------------------------------------------------------------------
 * Diagnostics.  sdllm_plan_attention reports the launch plan the library would use (host
 * only, no HIP call): number of key-range splits, query rows per workgroup, workgroups, the
 * workgroup shape and its ring depth.
 * Returns SDLLM_OK or the validation error.
 * ------------------------------------------------------------------------------------- */
typedef struct sdllm_attn_plan {
  int32_t kv_splits;
  int32_t rows_per_workgroup;
  int32_t workgroups;
  int32_t key_tiles_per_split;
  int32_t workgroup_shape;   /* 0: 4 waves; 1: 8 waves, two groups on the same rows alternating key tiles;
                                2: 8 waves, two groups on different rows sharing every key tile (bf16 only) */
  int32_t ring_stages;       /* K/V tiles the LDS ring of a workgroup holds per group (2..4) */
} sdllm_attn_plan;

int sdllm_plan_attention(const sdllm_attn_params* p, sdllm_attn_plan* plan);

const char* sdllm_status_string(int status);
const char* sdllm_last_error(void); /* calling thread's last failure text ("" if none) */
int sdllm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SDLLM_H */
