// Internal declarations shared by the host-side API and the kernel launchers.
// gfx950 only; no other backend.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>
#include "sdllm.h"
#include "sdllm_diag.h"

namespace sdllm {

constexpr int kNumCUs = 256;   // MI355X: 8 XCDs x 32 CUs
constexpr int kNumXCDs = 8;

// Opt-in of a kernel to its dynamic LDS size: done once per (kernel, device), safe when several threads
// make their first call at the same time (the runtime call is idempotent; the bit only saves repeating it).
// sdllm_init() runs every opt-in of the library for the current device, so that the calls that follow only launch.
struct LdsOptIn { std::atomic<unsigned long long> done{0}; };
inline hipError_t ensure_lds_opt_in(const void* kernel, size_t bytes, LdsOptIn& st) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ULL << (dev & 63);
  if (st.done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return e;
  st.done.fetch_or(bit, std::memory_order_release);
  return hipSuccess;
}
hipError_t prepare_attention_bf16();   // every opt-in of the module, for the current device
hipError_t prepare_attention_f32();
hipError_t prepare_lm_head();

// ---- attention launch plan (host, pure function of the parameters) ----
struct AttnPlan {
  int kv_splits;        // key-range splits (grid factor)
  int rb;               // 16-row query blocks per wave (rows per workgroup = 64 * rb)
  int stages;           // LDS ring depth of the K/V stream (2..4)
  int mode;             // 0: one 4-wave group; 1: two groups, same rows, alternating key tiles; 2: two groups,
                        // different rows, shared key tiles
  int q_tiles;          // query tiles per (batch, kv head) group
  int key_tiles;        // 64-key tiles over Nkv
  int tiles_per_split;  // key tiles handled by one split
  int workgroups;
};
AttnPlan plan_attention_bf16(const sdllm_attn_params& p);
size_t attention_bf16_workspace_bytes(const sdllm_attn_params& p, const AttnPlan& plan);

hipError_t launch_attention_bf16(const sdllm_attn_params& p, const AttnPlan& plan,
                                 const void* q_block, const void* q_suffix,
                                 const void* k_cache, const void* v_cache,
                                 const void* k_block, const void* v_block,
                                 const void* k_suffix, const void* v_suffix,
                                 const int32_t* keep_idx, void* out, void* workspace, hipStream_t stream);

hipError_t launch_attention_f32(const sdllm_attn_params& p,
                                const void* q_block, const void* q_suffix,
                                const void* k_cache, const void* v_cache,
                                const void* k_block, const void* v_block,
                                const void* k_suffix, const void* v_suffix,
                                const int32_t* keep_idx, void* out, hipStream_t stream);

// ---- unmask ----
int unmask_splits(const sdllm_unmask_params& p);   // vocabulary splits per row
size_t unmask_workspace_bytes(const sdllm_unmask_params& p);
hipError_t launch_unmask(const sdllm_unmask_params& p, const void* logits, int32_t* tokens, uint8_t* masked,
                         float* confidence, int32_t* n_committed, uint8_t* block_done, uint8_t* eos_seen,
                         void* workspace, hipStream_t stream);

// ---- vocabulary projection fused into the unmask ----
void lm_head_plan(const sdllm_lm_head_params& p, sdllm_lm_head_plan* plan);
size_t lm_head_workspace_bytes(const sdllm_lm_head_params& p);
size_t lm_head_packed_weight_bytes(int V, int Hd);
hipError_t launch_lm_head_pack_weight(int V, int Hd, long long ld_w, const void* weight, void* packed, hipStream_t stream);
hipError_t launch_lm_head_unmask(const sdllm_lm_head_params& p, const void* hidden, const void* weight,
                                 int32_t* tokens, uint8_t* masked, float* confidence, int32_t* n_committed,
                                 uint8_t* block_done, uint8_t* eos_seen, void* workspace, hipStream_t stream);

// ---- rope ----
hipError_t launch_rope(const sdllm_rope_params& p, const void* x_block, const void* x_suffix,
                       const int32_t* keep_idx, void* out_block, void* out_suffix, hipStream_t stream);

// ---- device ceilings (diagnostics) ----
hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t stream);
hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
hipError_t launch_probe_mfma(int iters, int kind, void* sink, hipStream_t stream);
double probe_mfma_flops(int iters);

// ---- kv append ----
hipError_t launch_kv_append(const sdllm_append_params& p, void* k_caches, void* v_caches,
                            const void* k_blocks, const void* v_blocks, const uint8_t* do_append,
                            hipStream_t stream);

}  // namespace sdllm
