// Host side of the C ABI: argument validation (before any HIP call), plan / workspace queries,
// error text, dispatch to the kernel launchers.
#include "common.h"
#include <cstdio>
#include <cstdarg>
#include <cstring>
#include <cmath>
#include <vector>
#include <atomic>

// ---- the device-resident scratch of sdllm_confidence_unmask_noalloc (file scope).  Every GPU the library runs on
// holds its own copy of the array at its own address; in host code the array's name is only a handle for the symbol
// lookup, never an address: the per-device address found by scratch_of_current_device() is what kernels and runtime
// calls are given.
static __device__ __align__(256) unsigned char scratch[SDLLM_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_attn_params(const sdllm_attn_params* p) {
  if (!p) return fail(SDLLM_ERR_INVALID_ARG, "attention: params is NULL");
  if (p->dtype != SDLLM_FP32 && p->dtype != SDLLM_BF16)
    return fail(SDLLM_ERR_UNSUPPORTED, "attention: dtype %d not supported (fp32=0, bf16=1)", p->dtype);
  if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->D < 1 || p->K < 1)
    return fail(SDLLM_ERR_INVALID_ARG, "attention: B, Hq, Hkv, D, K must be >= 1");
  if (p->Hq % p->Hkv != 0)
    return fail(SDLLM_ERR_INVALID_ARG, "attention: Hq (%d) must be a multiple of Hkv (%d)", p->Hq, p->Hkv);
  if (p->prefix_len < 0 || p->prefix_cap < p->prefix_len)
    return fail(SDLLM_ERR_INVALID_ARG, "attention: need 0 <= prefix_len (%d) <= prefix_cap (%d)", p->prefix_len, p->prefix_cap);
  if (p->S < 0 || p->n_keep < 0 || p->n_keep > p->S)
    return fail(SDLLM_ERR_INVALID_ARG, "attention: need 0 <= n_keep (%d) <= S (%d)", p->n_keep, p->S);
  if (p->kv_splits < 0) return fail(SDLLM_ERR_INVALID_ARG, "attention: kv_splits must be >= 0");
  if (!(p->scale == p->scale) || std::isinf(p->scale)) return fail(SDLLM_ERR_INVALID_ARG, "attention: scale is not finite");
  if (p->dtype == SDLLM_BF16) {
    if (p->D != 64 && p->D != 128)
      return fail(SDLLM_ERR_UNSUPPORTED, "attention: bf16 head_dim %d not compiled (64, 128)", p->D);
  } else {
    if (p->D % 4 != 0 || p->D > 256)
      return fail(SDLLM_ERR_UNSUPPORTED, "attention: fp32 head_dim %d not supported (multiple of 4, <= 256)", p->D);
    if (p->Hq > 65535 || p->B > 65535)
      return fail(SDLLM_ERR_UNSUPPORTED, "attention: fp32 path needs Hq, B <= 65535");
  }
  const long long nkv = (long long)p->prefix_len + p->K + p->n_keep;
  const long long rows = (long long)p->B * p->Hq * (p->K + p->n_keep);
  if (nkv > (1LL << 30) || rows > (1LL << 31) - 1)
    return fail(SDLLM_ERR_UNSUPPORTED, "attention: sequence or batch too large");
  return SDLLM_OK;
}

int check_unmask_params(const sdllm_unmask_params* p) {
  if (!p) return fail(SDLLM_ERR_INVALID_ARG, "unmask: params is NULL");
  if (p->dtype != SDLLM_FP32 && p->dtype != SDLLM_BF16)
    return fail(SDLLM_ERR_UNSUPPORTED, "unmask: dtype %d not supported (fp32=0, bf16=1)", p->dtype);
  if (p->B < 1 || p->K < 1 || p->V < 1) return fail(SDLLM_ERR_INVALID_ARG, "unmask: B, K, V must be >= 1");
  if (p->K > 4096) return fail(SDLLM_ERR_UNSUPPORTED, "unmask: K (%d) > 4096", p->K);
  if (p->ld < p->V) return fail(SDLLM_ERR_INVALID_ARG, "unmask: ld (%lld) < V (%d)", (long long)p->ld, p->V);
  const int elem = p->dtype == SDLLM_FP32 ? 4 : 2;
  if ((p->ld * elem) % 16 != 0)
    return fail(SDLLM_ERR_INVALID_ARG, "unmask: ld * element size (%lld bytes) must be a multiple of 16", (long long)p->ld * elem);
  if ((long long)p->B * p->K > (1LL << 24)) return fail(SDLLM_ERR_UNSUPPORTED, "unmask: B*K too large");
  if (p->r_extra_masked < 0 || p->r_extra_total < p->r_extra_masked)
    return fail(SDLLM_ERR_INVALID_ARG, "unmask: need 0 <= r_extra_masked <= r_extra_total");
  if (!(p->tau0 == p->tau0) || !(p->alpha == p->alpha) || !(p->tau_eos == p->tau_eos))
    return fail(SDLLM_ERR_INVALID_ARG, "unmask: tau0 / alpha / tau_eos is NaN");
  return SDLLM_OK;
}

int check_lm_head_params(const sdllm_lm_head_params* p) {
  if (!p) return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: params is NULL");
  if (p->B < 1 || p->K < 1 || p->V < 1 || p->Hd < 1)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: B, K, V, Hd must be >= 1");
  if (p->K > 4096) return fail(SDLLM_ERR_UNSUPPORTED, "lm_head_unmask: K (%d) > 4096", p->K);
  if ((long long)p->B * p->K > 65536) return fail(SDLLM_ERR_UNSUPPORTED, "lm_head_unmask: B*K > 65536");
  if (p->Hd % 32 != 0) return fail(SDLLM_ERR_UNSUPPORTED, "lm_head_unmask: Hd (%d) must be a multiple of 32", p->Hd);
  if (p->weight_packed != 0 && p->weight_packed != 1)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: weight_packed must be 0 or 1");
  const bool row_major = p->weight_packed == 0;      // ld_w is ignored for a packed weight
  if (p->ld_h < p->Hd || (row_major && p->ld_w < p->Hd))
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: ld_h (%lld) and ld_w (%lld) must be >= Hd (%d)",
                (long long)p->ld_h, (long long)p->ld_w, p->Hd);
  if (p->ld_h % 8 != 0 || (row_major && p->ld_w % 8 != 0))
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: ld_h and ld_w must be multiples of 8 elements (16 bytes)");
  if ((long long)p->B * p->K * p->ld_h >= (1LL << 31))
    return fail(SDLLM_ERR_UNSUPPORTED, "lm_head_unmask: B*K*ld_h must be below 2^31");
  if (p->r_extra_masked < 0 || p->r_extra_total < p->r_extra_masked)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: need 0 <= r_extra_masked <= r_extra_total");
  if (!(p->tau0 == p->tau0) || !(p->alpha == p->alpha) || !(p->tau_eos == p->tau_eos))
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: tau0 / alpha / tau_eos is NaN");
  return SDLLM_OK;
}

int check_append_params(const sdllm_append_params* p) {
  if (!p) return fail(SDLLM_ERR_INVALID_ARG, "kv_append: params is NULL");
  if (p->dtype != SDLLM_FP32 && p->dtype != SDLLM_BF16)
    return fail(SDLLM_ERR_UNSUPPORTED, "kv_append: dtype %d not supported (fp32=0, bf16=1)", p->dtype);
  if (p->n_layers < 1 || p->B < 1 || p->Hkv < 1 || p->D < 1 || p->K < 1)
    return fail(SDLLM_ERR_INVALID_ARG, "kv_append: n_layers, B, Hkv, D, K must be >= 1");
  if (p->prefix_len < 0 || (long long)p->prefix_len + p->K > p->prefix_cap)
    return fail(SDLLM_ERR_INVALID_ARG, "kv_append: prefix_len (%d) + K (%d) exceeds prefix_cap (%d)", p->prefix_len, p->K, p->prefix_cap);
  const int elem = p->dtype == SDLLM_FP32 ? 4 : 2;
  if ((p->D * elem) % 16 != 0)
    return fail(SDLLM_ERR_UNSUPPORTED, "kv_append: row size %d bytes must be a multiple of 16", p->D * elem);
  const long long dense_c = (long long)p->B * p->Hkv * p->prefix_cap * p->D;
  const long long dense_b = (long long)p->B * p->Hkv * p->K * p->D;
  if ((long long)p->n_layers * p->B * p->Hkv * (((long long)p->K * p->D * elem / 16 + 1023) / 1024) > 0x7fffffffLL ||
      (long long)p->K * p->D * elem / 16 > 0x7fffffffLL)
    return fail(SDLLM_ERR_UNSUPPORTED, "kv_append: problem too large for one launch");
  if (p->cache_layer_stride != 0 && (p->cache_layer_stride < dense_c || (p->cache_layer_stride * elem) % 16 != 0))
    return fail(SDLLM_ERR_INVALID_ARG, "kv_append: cache_layer_stride too small or not 16-byte aligned");
  if (p->block_layer_stride != 0 && (p->block_layer_stride < dense_b || (p->block_layer_stride * elem) % 16 != 0))
    return fail(SDLLM_ERR_INVALID_ARG, "kv_append: block_layer_stride too small or not 16-byte aligned");
  return SDLLM_OK;
}

int check_rope_params(const sdllm_rope_params* p) {
  if (!p) return fail(SDLLM_ERR_INVALID_ARG, "rope: params is NULL");
  if (p->dtype != SDLLM_FP32 && p->dtype != SDLLM_BF16)
    return fail(SDLLM_ERR_UNSUPPORTED, "rope: dtype %d not supported (fp32=0, bf16=1)", p->dtype);
  if (p->B < 1 || p->H < 1 || p->K < 1) return fail(SDLLM_ERR_INVALID_ARG, "rope: B, H, K must be >= 1");
  if (p->D < 16 || p->D % 16 != 0 || p->D > 512)
    return fail(SDLLM_ERR_UNSUPPORTED, "rope: head_dim %d not supported (multiple of 16, <= 512)", p->D);
  if (p->S < 0 || p->n_keep < 0 || p->n_keep > p->S)
    return fail(SDLLM_ERR_INVALID_ARG, "rope: need 0 <= n_keep (%d) <= S (%d)", p->n_keep, p->S);
  if (p->pos0 < 0 || (long long)p->pos0 + p->K + p->S > 0x7fffffffLL)
    return fail(SDLLM_ERR_INVALID_ARG, "rope: need pos0 >= 0 and pos0 + K + S within int32");
  if (!(p->theta_base > 1.0f) || std::isinf(p->theta_base))
    return fail(SDLLM_ERR_INVALID_ARG, "rope: theta_base must be finite and > 1");
  if ((long long)p->B * p->H > 0x7fffffffLL || p->K + p->n_keep > 0x7fffffff - 1)
    return fail(SDLLM_ERR_UNSUPPORTED, "rope: problem too large");
  return SDLLM_OK;
}

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

hipError_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {                      // first use on this device (two threads may both look it up: same answer)
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return hipSuccess;
}

}  // namespace

extern "C" {

int sdllm_version(void) { return SDLLM_VERSION; }

int sdllm_init(void) {
  hipError_t e = sdllm::prepare_attention_bf16();
  if (e == hipSuccess) e = sdllm::prepare_attention_f32();
  if (e == hipSuccess) e = sdllm::prepare_lm_head();
  void* ptr = nullptr;
  if (e == hipSuccess) e = scratch_of_current_device(&ptr);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "init: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

const char* sdllm_last_error(void) { return g_err; }

const char* sdllm_status_string(int status) {
  switch (status) {
    case SDLLM_OK: return "ok";
    case SDLLM_ERR_INVALID_ARG: return "invalid argument";
    case SDLLM_ERR_UNSUPPORTED: return "unsupported dtype / shape";
    case SDLLM_ERR_WORKSPACE: return "workspace missing or too small";
    case SDLLM_ERR_HIP: return "HIP launch failure";
    default: return "unknown status";
  }
}

int sdllm_plan_attention(const sdllm_attn_params* p, sdllm_attn_plan* plan) {
  int rc = check_attn_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!plan) return fail(SDLLM_ERR_INVALID_ARG, "plan_attention: plan is NULL");
  if (p->dtype == SDLLM_FP32) {
    plan->kv_splits = 1; plan->rows_per_workgroup = 4;
    plan->workgroups = ((p->K + p->n_keep + 3) / 4) * p->Hq * p->B;
    plan->key_tiles_per_split = (p->prefix_len + p->K + p->n_keep + 63) / 64;
    plan->workgroup_shape = 0; plan->ring_stages = 2;
    return SDLLM_OK;
  }
  sdllm::AttnPlan pl = sdllm::plan_attention_bf16(*p);
  plan->kv_splits = pl.kv_splits; plan->rows_per_workgroup = 64 * pl.rb * (pl.mode == 2 ? 2 : 1);
  plan->workgroups = pl.workgroups; plan->key_tiles_per_split = pl.tiles_per_split;
  plan->workgroup_shape = pl.mode; plan->ring_stages = pl.stages;
  return SDLLM_OK;
}

size_t sdllm_attention_workspace_bytes(const sdllm_attn_params* p) {
  if (check_attn_params(p) != SDLLM_OK) return (size_t)-1;
  if (p->dtype == SDLLM_FP32) return 0;
  return sdllm::attention_bf16_workspace_bytes(*p, sdllm::plan_attention_bf16(*p));
}

int sdllm_block_attention(const sdllm_attn_params* p,
                          const void* q_block, const void* q_suffix,
                          const void* k_cache, const void* v_cache,
                          const void* k_block, const void* v_block,
                          const void* k_suffix, const void* v_suffix,
                          const int32_t* keep_idx, void* out,
                          void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_attn_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!q_block || !k_block || !v_block || !out)
    return fail(SDLLM_ERR_INVALID_ARG, "attention: q_block, k_block, v_block, out must not be NULL");
  if (p->prefix_len > 0 && (!k_cache || !v_cache))
    return fail(SDLLM_ERR_INVALID_ARG, "attention: k_cache / v_cache is NULL with prefix_len > 0");
  if (p->n_keep > 0 && (!q_suffix || !k_suffix || !v_suffix || !keep_idx))
    return fail(SDLLM_ERR_INVALID_ARG, "attention: q_suffix / k_suffix / v_suffix / keep_idx is NULL with n_keep > 0");
  const void* ptrs[] = {q_block, q_suffix, k_cache, v_cache, k_block, v_block, k_suffix, v_suffix, out, workspace};
  for (const void* q : ptrs)
    if (q && !aligned16(q)) return fail(SDLLM_ERR_INVALID_ARG, "attention: a base pointer is not 16-byte aligned");
  if (p->dtype == SDLLM_FP32) {
    hipError_t e = sdllm::launch_attention_f32(*p, q_block, q_suffix, k_cache, v_cache, k_block, v_block,
                                               k_suffix, v_suffix, keep_idx, out, (hipStream_t)stream);
    if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "attention (fp32): %s", hipGetErrorString(e));
    return SDLLM_OK;
  }
  sdllm::AttnPlan pl = sdllm::plan_attention_bf16(*p);
  const size_t need = sdllm::attention_bf16_workspace_bytes(*p, pl);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(SDLLM_ERR_WORKSPACE, "attention: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
  hipError_t e = sdllm::launch_attention_bf16(*p, pl, q_block, q_suffix, k_cache, v_cache, k_block, v_block,
                                              k_suffix, v_suffix, keep_idx, out, need ? workspace : nullptr,
                                              (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "attention (bf16): %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_validate_keep_idx(const int32_t* keep_idx, int32_t n_keep, int32_t S, void* stream) {
  if (n_keep < 0 || S < 0 || n_keep > S)
    return fail(SDLLM_ERR_INVALID_ARG, "validate_keep_idx: need 0 <= n_keep (%d) <= S (%d)", n_keep, S);
  if (n_keep == 0) return SDLLM_OK;
  if (!keep_idx) return fail(SDLLM_ERR_INVALID_ARG, "validate_keep_idx: keep_idx is NULL with n_keep > 0");
  std::vector<int32_t> host((size_t)n_keep);
  hipError_t e = hipMemcpyAsync(host.data(), keep_idx, (size_t)n_keep * sizeof(int32_t), hipMemcpyDeviceToHost,
                                (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "validate_keep_idx: %s", hipGetErrorString(e));
  for (int32_t j = 0; j < n_keep; ++j) {
    if (host[j] < 0 || host[j] >= S)
      return fail(SDLLM_ERR_INVALID_ARG, "validate_keep_idx: keep_idx[%d] = %d is outside [0, %d)", j, host[j], S);
    if (j > 0 && host[j] <= host[j - 1])
      return fail(SDLLM_ERR_INVALID_ARG, "validate_keep_idx: keep_idx[%d] = %d does not exceed keep_idx[%d] = %d",
                  j, host[j], j - 1, host[j - 1]);
  }
  return SDLLM_OK;
}

int sdllm_suffix_keep_indices(int32_t S, int32_t K, int32_t w_blocks, int32_t keep_trailing,
                              int32_t* out_idx, int32_t cap, int32_t* n_keep) {
  if (!out_idx || !n_keep) return fail(SDLLM_ERR_INVALID_ARG, "suffix_keep_indices: out_idx / n_keep is NULL");
  if (S < 0 || w_blocks < 0 || K < 1) return fail(SDLLM_ERR_INVALID_ARG, "suffix_keep_indices: need S >= 0, w_blocks >= 0, K >= 1");
  const long long window = (long long)w_blocks * K < S ? (long long)w_blocks * K : S;
  const bool extra = keep_trailing && S > 0 && window < S;          // trailing position outside the window
  const long long n = window + (extra ? 1 : 0);
  if (n > cap) return fail(SDLLM_ERR_INVALID_ARG, "suffix_keep_indices: %lld indices do not fit the capacity %d", n, cap);
  for (long long i = 0; i < window; ++i) out_idx[i] = (int32_t)i;
  if (extra) out_idx[window] = S - 1;
  *n_keep = (int32_t)n;
  return SDLLM_OK;
}

size_t sdllm_unmask_workspace_bytes(const sdllm_unmask_params* p) {
  if (check_unmask_params(p) != SDLLM_OK) return (size_t)-1;
  return sdllm::unmask_workspace_bytes(*p);
}

int sdllm_confidence_unmask(const sdllm_unmask_params* p, const void* logits,
                            int32_t* tokens, uint8_t* masked, float* confidence,
                            int32_t* n_committed, uint8_t* block_done, uint8_t* eos_seen,
                            void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_unmask_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!logits || !tokens || !masked || !n_committed || !block_done)
    return fail(SDLLM_ERR_INVALID_ARG, "unmask: logits, tokens, masked, n_committed, block_done must not be NULL");
  if (!aligned16(logits)) return fail(SDLLM_ERR_INVALID_ARG, "unmask: logits is not 16-byte aligned");
  const size_t need = sdllm::unmask_workspace_bytes(*p);
  if (!workspace || workspace_bytes < need)
    return fail(SDLLM_ERR_WORKSPACE, "unmask: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
  if ((reinterpret_cast<uintptr_t>(workspace) & 3u) != 0)
    return fail(SDLLM_ERR_INVALID_ARG, "unmask: workspace is not 4-byte aligned");
  hipError_t e = sdllm::launch_unmask(*p, logits, tokens, masked, confidence, n_committed, block_done, eos_seen,
                                      workspace, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "unmask: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_confidence_unmask_noalloc(const sdllm_unmask_params* p, const void* logits,
                                    int32_t* tokens, uint8_t* masked, float* confidence,
                                    int32_t* n_committed, uint8_t* block_done, uint8_t* eos_seen, void* stream) {
  int rc = check_unmask_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!logits || !tokens || !masked || !n_committed || !block_done)
    return fail(SDLLM_ERR_INVALID_ARG, "unmask_noalloc: logits, tokens, masked, n_committed, block_done must not be NULL");
  if (!aligned16(logits)) return fail(SDLLM_ERR_INVALID_ARG, "unmask_noalloc: logits is not 16-byte aligned");
  const size_t need = sdllm::unmask_workspace_bytes(*p);
  if (need > (size_t)SDLLM_NOALLOC_SCRATCH_BYTES)
    return fail(SDLLM_ERR_UNSUPPORTED, "unmask_noalloc: %zu bytes of partial results exceed the library's %u-byte scratch "
                "(B*K = %lld rows); use sdllm_confidence_unmask with a workspace", need,
                (unsigned)SDLLM_NOALLOC_SCRATCH_BYTES, (long long)p->B * p->K);
  void* ptr = nullptr;
  hipError_t e = scratch_of_current_device(&ptr);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "unmask_noalloc: scratch lookup: %s", hipGetErrorString(e));
  e = sdllm::launch_unmask(*p, logits, tokens, masked, confidence, n_committed, block_done, eos_seen, ptr, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "unmask_noalloc: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

size_t sdllm_lm_head_packed_weight_bytes(int32_t V, int32_t Hd) {
  if (V < 1 || Hd < 32 || Hd % 32 != 0) return (size_t)-1;
  return sdllm::lm_head_packed_weight_bytes(V, Hd);
}

int sdllm_lm_head_pack_weight(int32_t V, int32_t Hd, int64_t ld_w, const void* weight, void* packed, void* stream) {
  if (V < 1 || Hd < 32 || Hd % 32 != 0)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_pack_weight: need V >= 1 and Hd a positive multiple of 32");
  if (ld_w < Hd || ld_w % 8 != 0)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_pack_weight: ld_w (%lld) must be >= Hd (%d) and a multiple of 8", (long long)ld_w, Hd);
  if (!weight || !packed) return fail(SDLLM_ERR_INVALID_ARG, "lm_head_pack_weight: weight and packed must not be NULL");
  if (((uintptr_t)weight | (uintptr_t)packed) & 15)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_pack_weight: weight / packed is not 16-byte aligned");
  hipError_t e = sdllm::launch_lm_head_pack_weight(V, Hd, ld_w, weight, packed, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "lm_head_pack_weight: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_plan_lm_head(const sdllm_lm_head_params* p, sdllm_lm_head_plan* plan) {
  int rc = check_lm_head_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!plan) return fail(SDLLM_ERR_INVALID_ARG, "plan_lm_head: plan is NULL");
  sdllm::lm_head_plan(*p, plan);
  return SDLLM_OK;
}

size_t sdllm_lm_head_unmask_workspace_bytes(const sdllm_lm_head_params* p) {
  if (check_lm_head_params(p) != SDLLM_OK) return (size_t)-1;
  return sdllm::lm_head_workspace_bytes(*p);
}

int sdllm_lm_head_unmask(const sdllm_lm_head_params* p, const void* hidden, const void* weight,
                         int32_t* tokens, uint8_t* masked, float* confidence,
                         int32_t* n_committed, uint8_t* block_done, uint8_t* eos_seen,
                         void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_lm_head_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!hidden || !weight || !tokens || !masked || !n_committed || !block_done)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: hidden, weight, tokens, masked, n_committed, block_done must not be NULL");
  if (!aligned16(hidden) || !aligned16(weight))
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: hidden / weight is not 16-byte aligned");
  const size_t need = sdllm::lm_head_workspace_bytes(*p);
  if (!workspace || workspace_bytes < need)
    return fail(SDLLM_ERR_WORKSPACE, "lm_head_unmask: workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
  if ((reinterpret_cast<uintptr_t>(workspace) & 3u) != 0)
    return fail(SDLLM_ERR_INVALID_ARG, "lm_head_unmask: workspace is not 4-byte aligned");
  hipError_t e = sdllm::launch_lm_head_unmask(*p, hidden, weight, tokens, masked, confidence, n_committed,
                                              block_done, eos_seen, workspace, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "lm_head_unmask: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_kv_append(const sdllm_append_params* p, void* k_caches, void* v_caches,
                    const void* k_blocks, const void* v_blocks, const uint8_t* do_append, void* stream) {
  int rc = check_append_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!k_caches || !v_caches || !k_blocks || !v_blocks)
    return fail(SDLLM_ERR_INVALID_ARG, "kv_append: caches and blocks must not be NULL");
  if (!aligned16(k_caches) || !aligned16(v_caches) || !aligned16(k_blocks) || !aligned16(v_blocks))
    return fail(SDLLM_ERR_INVALID_ARG, "kv_append: a base pointer is not 16-byte aligned");
  hipError_t e = sdllm::launch_kv_append(*p, k_caches, v_caches, k_blocks, v_blocks, do_append, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "kv_append: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_rope_gathered(const sdllm_rope_params* p, const void* x_block, const void* x_suffix,
                        const int32_t* keep_idx, void* out_block, void* out_suffix, void* stream) {
  int rc = check_rope_params(p);
  if (rc != SDLLM_OK) return rc;
  if (!x_block || !out_block) return fail(SDLLM_ERR_INVALID_ARG, "rope: x_block, out_block must not be NULL");
  if (p->n_keep > 0 && (!x_suffix || !out_suffix || !keep_idx))
    return fail(SDLLM_ERR_INVALID_ARG, "rope: x_suffix / out_suffix / keep_idx is NULL with n_keep > 0");
  const void* ptrs[] = {x_block, x_suffix, out_block, out_suffix};
  for (const void* q : ptrs)
    if (q && !aligned16(q)) return fail(SDLLM_ERR_INVALID_ARG, "rope: a base pointer is not 16-byte aligned");
  hipError_t e = sdllm::launch_rope(*p, x_block, x_suffix, keep_idx, out_block, out_suffix, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "rope: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_probe_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes == 0 || bytes % 16 != 0 || !aligned16(src))
    return fail(SDLLM_ERR_INVALID_ARG, "probe_read: need src (16-byte aligned), sink, bytes > 0 and a multiple of 16");
  hipError_t e = sdllm::launch_probe_read(src, bytes, sink, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "probe_read: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst))
    return fail(SDLLM_ERR_INVALID_ARG, "probe_copy: need dst, src (16-byte aligned), bytes > 0 and a multiple of 16");
  hipError_t e = sdllm::launch_probe_copy(dst, src, bytes, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "probe_copy: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

int sdllm_probe_mfma_bf16(int32_t iters, int32_t operand_kind, void* sink, void* stream, double* flops) {
  if (iters < 1 || (operand_kind != 0 && operand_kind != 1) || !sink)
    return fail(SDLLM_ERR_INVALID_ARG, "probe_mfma_bf16: need iters >= 1, operand_kind 0 or 1, sink");
  if (flops) *flops = sdllm::probe_mfma_flops(iters);
  hipError_t e = sdllm::launch_probe_mfma(iters, operand_kind, sink, (hipStream_t)stream);
  if (e != hipSuccess) return fail(SDLLM_ERR_HIP, "probe_mfma_bf16: %s", hipGetErrorString(e));
  return SDLLM_OK;
}

}  // extern "C"
