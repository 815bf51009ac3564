// KV append: cache[l][b,h,P+r,:] <- block[l][b,h,r,:] for every layer, K and V (paper section 3.3:
// the prefix K/V is kept across steps).  Pure HBM streaming: one 16-byte chunk per lane per
// access, source fully contiguous, destination contiguous in runs of K*D elements.
#include "common.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // native vector: usable with nontemporal builtins

struct AppendArgs {
  u32x4* kc; u32x4* vc;
  const u32x4* kb; const u32x4* vb;
  const uint8_t* do_append;
  long long cache_layer_stride16;   // in 16-byte chunks
  long long block_layer_stride16;
  long long seq_cache16;            // Hkv * cap * row16
  int run16;                        // K * row16: chunks per (layer, b, h) run
  int row16;                        // 16-byte chunks per row (D * elem / 16)
  int cap_rows; int P;
  int Hkv; int B; int L;
  long long total16;                // chunks per tensor (K or V): L*B*Hkv*run16
};

constexpr int kAppendUnroll = 4;

__global__ __launch_bounds__(256) void kv_append_kernel(AppendArgs a) {
  // blockIdx.y selects K (0) or V (1); each thread moves kAppendUnroll chunks spaced by the
  // block size so that every access instruction of a wave covers 1 KiB contiguous.
  const u32x4* __restrict__ src = blockIdx.y ? a.vb : a.kb;
  u32x4* __restrict__ dst = blockIdx.y ? a.vc : a.kc;
  long long base = ((long long)blockIdx.x * kAppendUnroll) * 256 + threadIdx.x;
  u32x4 v[kAppendUnroll];
  long long doff[kAppendUnroll];
  bool ok[kAppendUnroll];
#pragma unroll
  for (int u = 0; u < kAppendUnroll; ++u) {
    long long i = base + (long long)u * 256;
    ok[u] = i < a.total16;
    long long ii = ok[u] ? i : 0;
    // i -> (layer, b, h, chunk within run)
    long long run = ii / a.run16;
    int c = (int)(ii - run * a.run16);
    int h = (int)(run % a.Hkv);
    long long t = run / a.Hkv;
    int b = (int)(t % a.B);
    int l = (int)(t / a.B);
    if (ok[u] && a.do_append != nullptr && a.do_append[b] == 0) ok[u] = false;
    long long soff = (long long)l * a.block_layer_stride16 + ((long long)b * a.Hkv + h) * a.run16 + c;
    doff[u] = (long long)l * a.cache_layer_stride16 + (long long)b * a.seq_cache16 +
              ((long long)h * a.cap_rows + a.P) * a.row16 + c;
    if (ok[u]) v[u] = __builtin_nontemporal_load(src + soff);
  }
#pragma unroll
  for (int u = 0; u < kAppendUnroll; ++u)
    if (ok[u]) __builtin_nontemporal_store(v[u], dst + doff[u]);
}

hipError_t launch_kv_append(const sdllm_append_params& p, void* k_caches, void* v_caches,
                            const void* k_blocks, const void* v_blocks, const uint8_t* do_append,
                            hipStream_t stream) {
  const int elem = p.dtype == SDLLM_FP32 ? 4 : 2;
  AppendArgs a;
  a.kc = (u32x4*)k_caches; a.vc = (u32x4*)v_caches;
  a.kb = (const u32x4*)k_blocks; a.vb = (const u32x4*)v_blocks;
  a.do_append = do_append;
  a.row16 = p.D * elem / 16;
  a.run16 = p.K * a.row16;
  long long cls = p.cache_layer_stride ? p.cache_layer_stride : (long long)p.B * p.Hkv * p.prefix_cap * p.D;
  long long bls = p.block_layer_stride ? p.block_layer_stride : (long long)p.B * p.Hkv * p.K * p.D;
  a.cache_layer_stride16 = cls * elem / 16;
  a.block_layer_stride16 = bls * elem / 16;
  a.seq_cache16 = (long long)p.Hkv * p.prefix_cap * a.row16;
  a.cap_rows = p.prefix_cap; a.P = p.prefix_len;
  a.Hkv = p.Hkv; a.B = p.B; a.L = p.n_layers;
  a.total16 = (long long)p.n_layers * p.B * p.Hkv * a.run16;
  const long long per_block = 256LL * kAppendUnroll;
  long long blocks = (a.total16 + per_block - 1) / per_block;
  if (blocks <= 0) return hipSuccess;
  dim3 grid((unsigned)blocks, 2, 1);
  hipLaunchKernelGGL(kv_append_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace sdllm
