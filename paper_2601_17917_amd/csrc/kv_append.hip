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
  int run16;                        // K * row16: contiguous chunks per (layer, b, h) run
  int row16;                        // 16-byte chunks per row (D * elem / 16)
  int cap_rows; int P;
  int Hkv; int B;
  int parts;                        // workgroups per run
};


// One workgroup moves up to 16 KiB of one (layer, batch, head) run.  The run is decoded once per
// workgroup with scalar arithmetic; a lane only adds its offset.  Each access instruction of a
// wave covers 1 KiB contiguous; all loads are issued before the stores.
constexpr int kAppendUnroll = 4;
constexpr int kAppendChunksPerWG = 256 * kAppendUnroll;

__global__ __launch_bounds__(256) void kv_append_kernel(AppendArgs a) {
  const u32x4* __restrict__ src = blockIdx.y ? a.vb : a.kb;
  u32x4* __restrict__ dst = blockIdx.y ? a.vc : a.kc;
  const unsigned run = blockIdx.x / (unsigned)a.parts;
  const unsigned part = blockIdx.x - run * (unsigned)a.parts;
  const unsigned h = run % (unsigned)a.Hkv;
  const unsigned t = run / (unsigned)a.Hkv;
  const unsigned b = t % (unsigned)a.B;
  const unsigned l = t / (unsigned)a.B;
  if (a.do_append != nullptr && a.do_append[b] == 0) return;   // uniform
  const long long soff = (long long)l * a.block_layer_stride16 + ((long long)b * a.Hkv + h) * a.run16;
  const long long doff = (long long)l * a.cache_layer_stride16 + (long long)b * a.seq_cache16 +
                         ((long long)h * a.cap_rows + a.P) * a.row16;
  const int c0 = (int)part * kAppendChunksPerWG + (int)threadIdx.x;
  u32x4 v[kAppendUnroll];
#pragma unroll
  for (int u = 0; u < kAppendUnroll; ++u) {
    const int c = c0 + u * 256;
    if (c < a.run16) v[u] = src[soff + c];
  }
#pragma unroll
  for (int u = 0; u < kAppendUnroll; ++u) {
    const int c = c0 + u * 256;
    if (c < a.run16) dst[doff + c] = v[u];   // plain stores: measured 15 % faster than nontemporal ones here
  }
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
  a.Hkv = p.Hkv; a.B = p.B;
  a.parts = (a.run16 + 256 * kAppendUnroll - 1) / (256 * kAppendUnroll);
  const long long blocks = (long long)p.n_layers * p.B * p.Hkv * a.parts;
  dim3 grid((unsigned)blocks, 2, 1);
  hipLaunchKernelGGL(kv_append_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace sdllm
