// fp32 attention over [prefix cache | block | gathered suffix] (paper Eq. 8 and the paragraph
// after it).  Plain fp32 FMA arithmetic with an accurate exp: this is the correctness-grade
// path (max-abs error <= 1e-5 against the fp64 definition), not the throughput path.
//
// A workgroup = four query rows of one (batch, head), one wave per row.  Keys are visited in chunks of 64:
// the workgroup brings the chunk's K and V rows into LDS with coalesced 16-byte loads (the four waves share
// them), lane j scores key j of the chunk (dot product over D from LDS), the chunk's maximum and sum are formed
// with wave reductions (online softmax), and for the output lane l owns columns l, l+64, ...
#include "common.h"

namespace sdllm {

struct AttnF32Args {
  const float* q_block; const float* q_suffix;
  const float* k_cache; const float* v_cache;
  const float* k_block; const float* v_block;
  const float* k_suffix; const float* v_suffix;
  const int32_t* keep_idx;
  float* out;
  int B, Hq, Hkv, D, P, cap, K, S, n_keep;
  float scale;
};

constexpr int kF32MaxD = 256;
constexpr int kF32Waves = 4;

// row r of the pruned K/V sequence of KV head (b, kvh): pointer offset selection
__device__ __forceinline__ const float* kv_row(const AttnF32Args& a, const float* cache, const float* block,
                                               const float* suffix, int b, int kvh, int r) {
  const long long bh = (long long)b * a.Hkv + kvh;
  if (r < a.P) return cache + (bh * a.cap + r) * a.D;
  r -= a.P;
  if (r < a.K) return block + (bh * a.K + r) * a.D;
  r -= a.K;
  return suffix + (bh * a.S + a.keep_idx[r]) * a.D;
}

// LDS: K chunk [64][D + 4] (the pad keeps 16-byte alignment and spreads the rows over the banks), V chunk [64][D]
__host__ __device__ constexpr size_t f32_lds_bytes(int D) { return (size_t)64 * (2 * D + 4) * sizeof(float); }

__global__ __launch_bounds__(64 * kF32Waves) void attention_f32_kernel(AttnF32Args a) {
  __shared__ float q_s[kF32Waves][kF32MaxD];
  extern __shared__ __attribute__((aligned(16))) float kv_s[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int Nq = a.K + a.n_keep, Nkv = a.P + a.K + a.n_keep;
  const int qi = blockIdx.x * kF32Waves + wave;
  const int hq = blockIdx.y, b = blockIdx.z;
  const bool valid = qi < Nq;                // a wave without a row still helps to load and keeps the barriers
  const int kvh = hq / (a.Hq / a.Hkv);
  const int D = a.D, D4 = D / 4, KP = D + 4;
  float* k_s = kv_s;
  float* v_s = kv_s + 64 * KP;
  const long long qbh = (long long)b * a.Hq + hq;
  if (valid) {
    const float* qrow = (qi < a.K) ? a.q_block + (qbh * a.K + qi) * D
                                   : a.q_suffix + (qbh * a.S + a.keep_idx[qi - a.K]) * D;
    for (int d = lane; d < D; d += 64) q_s[wave][d] = qrow[d];
  }

  constexpr int kCols = kF32MaxD / 64;       // output columns per lane
  float o[kCols];
#pragma unroll
  for (int c = 0; c < kCols; ++c) o[c] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int k0 = 0; k0 < Nkv; k0 += 64) {
    const int nk = min(64, Nkv - k0);
    __syncthreads();                         // the previous chunk is consumed (first trip: q_s is written)
    for (int i = threadIdx.x; i < nk * D4; i += 64 * kF32Waves) {
      const int j = i / D4, c4 = i - j * D4;
      const float4 kk = reinterpret_cast<const float4*>(kv_row(a, a.k_cache, a.k_block, a.k_suffix, b, kvh, k0 + j))[c4];
      const float4 vv = reinterpret_cast<const float4*>(kv_row(a, a.v_cache, a.v_block, a.v_suffix, b, kvh, k0 + j))[c4];
      *reinterpret_cast<float4*>(k_s + j * KP + 4 * c4) = kk;
      *reinterpret_cast<float4*>(v_s + j * D + 4 * c4) = vv;
    }
    __syncthreads();
    if (!valid) continue;
    float sc = -INFINITY;
    if (lane < nk) {
      const float4* kr = reinterpret_cast<const float4*>(k_s + lane * KP);
      float acc = 0.f;
      for (int d4 = 0; d4 < D4; ++d4) {
        const float4 kk = kr[d4];
        const float* qq = &q_s[wave][4 * d4];
        acc = fmaf(qq[0], kk.x, acc); acc = fmaf(qq[1], kk.y, acc);
        acc = fmaf(qq[2], kk.z, acc); acc = fmaf(qq[3], kk.w, acc);
      }
      sc = acc * a.scale;
    }
    float cmax = sc;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off));
    const float m_new = fmaxf(m, cmax);
    const float corr = (m == -INFINITY) ? 0.f : expf(m - m_new);
    const float p = (lane < nk) ? expf(sc - m_new) : 0.f;
    float psum = p;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) psum += __shfl_xor(psum, off);
    l = l * corr + psum;
    m = m_new;
#pragma unroll
    for (int c = 0; c < kCols; ++c) o[c] *= corr;
    for (int j = 0; j < nk; ++j) {
      const float pj = __shfl(p, j);
      const float* vr = v_s + j * D;
#pragma unroll
      for (int c = 0; c < kCols; ++c) {
        const int d = lane + 64 * c;
        if (d < D) o[c] = fmaf(pj, vr[d], o[c]);
      }
    }
  }
  if (!valid) return;
  float* orow = a.out + (qbh * Nq + qi) * D;
  const float inv = 1.0f / l;
#pragma unroll
  for (int c = 0; c < kCols; ++c) {
    const int d = lane + 64 * c;
    if (d < D) orow[d] = o[c] * inv;
  }
}

hipError_t prepare_attention_f32() {
  static LdsOptIn st;
  return ensure_lds_opt_in(reinterpret_cast<const void*>(&attention_f32_kernel), f32_lds_bytes(kF32MaxD), st);
}

hipError_t launch_attention_f32(const sdllm_attn_params& p,
                                const void* q_block, const void* q_suffix,
                                const void* k_cache, const void* v_cache,
                                const void* k_block, const void* v_block,
                                const void* k_suffix, const void* v_suffix,
                                const int32_t* keep_idx, void* out, hipStream_t stream) {
  AttnF32Args a;
  a.q_block = (const float*)q_block; a.q_suffix = (const float*)q_suffix;
  a.k_cache = (const float*)k_cache; a.v_cache = (const float*)v_cache;
  a.k_block = (const float*)k_block; a.v_block = (const float*)v_block;
  a.k_suffix = (const float*)k_suffix; a.v_suffix = (const float*)v_suffix;
  a.keep_idx = keep_idx; a.out = (float*)out;
  a.B = p.B; a.Hq = p.Hq; a.Hkv = p.Hkv; a.D = p.D; a.P = p.prefix_len; a.cap = p.prefix_cap;
  a.K = p.K; a.S = p.S; a.n_keep = p.n_keep;
  a.scale = p.scale > 0.f ? p.scale : 1.0f / sqrtf((float)p.D);
  const int Nq = p.K + p.n_keep;
  dim3 grid((Nq + kF32Waves - 1) / kF32Waves, p.Hq, p.B);
  hipError_t e = prepare_attention_f32();     // opt-in to the LDS size of the largest head dim, once per device
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attention_f32_kernel, grid, dim3(64 * kF32Waves), f32_lds_bytes(p.D), stream, a);
  return hipGetLastError();
}

}  // namespace sdllm
