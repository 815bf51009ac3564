// Rotary position embedding of the pruned query / key rows with their original position ids
// (paper section 3.3, the sentence before Eq. 7: kept suffix tokens keep the logical order of the
// full sequence through their RoPE position ids).  Block row r is rotated for position pos0 + r,
// kept suffix row j for position pos0 + K + keep_idx[j]; suffix rows that are not kept are neither
// read nor written.
//
// Bandwidth-bound and tiny: one workgroup per (pruned row, chunk of batch*heads).  The D/2
// (cos, sin) pairs of the row's position are computed once per workgroup in double precision
// (angle = position * base^(-2i/D) reaches thousands of radians; in float the angle itself would
// carry an error of 1e-4), kept in LDS as floats, and applied to the same row of every (batch, head)
// of the chunk with 16-byte loads and stores.  In place is allowed: a lane reads both halves of its
// pairs before it writes them, and no other lane touches them.
#include "common.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

struct RopeArgs {
  const void* x_block; const void* x_suffix;
  void* out_block; void* out_suffix;
  const int32_t* keep_idx;
  int BH, D, K, S, n_keep, pos0, rows_per_chunk;
  double log2_base;
};

constexpr int kRopeMaxHalfD = 256;

template <typename T> struct RopeVec;
template <> struct RopeVec<float> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void unpack(const u32x4& r, float* x) {
    x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y); x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
  }
  __device__ static __forceinline__ u32x4 pack(const float* x) {
    return u32x4{__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
  }
};
template <> struct RopeVec<uint16_t> {   // bf16 bit patterns; results rounded to nearest even
  static constexpr int N = 8;
  __device__ static __forceinline__ void unpack(const u32x4& r, float* x) {
    x[0] = __uint_as_float(r.x << 16); x[1] = __uint_as_float(r.x & 0xffff0000u);
    x[2] = __uint_as_float(r.y << 16); x[3] = __uint_as_float(r.y & 0xffff0000u);
    x[4] = __uint_as_float(r.z << 16); x[5] = __uint_as_float(r.z & 0xffff0000u);
    x[6] = __uint_as_float(r.w << 16); x[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  __device__ static __forceinline__ unsigned pk(float lo, float hi) {
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
  }
  __device__ static __forceinline__ u32x4 pack(const float* x) {
    return u32x4{pk(x[0], x[1]), pk(x[2], x[3]), pk(x[4], x[5]), pk(x[6], x[7])};
  }
};

template <typename T, bool INTERLEAVED>
__global__ __launch_bounds__(256) void rope_kernel(RopeArgs a) {
  constexpr int N = RopeVec<T>::N;
  __shared__ float cos_s[kRopeMaxHalfD], sin_s[kRopeMaxHalfD];
  const int qi = blockIdx.x;                       // row of the pruned sequence: block rows, then kept suffix rows
  const int tid = threadIdx.x;
  const bool in_block = qi < a.K;
  const int srow = in_block ? qi : a.keep_idx[qi - a.K];
  const int pos = a.pos0 + (in_block ? qi : a.K + srow);
  const long long T_len = in_block ? a.K : a.S;    // rows per (batch, head) of the tensor this row lives in
  const T* src = reinterpret_cast<const T*>(in_block ? a.x_block : a.x_suffix);
  T* dst = reinterpret_cast<T*>(in_block ? a.out_block : a.out_suffix);
  const int D = a.D, H2 = D / 2;

  for (int i = tid; i < H2; i += 256) {
    const double theta = exp2(-(2.0 * i / D) * a.log2_base);
    double s, c;
    sincos((double)pos * theta, &s, &c);
    cos_s[i] = (float)c; sin_s[i] = (float)s;
  }
  __syncthreads();

  const int bh0 = blockIdx.y * a.rows_per_chunk;
  const int bh1 = min(bh0 + a.rows_per_chunk, a.BH);
  if (INTERLEAVED) {
    // pairs (2i, 2i+1): one vector holds N/2 whole pairs
    const int RV = D / N;
    const int items = (bh1 - bh0) * RV;
    for (int it = tid; it < items; it += 256) {
      const int bh = bh0 + it / RV, rv = it % RV;
      const long long off = ((long long)bh * T_len + srow) * D + (long long)rv * N;
      float x[N], y[N];
      RopeVec<T>::unpack(*reinterpret_cast<const u32x4*>(src + off), x);
#pragma unroll
      for (int e = 0; e < N / 2; ++e) {
        const float c = cos_s[rv * (N / 2) + e], s = sin_s[rv * (N / 2) + e];
        y[2 * e] = x[2 * e] * c - x[2 * e + 1] * s;
        y[2 * e + 1] = x[2 * e + 1] * c + x[2 * e] * s;
      }
      *reinterpret_cast<u32x4*>(dst + off) = RopeVec<T>::pack(y);
    }
  } else {
    // pairs (i, i + D/2): a vector of the first half and the matching vector of the second half
    const int HV = H2 / N;
    const int items = (bh1 - bh0) * HV;
    for (int it = tid; it < items; it += 256) {
      const int bh = bh0 + it / HV, hv = it % HV;
      const long long off = ((long long)bh * T_len + srow) * D + (long long)hv * N;
      float x1[N], x2[N], y1[N], y2[N];
      RopeVec<T>::unpack(*reinterpret_cast<const u32x4*>(src + off), x1);
      RopeVec<T>::unpack(*reinterpret_cast<const u32x4*>(src + off + H2), x2);
#pragma unroll
      for (int e = 0; e < N; ++e) {
        const float c = cos_s[hv * N + e], s = sin_s[hv * N + e];
        y1[e] = x1[e] * c - x2[e] * s;
        y2[e] = x2[e] * c + x1[e] * s;
      }
      *reinterpret_cast<u32x4*>(dst + off) = RopeVec<T>::pack(y1);
      *reinterpret_cast<u32x4*>(dst + off + H2) = RopeVec<T>::pack(y2);
    }
  }
}

hipError_t launch_rope(const sdllm_rope_params& p, const void* x_block, const void* x_suffix,
                       const int32_t* keep_idx, void* out_block, void* out_suffix, hipStream_t stream) {
  RopeArgs a;
  a.x_block = x_block; a.x_suffix = x_suffix; a.out_block = out_block; a.out_suffix = out_suffix;
  a.keep_idx = keep_idx;
  a.BH = p.B * p.H; a.D = p.D; a.K = p.K; a.S = p.S; a.n_keep = p.n_keep; a.pos0 = p.pos0;
  a.log2_base = log2((double)p.theta_base);
  const int elem = p.dtype == SDLLM_FP32 ? 4 : 2;
  const int nvec = 16 / elem;
  const int vec_items_per_row = p.interleaved ? p.D / nvec : (p.D / 2) / nvec;
  const int rows_per_pass = 256 / vec_items_per_row > 0 ? 256 / vec_items_per_row : 1;
  const int Nq = p.K + p.n_keep;
  // enough workgroups to fill the chip when the data allows it, but at least one full pass each
  int chunks = (4 * kNumCUs + Nq - 1) / Nq;
  const int max_chunks = (a.BH + rows_per_pass - 1) / rows_per_pass;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks < 1) chunks = 1;
  if (chunks > 65535) chunks = 65535;
  a.rows_per_chunk = (a.BH + chunks - 1) / chunks;
  chunks = (a.BH + a.rows_per_chunk - 1) / a.rows_per_chunk;
  dim3 grid(Nq, chunks);
  if (p.dtype == SDLLM_FP32) {
    if (p.interleaved) hipLaunchKernelGGL((rope_kernel<float, true>), grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((rope_kernel<float, false>), grid, dim3(256), 0, stream, a);
  } else {
    if (p.interleaved) hipLaunchKernelGGL((rope_kernel<uint16_t, true>), grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((rope_kernel<uint16_t, false>), grid, dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace sdllm
