// Diagnostics: what plain kernels reach on the device the library runs on -- a read-only stream, a copy,
// and a loop of independent bf16 matrix instructions.  The roofline fractions of the hot-path kernels are
// quoted against the published peaks; these three give the practical ceilings next to them.
#include "common.h"

namespace sdllm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4p;

constexpr int kProbeThreads = 256;
constexpr int kProbeVec = 8;            // 16-byte vectors per lane and workgroup

__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const u32x4p* __restrict__ p, unsigned* sink, long long n) {
  const long long i = (long long)blockIdx.x * kProbeVec * kProbeThreads + threadIdx.x;
  u32x4p v[kProbeVec];
#pragma unroll
  for (int u = 0; u < kProbeVec; ++u) {
    const long long j = i + (long long)u * kProbeThreads;
    v[u] = j < n ? __builtin_nontemporal_load(p + j) : u32x4p{0u, 0u, 0u, 0u};
  }
  unsigned acc = 0;
#pragma unroll
  for (int u = 0; u < kProbeVec; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  if (acc == 0x9e3779b9u) sink[0] = acc;          // keeps the loads alive; practically never taken
}

constexpr int kCopyVec = 4;
__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(u32x4p* __restrict__ q, const u32x4p* __restrict__ p, long long n) {
  const long long i = (long long)blockIdx.x * kCopyVec * kProbeThreads + threadIdx.x;
  u32x4p v[kCopyVec];
#pragma unroll
  for (int u = 0; u < kCopyVec; ++u) {
    const long long j = i + (long long)u * kProbeThreads;
    if (j < n) v[u] = __builtin_nontemporal_load(p + j);
  }
#pragma unroll
  for (int u = 0; u < kCopyVec; ++u) {
    const long long j = i + (long long)u * kProbeThreads;
    if (j < n) __builtin_nontemporal_store(v[u], q + j);
  }
}

// Every wave: 8 independent accumulators, `iters` rounds of 8 v_mfma_f32_16x16x32_bf16.  kind 0: smooth small
// operand values; kind 1: operands with pseudo-random sign, exponent and mantissa bits (values in about
// [-2, 2]), which draw more power per instruction and lower the sustained clock.
__global__ __launch_bounds__(kProbeThreads, 2) void probe_mfma_kernel(int iters, int kind, float* sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[8], b[8];                      // one operand pair per accumulator: consecutive instructions see different bits
  unsigned h = (unsigned)(threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
#pragma unroll
  for (int p = 0; p < 8; ++p)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (kind == 0) { a[p][i] = (__bf16)(0.001f * (lane + i)); b[p][i] = (__bf16)(0.002f * (lane - i)); }
      else {
        h = h * 1664525u + 1013904223u;
        const unsigned ea = 0x3e00u + ((h >> 8) & 0x1ffu);         // exponents 2^-3 .. 2^0, random mantissa
        a[p][i] = __builtin_bit_cast(__bf16, (unsigned short)(ea | ((h & 1u) << 15)));
        h = h * 1664525u + 1013904223u;
        const unsigned eb = 0x3e00u + ((h >> 8) & 0x1ffu);
        b[p][i] = __builtin_bit_cast(__bf16, (unsigned short)(eb | ((h & 1u) << 15)));
      }
    }
  f32x4 c[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) c[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[i], c[i], 0, 0, 0);
    // fold the accumulators back now and then so that random operands cannot run them to infinity
    if ((it & 63) == 63) {
#pragma unroll
      for (int i = 0; i < 8; ++i) c[i] = c[i] * 1.0e-3f;
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += c[i][0] + c[i][1] + c[i][2] + c[i][3];
  if (s == 123.456f) sink[0] = s;
}

hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t stream) {
  const long long n = (long long)(bytes / 16);
  const unsigned grid = (unsigned)((n + kProbeVec * kProbeThreads - 1) / (kProbeVec * kProbeThreads));
  hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(kProbeThreads), 0, stream, (const u32x4p*)src, (unsigned*)sink, n);
  return hipGetLastError();
}

hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const long long n = (long long)(bytes / 16);
  const unsigned grid = (unsigned)((n + kCopyVec * kProbeThreads - 1) / (kCopyVec * kProbeThreads));
  hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(kProbeThreads), 0, stream, (u32x4p*)dst, (const u32x4p*)src, n);
  return hipGetLastError();
}

double probe_mfma_flops(int iters) {   // per launch
  const double waves = 2.0 * kNumCUs * (kProbeThreads / 64);
  return waves * iters * 8.0 * (2.0 * 16 * 16 * 32);
}

hipError_t launch_probe_mfma(int iters, int kind, void* sink, hipStream_t stream) {
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(2 * kNumCUs), dim3(kProbeThreads), 0, stream, iters, kind, (float*)sink);
  return hipGetLastError();
}

}  // namespace sdllm
