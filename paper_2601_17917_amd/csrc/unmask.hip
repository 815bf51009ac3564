// Confidence-aware unmasking (paper Eq. 4, 5, 9, 10; block termination; EOS early exit).
//
// Two launches on the caller's stream:
//  1. unmask_rows: a bandwidth-bound streaming reduction.  Every masked row of logits is
//     split over `nsplit` workgroups; each streams its vocabulary slice once with 16-byte
//     loads and reduces it to a (max, sum of exp relative to that max, lowest argmax id)
//     triple.  Rows of unmasked positions are never read.
//  2. unmask_commit: one workgroup per sequence merges the triples in a fixed pattern,
//     forms c_i = 1 / sum, evaluates the threshold, commits, and writes the flags.
// The rows kernel is bound by its vector arithmetic, not by the stream: per 32 logits of a lane (one trip of four
// 16-byte bf16 vectors) it issues 189 instructions -- unpack 32, max 16, FMA 31, exp 33, add 31, addressing and
// bookkeeping 46 -- i.e. (156 + 33 * 2.4) / 32 = 7.35 issue slots per logit with v_exp_f32 at the 2.4 slots it costs
// against an FMA (fp32 logits need no unpack: 6.35).  On 256 CUs x 4 SIMDs at 2.4 GHz, one wave-wide instruction per
// four cycles, that is the plain-ALU roof the benchmark quotes next to the HBM one.
// (A single launch in which the last workgroup to arrive commits its sequence was measured
// and dropped: the device-scope release/acquire fences it needs write back and invalidate
// the L2 of an XCD on every workgroup and cost several times the second launch.)
#include "common.h"
#include "unmask_common.h"

namespace sdllm {

constexpr int kRowThreads = 256;
constexpr int kVecPerIter = 4;        // 16-byte vectors in flight per lane

template <typename T> struct Vec;
template <> struct Vec<uint16_t> {   // bf16 bit patterns, 8 per 16 bytes
  static constexpr int N = 8;
  __device__ static __forceinline__ void unpack(const u32x4& r, float* x) {
    x[0] = __uint_as_float(r.x << 16); x[1] = __uint_as_float(r.x & 0xffff0000u);
    x[2] = __uint_as_float(r.y << 16); x[3] = __uint_as_float(r.y & 0xffff0000u);
    x[4] = __uint_as_float(r.z << 16); x[5] = __uint_as_float(r.z & 0xffff0000u);
    x[6] = __uint_as_float(r.w << 16); x[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};
template <> struct Vec<float> {      // 4 per 16 bytes
  static constexpr int N = 4;
  __device__ static __forceinline__ void unpack(const u32x4& r, float* x) {
    x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
    x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
  }
};

// Maximum of the N values of one vector with the three-input instruction, written out: through fmaxf the compiler
// first canonicalises every value it cannot prove canonical (an extra v_max x, x per unpacked logit pair).  The
// instruction itself returns the other operand when one is NaN, like fmaxf.
__device__ __forceinline__ float max3_raw(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
template <int N>
__device__ __forceinline__ float vector_max(const float (&x)[N]) {
  static_assert(N == 4 || N == 8, "16-byte vectors of fp32 / bf16");
  float c = max3_raw(x[0], x[1], x[2]);
  if constexpr (N == 8) {
    c = max3_raw(c, x[3], x[4]);
    c = max3_raw(c, x[5], x[6]);
    return max3_raw(c, x[7], x[7]);
  } else {
    return max3_raw(c, x[3], x[3]);
  }
}

// Folds kVecPerIter unpacked vectors per lane (vector indices v0, v0 + 256, ...) into the lane's running
// (max, sum of exp2 relative to that max, first vector holding the max).  Elements that do not exist
// hold -inf: they never win the maximum and add exp2(-inf) = 0.
template <int N>
__device__ __forceinline__ void accumulate_trip(const float (&x)[kVecPerIter][N], int v0, float& m, float& s, int& mvec) {
  float bm = m;
#pragma unroll
  for (int u = 0; u < kVecPerIter; ++u) {
    const float c = vector_max<N>(x[u]);
    const bool up = c > bm;                // strict: the earliest vector keeps the maximum
    mvec = up ? v0 + u * kRowThreads : mvec;
    bm = up ? c : bm;
  }
  s *= fast_exp2((m - bm) * kLog2e);
  m = bm;
  const float ml = m * kLog2e;
#pragma unroll
  for (int u = 0; u < kVecPerIter; ++u) {
#pragma unroll
    for (int j = 0; j < N; ++j) s += fast_exp2(fmaf(x[u][j], kLog2e, -ml));
  }
}

// Streams vocabulary slice `split` of one row; the merged triple of the workgroup ends in thread 0.
template <typename T>
__device__ __forceinline__ Partial reduce_row_slice(const UnmaskArgs& a, int row, int split, Partial* red) {
  constexpr int N = Vec<T>::N;
  constexpr int kStride = kRowThreads * kVecPerIter;
  constexpr unsigned kNegInfWord = (N == 8) ? 0xff80ff80u : 0xff800000u;   // -inf: two bf16 / one fp32
  const u32x4* __restrict__ base = reinterpret_cast<const u32x4*>(reinterpret_cast<const T*>(a.logits) + (long long)row * a.ld);
  const int v_begin = split * a.vec_per_split;
  const int v_end = min(v_begin + a.vec_per_split, a.nvec);
  const int tid = threadIdx.x;

  float m = kNegBig, s = 0.f;
  int mvec = 0x7fffffff;                   // vector index holding this lane's maximum (first one)

  // The arithmetic, not the stream, bounds this kernel (its loads hide behind it), so the trips that
  // lie wholly inside the slice and hold only complete vectors run without any bounds handling:
  // unconditional loads, unpack, max, exp2-sum.  What is left (less than one trip, and the row's last
  // vector when V is not a multiple of the vector length) goes through one guarded trip.
  const bool ragged_row_end = (v_end == a.nvec) && (a.V % N != 0);             // uniform
  const int n_bulk = max((v_end - (ragged_row_end ? 1 : 0)) - v_begin, 0) / kStride;   // uniform
  int v0 = v_begin + tid;
  for (int t = 0; t < n_bulk; ++t, v0 += kStride) {
    u32x4 r[kVecPerIter];
#pragma unroll
    for (int u = 0; u < kVecPerIter; ++u) r[u] = __builtin_nontemporal_load(base + v0 + u * kRowThreads);
    float x[kVecPerIter][N];
#pragma unroll
    for (int u = 0; u < kVecPerIter; ++u) Vec<T>::unpack(r[u], x[u]);
    accumulate_trip<N>(x, v0, m, s, mvec);
  }
  if (v0 - tid < v_end) {                  // uniform: the guarded trip
    u32x4 r[kVecPerIter];
#pragma unroll
    for (int u = 0; u < kVecPerIter; ++u) {
      r[u] = u32x4{kNegInfWord, kNegInfWord, kNegInfWord, kNegInfWord};
      const int v = v0 + u * kRowThreads;
      if (v < v_end) r[u] = __builtin_nontemporal_load(base + v);
    }
    float x[kVecPerIter][N];
#pragma unroll
    for (int u = 0; u < kVecPerIter; ++u) Vec<T>::unpack(r[u], x[u]);
    if (ragged_row_end) {                  // uniform: the row's last vector runs past V
#pragma unroll
      for (int u = 0; u < kVecPerIter; ++u) {
        const int v = v0 + u * kRowThreads;
        if (v == a.nvec - 1) {
#pragma unroll
          for (int j = 0; j < N; ++j) if (v * N + j >= a.V) x[u][j] = -INFINITY;
        }
      }
    }
    if (v0 < v_end) accumulate_trip<N>(x, v0, m, s, mvec);   // lanes past the end have nothing to add
  }

  // merge (max, sum, first vector holding the max) across the wave, then across the waves through
  // LDS.  Vectors cover disjoint, increasing id ranges, so the lowest vector index among equal
  // maxima contains the lowest arg-max id; it is located at the end by ONE lane re-reading ONE
  // vector (a per-lane re-read would add a scattered 64-byte fetch per lane to the stream).
  wave_merge_triples(m, s, mvec);
  if ((tid & 63) == 0) red[tid >> 6] = Partial{m, s, mvec};
  __syncthreads();
  int idx = 0x7fffffff;
  if (tid == 0) {
#pragma unroll
    for (int w = 1; w < kRowThreads / 64; ++w) merge_partial(m, s, mvec, red[w].m, red[w].s, red[w].idx);
    if (mvec != 0x7fffffff) {
      u32x4 r = base[mvec];
      float x[N];
      Vec<T>::unpack(r, x);
#pragma unroll
      for (int j = N - 1; j >= 0; --j) if (x[j] == m && mvec * N + j < a.V) idx = mvec * N + j;
    }
  }
  return Partial{m, s, idx};
}

// Threshold, selection, update and flags of sequence b (Eq. 10, 9, 5), run by one whole workgroup
// once every triple of the sequence is visible.
template <int THREADS>
__device__ __forceinline__ void commit_sequence(const UnmaskArgs& a, int b, float* conf_s, int* xhat_s) {
  __shared__ int cnt_masked, cnt_thr, eos_hit;
  __shared__ float best_c[THREADS / 64];
  __shared__ int best_i[THREADS / 64];
  const int tid = threadIdx.x, K = a.K;
  if (tid == 0) { cnt_masked = 0; cnt_thr = 0; eos_hit = 0; }
  __syncthreads();

  // pass 1: P2 adjacent lanes (at most one wave) hold the triples of one position and merge them with a
  // butterfly (fixed pattern); all loads of a pass are independent.  With more than 64 triples per
  // position (the vocabulary projection writes one per vocabulary tile) a lane first folds every 64th.
  const int P2 = a.nsplit_p2;
  const int pos_per_pass = THREADS / P2;
  const int k = tid & (P2 - 1);
  int my_masked = 0;
  for (int i0 = 0; i0 < K; i0 += pos_per_pass) {
    const int i = i0 + tid / P2;
    const bool in = i < K;
    const long long pos = (long long)b * K + (in ? i : 0);
    const bool is_masked = in && a.masked[pos] != 0;
    // the triple is loaded without waiting for the mask byte (its slot is valid memory either way;
    // for an unmasked position it holds garbage that is discarded): one memory round trip, not two
    const Partial pr = a.partials[pos * a.nsplit + min(k, a.nsplit - 1)];
    float m = kNegBig, s = 0.f; int idx = 0x7fffffff;
    if (is_masked && k < a.nsplit) { m = pr.m; s = pr.s; idx = pr.idx; }
    if (a.nsplit > P2 && is_masked) {
      constexpr int kBatch = 16;                      // independent loads in flight per lane
      for (int k0 = k + P2; k0 < a.nsplit; k0 += kBatch * P2) {
        Partial q[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) q[u] = a.partials[pos * a.nsplit + min(k0 + u * P2, a.nsplit - 1)];
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
          if (k0 + u * P2 < a.nsplit) merge_partial(m, s, idx, q[u].m, q[u].s, q[u].idx);
      }
    }
    // butterfly over the P2 adjacent lanes of a position (P2 is uniform), fixed pattern, lane network only
    if (P2 >= 2)  merge_partial(m, s, idx, lane_partner<0>(m), lane_partner<0>(s), lane_partner<0>(idx));
    if (P2 >= 4)  merge_partial(m, s, idx, lane_partner<1>(m), lane_partner<1>(s), lane_partner<1>(idx));
    if (P2 >= 8)  merge_partial(m, s, idx, lane_partner<2>(m), lane_partner<2>(s), lane_partner<2>(idx));
    if (P2 >= 16) merge_partial(m, s, idx, lane_partner<3>(m), lane_partner<3>(s), lane_partner<3>(idx));
    if (P2 >= 32) merge_partial(m, s, idx, lane_partner<4>(m), lane_partner<4>(s), lane_partner<4>(idx));
    if (P2 >= 64) merge_partial(m, s, idx, lane_partner<5>(m), lane_partner<5>(s), lane_partner<5>(idx));
    if (in && k == 0) {
      float c = 0.f;
      if (is_masked) {
        c = 1.0f / s;
        my_masked++;
        if (a.confidence) a.confidence[pos] = c;
        // a row without any finite logit has no arg-max: id 0 stands in, so that a committed id is always < V
        xhat_s[i] = (unsigned)idx < (unsigned)a.V ? idx : 0;
        // the selection below works on a strictly positive NORMAL number (it survives a flush of denormals):
        // a row of NaN logits (garbage in) ranks last instead of leaving the fallback without a candidate
        if (!(c > 0.f)) c = 1.17549435e-38f;
      }
      conf_s[i] = c;
    }
  }
  if (my_masked) atomicAdd(&cnt_masked, my_masked);
  __syncthreads();
  const int m_b = cnt_masked;
  if (m_b == 0) {
    if (tid == 0) { a.n_committed[b] = 0; a.block_done[b] = 1; }
    return;
  }
  // Eq. 10 in double, in the written order of operations
  const double r_mask = (double)(m_b + a.r_extra_masked) / (double)(K + a.r_extra_total);
  const double tau = __dmul_rn((double)a.tau0, __dsub_rn(1.0, __dmul_rn((double)a.alpha, __dsub_rn(1.0, r_mask))));

  // pass 2: threshold commits + candidates for the fallback
  float bc = -1.f; int bi = 0x7fffffff; int my_thr = 0;
  for (int i = tid; i < K; i += THREADS) {
    const long long pos = (long long)b * K + i;
    // pass 1 left 0 for an unmasked position and 1 / sum > 0 for a masked one: no second look at the
    // mask bytes (one memory round trip less)
    const float c = conf_s[i];
    if (c == 0.f) continue;
    if ((double)c >= tau) {
      const int xhat = xhat_s[i];
      a.tokens[pos] = xhat;
      a.masked[pos] = 0;
      my_thr++;
      if (a.eos_id >= 0 && xhat == a.eos_id && c >= a.tau_eos) eos_hit = 1;
    }
    if (c > bc) { bc = c; bi = i; }       // ascending i: strict > keeps the lowest position
  }
  if (my_thr) atomicAdd(&cnt_thr, my_thr);
  {   // the wave's best candidate: highest confidence, lowest position among equals
    const float wave_c = wave_allreduce(bc, [](float x, float y) { return fmaxf(x, y); });
    bi = wave_allreduce(bc == wave_c ? bi : 0x7fffffff, [](int x, int y) { return min(x, y); });
    bc = wave_c;
  }
  if ((tid & 63) == 0) { best_c[tid >> 6] = bc; best_i[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    int ncommit = cnt_thr;
    if (ncommit == 0) {                     // fallback: single most confident masked position
      for (int w = 1; w < THREADS / 64; ++w)
        if (best_c[w] > bc || (best_c[w] == bc && best_i[w] < bi)) { bc = best_c[w]; bi = best_i[w]; }
      if (bi < K) {                         // always true with m_b > 0; no store can leave the block regardless
        const long long pos = (long long)b * K + bi;
        const int xhat = xhat_s[bi];
        a.tokens[pos] = xhat;
        a.masked[pos] = 0;
        ncommit = 1;
        if (a.eos_id >= 0 && xhat == a.eos_id && bc >= a.tau_eos) eos_hit = 1;
      }
    }
    a.n_committed[b] = ncommit;
    a.block_done[b] = (m_b - ncommit == 0) ? 1 : 0;
    if (a.eos_seen && eos_hit) a.eos_seen[b] = 1;
  }
}

template <typename T>
__global__ __launch_bounds__(kRowThreads) void unmask_rows_kernel(UnmaskArgs a) {
  __shared__ Partial red[kRowThreads / 64];
  const int row = blockIdx.x / a.nsplit;
  const int split = blockIdx.x - row * a.nsplit;
  // The row's mask byte through the scalar data cache: the aligned dword that holds it (an aligned dword lies inside
  // one page, so reading it cannot fault even where the byte array does not fill it; only the row's own byte is
  // used).  A vector load of the byte costs every workgroup a longer round trip before its first logits load.
  typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;
  const uintptr_t mb = reinterpret_cast<uintptr_t>(a.masked) + (uintptr_t)row;
  const uint32_t mword = *reinterpret_cast<const_u32_ptr>(mb & ~(uintptr_t)3);
  if (((mword >> (8 * (unsigned)(mb & 3))) & 0xffu) == 0) return;            // uniform per workgroup
  const Partial p = reduce_row_slice<T>(a, row, split, red);
  if (threadIdx.x == 0) a.partials[(long long)row * a.nsplit + split] = p;
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void unmask_commit_kernel(UnmaskArgs a) {
  extern __shared__ float conf_s[];          // K confidences, then K predicted ids
  int* xhat_s = reinterpret_cast<int*>(conf_s + a.K);
  commit_sequence<THREADS>(a, blockIdx.x, conf_s, xhat_s);
}

hipError_t launch_unmask_commit(const UnmaskArgs& args, int B, hipStream_t stream) {
  UnmaskArgs r = args;
  r.nsplit_p2 = 1;
  while (r.nsplit_p2 < r.nsplit && r.nsplit_p2 < 64) r.nsplit_p2 <<= 1;
  const size_t lds = (size_t)r.K * (sizeof(float) + sizeof(int));
  // many triples per position: 1024 threads, and no more lanes per position than lets all K positions go
  // in one pass when that is possible (every pass is another chain of dependent memory round trips)
  if (r.nsplit > 64) {
    while (r.nsplit_p2 > 1 && r.nsplit_p2 * r.K > 1024) r.nsplit_p2 >>= 1;
    hipLaunchKernelGGL(unmask_commit_kernel<1024>, dim3(B), dim3(1024), lds, stream, r);
  }
  else hipLaunchKernelGGL(unmask_commit_kernel<kRowThreads>, dim3(B), dim3(kRowThreads), lds, stream, r);
  return hipGetLastError();
}

int unmask_splits(const sdllm_unmask_params& p) {
  const int N = p.dtype == SDLLM_FP32 ? 4 : 8;
  const long long nvec = ((long long)p.V + N - 1) / N;
  // aim at >= 8 workgroups per CU over the rows, but keep >= 2 main-loop iterations per split
  const long long rows = (long long)p.B * p.K;
  long long want = (8LL * kNumCUs + rows - 1) / rows;
  // usually only part of the rows is masked (the others' workgroups exit at once): keep at least 6 slices
  // per row while that stays below 16 workgroups per CU (512 rows, about half masked: 49.6 -> 48.3 us per step)
  if (want < 6 && rows * 6 <= 16LL * kNumCUs) want = 6;
  long long max_by_len = nvec / (kRowThreads * kVecPerIter);
  if (max_by_len < 1) max_by_len = 1;
  long long n = want < max_by_len ? want : max_by_len;
  if (n < 1) n = 1;
  if (n > 64) n = 64;
  return (int)n;
}

size_t unmask_workspace_bytes(const sdllm_unmask_params& p) {
  return (size_t)p.B * p.K * unmask_splits(p) * sizeof(Partial);
}

hipError_t launch_unmask(const sdllm_unmask_params& p, const void* logits, int32_t* tokens, uint8_t* masked,
                         float* confidence, int32_t* n_committed, uint8_t* block_done, uint8_t* eos_seen,
                         void* workspace, hipStream_t stream) {
  const int N = p.dtype == SDLLM_FP32 ? 4 : 8;
  UnmaskArgs r;
  r.logits = logits; r.masked = masked;
  r.partials = (Partial*)workspace;
  r.tokens = tokens; r.confidence = confidence;
  r.n_committed = n_committed; r.block_done = block_done; r.eos_seen = eos_seen;
  r.ld = p.ld; r.V = p.V; r.K = p.K;
  r.nvec = (p.V + N - 1) / N;
  r.nsplit = unmask_splits(p);
  r.nsplit_p2 = 1;
  r.vec_per_split = (r.nvec + r.nsplit - 1) / r.nsplit;
  r.tau0 = p.tau0; r.alpha = p.alpha; r.r_extra_masked = p.r_extra_masked; r.r_extra_total = p.r_extra_total;
  r.eos_id = p.eos_id; r.tau_eos = p.tau_eos;
  dim3 grid((unsigned)((long long)p.B * p.K * r.nsplit), 1, 1);
  if (p.dtype == SDLLM_FP32) hipLaunchKernelGGL(unmask_rows_kernel<float>, grid, dim3(kRowThreads), 0, stream, r);
  else hipLaunchKernelGGL(unmask_rows_kernel<uint16_t>, grid, dim3(kRowThreads), 0, stream, r);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_unmask_commit(r, p.B, stream);
}

}  // namespace sdllm
