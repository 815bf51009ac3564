// Pieces shared by the two producers of per-row softmax partials (the streaming reduction over stored
// logits and the vocabulary projection that never stores them) and by the commit kernel.
#pragma once
#include "common.h"
#include <type_traits>

namespace sdllm {

constexpr float kLog2e = 1.4426950408889634f;
// finite stand-in for -inf as the initial running maximum: keeps (m - m) and m * log2(e) free of NaN
// and overflow (a lane or a vector whose logits are all -inf then contributes exp2(-inf) = 0)
constexpr float kNegBig = -1.0e30f;

struct Partial { float m; float s; int idx; };
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // native vector: usable with nontemporal builtins

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// merge (m2,s2,i2) into (m,s,i); ties on the maximum keep the lower id
__device__ __forceinline__ void merge_partial(float& m, float& s, int& i, float m2, float s2, int i2) {
  float M = fmaxf(m, m2);
  float a = fast_exp2((m - M) * kLog2e);
  float b = fast_exp2((m2 - M) * kLog2e);
  s = s * a + s2 * b;
  i = (m2 > m) ? i2 : ((m2 == m) ? min(i, i2) : i);
  m = M;
}

// Wave-wide reductions on the vector ALU's own lane network (DPP row operations inside each row of 16 lanes, then
// the two row swaps): ~10 cycles per step where a shuffle through the LDS crossbar is a memory-pipe round trip.
// Every lane ends with the result.
template <typename T, typename F>
__device__ __forceinline__ T wave_allreduce(T v, F op) {
  static_assert(sizeof(T) == 4, "32-bit values");
  auto dpp = [](T x, auto ctrl_c) {
    constexpr int CTRL = decltype(ctrl_c)::value;
    return __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
  };
  v = op(v, dpp(v, std::integral_constant<int, 0xB1>{}));    // quad_perm [1,0,3,2]
  v = op(v, dpp(v, std::integral_constant<int, 0x4E>{}));    // quad_perm [2,3,0,1]
  v = op(v, dpp(v, std::integral_constant<int, 0x141>{}));   // row_half_mirror: the other quad of each 8
  v = op(v, dpp(v, std::integral_constant<int, 0x140>{}));   // row_mirror: the other half of each row of 16
  // the two swaps exchange rows 1 <-> 0, 3 <-> 2 and then the halves between their two operands (the same value
  // twice here); the results are copied into scalars before the bit casts (a bit cast applied to a vector element
  // expression reads element 0 with this compiler)
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned a0 = r16[0], a1 = r16[1];
  v = op(__builtin_bit_cast(T, a0), __builtin_bit_cast(T, a1));
  const unsigned w = __builtin_bit_cast(unsigned, v);
  const auto r32 = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  const unsigned b0 = r32[0], b1 = r32[1];
  return op(__builtin_bit_cast(T, b0), __builtin_bit_cast(T, b1));
}

// The value a partner lane holds, for a butterfly over groups of 2^(LEVEL+1) adjacent lanes: level 0 / 1 pair lane i
// with i ^ 1 / i ^ 2, level 2 / 3 mirror inside 8 / 16 lanes (lane i with 7 - i / 15 - i: the partner lies in the other
// half of the group, which is all a butterfly needs once both halves are reduced), level 4 / 5 take the same lane of
// the neighbouring row of 16 / the other half of the wave.  All on the vector ALU's lane network.
template <int LEVEL, typename T>
__device__ __forceinline__ T lane_partner(T x) {
  static_assert(sizeof(T) == 4 && LEVEL >= 0 && LEVEL <= 5, "32-bit values, 64 lanes");
  const int xi = __builtin_bit_cast(int, x);
  if constexpr (LEVEL < 4) {
    constexpr int CTRL = LEVEL == 0 ? 0xB1 : LEVEL == 1 ? 0x4E : LEVEL == 2 ? 0x141 : 0x140;
    return __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(0, xi, CTRL, 0xf, 0xf, true));
  } else if constexpr (LEVEL == 4) {
    const auto r = __builtin_amdgcn_permlane16_swap((unsigned)xi, (unsigned)xi, false, false);
    const unsigned even_rows = r[1], odd_rows = r[0];      // [r1,r1,r3,r3] and [r0,r0,r2,r2]
    const bool odd = (__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) >> 4) & 1;
    return __builtin_bit_cast(T, odd ? odd_rows : even_rows);
  } else {
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)xi, (unsigned)xi, false, false);
    const unsigned lo_half = r[1], hi_half = r[0];         // [hi,hi] and [lo,lo]
    const bool hi = (__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) >> 5) & 1;
    return __builtin_bit_cast(T, hi ? hi_half : lo_half);
  }
}

// (max, sum of exp relative to the max, lowest index among the lanes that hold the max) of a wave's 64 lane triples:
// maximum first, one rescale per lane, then plain sums -- the same result as 63 pairwise merges up to rounding order
__device__ __forceinline__ void wave_merge_triples(float& m, float& s, int& idx) {
  const float M = wave_allreduce(m, [](float a, float b) { return fmaxf(a, b); });
  s *= fast_exp2((m - M) * kLog2e);
  idx = (m == M) ? idx : 0x7fffffff;
  s = wave_allreduce(s, [](float a, float b) { return a + b; });
  idx = wave_allreduce(idx, [](int a, int b) { return min(a, b); });
  m = M;
}

struct UnmaskArgs {
  const void* logits;
  Partial* partials;       // [rows][nsplit]
  int32_t* tokens; uint8_t* masked; float* confidence;
  int32_t* n_committed; uint8_t* block_done; uint8_t* eos_seen;
  long long ld;            // elements
  int V;
  int nvec;                // 16-byte vectors covering V (last one may be partial)
  int vec_per_split;
  int nsplit;
  int nsplit_p2;           // nsplit rounded up to a power of two (<= 64)
  int K;
  float tau0, alpha; int r_extra_masked, r_extra_total; int eos_id; float tau_eos;
};

// Second launch of both paths: merges the triples of every masked position in a fixed pattern and commits
// (Eq. 10, 9, 5, exit flags).  r.partials is [B*K][r.nsplit]; r.nsplit may be any count >= 1.
hipError_t launch_unmask_commit(const UnmaskArgs& r, int B, hipStream_t stream);

}  // namespace sdllm
