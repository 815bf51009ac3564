// Pieces shared by the two producers of per-row softmax partials (the streaming reduction over stored
// logits and the vocabulary projection that never stores them) and by the commit kernel.
#pragma once
#include "common.h"

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
