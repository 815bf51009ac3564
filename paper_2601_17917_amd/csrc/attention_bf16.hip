// bf16 attention over [prefix cache | block | gathered suffix] for gfx950 (paper Eq. 8 and the
// paragraph after it: block + kept-suffix queries attend, unmasked, to the whole pruned sequence).
//
// Work decomposition
//   group   = (batch, KV head).  The g = Hq/Hkv query heads of a group share its K/V, so their
//             g*Nq query rows are treated as one list of "virtual rows" and tiled together.
//   workgroup = (group, query tile of 64*RB rows, key-range split); 4 waves, wave w owns the
//             16*RB rows  [w*16*RB, (w+1)*16*RB) of the tile for all keys of the split.  Two 8-wave shapes
//             (template MODE, see the kernel): two 4-wave groups on the same rows that alternate key tiles,
//             or two groups on different rows that share every key tile.
//   K/V tiles of 64 keys stream through a two-stage LDS ring.  They are moved global -> LDS
//             directly (global_load_lds_dwordx4: no register staging), one tile ahead of the
//             one being computed, one workgroup barrier per tile.  Rows come from three places
//             (cache, block, suffix[keep_idx]) and are addressed per row, so the gather costs
//             nothing extra: a row is 16 lanes x 16 B, fully coalesced.
// Math (all MFMA v_mfma_f32_16x16x32_bf16, fp32 accumulate)
//   S^T = K Q^T  : A = K rows from LDS, B = Q rows from registers.  The accumulator of lane
//                  (q = lane%16, G = lane/16) holds keys 16*kb + 4*G + i of query row q, so a
//                  softmax row reduction is 15 in-lane ops + 2 cross-lane steps.
//   O^T = V^T P^T: A = V^T through the LDS transpose read (ds_read_b64_tr_b16), B = P^T taken
//                  straight from the S^T accumulators (same lane layout), converted to bf16.
//   Online softmax in the log2 domain; a split writes (unnormalised O, m, l) and a second
//   kernel merges the splits in a fixed order (deterministic, no atomics).
#include "common.h"
#include <type_traits>

namespace sdllm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kKeyTile = 64;
constexpr bool kShareTiles = true;   // 8-wave workgroups with row-split groups for heads with many query rows
constexpr int kShareMinRows = 512;   // ... from this many query rows per K/V head
constexpr int kShareStages = 3;
constexpr float kLog2eA = 1.4426950408889634f;
constexpr float kNegBigA = -3.0e38f;

struct AttnArgs {
  const uint16_t* q_block; const uint16_t* q_suffix;
  const uint16_t* k_cache; const uint16_t* v_cache;
  const uint16_t* k_block; const uint16_t* v_block;
  const uint16_t* k_suffix; const uint16_t* v_suffix;
  const int32_t* keep_idx;
  uint16_t* out;
  float* ws_o;    // [group][virtual row][split][D]   unnormalised partial outputs
  float* ws_ml;   // [group][virtual row][split][2]   (running max in log2 units, sum)
  int B, Hq, Hkv, g, P, cap, K, S, n_keep, Nq, Nkv, Rtot;
  int nsplit, tiles_per_split, key_tiles, q_tiles, n_units;
  float scale_log2, inv_scale_log2;
};

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  // one v_cvt_pk_bf16_f32 (round to nearest even)
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// One 16-byte-per-lane global -> LDS transfer (the data never passes through registers): lane i's
// 16 bytes land at lds_addr + 16*i.  Issued through inline assembly so that the compiler's
// wait-count insertion does not serialise a multi-stage pipeline; completion is tracked by hand
// with s_waitcnt vmcnt(n) before the workgroup barrier (transfers complete in issue order).
__device__ __forceinline__ void dma16_sbase(unsigned lds_addr, const void* sbase, unsigned voff) {
  // the base is the same in every lane; say so, so that it is held in a scalar register pair
  const unsigned long long p = reinterpret_cast<unsigned long long>(sbase);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)p);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(p >> 32));
  const unsigned long long pu = ((unsigned long long)hi << 32) | lo;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(pu) : "memory", "m0");
}
// One 16-row slab of one tensor: NT transfers of 1 KiB to consecutive KiB of LDS from one scalar
// base.  m0 (the LDS base of a transfer) is written once: the instruction's immediate offset moves
// the LDS address and the global address alike, so transfer j carries offset j KiB and its lane offset
// voffj has those j KiB taken off beforehand.  One wait state separates the write of m0 from the
// first transfer that reads it.
// ONCE: every byte of K/V is read by exactly one workgroup of the launch (one query tile per K/V head and
// split); the transfers then carry the nontemporal hint (cfg3A 31.1 -> 28.6 us).  Where query tiles share a
// K/V stream through L2 the hint costs 4-6 %, so it is left off there.
template <int NT, bool ONCE>
__device__ __forceinline__ void dma_slab(unsigned lds_addr, const void* sbase, const unsigned (&voffj)[4]) {
  static_assert(NT == 2 || NT == 4, "transfers per slab");
  if constexpr (NT == 4 && ONCE)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %1 nt\n\t"
                 "global_load_lds_dwordx4 %3, %1 offset:1024 nt\n\t"
                 "global_load_lds_dwordx4 %4, %1 offset:2048 nt\n\t"
                 "global_load_lds_dwordx4 %5, %1 offset:3072 nt"
                 :: "s"(lds_addr), "s"(sbase), "v"(voffj[0]), "v"(voffj[1]), "v"(voffj[2]), "v"(voffj[3]) : "memory", "m0");
  else if constexpr (NT == 4)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %1\n\t"
                 "global_load_lds_dwordx4 %3, %1 offset:1024\n\t"
                 "global_load_lds_dwordx4 %4, %1 offset:2048\n\t"
                 "global_load_lds_dwordx4 %5, %1 offset:3072"
                 :: "s"(lds_addr), "s"(sbase), "v"(voffj[0]), "v"(voffj[1]), "v"(voffj[2]), "v"(voffj[3]) : "memory", "m0");
  else if constexpr (ONCE)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %1 nt\n\t"
                 "global_load_lds_dwordx4 %3, %1 offset:1024 nt"
                 :: "s"(lds_addr), "s"(sbase), "v"(voffj[0]), "v"(voffj[1]) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %1\n\t"
                 "global_load_lds_dwordx4 %3, %1 offset:1024"
                 :: "s"(lds_addr), "s"(sbase), "v"(voffj[0]), "v"(voffj[1]) : "memory", "m0");
}
template <bool ONCE>
__device__ __forceinline__ void dma16_vaddr(unsigned lds_addr, const void* vaddr) {
  if constexpr (ONCE)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(vaddr) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(vaddr) : "memory", "m0");
}
// A pointer that is the same in every lane, moved into a scalar register pair (64-bit address
// arithmetic with products is done on the vector ALU; everything derived from the result would
// otherwise stay there too)
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const T*>(((unsigned long long)hi << 32) | lo);
}
// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt fields left at "no wait")
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Compile-time shape constants shared by the helpers below (NST = stages of the K/V ring in LDS; NG = 4-wave
// groups of the workgroup, each of which has a key tile of its own in every stage)
template <int D, int NST = 2, int NG = 1> struct Shape {
  static constexpr int CPR = D / 8;                // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;             // rows covered by one wave-wide transfer
  static constexpr int IPT = 16 / RPI;             // transfers per wave per tile per tensor (a wave loads 16 rows)
  static constexpr int R256 = 16 / CPR;            // rows per 256 bytes of LDS
  static constexpr int NS = D / 32;                // 32-wide d slices (QK^T contraction steps)
  static constexpr int NDB = D / 16;               // 16-wide d blocks of the output
  static constexpr int ROWB = D * 2;               // bytes per row
  static constexpr int TILEB = kKeyTile * ROWB;    // bytes per tile per tensor
  static constexpr int STAGEB = NG * TILEB;        // bytes per ring stage per tensor
  // LDS: [K stage 0] .. [K stage NST-1][V stage 0] .. [V stage NST-1], a stage = the groups' tiles one after the
  // other; a stage offset plus any row offset of a tile fits the 16-bit immediate of a DS instruction, so a lane
  // needs one base register per d slice / d block and no address arithmetic inside the loop.
  static constexpr int VBASE = NST * STAGEB;
  static constexpr int LDS_BYTES = 2 * NST * STAGEB;
  static_assert(NST >= 2 && NST <= 4 && (NG == 1 || NG == 2), "ring stages, wave groups");
  static_assert((NST - 1) * STAGEB + kKeyTile * ROWB <= 65536, "stage offset as a DS immediate");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS of a CU");
};

// Per-lane constants of the K/V stream
template <int D> struct Lane {
  // byte offset of the lane's (swizzled) source chunk of transfer j within a tile, minus j KiB (see
  // dma_slab); entries past IPT unused
  unsigned kgj[4], vgj[4];
  unsigned kro[Shape<D>::NS], vro[Shape<D>::NDB];  // LDS read bases (bytes), before compile-time offsets
  unsigned lds_base; int wave, grp, lane, G;        // wave: index within its 4-wave group; grp: the group
};

typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;   // scalar (constant-cache) loads

// keep_idx values of the first and the last of the 16 rows a wave moves for one key tile, loaded one
// tile ahead (scalar loads that complete behind the tile being computed).  Indices are clamped, so
// asking for a tile past the end is harmless.
struct KeepAhead { int first, last; };

__device__ __forceinline__ void load_keep_ahead(const AttnArgs& a, int wave, int tile, KeepAhead& ka) {
  ka.first = 0; ka.last = 0;
  const int s0 = tile * kKeyTile + 16 * wave - a.P - a.K;
  if (a.n_keep > 0 && s0 >= 0) {                   // only slabs that start in the suffix use the bounds
    const const_i32_ptr keep_c = (const_i32_ptr)(uintptr_t)a.keep_idx;
    ka.first = keep_c[min(s0, a.n_keep - 1)];
    ka.last = keep_c[min(s0 + 15, a.n_keep - 1)];
  }
}

// Loop-invariant tile ranges of a wave's 16-row slab (rows 64 t + 16 w .. + 15 of key tile t): the slab
// lies wholly in the cache for t <= tc, wholly in the block for tb0 <= t <= tb1, wholly in the kept
// suffix for ts0 <= t <= ts1 (a range is empty when its bounds cross).
struct SlabRanges { int tc, tb0, tb1, ts0, ts1; };

__device__ __forceinline__ SlabRanges slab_ranges(const AttnArgs& a, int wave) {
  SlabRanges r;
  const int w16 = 16 * wave;                       // arithmetic shifts: floor division also below zero
  r.tc = (a.P - w16 - 16) >> 6;
  r.tb0 = (a.P - w16 + 63) >> 6;   r.tb1 = (a.P + a.K - w16 - 16) >> 6;
  r.ts0 = (a.P + a.K - w16 + 63) >> 6;   r.ts1 = (a.Nkv - w16 - 16) >> 6;
  return r;
}

// 16 consecutive rows of one source tensor starting at source row `row0`: scalar bases, the lane's
// constant offsets, no per-lane address arithmetic.  The lane offsets kgj / vgj count rows from the
// start of the tile, hence the step back by the wave's 16*wave rows.
template <int D, bool ONCE, int NST, int NG>
__device__ __forceinline__ void issue_slab(const Lane<D>& L, unsigned sk, const uint16_t* kp, const uint16_t* vp, long long row0) {
  using S = Shape<D, NST, NG>;
  const unsigned char* kt = reinterpret_cast<const unsigned char*>(kp) + (row0 - 16 * L.wave) * S::ROWB;
  const unsigned char* vt = reinterpret_cast<const unsigned char*>(vp) + (row0 - 16 * L.wave) * S::ROWB;
  static_assert(S::RPI * S::ROWB == 1024, "a transfer moves 1 KiB");
  dma_slab<S::IPT, ONCE>(sk, kt, L.kgj);
  dma_slab<S::IPT, ONCE>(sk + S::VBASE, vt, L.vgj);
}

// Puts key tile `tile` (a tile this wave's group moves) in flight into ring stage `stage` (the group's part of it
// when a stage holds NG tiles): 2 * IPT transfers per wave, which moves rows 16*wave .. 16*wave+15 of the tile.
// `ka` holds the keep_idx bounds of these rows on entry and those of the group's next tile (tile + STEP) on return.
template <int D, bool ONCE, int NST, int NG, int STEP>
__device__ __forceinline__ void issue_tile(const AttnArgs& a, const Lane<D>& L, const SlabRanges& R,
                                           const uint16_t* kc, const uint16_t* vc,
                                           const uint16_t* kb, const uint16_t* vb, const uint16_t* ks, const uint16_t* vs,
                                           int tile, int stage, KeepAhead& ka) {
  using S = Shape<D, NST, NG>;
  const unsigned sk = L.lds_base + stage * S::STAGEB + L.grp * S::TILEB + 16 * L.wave * S::ROWB;
  const unsigned sv = sk + S::VBASE;
  const int r0 = tile * kKeyTile + 16 * L.wave;    // uniform: first of the wave's 16 rows
  // Uniform classification of the wave's slab.  Sixteen consecutive rows of one source tensor (the
  // cache, the block, or a run of the suffix that keep_idx maps to consecutive rows: increasing
  // indices whose ends differ by 15) are one contiguous slab.
  if (tile <= R.tc) {
    issue_slab<D, ONCE, NST, NG>(L, sk, kc, vc, r0);
  } else if (tile >= R.tb0 && tile <= R.tb1) {
    issue_slab<D, ONCE, NST, NG>(L, sk, kb, vb, r0 - a.P);
  } else if (tile >= R.ts0 && tile <= R.ts1 && ka.last - ka.first == 15) {
    issue_slab<D, ONCE, NST, NG>(L, sk, ks, vs, ka.first);
  } else {
    // rows from more than one place, a gap in keep_idx, the ragged tail: per-row addresses without a
    // divergent branch.  keep_idx is read through the constant address space with uniform indices
    // (scalar loads: they do not touch the vector-memory counter that tracks the transfers in flight);
    // rows past the end repeat the last row (finite data; their scores are masked).
    int kidx[S::IPT];
#pragma unroll
    for (int j = 0; j < S::IPT; ++j) kidx[j] = 0;
    if (a.n_keep > 0) {
      const const_i32_ptr keep_c = (const_i32_ptr)(uintptr_t)a.keep_idx;
      // the lane's own row is picked with and/or masks (a select would let the compiler move each
      // load under a branch of its own and wait for them one by one)
      int pick[S::RPI];
#pragma unroll
      for (int q2 = 0; q2 < S::RPI; ++q2) pick[q2] = -(int)(L.lane / S::CPR == q2);
#pragma unroll
      for (int j = 0; j < S::IPT; ++j)
#pragma unroll
        for (int q2 = 0; q2 < S::RPI; ++q2) {
          const int si = min(max(r0 + S::RPI * j + q2 - a.P - a.K, 0), a.n_keep - 1);
          kidx[j] |= keep_c[si] & pick[q2];
        }
    }
    const unsigned char* kpp[S::IPT]; const unsigned char* vpp[S::IPT];
#pragma unroll
    for (int j = 0; j < S::IPT; ++j) {
      const int rl = S::RPI * j + L.lane / S::CPR;
      const int r = min(r0 + rl, a.Nkv - 1);
      const bool in_c = r < a.P, in_b = r < a.P + a.K;
      const uint16_t* kp = in_c ? kc : (in_b ? kb : ks);
      const uint16_t* vp = in_c ? vc : (in_b ? vb : vs);
      const long long off = (long long)(in_c ? r : (in_b ? r - a.P : kidx[j])) * D;
      kpp[j] = reinterpret_cast<const unsigned char*>(kp + off) + (L.kgj[j] + 1024 * j - (16 * L.wave + rl) * S::ROWB);
      vpp[j] = reinterpret_cast<const unsigned char*>(vp + off) + (L.vgj[j] + 1024 * j - (16 * L.wave + rl) * S::ROWB);
    }
#pragma unroll
    for (int j = 0; j < S::IPT; ++j) dma16_vaddr<ONCE>(sk + j * S::RPI * S::ROWB, kpp[j]);
#pragma unroll
    for (int j = 0; j < S::IPT; ++j) dma16_vaddr<ONCE>(sv + j * S::RPI * S::ROWB, vpp[j]);
  }
  load_keep_ahead(a, L.wave, tile + STEP, ka);
}

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

// V^T operand (16 d x 32 keys) of d block `db`, key half `u`, through two LDS transpose reads
template <int D, int STAGE, int NG>
__device__ __forceinline__ s16x8 read_vt(const unsigned char* lds, const Lane<D>& L, int db, int u) {
  using S = Shape<D, 2, NG>;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (lds_s16x4_ptr)(lds + L.vro[db] + STAGE * S::STAGEB + (32 * u) * S::ROWB));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (lds_s16x4_ptr)(lds + L.vro[db] + STAGE * S::STAGEB + (32 * u + 16) * S::ROWB));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// One key tile (ring stage STAGE, a compile-time constant so that every LDS address is base + immediate)
template <int D, int RB, int STAGE, int NG>
__device__ __forceinline__ void compute_tile(const AttnArgs& a, const Lane<D>& L, const unsigned char* lds, int t,
                                             const bf16x8 (&qreg)[RB][Shape<D>::NS], f32x4 (&o)[RB][Shape<D>::NDB],
                                             float (&m)[RB], float (&thr)[RB], float (&lsum)[RB]) {
  using S = Shape<D, 2, NG>;
  constexpr int NS = S::NS, NDB = S::NDB;
  constexpr bool kMfmaRowSum = (RB == 1);
  // the compiler's interleaving strategy for matrix instructions and LDS reads in this block (dense-suffix shape
  // 269 -> 263 us; the stream-bound shapes do not notice)
  __builtin_amdgcn_iglp_opt(0);
  // ---- S^T = K Q^T
  f32x4 sacc[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int kb4 = 0; kb4 < 4; ++kb4) sacc[rb][kb4] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kb4 = 0; kb4 < 4; ++kb4) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const bf16x8 kop = *reinterpret_cast<const bf16x8*>(lds + L.kro[s] + STAGE * S::STAGEB + kb4 * 16 * S::ROWB);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        sacc[rb][kb4] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qreg[rb][s], sacc[rb][kb4], 0, 0, 0);
    }
  }

  // ---- with 16 query rows per wave the V^T operands go in flight now: they do not depend on the
  // softmax, so their LDS latency hides behind it
  constexpr int NPRE = (RB == 1) ? 2 : 0;           // 32 rows per wave: no registers to spare for it
  s16x8 vpre[NPRE > 0 ? NPRE : 1][NDB];
#pragma unroll
  for (int u = 0; u < NPRE; ++u)
#pragma unroll
    for (int db = 0; db < NDB; ++db) vpre[u][db] = read_vt<D, STAGE, NG>(lds, L, db, u);

  // ---- online softmax (log2 domain: p = exp2(s * scale_log2 - m)); keys past Nkv only exist in the last tile
  const int key0 = t * kKeyTile;
  if (key0 + kKeyTile > a.Nkv) {                   // uniform branch
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int kb4 = 0; kb4 < 4; ++kb4)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (key0 + kb4 * 16 + 4 * L.G + i >= a.Nkv) sacc[rb][kb4][i] = kNegBigA;
  }
  s16x8 pk[RB][2];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float mx = fmaxf(fmaxf(sacc[rb][0][0], sacc[rb][0][1]), sacc[rb][0][2]);
    mx = fmaxf(fmaxf(mx, sacc[rb][0][3]), sacc[rb][1][0]);
    mx = fmaxf(fmaxf(mx, sacc[rb][1][1]), sacc[rb][1][2]);
    mx = fmaxf(fmaxf(mx, sacc[rb][1][3]), sacc[rb][2][0]);
    mx = fmaxf(fmaxf(mx, sacc[rb][2][1]), sacc[rb][2][2]);
    mx = fmaxf(fmaxf(mx, sacc[rb][2][3]), sacc[rb][3][0]);
    mx = fmaxf(fmaxf(mx, sacc[rb][3][1]), sacc[rb][3][2]);
    mx = fmaxf(mx, sacc[rb][3][3]);
    // Lazy reference: the row's reference exponent only moves when the new maximum exceeds it by
    // more than 8 (log2 units), so probabilities stay below 2^8 (exact in fp32 sums, same relative
    // precision in bf16) and the accumulator rescale below runs in a handful of tiles instead of
    // most of them.  The final O / l is unchanged: both carry the same reference.
    // A row's maximum exceeds the reference by 8 iff the in-lane maximum of one of its four lanes
    // does, so the common case needs no cross-lane reduction at all: one wave-wide test against
    // thr = (m + 8) / scale_log2 (kept beside m; a rounding-sized miss of the test only lets a
    // probability reach 2^8 (1 + eps), a spurious hit leaves m unchanged).
    if (__builtin_amdgcn_ballot_w64(mx > thr[rb]) != 0) {      // uniform branch
      // across the four 16-lane groups that hold the other keys of the same query row: VALU lane swaps
      const auto s16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = fmaxf(__uint_as_float(s16[0]), __uint_as_float(s16[1]));
      const auto s32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = fmaxf(__uint_as_float(s32[0]), __uint_as_float(s32[1]));
      const float cand = mx * a.scale_log2;
      const float m_up = (cand > m[rb] + 8.0f) ? cand : m[rb];
      const float corr = exp2_fast(m[rb] - m_up);  // 1 for the rows that stay
      lsum[rb] *= corr;
#pragma unroll
      for (int db = 0; db < NDB; ++db) o[rb][db] *= corr;
      m[rb] = m_up;
      thr[rb] = (m_up + 8.0f) * a.inv_scale_log2;
    }
    const float m_new = m[rb];
    float ps = 0.f;
#pragma unroll
    for (int kb4 = 0; kb4 < 4; ++kb4)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = exp2_fast(fmaf(sacc[rb][kb4][i], a.scale_log2, -m_new));
        sacc[rb][kb4][i] = p;
        if (!kMfmaRowSum) ps += p;
      }
    if (!kMfmaRowSum) lsum[rb] += ps;              // per-lane partial sum, reduced across lanes in the epilogue
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      union { uint32_t w[4]; s16x8 v; } cv;
      cv.w[0] = pack_bf16x2(sacc[rb][2 * u][0], sacc[rb][2 * u][1]);
      cv.w[1] = pack_bf16x2(sacc[rb][2 * u][2], sacc[rb][2 * u][3]);
      cv.w[2] = pack_bf16x2(sacc[rb][2 * u + 1][0], sacc[rb][2 * u + 1][1]);
      cv.w[3] = pack_bf16x2(sacc[rb][2 * u + 1][2], sacc[rb][2 * u + 1][3]);
      pk[rb][u] = cv.v;
    }
  }

  // ---- row sums on the matrix pipe (16 rows per wave; with 32 there are no registers to spare):
  // ones^T P^T adds the (bf16-rounded) probabilities of all 32 keys of a half tile for every query
  // row; each lane receives its row's complete sum
  if (kMfmaRowSum) {
    union { uint32_t w[4]; s16x8 v; } ones;
    ones.w[0] = ones.w[1] = ones.w[2] = ones.w[3] = 0x3f803f80u;   // bf16 1.0 pairs
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      f32x4 ls = {lsum[rb], 0.f, 0.f, 0.f};
#pragma unroll
      for (int u = 0; u < 2; ++u)
        ls = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ones.v),
                                                     __builtin_bit_cast(bf16x8, pk[rb][u]), ls, 0, 0, 0);
      lsum[rb] = ls[0];
    }
  }

  // ---- O^T += V^T P^T
#pragma unroll
  for (int u = 0; u < 2; ++u) {
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const s16x8 vop = (u < NPRE) ? vpre[u < NPRE ? u : 0][db] : read_vt<D, STAGE, NG>(lds, L, db, u);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        o[rb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vop),
                                                             __builtin_bit_cast(bf16x8, pk[rb][u]),
                                                             o[rb][db], 0, 0, 0);
    }
  }
}

// NST ring stages: NST - 1 tiles are in flight ahead of the one being computed.  Two stages (64 KiB for D = 128)
// let two workgroups share a CU, i.e. two tiles in flight per CU; a deeper ring keeps as many bytes in flight from
// a single workgroup.
// MODE 0: one group of 4 waves, wave w owns query rows 16 RB w .. of the workgroup's 64 RB rows.
// MODE 1: two groups of 4 waves own the SAME query rows and alternate key tiles of the split (group g takes tiles
//   t0 + g, t0 + g + 2, ...), each with its own part of every ring stage, and merge their (O, m, l) through LDS at
//   the end.  A launch that has one workgroup per CU then runs two waves per SIMD -- one wave's MFMA chain fills
//   the gaps of the other's softmax and LDS waits -- without a second split's partial results going through HBM.
//   Measured on 32 layers x 5248 keys x 128 rows with the transfers removed: the tile arithmetic alone takes 55 us
//   with one wave per SIMD, as long as the K/V stream alone (57 us).
// MODE 2: two groups of 4 waves own DIFFERENT query rows (128 RB per workgroup) and share every key tile; the
//   groups take turns moving tiles into the ring (group g moves tiles t0 + g, t0 + g + 2, ...).  Two waves per SIMD
//   from one workgroup, and a K/V tile is brought into LDS once per 128 RB query rows instead of once per 64 RB.
template <int D, int RB, bool ONCE, int NST, int MODE>
__global__ __launch_bounds__(MODE ? 512 : 256, MODE ? 1 : 2) void attn_bf16_kernel(AttnArgs a) {
  constexpr int NG = (MODE == 1) ? 2 : 1;          // key tiles per ring stage
  constexpr int STEP = MODE ? 2 : 1;               // distance between the tiles one group moves
  using S = Shape<D, NST, NG>;
  static_assert(MODE == 2 ? (NST == 2 || NST == 3) : NST == 2, "ring depths that are built");
  constexpr int CPR = S::CPR, RPI = S::RPI, IPT = S::IPT, R256 = S::R256, NS = S::NS, NDB = S::NDB, ROWB = S::ROWB;
  // LDS rows are unpadded (a transfer writes 1 KiB contiguous); bank conflicts are avoided by
  // storing chunk c of row r at position c ^ f(r):  f_K(r) = (r / R256) % CPR makes the 16 rows of
  // one b128 read phase hit 16 different positions, f_V(r) = 2 * ((r / R256) % (CPR/2)) does the
  // same for the 8 rows x 32 bytes of one transpose-read phase.
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

  // ---- which piece of work: workgroups that share K/V (query tiles of one unit) sit on one XCD
  const int xcd = blockIdx.x % kNumXCDs, slot = blockIdx.x / kNumXCDs;
  const int unit = (slot / a.q_tiles) * kNumXCDs + xcd;
  const int qt = slot % a.q_tiles;
  if (unit >= a.n_units) return;
  const int grp = unit / a.nsplit, split = unit - grp * a.nsplit;
  const int b = grp / a.Hkv, kvh = grp - b * a.Hkv;
  const int t0 = split * a.tiles_per_split;
  const int t1 = min(t0 + a.tiles_per_split, a.key_tiles);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_wg = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave = wave_wg & 3, wgrp = wave_wg >> 2;   // wave within its group, group within the workgroup
  const int l16 = lane & 15, G = lane >> 4;

  // The query rows of this wave (both groups of MODE 1 hold the same rows).  A kept suffix row needs its keep_idx
  // entry before its address is known: those entries are requested first of all, for every row block at once, so
  // that their round trip overlaps the set-up below.
  const int row_base = (MODE == 2) ? qt * (128 * RB) + wgrp * (64 * RB) + wave * (16 * RB)
                                   : qt * (64 * RB) + wave * (16 * RB);
  int q_hl[RB], q_qi[RB], q_keep[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int R = min(row_base + rb * 16 + l16, a.Rtot - 1);
    q_hl[rb] = R / a.Nq; q_qi[rb] = R - q_hl[rb] * a.Nq;
    q_keep[rb] = 0;
    if (q_qi[rb] >= a.K) q_keep[rb] = a.keep_idx[q_qi[rb] - a.K];
  }

  Lane<D> L;
  L.lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
  L.wave = wave; L.grp = (MODE == 1) ? wgrp : 0; L.lane = lane; L.G = G;
  const long long bh = (long long)b * a.Hkv + kvh;
  // base pointers of this (batch, KV head); kept as separate values (in a struct the compiler turns
  // the three-way source select of the gather path into a table lookup in scratch memory)
  const uint16_t* kc = uniform_ptr(a.k_cache + bh * a.cap * D);  const uint16_t* vc = uniform_ptr(a.v_cache + bh * a.cap * D);
  const uint16_t* kb = uniform_ptr(a.k_block + bh * a.K * D);    const uint16_t* vb = uniform_ptr(a.v_block + bh * a.K * D);
  const uint16_t* ks = uniform_ptr(a.k_suffix + bh * a.S * D);   const uint16_t* vs = uniform_ptr(a.v_suffix + bh * a.S * D);
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const int r = 16 * wave + RPI * j + lane / CPR, q = lane % CPR;
    // r * ROWB >= j KiB, so the offsets stay non-negative
    L.kgj[j] = r * ROWB + ((q ^ ((r / R256) % CPR)) << 4) - 1024 * j;
    L.vgj[j] = r * ROWB + ((q ^ (2 * ((r / R256) % (CPR / 2)))) << 4) - 1024 * j;
  }
#pragma unroll
  for (int j = IPT; j < 4; ++j) { L.kgj[j] = 0; L.vgj[j] = 0; }
  {
    const int fk = (D == 128) ? l16 : (l16 >> 1);
    const unsigned gofs = (unsigned)L.grp * S::TILEB; // the group's tile inside a stage
#pragma unroll
    for (int s2 = 0; s2 < NS; ++s2) L.kro[s2] = gofs + l16 * ROWB + (((4 * s2 + G) ^ fk) << 4);
    const int e4 = l16 >> 2, c4 = l16 & 3;
    const int fv = (D == 128) ? 2 * (4 * (G & 1) + e4) : 2 * (2 * (G & 1) + (e4 >> 1));
#pragma unroll
    for (int db = 0; db < NDB; ++db)
      L.vro[db] = gofs + S::VBASE + (4 * G + e4) * ROWB + (((2 * db + (c4 >> 1)) ^ fv) << 4) + ((c4 & 1) << 3);
  }

  // ---- query rows of this wave, as MFMA B operands (lane: row l16, d = 32*s + 8*G .. +7).  Requested BEFORE the
  // first K/V transfers: the wait for the keep_idx entries covers everything older in the vector-memory queue --
  // behind the first tile's transfers the query rows would only be requested once that tile had landed (two memory
  // round trips in a row instead of one short one and two in parallel).  All row blocks' addresses first, then all
  // loads, so that one block's loads do not wait for the other's.
  const uint16_t* qp[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const long long qbh = (long long)b * a.Hq + (long long)kvh * a.g + q_hl[rb];
    qp[rb] = (q_qi[rb] < a.K) ? a.q_block + (qbh * a.K + q_qi[rb]) * D
                              : a.q_suffix + (qbh * a.S + q_keep[rb]) * D;
  }
  bf16x8 qreg[RB][NS];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int s = 0; s < NS; ++s)
      qreg[rb][s] = *reinterpret_cast<const bf16x8*>(qp[rb] + 32 * s + 8 * G);

  // ---- the first NST - 1 steps' tiles go in flight
  const int tg0 = t0 + (MODE ? wgrp : 0);          // the tiles this wave's group moves: tg0, tg0 + STEP, ...
  const SlabRanges R = slab_ranges(a, wave);
  KeepAhead ka;
  load_keep_ahead(a, wave, tg0, ka);
  if constexpr (MODE == 2) {
#pragma unroll
    for (int j = 0; j < NST - 1; ++j)              // tile t0 + j belongs to group j & 1
      if ((j & 1) == wgrp && t0 + j < t1)
        issue_tile<D, ONCE, NST, NG, STEP>(a, L, R, kc, vc, kb, vb, ks, vs, t0 + j, j, ka);
  } else {
#pragma unroll
    for (int j = 0; j < NST - 1; ++j)
      if (tg0 + NG * j < t1) issue_tile<D, ONCE, NST, NG, STEP>(a, L, R, kc, vc, kb, vb, ks, vs, tg0 + NG * j, j, ka);
  }

  f32x4 o[RB][NDB];
  float m[RB], thr[RB], lsum[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m[rb] = kNegBigA; thr[rb] = kNegBigA; lsum[rb] = 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db) o[rb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // NST steps per trip so that the ring stage is a compile-time constant.  Per step: wait for the tile's transfers
  // (transfers complete in issue order; a wave never has a younger tile in flight when it waits, so the wait is
  // vmcnt(0)), barrier (every wave's part has landed and the previous step's tiles are consumed), put the next tile
  // in flight into the stage just freed, compute.  The query-row loads are complete after the first wait, so the
  // compiler places no vector-memory wait of its own inside the loop; in MODE 2 half of the waves skip that first
  // wait, so everything is completed once before the loop.
  if constexpr (MODE == 2) wait_vmcnt<0>();
  if constexpr (MODE == 2) {
    // step s works on tile t0 + s in stage s % NST; the tile was moved by group s & 1, whose waves have nothing
    // younger in flight when they wait for it (their next tile, t0 + s + 2, goes in flight during this step or later)
    auto tile_step = [&](auto stage_c, int t) {
      constexpr int STAGE = decltype(stage_c)::value;
      const int par = (t - t0) & 1;
      if (par == wgrp) wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      if (((par + NST - 1) & 1) == wgrp && t + NST - 1 < t1)
        issue_tile<D, ONCE, NST, NG, STEP>(a, L, R, kc, vc, kb, vb, ks, vs, t + NST - 1, (STAGE + NST - 1) % NST, ka);
      compute_tile<D, RB, STAGE, NG>(a, L, lds, t, qreg, o, m, thr, lsum);
    };
    for (int t = t0; t < t1; t += NST) {
      tile_step(std::integral_constant<int, 0>{}, t);
      if (t + 1 >= t1) break;
      tile_step(std::integral_constant<int, 1>{}, t + 1);
      if constexpr (NST >= 3) {
        if (t + 2 >= t1) break;
        tile_step(std::integral_constant<int, 2>{}, t + 2);
      }
    }
  } else {
    static_assert(NST == 2, "modes 0 and 1 are built with two ring stages");
    auto tile_step = [&](auto stage_c, int t) {    // t: this group's tile of the step
      constexpr int STAGE = decltype(stage_c)::value;
      wait_vmcnt<0>();                             // only this tile's transfers are in flight
      __builtin_amdgcn_s_barrier();
      if (t + NG < t1)
        issue_tile<D, ONCE, NST, NG, STEP>(a, L, R, kc, vc, kb, vb, ks, vs, t + NG, (STAGE + 1) % 2, ka);
      if (NG == 1 || t < t1) compute_tile<D, RB, STAGE, NG>(a, L, lds, t, qreg, o, m, thr, lsum);
    };
    // the trip count depends on the split only (t0, t1), not on the group: every wave meets every barrier
    for (int t = t0; t < t1; t += NG * NST) {
      tile_step(std::integral_constant<int, 0>{}, t + L.grp);
      if (t + NG >= t1) break;
      tile_step(std::integral_constant<int, 1>{}, t + NG + L.grp);
    }
  }

  // ---- two groups: the second hands its (O, m, l) to the first through LDS (the ring is free once every wave is
  // past its last tile); fixed order, so the result does not depend on timing
  if constexpr (MODE == 1) {
    constexpr int WAVE_O = RB * NDB * 64 * 16;     // bytes of one wave's accumulators, lane-contiguous 16-byte pieces
    static_assert(4 * (WAVE_O + RB * 64 * 8) <= S::LDS_BYTES, "exchange area fits the ring");
    __builtin_amdgcn_s_barrier();
    f32x4* xo = reinterpret_cast<f32x4*>(lds + wave * WAVE_O);
    float2* xml = reinterpret_cast<float2*>(lds + 4 * WAVE_O + wave * (RB * 64 * 8));
    if (wgrp == 1) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int db = 0; db < NDB; ++db) xo[(rb * NDB + db) * 64 + lane] = o[rb][db];
        xml[rb * 64 + lane] = make_float2(m[rb], lsum[rb]);
      }
    }
    __syncthreads();
    if (wgrp == 1) return;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float2 ml = xml[rb * 64 + lane];
      const float M = fmaxf(m[rb], ml.x);
      const float w0 = exp2_fast(m[rb] - M), w1 = exp2_fast(ml.x - M);
      lsum[rb] = lsum[rb] * w0 + ml.y * w1;
      m[rb] = M;
#pragma unroll
      for (int db = 0; db < NDB; ++db) o[rb][db] = o[rb][db] * w0 + xo[(rb * NDB + db) * 64 + lane] * w1;
    }
  }

  // ---- epilogue
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float l = lsum[rb];
    if (RB != 1) {                                 // per-lane partial sums (see compute_tile): reduce across the row's lanes
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
    }
    const int R = row_base + rb * 16 + l16;
    if (R >= a.Rtot) continue;
    if (a.nsplit == 1) {
      const float inv = 1.0f / l;
      uint16_t* orow = a.out + (((long long)b * a.Hq + (long long)kvh * a.g) * a.Nq + R) * D;
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        uint2 w;
        w.x = pack_bf16x2(o[rb][db][0] * inv, o[rb][db][1] * inv);
        w.y = pack_bf16x2(o[rb][db][2] * inv, o[rb][db][3] * inv);
        *reinterpret_cast<uint2*>(orow + 16 * db + 4 * G) = w;
      }
    } else {
      const long long slot_i = ((long long)grp * a.Rtot + R) * a.nsplit + split;
      float* wo = a.ws_o + slot_i * D;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
        *reinterpret_cast<f32x4*>(wo + 16 * db + 4 * G) = o[rb][db];
      if (G == 0) { a.ws_ml[slot_i * 2] = m[rb]; a.ws_ml[slot_i * 2 + 1] = l; }
    }
  }
}

// merge the key-range splits of every output row: fixed (index) order, fp32.  The loads of up to
// four splits are issued together so that a row costs about one memory round trip.
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a, long long total_rows) {
  constexpr int TPR = D / 4;                       // threads per row
  constexpr int RPB = 256 / TPR;                   // rows per workgroup
  const long long row = (long long)blockIdx.x * RPB + threadIdx.x / TPR;   // = grp * Rtot + R
  if (row >= total_rows) return;
  const int d = (threadIdx.x % TPR) * 4;
  const float* ml = a.ws_ml + row * a.nsplit * 2;
  const float* po = a.ws_o + row * a.nsplit * D + d;
  // the first four splits' loads go out together with their (max, sum) pairs: the common maximum needs only the
  // latter, so a row costs one memory round trip (more than four splits: the remaining maxima are read first)
  f32x4 ov[4]; float mk[4], lk[4];
  auto load_batch = [&](int k0) {                  // splits past the last one: weight 0 (uniform branches, no loads)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ov[u] = f32x4{0.f, 0.f, 0.f, 0.f}; mk[u] = kNegBigA; lk[u] = 0.f;
      if (k0 + u < a.nsplit) {
        const int k = k0 + u;
        ov[u] = *reinterpret_cast<const f32x4*>(po + (long long)k * D);
        mk[u] = ml[2 * k]; lk[u] = ml[2 * k + 1];
      }
    }
  };
  load_batch(0);
  float M = kNegBigA;
  for (int k = 4; k < a.nsplit; ++k) M = fmaxf(M, ml[2 * k]);
#pragma unroll
  for (int u = 0; u < 4; ++u) M = fmaxf(M, mk[u]);
  float L = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < a.nsplit; k0 += 4) {
    if (k0 > 0) load_batch(k0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float w = (k0 + u < a.nsplit) ? exp2_fast(mk[u] - M) : 0.f;
      L += w * lk[u];
      acc += ov[u] * w;
    }
  }
  const float inv = 1.0f / L;
  const long long grp = row / a.Rtot;
  const int R = (int)(row - grp * a.Rtot);
  const int b = (int)(grp / a.Hkv), kvh = (int)(grp - (long long)b * a.Hkv);
  uint16_t* orow = a.out + (((long long)b * a.Hq + (long long)kvh * a.g) * a.Nq + R) * D;
  uint2 w2;
  w2.x = pack_bf16x2(acc[0] * inv, acc[1] * inv);
  w2.y = pack_bf16x2(acc[2] * inv, acc[3] * inv);
  *reinterpret_cast<uint2*>(orow + d) = w2;
}

AttnPlan plan_attention_bf16(const sdllm_attn_params& p) {
  AttnPlan pl;
  const int g = p.Hq / p.Hkv;
  const long long Rtot = (long long)g * (p.K + p.n_keep);
  const long long Nkv = (long long)p.prefix_len + p.K + p.n_keep;
  // 32 query rows per wave (128 per workgroup) pay off only when many query rows share one K/V
  // stream (dense suffix); measured: 1024 rows -> 1.4x faster, 448 rows (GQA 7:1) -> 8 % slower
  pl.rb = Rtot >= 512 ? 2 : 1;
  // ... and when one 128-row tile then covers a K/V head with a long key stream: every K/V byte is read by
  // one workgroup only, which lets the transfers carry the nontemporal hint (32 layers x 5248 keys, 128 rows:
  // 2650 -> 2510 us per step; with 1312 keys the extra key splits it takes cost more than it gains)
  if (Rtot > 64 && Rtot <= 128 && Nkv >= 64 * kKeyTile) pl.rb = 2;
  // Many query tiles per K/V head: 8-wave workgroups whose two groups own 64 rb rows each and share every key tile
  // (mode 2) bring a tile into LDS half as often, with three ring stages (one such workgroup per CU).
  pl.mode = 0;
  pl.stages = 2;
  if (kShareTiles && Rtot >= kShareMinRows) { pl.mode = 2; pl.stages = kShareStages; }
  const int rows_wg = 64 * pl.rb * (pl.mode == 2 ? 2 : 1);
  pl.q_tiles = (int)((Rtot + rows_wg - 1) / rows_wg);
  pl.key_tiles = (int)((Nkv + kKeyTile - 1) / kKeyTile);
  const long long base = (long long)p.B * p.Hkv * pl.q_tiles;
  long long ns;
  if (p.kv_splits > 0) {
    ns = p.kv_splits;
  } else {
    // aim at two workgroups per CU (one when they are 128-row tiles: 32 layers x 5248 keys x 128 rows
    // measured 2402 us per step with 2 splits, 2480 with 4) ...
    ns = ((pl.rb == 2 ? 1LL : 2LL) * kNumCUs + base - 1) / base;
    // ... but keep a split long enough to amortise its merge: 16 key tiles once there is a workgroup
    // per CU without splitting, 8 with one per two CUs, 2 when the launch would otherwise leave most
    // of the chip idle (sweeps: 256 workgroups x 17 tiles -> 1 split, x 82 -> 2; 128 x 20 -> 2; 32 x 11 -> 4)
    const long long cap2 = pl.key_tiles / (base >= kNumCUs ? 16 : (base >= kNumCUs / 2 ? 8 : 2));
    if (ns > cap2) ns = cap2;
  }
  if (ns > pl.key_tiles) ns = pl.key_tiles;
  if (ns > 64) ns = 64;
  if (ns < 1) ns = 1;
  pl.tiles_per_split = (int)((pl.key_tiles + ns - 1) / ns);
  pl.kv_splits = (pl.key_tiles + pl.tiles_per_split - 1) / pl.tiles_per_split;   // no empty split
  const long long units = (long long)p.B * p.Hkv * pl.kv_splits;
  pl.workgroups = (int)(((units + kNumXCDs - 1) / kNumXCDs) * kNumXCDs * pl.q_tiles);
  // Two ring stages let two 4-wave workgroups share a CU (two tiles in flight per CU).  Where the launch has at most
  // one workgroup per CU anyway and a split is long enough, two 4-wave groups of one workgroup alternate its key
  // tiles instead (two waves per SIMD, the groups' partial results merged in LDS: mode 1).  (A deeper ring in the
  // 4-wave workgroup, three or four stages, measured no faster on any shape.)
  if (pl.mode == 0 && pl.workgroups <= kNumCUs && pl.tiles_per_split >= 4) pl.mode = 1;
  return pl;
}

size_t attention_bf16_workspace_bytes(const sdllm_attn_params& p, const AttnPlan& pl) {
  if (pl.kv_splits <= 1) return 0;
  const size_t rows = (size_t)p.B * p.Hq * (p.K + p.n_keep);
  return rows * pl.kv_splits * (size_t)(p.D + 2) * sizeof(float);
}

template <int D, int RB, bool ONCE, int NST, int MODE>
static hipError_t opt_in_main() {
  static LdsOptIn st;
  return ensure_lds_opt_in(reinterpret_cast<const void*>(&attn_bf16_kernel<D, RB, ONCE, NST, MODE>),
                           Shape<D, NST, MODE == 1 ? 2 : 1>::LDS_BYTES, st);
}

// launch == false: only the kernel's LDS opt-in on the current device (the preparation pass of sdllm_init)
template <int D, int RB, bool ONCE, int NST, int MODE>
static hipError_t launch_main(const AttnArgs& a, const AttnPlan& pl, hipStream_t stream, bool launch) {
  constexpr size_t lds_bytes = Shape<D, NST, MODE == 1 ? 2 : 1>::LDS_BYTES;
  hipError_t e = opt_in_main<D, RB, ONCE, NST, MODE>();
  if (e != hipSuccess || !launch) return e;
  hipLaunchKernelGGL((attn_bf16_kernel<D, RB, ONCE, NST, MODE>), dim3(pl.workgroups), dim3(MODE ? 512 : 256), lds_bytes,
                     stream, a);
  return hipGetLastError();
}

template <int D, int RB>
static hipError_t launch_rb(const AttnArgs& a, const AttnPlan& pl, hipStream_t stream, bool launch) {
  if (pl.mode == 2)           // row-split groups sharing the tiles (several query tiles per K/V head)
    return pl.stages == 3 ? launch_main<D, RB, false, 3, 2>(a, pl, stream, launch)
                          : launch_main<D, RB, false, 2, 2>(a, pl, stream, launch);
  // one query tile per K/V head (and split): every K/V byte is read by one workgroup only (nontemporal hint)
  if (pl.q_tiles == 1) {
    if (pl.mode == 1) return launch_main<D, RB, true, 2, 1>(a, pl, stream, launch);
    return launch_main<D, RB, true, 2, 0>(a, pl, stream, launch);
  }
  if (pl.mode == 1) return launch_main<D, RB, false, 2, 1>(a, pl, stream, launch);
  return launch_main<D, RB, false, 2, 0>(a, pl, stream, launch);
}

template <int D>
static hipError_t launch_d(const AttnArgs& a, const AttnPlan& pl, hipStream_t stream, bool launch = true) {
  return pl.rb == 2 ? launch_rb<D, 2>(a, pl, stream, launch) : launch_rb<D, 1>(a, pl, stream, launch);
}

hipError_t prepare_attention_bf16() {
  AttnArgs a{};
  AttnPlan pl{};
  hipError_t e = hipSuccess;
  for (int rb = 1; rb <= 2; ++rb)
    for (int q_tiles = 1; q_tiles <= 2; ++q_tiles)
      for (int mode = 0; mode <= 2; ++mode)
        for (int stages = 2; stages <= 3; ++stages) {
          if (mode != 2 && stages > 2) continue;
          if (mode == 2 && q_tiles == 1) continue;
          pl.rb = rb; pl.q_tiles = q_tiles; pl.stages = stages; pl.mode = mode;
          if (e == hipSuccess) e = launch_d<128>(a, pl, nullptr, false);
          if (e == hipSuccess) e = launch_d<64>(a, pl, nullptr, false);
        }
  return e;
}

hipError_t launch_attention_bf16(const sdllm_attn_params& p, const AttnPlan& pl,
                                 const void* q_block, const void* q_suffix,
                                 const void* k_cache, const void* v_cache,
                                 const void* k_block, const void* v_block,
                                 const void* k_suffix, const void* v_suffix,
                                 const int32_t* keep_idx, void* out, void* workspace, hipStream_t stream) {
  AttnArgs a;
  a.q_block = (const uint16_t*)q_block; a.q_suffix = (const uint16_t*)q_suffix;
  a.k_cache = (const uint16_t*)k_cache; a.v_cache = (const uint16_t*)v_cache;
  a.k_block = (const uint16_t*)k_block; a.v_block = (const uint16_t*)v_block;
  a.k_suffix = (const uint16_t*)k_suffix; a.v_suffix = (const uint16_t*)v_suffix;
  a.keep_idx = keep_idx; a.out = (uint16_t*)out;
  a.B = p.B; a.Hq = p.Hq; a.Hkv = p.Hkv; a.g = p.Hq / p.Hkv;
  a.P = p.prefix_len; a.cap = p.prefix_cap; a.K = p.K; a.S = p.S; a.n_keep = p.n_keep;
  a.Nq = p.K + p.n_keep; a.Nkv = p.prefix_len + p.K + p.n_keep; a.Rtot = a.g * a.Nq;
  a.nsplit = pl.kv_splits; a.tiles_per_split = pl.tiles_per_split; a.key_tiles = pl.key_tiles;
  a.q_tiles = pl.q_tiles; a.n_units = p.B * p.Hkv * pl.kv_splits;
  const float scale = p.scale > 0.f ? p.scale : 1.0f / sqrtf((float)p.D);
  a.scale_log2 = scale * kLog2eA;
  a.inv_scale_log2 = 1.0f / a.scale_log2;
  const size_t rows = (size_t)p.B * p.Hq * a.Nq;
  a.ws_o = (float*)workspace;
  a.ws_ml = a.ws_o ? a.ws_o + rows * pl.kv_splits * (size_t)p.D : nullptr;

  hipError_t e;
  e = p.D == 128 ? launch_d<128>(a, pl, stream) : launch_d<64>(a, pl, stream);
  if (e != hipSuccess) return e;
  if (pl.kv_splits > 1) {
    const long long total_rows = (long long)rows;
    if (p.D == 128) {
      const int rpb = 256 / (128 / 4);
      hipLaunchKernelGGL(attn_combine_kernel<128>, dim3((unsigned)((total_rows + rpb - 1) / rpb)), dim3(256), 0, stream, a, total_rows);
    } else {
      const int rpb = 256 / (64 / 4);
      hipLaunchKernelGGL(attn_combine_kernel<64>, dim3((unsigned)((total_rows + rpb - 1) / rpb)), dim3(256), 0, stream, a, total_rows);
    }
    e = hipGetLastError();
  }
  return e;
}

}  // namespace sdllm
