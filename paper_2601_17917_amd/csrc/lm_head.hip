// Vocabulary projection fused into the confidence-aware unmask (paper Eq. 3 -> Eq. 4): the logits
// z_i = W h_i of the masked positions are formed tile by tile on the matrix cores and reduced to
// (max, sum of exp, lowest argmax id) triples in registers; they are never written to memory.
// The triples go to the same commit kernel as those of the streaming reduction over stored logits.
//
// One workgroup = one vocabulary tile (BN rows of W) x one chunk of BM masked rows, the whole of Hd.
//   * Masked rows are compacted inside the kernel (every workgroup scans the mask bytes), so the
//     matrix cores only see rows that Eq. 4 asks for; a chunk beyond the masked count exits at once.
//   * W is the streamed operand and has no reuse inside a workgroup: every wave owns WNB x 16
//     vocabulary rows and loads its MFMA A operands straight from global memory into registers
//     (16 bytes per lane = the operand layout itself), PF k-steps ahead; W never touches LDS.
//   * The hidden rows are the shared operand: chunks of KC elements per row go through an LDS ring
//     (registers -> LDS ahead of use, one barrier per chunk), XOR-swizzled so that the 16-byte
//     B-operand reads are bank-conflict free.
//   * logits^T tile = W_tile h^T (v_mfma_f32_16x16x32_bf16, fp32 accumulate): a lane ends up with
//     vocabulary ids 4 (lane / 16) + r of row lane % 16, so the row reduction is in-lane first, then two
//     lane exchanges, then across the four waves through LDS.
//   * Row chunks of one vocabulary tile get workgroup ids that are equal mod 8 and adjacent in
//     dispatch order: same XCD, same L2, so W comes from HBM once.
//   * Shapes: with 256 rows per chunk (more than 128 masked positions) lm_head_rows_kernel is bound by
//     the matrix pipe (one wave per SIMD, accumulators in the accumulation registers, B operands through
//     a register ring fed across chunk boundaries).  Calls with at most 128 masked positions are a read
//     of W and take the stream kernels further down, which turn the roles around: the hidden operands
//     stay in registers and W goes through LDS (1 KB row pieces through registers up to 64 positions,
//     global -> LDS transfers up to 128), or, when W is the packed image, comes straight from it.
//   * The masked count is device data: the host launches every shape that B x K admits and each launch
//     exits unless the count is in its range.
#include "common.h"
#include "unmask_common.h"
#include <climits>
#include <type_traits>

namespace sdllm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kLmThreads = 256;
constexpr int kLmWaves = kLmThreads / 64;
constexpr int kLmStageBytes = 32768;      // one LDS stage of hidden rows

struct LmHeadArgs {
  const uint16_t* hidden;     // [rows_total][ld_h]
  const uint16_t* weight;     // [V][ld_w], or the packed image [ceil(V/16)][Hd/32][64 lanes][8] (packed != 0)
  const uint8_t* masked;      // [rows_total]
  Partial* partials;          // [rows_total][ntile]
  long long ld_h, ld_w;       // elements
  int rows_total, V, Hd;
  int ntile;                  // vocabulary tiles
  int nchunk;                 // row chunks in the grid (upper bound of ceil(masked rows / BM))
  // The masked count is device data, the shape that suits it is not known to the host: a call launches every
  // shape its B x K admits and each launch exits at once unless min_masked <= masked count <= max_masked.
  int min_masked, max_masked;
  // a position's triples are [ntile_out] (the largest tile count among the call's launches); the launch that
  // runs writes its ntile of them and neutral triples into the rest (slot tile + j ntile from workgroup tile)
  int ntile_out;
  int packed;                 // weight is the packed image: the A operand of 16-row block nb and k-step ks is
                              // the kilobyte at ((nb * Hd/32 + ks) * 64 + lane) * 8 elements
};

__device__ __forceinline__ void store_partial(const LmHeadArgs& a, int row, int tile, const Partial& p) {
  Partial* out = a.partials + (long long)row * a.ntile_out;
  out[tile] = p;
  for (int j = tile + a.ntile; j < a.ntile_out; j += a.ntile) out[j] = Partial{kNegBig, 0.f, 0x7fffffff};
}

// Number of masked positions of the call (uniform over the workgroup): one pass over the mask bytes without
// barriers, then one reduction.  wsum: kLmWaves ints of LDS, free for other use on return.
__device__ __forceinline__ int lm_masked_count(const LmHeadArgs& a, int* wsum) {
  const int tid = threadIdx.x;
  int mine = 0;
  for (int i = tid; i < a.rows_total; i += kLmThreads) mine += a.masked[i] != 0;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) mine += __shfl_xor(mine, off);
  if ((tid & 63) == 0) wsum[tid >> 6] = mine;
  __syncthreads();
  int total = 0;
#pragma unroll
  for (int w = 0; w < kLmWaves; ++w) total += wsum[w];
  __syncthreads();
  return total;
}


template <int BM, int WNB, int PF_>
struct LmShape {
  static constexpr int JB = BM / 16;                        // 16-row blocks (B operands) per chunk
  static constexpr int BN = kLmWaves * WNB * 16;            // vocabulary rows per workgroup
  static constexpr int KC = kLmStageBytes / 2 / BM;         // hidden elements per row and stage
  static constexpr int KSTEPS = KC / 32;                    // MFMA k-steps per stage
  static constexpr int PIECES = KC / 8;                     // 16-byte pieces per LDS row
  static constexpr int PF = PF_;                            // k-steps of W in flight per wave
  static constexpr int U = PF > KSTEPS ? PF / KSTEPS : 1;   // chunks per unrolled loop body (static ring slots)
  static constexpr int ROWS_PER_PASS = kLmThreads / PIECES; // rows one staging pass of the workgroup covers
  static constexpr int NPASS = BM / ROWS_PER_PASS;          // 16-byte staging loads per thread and chunk
  static constexpr int MIN_WAVES = BM <= 64 ? 2 : 1;        // waves per SIMD the register budget must allow
  // The wide shapes are bound by the matrix pipe with one wave per SIMD.  Their 128 / 256 accumulator
  // registers sit in the accumulation half of the register file by construction (left to the register
  // allocator they were shuffled between the halves inside the loop, or spilled), and their B operands
  // run through a register ring DB deep that is fed across chunk boundaries, which takes a third LDS
  // stage (a chunk is complete one barrier before it is first read).
  static constexpr bool WIDE = BM >= 128;
  static constexpr int NST = WIDE ? 3 : 2;
  static constexpr int DB = 4;
  static constexpr int HDEPTH = KSTEPS >= 4 ? 1 : 4 / KSTEPS;   // chunks a hidden chunk waits in registers (wide)
  static_assert((PIECES == 8 || PIECES % 16 == 0) && kLmThreads % PIECES == 0, "shape");
  static_assert((KSTEPS * U) % PF == 0 && (U == 1 || U % 2 == 0) && (!WIDE || U % HDEPTH == 0), "ring");
  // LDS rows are unpadded; piece p of row r sits at slot swz(r, p), chosen so that the 16 lanes of a
  // B-operand read (rows r..r+15, same piece) fall into 16 different 16-byte bank groups
  __device__ static __forceinline__ int swz(int r, int p) {
    return PIECES == 8 ? (p ^ ((r >> 1) & 7)) : (p ^ (r & 15));
  }
};

template <bool NT = false>
__device__ __forceinline__ bf16x8 load_w(const uint16_t* p) {
  if constexpr (NT) return __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
  else return *reinterpret_cast<const bf16x8*>(p);
}

// acc += A B, with the accumulator either left to the compiler or pinned to the accumulation registers
template <bool ACC_IN_AGPR>
__device__ __forceinline__ void mfma_acc(f32x4& acc, const bf16x8& a, const bf16x8& b) {
  if constexpr (ACC_IN_AGPR) asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
  else acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
}

// PACKED: W is the packed image (a lane's operand pieces of consecutive k-steps are 1 KB apart, a wave's load is
// one contiguous kilobyte that no other load touches: nontemporal)
template <int BM, int WNB, int PF_, bool PACKED>
__global__ __launch_bounds__(kLmThreads, (LmShape<BM, WNB, PF_>::MIN_WAVES)) void lm_head_rows_kernel(LmHeadArgs a) {
  using S = LmShape<BM, WNB, PF_>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  unsigned char* stage = lds_raw;                                          // NST x kLmStageBytes
  int* row_of = reinterpret_cast<int*>(lds_raw + S::NST * kLmStageBytes);  // BM compacted row ids (-1 = none)
  Partial* red = reinterpret_cast<Partial*>(row_of + BM);                  // [waves][BM]
  __shared__ int wsum[kLmWaves];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // ---- the masked count decides how many row chunks there are
  const int total = lm_masked_count(a, wsum);
  if (total < max(a.min_masked, 1)) return;        // another shape's launch has this call, or nothing is masked
  const int nact = (total + BM - 1) / BM;          // <= a.nchunk, since total <= rows_total
  // ---- workgroup -> (vocabulary tile, row chunk): chunks of a tile share id mod 8 (the XCD) and are adjacent
  // in dispatch order.  Only chunks that hold rows get workgroup ids: the idle workgroups of a grid sized for
  // B x K rows are its last ones (interleaved with the working ones they kept half of the chip idle: 256 of
  // 512 positions masked took 497 us, not the 320 us of 256 of 256).
  const int slot = blockIdx.x >> 3;
  const int tile = (slot / nact) * kNumXCDs + (blockIdx.x & 7);
  const int chunk = slot % nact;
  if (tile >= a.ntile) return;

  // ---- compact the masked rows; this workgroup takes compacted rows [lo, lo + BM)
  const int lo = chunk * BM;
  int running = 0;
  for (int base = 0; base < a.rows_total; base += kLmThreads) {
    const int i = base + tid;
    const bool f = i < a.rows_total && a.masked[i] != 0;
    const unsigned long long bal = __ballot(f);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[wave] = __popcll(bal);
    __syncthreads();
    int pre = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kLmWaves; ++w) { const int c = wsum[w]; pre += (w < wave) ? c : 0; tot += c; }
    const int ci = running + pre + rank - lo;
    if (f && ci >= 0 && ci < BM) row_of[ci] = i;
    running += tot;
    __syncthreads();
    if (running >= lo + BM) break;                 // uniform: the chunk is full
  }
  const int n_valid = min(running - lo, BM);       // uniform, >= 1 because chunk < nact
  if (tid < BM && tid >= n_valid) row_of[tid] = -1;
  __syncthreads();

  // ---- operand addressing
  const int NK = a.Hd / 32;                                    // k-steps
  const int NCH = (NK + S::KSTEPS - 1) / S::KSTEPS;            // LDS chunks
  const int q = lane >> 4, l16 = lane & 15;
  // every workgroup walks the chunks of Hd in its own rotation, so that the workgroups resident at one
  // time do not all ask for the same columns of W at once
  const int c0 = tile % NCH;
  auto kstep_at = [&](int t) {                                 // k-step at position t of this workgroup's walk
    const int cc = t / S::KSTEPS, ss = t - cc * S::KSTEPS;
    const int ch = (cc + c0) % NCH;
    return min(ch * S::KSTEPS + ss, NK - 1);
  };
  auto chunk_at = [&](int c) { int ch = c + c0; ch -= (ch >= NCH) ? NCH : 0; return ch; };   // c < NCH
  const uint16_t* wrow[WNB];                                   // this lane's operand piece of k-step 0
  constexpr int wks = PACKED ? 512 : 32;                       // elements from one k-step's piece to the next
#pragma unroll
  for (int ib = 0; ib < WNB; ++ib) {
    if constexpr (PACKED) {
      const int nb = min(tile * (S::BN / 16) + wave * WNB + ib, (a.V + 15) / 16 - 1);   // blocks past V: the last one
      wrow[ib] = a.weight + ((long long)nb * NK * 64 + lane) * 8;
    } else {
      const int n = min(tile * S::BN + (wave * WNB + ib) * 16 + l16, a.V - 1);   // rows past V: any valid row
      wrow[ib] = a.weight + (long long)n * a.ld_w + 8 * q;
    }
  }
  // staging: this thread moves piece `pc` of rows srow0 + ROWS_PER_PASS * i
  const int pc = tid % S::PIECES, srow0 = tid / S::PIECES;
  unsigned hoff[S::NPASS];       // element offset of the thread's rows
  unsigned soff[S::NPASS];       // byte offset inside a stage
#pragma unroll
  for (int i = 0; i < S::NPASS; ++i) {
    const int r = srow0 + S::ROWS_PER_PASS * i;
    hoff[i] = (unsigned)((long long)max(row_of[r], 0) * a.ld_h);
    soff[i] = (unsigned)(r * S::KC * 2 + (S::swz(r, pc) << 4));
  }
  // B-operand read of 16-row block jb, k-step ks: row jb * 16 + l16, piece 4 ks + q
  const unsigned boff = (unsigned)(l16 * S::KC * 2);

  f32x4 acc[WNB][S::JB];
#pragma unroll
  for (int ib = 0; ib < WNB; ++ib)
#pragma unroll
    for (int jb = 0; jb < S::JB; ++jb) acc[ib][jb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- prologue: first W k-steps in flight, first hidden chunk(s) into LDS
  bf16x8 abuf[S::PF][WNB];
#pragma unroll
  for (int s = 0; s < S::PF; ++s)
#pragma unroll
    for (int ib = 0; ib < WNB; ++ib) abuf[s][ib] = load_w<PACKED>(wrow[ib] + wks * kstep_at(s));
  // A chunk's pieces past Hd are staged as zeros and its k-steps past Hd are computed like the others
  // (finite W times zero adds nothing): the loop body has no branch, so the compiler's wait counters
  // see one straight line and keep the W loads PF steps ahead.
  const unsigned klast = (unsigned)(a.Hd - 8);          // last whole piece of a row
  auto stage_now = [&](int c, unsigned char* dst) {     // chunk at walk position c straight into LDS
    const unsigned k = (unsigned)(chunk_at(c < NCH ? c : 0) * S::KC) + 8u * pc;
    const bool keep = c < NCH && k < (unsigned)a.Hd;
#pragma unroll
    for (int i = 0; i < S::NPASS; ++i) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(a.hidden + (hoff[i] + min(k, klast)));
      *reinterpret_cast<u32x4*>(dst + soff[i]) = keep ? v : u32x4{0u, 0u, 0u, 0u};
    }
  };
  stage_now(0, stage);
  static_assert(S::WIDE, "only the 256-row shape is built: fewer positions take the stream kernels");
  stage_now(1, stage + kLmStageBytes);
  __syncthreads();

  const int NCHU = (NCH + S::U - 1) / S::U * S::U;      // chunks past NCH see zeros
  if constexpr (S::WIDE) {
    // ---- main loop, wide shapes: three LDS stages (read c, already complete c + 1, being written c + 2)
    constexpr int CH = S::KSTEPS * S::JB;               // B operands per chunk
    static_assert(CH % S::DB == 0, "B ring");
    unsigned pv[S::KSTEPS];                             // per-lane part of a B-operand address, by k-step
#pragma unroll
    for (int ks = 0; ks < S::KSTEPS; ++ks) pv[ks] = boff + (unsigned)(S::swz(l16, 4 * ks + q) << 4);
    auto read_b = [&](unsigned st_off, int ks, int jb) {
      return *reinterpret_cast<const bf16x8*>(stage + st_off + pv[ks] + jb * 16 * S::KC * 2);
    };
    unsigned cur_off = 0, nxt_off = kLmStageBytes, wr_off = 2 * kLmStageBytes;    // uniform
    bf16x8 bq[S::DB];
#pragma unroll
    for (int d = 0; d < S::DB; ++d) bq[d] = read_b(cur_off, d / S::JB, d % S::JB);
    // Loads return in issue order, so waiting for a young load also waits for every older one: a hidden
    // chunk that is consumed at the end of the chunk it was asked for in would drain the W ring down to
    // the loads of that chunk, however far ahead the ring runs.  The hidden chunks therefore travel HD
    // chunks ahead in registers, so that nothing younger than about PF k-steps is ever waited for.
    constexpr int HD = S::HDEPTH;                       // chunks a hidden chunk waits in registers
    u32x4 hreg[HD][S::NPASS];
    auto load_hidden = [&](int c, u32x4 (&dst)[S::NPASS]) {      // chunk at walk position c (zeros past the end)
      const unsigned k = (unsigned)(chunk_at(c < NCH ? c : 0) * S::KC) + 8u * pc;
      const unsigned kc = min(k, klast);
#pragma unroll
      for (int i = 0; i < S::NPASS; ++i) dst[i] = *reinterpret_cast<const u32x4*>(a.hidden + (hoff[i] + kc));
    };
    auto keep_mask = [&](int c) -> unsigned {
      const unsigned k = (unsigned)(chunk_at(c < NCH ? c : 0) * S::KC) + 8u * pc;
      return (c < NCH && k < (unsigned)a.Hd) ? 0xffffffffu : 0u;
    };
#pragma unroll
    for (int d = 1; d < HD; ++d) load_hidden(1 + d, hreg[d % HD]);     // chunks 2 .. HD: as if asked for earlier
    for (int cb = 0; cb < NCHU; cb += S::U) {
#pragma unroll
      for (int uu = 0; uu < S::U; ++uu) {
        const int c = cb + uu;
        // asked for now: chunk c + 1 + HD; written to LDS at the end of this chunk: chunk c + 2
        load_hidden(c + 1 + HD, hreg[uu % HD]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < S::KSTEPS; ++ks) {
          const int g = c * S::KSTEPS + ks;
          const int slot_a = (uu * S::KSTEPS + ks) % S::PF;
          bf16x8 aop[WNB];
#pragma unroll
          for (int ib = 0; ib < WNB; ++ib) aop[ib] = abuf[slot_a][ib];
#pragma unroll
          for (int ib = 0; ib < WNB; ++ib) abuf[slot_a][ib] = load_w<PACKED>(wrow[ib] + wks * kstep_at(g + S::PF));
#pragma unroll
          for (int jb = 0; jb < S::JB; ++jb) {
            const int t = ks * S::JB + jb, tn = t + S::DB;
            const bf16x8 bop = bq[t % S::DB];
            bq[t % S::DB] = tn < CH ? read_b(cur_off, tn / S::JB, tn % S::JB)
                                    : read_b(nxt_off, (tn - CH) / S::JB, (tn - CH) % S::JB);
#pragma unroll
            for (int ib = 0; ib < WNB; ++ib) mfma_acc<true>(acc[ib][jb], aop[ib], bop);
            __builtin_amdgcn_sched_barrier(0);          // keep the ring's distance as written
          }
        }
        // chunk c + 2 (asked for HD - 1 chunks ago) into the free stage.  Pieces past Hd become zeros by
        // masking, not by a select: a select would let the compiler turn the loads into conditional ones
        // and sink them down here
        const unsigned keep = keep_mask(c + 2);
#pragma unroll
        for (int i = 0; i < S::NPASS; ++i)
          *reinterpret_cast<u32x4*>(stage + wr_off + soff[i]) = hreg[(uu + 1) % HD][i] & u32x4{keep, keep, keep, keep};
        __syncthreads();
        const unsigned tmp = cur_off; cur_off = nxt_off; nxt_off = wr_off; wr_off = tmp;
      }
    }
    // the accumulators written by the last matrix instructions are read by vector instructions next; the
    // compiler does not see an MFMA inside the asm statement, so the required wait states are spelled out
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  }

  // ---- row reduction of the tile: in-lane over this lane's vocabulary ids (ascending), then over the
  // four lane groups, then over the waves
#pragma unroll
  for (int jb = 0; jb < S::JB; ++jb) {
    float m = kNegBig; int idx = 0x7fffffff;
#pragma unroll
    for (int ib = 0; ib < WNB; ++ib)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int n = tile * S::BN + (wave * WNB + ib) * 16 + 4 * q + r;
        float v = acc[ib][jb][r];
        if (n >= a.V) v = -INFINITY;
        acc[ib][jb][r] = v;
        if (v > m) { m = v; idx = n; }               // strict: the lowest id keeps a tie
      }
    const float ml = m * kLog2e;
    float s = 0.f;
#pragma unroll
    for (int ib = 0; ib < WNB; ++ib)
#pragma unroll
      for (int r = 0; r < 4; ++r) s += fast_exp2(fmaf(acc[ib][jb][r], kLog2e, -ml));
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float m2 = __shfl_xor(m, off); const float s2 = __shfl_xor(s, off); const int i2 = __shfl_xor(idx, off);
      merge_partial(m, s, idx, m2, s2, i2);
    }
    if (q == 0) red[wave * BM + jb * 16 + l16] = Partial{m, s, idx};
  }
  __syncthreads();
  if (tid < BM && row_of[tid] >= 0) {
    Partial p = red[tid];
#pragma unroll
    for (int w = 1; w < kLmWaves; ++w) {
      const Partial p2 = red[w * BM + tid];
      merge_partial(p.m, p.s, p.idx, p2.m, p2.s, p2.idx);
    }
    store_partial(a, row_of[tid], tile, p);
  }
}


// ---------------------------------------------------------------------------------------------------
// Stream shape (at most 32 positions in the block): the call is a read of W, so the kernel is built around
// that stream.  A workgroup owns 32 TT consecutive vocabulary rows (TT = 16: 512) and walks Hd in chunks of 512
// elements; within a chunk it visits its 16 sub-tiles of 32 rows one after the other, so that every
// wave-wide load is ONE KILOBYTE OF ONE ROW of W (registers -> LDS, swizzled, two stages, one barrier per
// sub-tile), and the matrix instructions read W back from LDS in operand layout.  The hidden rows never
// touch LDS: wave (ib, jb) computes vocabulary block ib x row block jb of every sub-tile, its B operands of
// a chunk (16 k-steps) sit in registers for all 16 sub-tiles and the next chunk's are asked for two
// sub-tiles ahead.  All 16 x (16 x 16) accumulators of a wave stay in registers until the end: one triple
// per (position, 512 vocabulary rows), a quarter of what the 128-row tiles of the other shapes write.
constexpr int kStSub = 32;                 // vocabulary rows per sub-tile
constexpr int kStTTMax = 20;               // most sub-tiles per workgroup: the accumulators a wave can hold
constexpr int kSt2TTMax = 16;              // the same with two row blocks per wave (33..64 positions)
constexpr int kStKC = 512;                 // elements of Hd per chunk (1 KB per row)
constexpr int kStKS = kStKC / 32;          // k-steps per chunk
constexpr int kStStage = kStSub * kStKC * 2;   // 32 KB

template <int TT>   // sub-tiles per workgroup (even: the two W stages alternate across chunk boundaries)
__global__ __launch_bounds__(kLmThreads) void lm_head_stream_kernel(LmHeadArgs a) {
  static_assert(TT % 2 == 0 && TT >= 2 && TT <= kStTTMax, "sub-tiles per workgroup");
  constexpr int kStTT = TT, kStRows = TT * kStSub;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  unsigned char* stage = lds_raw;                                            // 2 x kStStage
  int* row_of = reinterpret_cast<int*>(lds_raw + 2 * kStStage);              // 32 compacted row ids (-1 = none)
  Partial* red = reinterpret_cast<Partial*>(row_of + 32);                    // [waves][16]
  __shared__ int wsum[kLmWaves];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = blockIdx.x;                                               // < a.ntile by the grid size

  // ---- this launch works only if the masked count is in its range (another shape's launch has the call
  // otherwise); then the masked rows are compacted
  {
    const int total = lm_masked_count(a, wsum);
    if (total < a.min_masked || total > a.max_masked) return;
  }
  int running = 0;
  for (int base = 0; base < a.rows_total; base += kLmThreads) {
    const int i = base + tid;
    const bool f = i < a.rows_total && a.masked[i] != 0;
    const unsigned long long bal = __ballot(f);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[wave] = __popcll(bal);
    __syncthreads();
    int pre = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kLmWaves; ++w) { const int c = wsum[w]; pre += (w < wave) ? c : 0; tot += c; }
    const int ci = running + pre + rank;
    if (f && ci < 32) row_of[ci] = i;
    running += tot;
    __syncthreads();
  }
  const int n_valid = min(running, 32);            // uniform
  if (n_valid <= 0) return;
  if (tid < 32 && tid >= n_valid) row_of[tid] = -1;
  __syncthreads();

  const int NCH = (a.Hd + kStKC - 1) / kStKC;      // chunks of Hd
  const int NU = NCH * kStTT;                      // (chunk, sub-tile) steps of the walk
  const int c0 = tile % NCH;                       // this workgroup's rotation of the chunk order
  const int q = lane >> 4, l16 = lane & 15;
  const int ib = wave & 1, jb = wave >> 1;
  const unsigned klast = (unsigned)(a.Hd - 8);     // last whole 16-byte piece of a row

  // W staging: this wave moves rows 8 wave + i (i = 0..7) of a sub-tile, lane l the l-th 16 bytes of the chunk
  const long long vrow0 = (long long)tile * kStRows + 8 * wave;
  unsigned sdst[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = 8 * wave + i;
    sdst[i] = (unsigned)(r * (kStKC * 2) + ((lane ^ (r & 15)) << 4));
  }
  auto load_w_sub = [&](int u, u32x4 (&dst)[8]) {          // step u of the walk (clamped to the last one)
    const int uc = min(u, NU - 1);
    const int kc = uc / kStTT, t = uc - kc * kStTT;
    int kcw = kc + c0; kcw -= (kcw >= NCH) ? NCH : 0;
    const unsigned k = min((unsigned)(kcw * kStKC + 8 * lane), klast);     // pieces past Hd: any valid piece
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const long long n = min(vrow0 + t * kStSub + i, (long long)a.V - 1);   // rows past V: any valid row
      // every byte of W is read once and whole lines at a time here: streaming loads (cfg2: 182 -> 172 us)
      dst[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a.weight + n * a.ld_w + k));
    }
  };
  // B operands of a chunk for this wave's row block: row jb * 16 + l16, k-step ks, elements 8 q .. 8 q + 7
  const long long hrow = (long long)max(row_of[jb * 16 + l16], 0) * a.ld_h;
  auto load_b_chunk = [&](int kc, bf16x8 (&dst)[kStKS]) {  // chunk at walk position kc (clamped); zeros past Hd
    int kcw = min(kc, NCH - 1) + c0; kcw -= (kcw >= NCH) ? NCH : 0;
#pragma unroll
    for (int ks = 0; ks < kStKS; ++ks) {
      const unsigned k = (unsigned)(kcw * kStKC + 32 * ks + 8 * q);
      const unsigned keep = (k < (unsigned)a.Hd) ? 0xffffffffu : 0u;
      const u32x4 v = *reinterpret_cast<const u32x4*>(a.hidden + hrow + min(k, klast));
      dst[ks] = __builtin_bit_cast(bf16x8, v & u32x4{keep, keep, keep, keep});
    }
  };
  // A operand of k-step ks: row ib * 16 + l16 of the sub-tile, piece 4 ks + q, swizzled by the row
  const unsigned aoff = (unsigned)((ib * 16 + l16) * (kStKC * 2));

  f32x4 acc[kStTT];
#pragma unroll
  for (int t = 0; t < kStTT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- prologue: step 0 into stage 0, step 1 into registers, the first chunk's B operands
  u32x4 wreg[2][8];
  load_w_sub(0, wreg[0]);
  load_w_sub(1, wreg[1]);
  bf16x8 bcur[kStKS], bnext[kStKS];
  load_b_chunk(0, bcur);
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(stage + sdst[i]) = wreg[0][i];
  __syncthreads();

  // ---- main loop: chunks of Hd (rotated), 16 sub-tiles each; step u = kc * 16 + t reads stage u & 1
  for (int kc = 0; kc < NCH; ++kc) {
#pragma unroll
    for (int t = 0; t < kStTT; ++t) {
      const int u = kc * kStTT + t;
      // two steps ahead into the register set that was written to LDS one step ago
      load_w_sub(u + 2, wreg[t & 1]);
      if (t == kStTT - 2) load_b_chunk(kc + 1, bnext);
      __builtin_amdgcn_sched_barrier(0);
      const unsigned char* cur = stage + (t & 1) * kStStage;
#pragma unroll
      for (int ks = 0; ks < kStKS; ++ks) {
        const bf16x8 aop = *reinterpret_cast<const bf16x8*>(cur + aoff + (unsigned)(((4 * ks + q) ^ l16) << 4));
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bcur[ks], acc[t], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      // step u + 1 (asked for one step ago) into the other stage, which step u - 1 has finished reading
      unsigned char* nxt = stage + ((t + 1) & 1) * kStStage;
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(nxt + sdst[i]) = wreg[(t + 1) & 1][i];
      __syncthreads();
    }
#pragma unroll
    for (int ks = 0; ks < kStKS; ++ks) bcur[ks] = bnext[ks];
  }

  // ---- row reduction: this lane holds, for row jb * 16 + l16, the ids t * 32 + ib * 16 + 4 q + r of the tile
  float m = kNegBig; int idx = 0x7fffffff;
#pragma unroll
  for (int t = 0; t < kStTT; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n = tile * kStRows + t * kStSub + ib * 16 + 4 * q + r;
      float v = acc[t][r];
      if (n >= a.V) v = -INFINITY;
      acc[t][r] = v;
      if (v > m) { m = v; idx = n; }                 // ascending ids, strict: the lowest id keeps a tie
    }
  const float ml = m * kLog2e;
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < kStTT; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) s += fast_exp2(fmaf(acc[t][r], kLog2e, -ml));
#pragma unroll
  for (int off = 16; off <= 32; off <<= 1) {
    const float m2 = __shfl_xor(m, off); const float s2 = __shfl_xor(s, off); const int i2 = __shfl_xor(idx, off);
    merge_partial(m, s, idx, m2, s2, i2);
  }
  if (q == 0) red[wave * 16 + l16] = Partial{m, s, idx};
  __syncthreads();
  if (tid < 32 && row_of[tid] >= 0) {
    const int rb = tid >> 4, l = tid & 15;           // row block, row inside it; its two waves are 2 rb and 2 rb + 1
    Partial p0 = red[(2 * rb) * 16 + l];
    const Partial p1 = red[(2 * rb + 1) * 16 + l];
    merge_partial(p0.m, p0.s, p0.idx, p1.m, p1.s, p1.idx);
    store_partial(a, row_of[tid], tile, p0);
  }
}

// Stream shape for 33..64 positions: same walk and the same W route as lm_head_stream_kernel, but a wave owns two
// 16-row blocks of positions, and the B operands of two chunks for two blocks (256 registers) do not fit beside
// its 128 accumulator registers.  The hidden chunk (64 rows x 1 KB) therefore lives in LDS, one stage: the next
// chunk is asked for at the start of a chunk, waits in registers, and is written between two barriers at the
// chunk's end; B operands are read from LDS per matrix instruction (a stream-bound kernel has the LDS cycles).
constexpr int kSt2Rows = 64;                               // positions per workgroup
constexpr int kSt2Hid = kSt2Rows * kStKC * 2;              // 64 KB: one hidden chunk

template <int TT>
__global__ __launch_bounds__(kLmThreads) void lm_head_stream64_kernel(LmHeadArgs a) {
  static_assert(TT % 2 == 0 && TT >= 2 && TT <= kSt2TTMax, "sub-tiles per workgroup");
  constexpr int kStTT = TT, kStRows = TT * kStSub;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  unsigned char* stage = lds_raw;                                            // 2 x kStStage (W ring)
  unsigned char* hid = lds_raw + 2 * kStStage;                               // kSt2Hid (hidden chunk)
  int* row_of = reinterpret_cast<int*>(hid + kSt2Hid);                       // 64 compacted row ids (-1 = none)
  Partial* red = reinterpret_cast<Partial*>(row_of + kSt2Rows);              // [waves][32]
  __shared__ int wsum[kLmWaves];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = blockIdx.x;                                               // < a.ntile by the grid size

  // ---- this launch works only if the masked count is in its range (another shape's launch has the call
  // otherwise); then the masked rows are compacted
  {
    const int total = lm_masked_count(a, wsum);
    if (total < a.min_masked || total > a.max_masked) return;
  }
  int running = 0;
  for (int base = 0; base < a.rows_total; base += kLmThreads) {
    const int i = base + tid;
    const bool f = i < a.rows_total && a.masked[i] != 0;
    const unsigned long long bal = __ballot(f);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[wave] = __popcll(bal);
    __syncthreads();
    int pre = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kLmWaves; ++w) { const int c = wsum[w]; pre += (w < wave) ? c : 0; tot += c; }
    const int ci = running + pre + rank;
    if (f && ci < kSt2Rows) row_of[ci] = i;
    running += tot;
    __syncthreads();
  }
  const int n_valid = min(running, kSt2Rows);      // uniform
  if (n_valid <= 0) return;
  if (tid < kSt2Rows && tid >= n_valid) row_of[tid] = -1;
  __syncthreads();

  const int NCH = (a.Hd + kStKC - 1) / kStKC;      // chunks of Hd
  const int NU = NCH * kStTT;                      // (chunk, sub-tile) steps of the walk
  const int c0 = tile % NCH;                       // this workgroup's rotation of the chunk order
  const int q = lane >> 4, l16 = lane & 15;
  const int ib = wave & 1, jw = wave >> 1;         // vocabulary block of a sub-tile; row blocks 2 jw, 2 jw + 1
  const unsigned klast = (unsigned)(a.Hd - 8);     // last whole 16-byte piece of a row

  // W staging: this wave moves rows 8 wave + i (i = 0..7) of a sub-tile, lane l the l-th 16 bytes of the chunk
  const long long vrow0 = (long long)tile * kStRows + 8 * wave;
  unsigned sdst[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = 8 * wave + i;
    sdst[i] = (unsigned)(r * (kStKC * 2) + ((lane ^ (r & 15)) << 4));
  }
  auto load_w_sub = [&](int u, u32x4 (&dst)[8]) {          // step u of the walk (clamped to the last one)
    const int uc = min(u, NU - 1);
    const int kc = uc / kStTT, t = uc - kc * kStTT;
    int kcw = kc + c0; kcw -= (kcw >= NCH) ? NCH : 0;
    const unsigned k = min((unsigned)(kcw * kStKC + 8 * lane), klast);     // pieces past Hd: any valid piece
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const long long n = min(vrow0 + t * kStSub + i, (long long)a.V - 1);   // rows past V: any valid row
      dst[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a.weight + n * a.ld_w + k));
    }
  };
  // hidden staging: this wave moves rows 16 wave + i (i = 0..15) of the chunk, lane l the l-th 16 bytes
  unsigned hsrc[16], hdst[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = 16 * wave + i;
    hsrc[i] = (unsigned)((long long)max(row_of[r], 0) * a.ld_h);           // B*K*ld_h < 2^31 is validated
    hdst[i] = (unsigned)(r * (kStKC * 2) + ((lane ^ (r & 15)) << 4));
  }
  auto load_hidden = [&](int kc, u32x4 (&dst)[16]) {       // chunk at walk position kc (clamped); zeros past Hd
    int kcw = min(kc, NCH - 1) + c0; kcw -= (kcw >= NCH) ? NCH : 0;
    const unsigned k = (unsigned)(kcw * kStKC + 8 * lane);
    const unsigned keep = (k < (unsigned)a.Hd) ? 0xffffffffu : 0u;
    const unsigned kk = min(k, klast);
#pragma unroll
    for (int i = 0; i < 16; ++i)
      dst[i] = *reinterpret_cast<const u32x4*>(a.hidden + hsrc[i] + kk) & u32x4{keep, keep, keep, keep};
  };
  // operands of k-step ks: A = row ib * 16 + l16 of the sub-tile, B = row (2 jw + rb) * 16 + l16 of the hidden
  // chunk; both piece 4 ks + q, swizzled by the row (row & 15 = l16 for both)
  const unsigned aoff = (unsigned)((ib * 16 + l16) * (kStKC * 2));
  const unsigned boff0 = (unsigned)(((2 * jw) * 16 + l16) * (kStKC * 2));
  const unsigned boff1 = boff0 + 16 * (kStKC * 2);

  f32x4 acc[kStTT][2];
#pragma unroll
  for (int t = 0; t < kStTT; ++t) { acc[t][0] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[t][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }

  // ---- prologue: W step 0 into stage 0, step 1 into registers, the first hidden chunk into LDS
  u32x4 wreg[2][8];
  u32x4 hreg[16];
  load_w_sub(0, wreg[0]);
  load_w_sub(1, wreg[1]);
  load_hidden(0, hreg);
#pragma unroll
  for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(stage + sdst[i]) = wreg[0][i];
#pragma unroll
  for (int i = 0; i < 16; ++i) *reinterpret_cast<u32x4*>(hid + hdst[i]) = hreg[i];
  __syncthreads();

  for (int kc = 0; kc < NCH; ++kc) {
    load_hidden(kc + 1, hreg);                     // waits in registers until the end of this chunk
#pragma unroll
    for (int t = 0; t < kStTT; ++t) {
      const int u = kc * kStTT + t;
      load_w_sub(u + 2, wreg[t & 1]);
      __builtin_amdgcn_sched_barrier(0);
      const unsigned char* cur = stage + (t & 1) * kStStage;
#pragma unroll
      for (int ks = 0; ks < kStKS; ++ks) {
        const unsigned po = (unsigned)(((4 * ks + q) ^ l16) << 4);
        const bf16x8 aop = *reinterpret_cast<const bf16x8*>(cur + aoff + po);
        const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(hid + boff0 + po);
        const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(hid + boff1 + po);
        acc[t][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, b0, acc[t][0], 0, 0, 0);
        acc[t][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, b1, acc[t][1], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      unsigned char* nxt = stage + ((t + 1) & 1) * kStStage;
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(nxt + sdst[i]) = wreg[(t + 1) & 1][i];
      __syncthreads();
    }
    // every wave has passed the barrier of the last sub-tile: nobody reads the hidden chunk any more
#pragma unroll
    for (int i = 0; i < 16; ++i) *reinterpret_cast<u32x4*>(hid + hdst[i]) = hreg[i];
    __syncthreads();
  }

  // ---- row reduction: this lane holds, for row (2 jw + rb) * 16 + l16, the ids t * 32 + ib * 16 + 4 q + r
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    float m = kNegBig; int idx = 0x7fffffff;
#pragma unroll
    for (int t = 0; t < kStTT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int n = tile * kStRows + t * kStSub + ib * 16 + 4 * q + r;
        float v = acc[t][rb][r];
        if (n >= a.V) v = -INFINITY;
        acc[t][rb][r] = v;
        if (v > m) { m = v; idx = n; }               // ascending ids, strict: the lowest id keeps a tie
      }
    const float ml = m * kLog2e;
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < kStTT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) s += fast_exp2(fmaf(acc[t][rb][r], kLog2e, -ml));
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float m2 = __shfl_xor(m, off); const float s2 = __shfl_xor(s, off); const int i2 = __shfl_xor(idx, off);
      merge_partial(m, s, idx, m2, s2, i2);
    }
    if (q == 0) red[wave * 32 + rb * 16 + l16] = Partial{m, s, idx};
  }
  __syncthreads();
  if (tid < kSt2Rows && row_of[tid] >= 0) {
    // position tid sits in row block tid / 16 = 2 jw + rb; its two waves are 2 jw (ib = 0) and 2 jw + 1 (ib = 1)
    const int blk = tid >> 4, l = tid & 15;
    const int w0 = 2 * (blk >> 1), rb = blk & 1;
    Partial p0 = red[w0 * 32 + rb * 16 + l];
    const Partial p1 = red[(w0 + 1) * 32 + rb * 16 + l];
    merge_partial(p0.m, p0.s, p0.idx, p1.m, p1.s, p1.idx);
    store_partial(a, row_of[tid], tile, p0);
  }
}

// Stream shape for 64 RB positions (RB = 2: 128).  The walk is the same, the route is not: W and the hidden rows
// go from global memory straight into LDS (global_load_lds_dwordx4, no staging registers, no LDS store
// instructions), so the registers hold accumulators and B operands only and the number of sub-tiles per
// workgroup needs no parity.  A chunk is 256 elements of Hd (8 k-steps), a sub-tile 32 vocabulary rows x 512
// bytes (16 KB; a transfer of one wave = two rows), the W ring has five stages and is filled four steps
// ahead.  A wave owns RB 16-row blocks of positions and both vocabulary blocks of a sub-tile; its hidden rows of
// the next chunk are transferred into a region of LDS that only this wave touches, as soon as it has read the
// current chunk's B operands from there into registers (8 RB reads per chunk).  No wave shares a position
// with another, so the row reduction ends in the wave.
// The transfers are inline assembly, invisible to the compiler's wait-count insertion: every wait for them
// is written out below, counted in transfers issued by the same wave after the one waited for (they complete
// in issue order), and the kernel has no other global load after its prologue.
constexpr int kDmSub = 32;                     // vocabulary rows per sub-tile
constexpr int kDmKC = 256;                     // elements of Hd per chunk (512 bytes per row)
constexpr int kDmKS = kDmKC / 32;              // k-steps per chunk
constexpr int kDmStage = kDmSub * kDmKC * 2;   // 16 KB
constexpr int kDmNST = 5;                      // W ring stages: filled kDmNST - 1 steps ahead (64 KB per CU in flight)
constexpr int kDmWT = kDmStage / 1024 / kLmWaves;   // W transfers per wave and step (4)
constexpr int kDmTTMax = 16;

template <int N> __device__ __forceinline__ void lm_wait_vmcnt() {
  static_assert(N >= 0 && N <= 63, "vmcnt is a six-bit field");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));    // expcnt / lgkmcnt: no wait
}
// one transfer: lane i's 16 bytes at vaddr land at lds_addr + 16 i (lds_addr uniform)
template <bool NT>
__device__ __forceinline__ void lm_dma16(unsigned lds_addr, const void* vaddr) {
  if constexpr (NT)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(vaddr) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(vaddr) : "memory", "m0");
}

// PACKED: W is the packed image; a transfer is then one operand tile (16 rows x one k-step, a contiguous
// kilobyte), the ring holds the tiles as they are and an A operand is read lane by lane, without a swizzle.
template <int TT, int RB, bool PACKED>
__global__ __launch_bounds__(kLmThreads) void lm_head_dma_kernel(LmHeadArgs a) {
  static_assert(TT >= 1 && TT <= kDmTTMax && (RB == 1 || RB == 2), "shape");
  constexpr int ROWS = kLmWaves * RB * 16;                                   // positions per workgroup
  constexpr int BT = RB * 8;                                                 // hidden transfers per wave and chunk
  constexpr int kHidWave = RB * 16 * kDmKC * 2;                              // bytes of a wave's hidden region
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  int* row_of = reinterpret_cast<int*>(lds_raw + kDmNST * kDmStage + kLmWaves * kHidWave);   // ROWS ids (-1 = none)
  __shared__ int wsum[kLmWaves];
  // LDS byte addresses (what m0 and the read instructions take)
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds_raw;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const unsigned hid0 = lds0 + kDmNST * kDmStage + wave * kHidWave;          // this wave's hidden region
  const int tile = blockIdx.x;                                               // < a.ntile by the grid size

  // ---- this launch works only if the masked count is in its range (another shape's launch has the call
  // otherwise); then the masked rows are compacted
  {
    const int total = lm_masked_count(a, wsum);
    if (total < a.min_masked || total > a.max_masked) return;
  }
  int running = 0;
  for (int base = 0; base < a.rows_total; base += kLmThreads) {
    const int i = base + tid;
    const bool f = i < a.rows_total && a.masked[i] != 0;
    const unsigned long long bal = __ballot(f);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[wave] = __popcll(bal);
    __syncthreads();
    int pre = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kLmWaves; ++w) { const int c = wsum[w]; pre += (w < wave) ? c : 0; tot += c; }
    const int ci = running + pre + rank;
    if (f && ci < ROWS) row_of[ci] = i;
    running += tot;
    __syncthreads();
  }
  const int n_valid = min(running, ROWS);          // uniform
  if (n_valid <= 0) return;
  if (tid < ROWS && tid >= n_valid) row_of[tid] = -1;
  __syncthreads();

  const int NCH = (a.Hd + kDmKC - 1) / kDmKC;      // chunks of Hd
  const int NU = NCH * TT;                         // (chunk, sub-tile) steps of the walk
  const int c0 = tile % NCH;                       // this workgroup's rotation of the chunk order
  const int q = lane >> 4, l16 = lane & 15;
  const unsigned klast = (unsigned)(a.Hd - 8);     // last whole 16-byte piece of a row
  const int half = lane >> 5, slot = lane & 31;    // a transfer covers two LDS rows of 32 slots
  auto chunk_at = [&](int kc) { int c = min(kc, NCH - 1) + c0; return c - ((c >= NCH) ? NCH : 0); };

  // W transfer j (0..3) of this wave fills rows 8 wave + 2 j + half of a sub-tile; LDS slot s of row r
  // holds piece s ^ (r & 15)
  unsigned wpiece[kDmWT];
#pragma unroll
  for (int j = 0; j < kDmWT; ++j) {
    const int r = 8 * wave + 2 * j + half;
    wpiece[j] = (unsigned)(slot ^ (r & 15));
  }
  const long long vrow0 = (long long)tile * (TT * kDmSub) + 8 * wave + half;
  const int NKS = a.Hd / 32, NB = (a.V + 15) / 16;             // k-steps, 16-row blocks (packed image)
  auto issue_w = [&](int u) {                      // step u of the walk (clamped to the last one) into stage u % 5
    const int uc = min(u, NU - 1);
    const int kc = uc / TT, t = uc - kc * TT;
    const unsigned st = lds0 + (unsigned)(u % kDmNST) * kDmStage + wave * (kDmWT * 1024);
    if constexpr (PACKED) {
      // transfer j of this wave is tile x = 4 wave + j of the 16 in a step: vocabulary block x / 8, k-step x % 8
      const int ks0 = chunk_at(kc) * kDmKS;
#pragma unroll
      for (int j = 0; j < kDmWT; ++j) {
        const int x = kDmWT * wave + j;
        const int nb = min((tile * TT + t) * 2 + x / kDmKS, NB - 1);           // blocks past V: the last one
        const int ks = min(ks0 + x % kDmKS, NKS - 1);                           // k-steps past Hd: the last one
        lm_dma16<true>(st + j * 1024, a.weight + (((long long)nb * NKS + ks) * 64 + lane) * 8);
      }
    } else {
      const unsigned kb = (unsigned)(chunk_at(kc) * kDmKC);
#pragma unroll
      for (int j = 0; j < kDmWT; ++j) {
        const long long n = min(vrow0 + t * kDmSub + 2 * j, (long long)a.V - 1);   // rows past V: any valid row
        const unsigned k = min(kb + 8 * wpiece[j], klast);                          // pieces past Hd: any valid piece
        lm_dma16<true>(st + j * 1024, a.weight + n * a.ld_w + k);
      }
    }
  };
  // hidden transfer j (0..BT-1) fills rows 2 j + half of this wave's region (row = rb * 16 + position in block)
  unsigned hoff[BT], hpiece[BT];
#pragma unroll
  for (int j = 0; j < BT; ++j) {
    const int r = 2 * j + half;                    // 0 .. RB * 16 - 1
    hoff[j] = (unsigned)((long long)max(row_of[wave * RB * 16 + r], 0) * a.ld_h);   // B*K*ld_h < 2^31 is validated
    hpiece[j] = (unsigned)(slot ^ (r & 15));
  }
  auto issue_b = [&](int kc) {                     // chunk at walk position kc (clamped to the last one)
    const unsigned kb = (unsigned)(chunk_at(kc) * kDmKC);
#pragma unroll
    for (int j = 0; j < BT; ++j)
      lm_dma16<false>(hid0 + j * 1024, a.hidden + hoff[j] + min(kb + 8 * hpiece[j], klast));
  };
  // operand reads: row (block * 16 + l16), piece 4 ks + q, swizzled by the row (row & 15 = l16)
  bf16x8 bcur[kDmKS][RB];
  auto read_b = [&](int kc) {                      // this wave's region -> registers; zeros past Hd
    const unsigned kb = (unsigned)(chunk_at(kc) * kDmKC);
#pragma unroll
    for (int ks = 0; ks < kDmKS; ++ks) {
      const unsigned keep = (kb + 32 * ks + 8 * q < (unsigned)a.Hd) ? 0xffffffffu : 0u;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const unsigned off = (unsigned)((rb * 16 + l16) * (kDmKC * 2) + (((4 * ks + q) ^ l16) << 4));
        const u32x4 v = *reinterpret_cast<const u32x4*>(lds_raw + kDmNST * kDmStage + wave * kHidWave + off);
        bcur[ks][rb] = __builtin_bit_cast(bf16x8, v & u32x4{keep, keep, keep, keep});
      }
    }
  };

  f32x4 acc[TT][2][RB];
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int ib = 0; ib < 2; ++ib)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) acc[t][ib][rb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- prologue: the first chunk's hidden rows, steps 0..2 of W
  issue_b(0);
#pragma unroll
  for (int u = 0; u < kDmNST - 1; ++u) issue_w(u);
  lm_wait_vmcnt<0>();
  __syncthreads();

  for (int kc = 0; kc < NCH; ++kc) {
    // the hidden rows of this chunk were asked for at the start of the chunk before (or in the prologue);
    // issued after them by this wave: that chunk's TT steps of W
    lm_wait_vmcnt<(TT * kDmWT < 63 ? TT * kDmWT : 63)>();
    read_b(kc);
    // the next chunk's rows may only start to arrive in the region once these reads have returned
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    issue_b(kc + 1);
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const int u = kc * TT + t;
      issue_w(u + kDmNST - 1);                     // into the stage that step u - 1 has finished reading
      __builtin_amdgcn_sched_barrier(0);
      const unsigned char* cur = lds_raw + (unsigned)(u % kDmNST) * kDmStage;
      // all A operands of the step are asked for at once: the matrix instructions then run back to back,
      // each waiting only for its own operand
      bf16x8 aop[kDmKS][2];
#pragma unroll
      for (int ks = 0; ks < kDmKS; ++ks) {
        if constexpr (PACKED) {
          aop[ks][0] = *reinterpret_cast<const bf16x8*>(cur + ks * 1024 + lane * 16);
          aop[ks][1] = *reinterpret_cast<const bf16x8*>(cur + (kDmKS + ks) * 1024 + lane * 16);
        } else {
          const unsigned po = (unsigned)(l16 * (kDmKC * 2) + (((4 * ks + q) ^ l16) << 4));
          aop[ks][0] = *reinterpret_cast<const bf16x8*>(cur + po);
          aop[ks][1] = *reinterpret_cast<const bf16x8*>(cur + 16 * (kDmKC * 2) + po);
        }
      }
      __builtin_amdgcn_sched_barrier(0);           // (the scheduler would sink the reads back between the MFMAs)
#pragma unroll
      for (int ks = 0; ks < kDmKS; ++ks)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          acc[t][0][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop[ks][0], bcur[ks][rb], acc[t][0][rb], 0, 0, 0);
          acc[t][1][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop[ks][1], bcur[ks][rb], acc[t][1][rb], 0, 0, 0);
        }
      __builtin_amdgcn_sched_barrier(0);
      // step u + 1 must have landed before the barrier: issued after it by this wave are the D = kDmNST - 2
      // steps u + 2 .. u + kDmNST - 1 (one in each of the steps u - D + 1 .. u), and the next chunk's hidden
      // rows wherever one of those steps began a chunk (t < D; with TT < D more than one of them may have)
      constexpr int D = kDmNST - 2;
      const int chunk_starts = TT >= D ? (t < D ? 1 : 0) : (D - 1 - t) / TT + 1;
      static_assert(D * kDmWT + D * BT <= 63, "vmcnt");
      if (chunk_starts == 0) lm_wait_vmcnt<D * kDmWT>();
      else if (chunk_starts == 1) lm_wait_vmcnt<D * kDmWT + BT>();
      else if (chunk_starts == 2) lm_wait_vmcnt<D * kDmWT + 2 * BT>();
      else lm_wait_vmcnt<D * kDmWT + 3 * BT>();
      __syncthreads();
    }
  }
  lm_wait_vmcnt<0>();                              // nothing of this workgroup's is in flight when it ends

  // ---- row reduction: this lane holds, for row (wave RB + rb) * 16 + l16, the ids t * 32 + ib * 16 + 4 q + r
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float m = kNegBig; int idx = 0x7fffffff;
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int n = tile * (TT * kDmSub) + t * kDmSub + ib * 16 + 4 * q + r;
          float v = acc[t][ib][rb][r];
          if (n >= a.V) v = -INFINITY;
          acc[t][ib][rb][r] = v;
          if (v > m) { m = v; idx = n; }             // ascending ids, strict: the lowest id keeps a tie
        }
    const float ml = m * kLog2e;
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += fast_exp2(fmaf(acc[t][ib][rb][r], kLog2e, -ml));
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float m2 = __shfl_xor(m, off); const float s2 = __shfl_xor(s, off); const int i2 = __shfl_xor(idx, off);
      merge_partial(m, s, idx, m2, s2, i2);
    }
    const int row = row_of[(wave * RB + rb) * 16 + l16];
    if (q == 0 && row >= 0) store_partial(a, row, tile, Partial{m, s, idx});
  }
}

// ---------------------------------------------------------------------------------------------------
// The packed image of W: one wave per operand tile (16 vocabulary rows x one k-step = one kilobyte).
__global__ __launch_bounds__(kLmThreads) void lm_head_pack_kernel(const uint16_t* __restrict__ W, long long ld_w,
                                                                  int V, int NK, long long ntiles, u32x4* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const long long g = (long long)blockIdx.x * kLmWaves + (threadIdx.x >> 6);     // tile: block g / NK, k-step g % NK
  if (g >= ntiles) return;
  const long long nb = g / NK;
  const int ks = (int)(g - nb * NK);
  const long long row = min(nb * 16 + (lane & 15), (long long)V - 1);             // rows past V repeat the last row
  out[g * 64 + lane] = *reinterpret_cast<const u32x4*>(W + row * ld_w + ks * 32 + 8 * (lane >> 4));
}

// Stream shape for at most 32 positions over a packed W.  Nothing is shared between the waves but the list of
// masked rows: a wave owns TT 16-row vocabulary blocks and both row blocks of positions, loads its A operands
// straight from the image (every load of a wave is one contiguous kilobyte, nontemporal, two k-steps ahead in
// registers) and keeps the B operands of a chunk of 8 k-steps in registers, the next chunk's beside them.  No
// LDS and no barrier in the loop; the compiler's wait counts see one straight line per chunk.
constexpr int kPkKS = 8;                       // k-steps per chunk of B operands
constexpr int kPkPF = 2;                       // k-steps of A operands in flight per wave
constexpr int kPkTTMax = 10;

template <int TT>
__global__ __launch_bounds__(kLmThreads) void lm_head_packed_kernel(LmHeadArgs a) {
  static_assert(TT >= 1 && TT <= kPkTTMax && kPkKS % kPkPF == 0, "shape");
  __shared__ int row_of[32];                     // compacted row ids (-1 = none)
  __shared__ Partial red[kLmWaves][32];
  __shared__ int wsum[kLmWaves];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = blockIdx.x;                   // < a.ntile by the grid size

  {
    const int total = lm_masked_count(a, wsum);
    if (total < a.min_masked || total > a.max_masked) return;
  }
  int running = 0;
  for (int base = 0; base < a.rows_total; base += kLmThreads) {
    const int i = base + tid;
    const bool f = i < a.rows_total && a.masked[i] != 0;
    const unsigned long long bal = __ballot(f);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[wave] = __popcll(bal);
    __syncthreads();
    int pre = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kLmWaves; ++w) { const int c = wsum[w]; pre += (w < wave) ? c : 0; tot += c; }
    const int ci = running + pre + rank;
    if (f && ci < 32) row_of[ci] = i;
    running += tot;
    __syncthreads();
  }
  const int n_valid = min(running, 32);            // uniform
  if (n_valid <= 0) return;
  if (tid < 32 && tid >= n_valid) row_of[tid] = -1;
  __syncthreads();

  const int NK = a.Hd / 32;                        // k-steps
  const int NCH = (NK + kPkKS - 1) / kPkKS;        // chunks
  const int NB = (a.V + 15) / 16;                  // 16-row blocks of the image
  const int q = lane >> 4, l16 = lane & 15;
  const int c0 = tile % NCH;                       // this workgroup's rotation of the chunk order
  auto chunk_at = [&](int c) { int ch = min(c, NCH - 1) + c0; return ch - ((ch >= NCH) ? NCH : 0); };
  auto kstep_at = [&](int s) {                     // k-step at position s of the walk (past the end: the last position)
    const int sc = min(s, NCH * kPkKS - 1);
    const int cc = sc / kPkKS, ss = sc - cc * kPkKS;
    return min(chunk_at(cc) * kPkKS + ss, NK - 1); // k-steps past Hd: the last one (its B operands are zeros)
  };
  // A operands: block nb0 + t of the image, this lane's 16 bytes of every k-step 512 elements apart
  const int nb0 = (tile * kLmWaves + wave) * TT;
  const uint16_t* wblk[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) wblk[t] = a.weight + ((long long)min(nb0 + t, NB - 1) * NK * 64 + lane) * 8;
  auto load_a = [&](int s, bf16x8 (&dst)[TT]) {
    const long long off = (long long)kstep_at(s) * 512;
#pragma unroll
    for (int t = 0; t < TT; ++t)
      dst[t] = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wblk[t] + off)));
  };
  // B operands: hidden row of position rb * 16 + l16, elements 8 q .. 8 q + 7 of every k-step of a chunk
  const uint16_t* hrow[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) hrow[rb] = a.hidden + (long long)max(row_of[rb * 16 + l16], 0) * a.ld_h + 8 * q;
  // (loaded as they are; k-steps past Hd are zeroed when the chunk becomes the current one: a mask applied at
  // the load would make the compiler wait for it there, behind every A load in flight)
  auto load_b = [&](int c, u32x4 (&dst)[kPkKS][2]) {             // chunk at walk position c
    const int k0 = chunk_at(c) * kPkKS;
#pragma unroll
    for (int ks = 0; ks < kPkKS; ++ks) {
      const int kk = min(k0 + ks, NK - 1);
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) dst[ks][rb] = *reinterpret_cast<const u32x4*>(hrow[rb] + 32 * kk);
    }
  };
  auto take_b = [&](int c, const u32x4 (&src)[kPkKS][2], bf16x8 (&dst)[kPkKS][2]) {   // zeros past Hd
    const int k0 = chunk_at(c) * kPkKS;
#pragma unroll
    for (int ks = 0; ks < kPkKS; ++ks) {
      const unsigned keep = (k0 + ks < NK) ? 0xffffffffu : 0u;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) dst[ks][rb] = __builtin_bit_cast(bf16x8, src[ks][rb] & u32x4{keep, keep, keep, keep});
    }
  };

  f32x4 acc[TT][2];
#pragma unroll
  for (int t = 0; t < TT; ++t) { acc[t][0] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[t][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }
  bf16x8 abuf[kPkPF][TT];
  bf16x8 bcur[kPkKS][2];
  u32x4 bnext[kPkKS][2];
  load_b(0, bnext);
#pragma unroll
  for (int s = 0; s < kPkPF; ++s) load_a(s, abuf[s]);
  take_b(0, bnext, bcur);

  for (int kc = 0; kc < NCH; ++kc) {
    load_b(kc + 1, bnext);                         // older than every A load below: it is back before they are
#pragma unroll
    for (int ks = 0; ks < kPkKS; ++ks) {
      bf16x8 acur[TT];
#pragma unroll
      for (int t = 0; t < TT; ++t) acur[t] = abuf[ks % kPkPF][t];
      load_a(kc * kPkKS + ks + kPkPF, abuf[ks % kPkPF]);
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        acc[t][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[t], bcur[ks][0], acc[t][0], 0, 0, 0);
        acc[t][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[t], bcur[ks][1], acc[t][1], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    take_b(kc + 1, bnext, bcur);
  }

  // ---- row reduction: this lane holds, for position rb * 16 + l16, the ids (nb0 + t) * 16 + 4 q + r
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    float m = kNegBig; int idx = 0x7fffffff;
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int n = (nb0 + t) * 16 + 4 * q + r;
        float v = acc[t][rb][r];
        if (n >= a.V) v = -INFINITY;
        acc[t][rb][r] = v;
        if (v > m) { m = v; idx = n; }               // ascending ids, strict: the lowest id keeps a tie
      }
    const float ml = m * kLog2e;
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) s += fast_exp2(fmaf(acc[t][rb][r], kLog2e, -ml));
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float m2 = __shfl_xor(m, off); const float s2 = __shfl_xor(s, off); const int i2 = __shfl_xor(idx, off);
      merge_partial(m, s, idx, m2, s2, i2);
    }
    if (q == 0) red[wave][rb * 16 + l16] = Partial{m, s, idx};
  }
  __syncthreads();
  if (tid < 32 && row_of[tid] >= 0) {
    Partial p = red[0][tid];                         // waves hold ascending vocabulary ranges
#pragma unroll
    for (int w = 1; w < kLmWaves; ++w) merge_partial(p.m, p.s, p.idx, red[w][tid].m, red[w][tid].s, red[w][tid].idx);
    store_partial(a, row_of[tid], tile, p);
  }
}

// ---- host side ----
// The kernel shapes, by the masked counts they serve.  Row-major W: up to 32 (stream, B operands in
// registers), up to 64 (stream, hidden chunk in LDS), up to 128 (stream, global -> LDS transfers), any (256-row
// chunks).  Packed W: up to 32 (operands straight from the image), up to 64 and up to 128 (global -> LDS
// transfers of operand tiles), any (256-row chunks).
enum { kShape32 = 0, kShape64, kShape128, kShapeRows, kNumShapes };
constexpr int kShapeMax[kNumShapes] = {32, kSt2Rows, 128, INT_MAX};

// Sub-tiles per workgroup of a stream kernel, out of the counts it is compiled for.  One workgroup per CU is
// resident, so a launch runs in rounds of kNumCUs workgroups and costs about rounds x (sub-tiles + a half for
// the prologue): 126464 vocabulary rows take 16 sub-tiles (247 workgroups), 152064 take 20 (238 workgroups; 16
// would leave 41 of 297 for a second round) or, where the accumulators allow no more, 10 (476, two rounds).
constexpr int kStTTs[] = {2, 4, 8, 12, 16, 20};
constexpr int kSt2TTs[] = {2, 4, 8, 10, 12, 16};
constexpr int kDmTTs[] = {1, 2, 3, 4, 6, 8, 10, 16};
constexpr int kPkTTs[] = {1, 2, 4, 6, 8, 10};      // 16-row blocks per wave: 64 rows per workgroup each
constexpr int kPkSub = kLmWaves * 16;
static_assert(kStSub == kDmSub, "one sub-tile size for the tile-size choice");

template <size_t N>
static int stream_tt(int V, const int (&tts)[N], int sub = kStSub) {
  const int nsub = (V + sub - 1) / sub;
  int best = tts[0];
  long long best_cost = LLONG_MAX;
  for (int tt : tts) {
    const int ntile = (nsub + tt - 1) / tt;
    const long long cost = (long long)((ntile + kNumCUs - 1) / kNumCUs) * (2 * tt + 1);
    if (cost <= best_cost) { best_cost = cost; best = tt; }     // ties: fewer, larger tiles
  }
  return best;
}

// top: the shape for B x K positions all masked; the shapes below it are launched too and serve the smaller
// masked counts; ntile_out is the largest tile count among the launched shapes.
// first: the smallest shape launched.  Over a packed W the 64-position kernel streams as fast as the
// 32-position one (161 against 167 us for 126464 x 4096), so where both would be launched the former serves
// 1..64 masked positions and the call has one idle launch less.
struct LmPlan { int first, top, nchunk, packed, tt[kNumShapes], bn[kNumShapes], ntile[kNumShapes], ntile_out; };

static LmPlan lm_plan(const sdllm_lm_head_params& p) {
  const long long rows = (long long)p.B * p.K;
  LmPlan pl;
  pl.packed = p.weight_packed;
  int sub[kNumShapes] = {kStSub, kStSub, kStSub, 256};
  if (pl.packed) {
    pl.tt[kShape32] = stream_tt(p.V, kPkTTs, kPkSub); sub[kShape32] = kPkSub;
    pl.tt[kShape64] = stream_tt(p.V, kDmTTs);
  } else {
    pl.tt[kShape32] = stream_tt(p.V, kStTTs);
    pl.tt[kShape64] = stream_tt(p.V, kSt2TTs);
  }
  pl.tt[kShape128] = stream_tt(p.V, kDmTTs);
  pl.tt[kShapeRows] = 1;                  // 256-row tiles (also for a half-empty chunk: it beat 128-row tiles)
  pl.top = 0;
  while (rows > kShapeMax[pl.top]) ++pl.top;
  pl.first = (pl.packed && pl.top > kShape32) ? kShape64 : kShape32;
  pl.ntile_out = 0;
  for (int i = 0; i < kNumShapes; ++i) {
    pl.bn[i] = pl.tt[i] * sub[i];
    pl.ntile[i] = (p.V + pl.bn[i] - 1) / pl.bn[i];
    if (i >= pl.first && i <= pl.top) pl.ntile_out = std::max(pl.ntile_out, pl.ntile[i]);
  }
  pl.nchunk = pl.top == kShapeRows ? (int)((rows + 255) / 256) : 1;
  return pl;
}

constexpr size_t dma_lds_bytes(int rb) {
  return (size_t)kDmNST * kDmStage + (size_t)kLmWaves * (rb * 16 * kDmKC * 2) + (size_t)kLmWaves * rb * 16 * sizeof(int);
}

static size_t lm_lds_bytes(int shape, int packed) {
  switch (shape) {
    case kShape32: return packed ? 0 : 2 * (size_t)kStStage + 32 * sizeof(int) + (size_t)kLmWaves * 16 * sizeof(Partial);
    case kShape64: return packed ? dma_lds_bytes(1)
                                 : 2 * (size_t)kStStage + kSt2Hid + kSt2Rows * sizeof(int) + (size_t)kLmWaves * 32 * sizeof(Partial);
    case kShape128: return dma_lds_bytes(2);
    default: return (size_t)3 * kLmStageBytes + 256 * sizeof(int) + (size_t)kLmWaves * 256 * sizeof(Partial);   // LmShape::NST
  }
}

void lm_head_plan(const sdllm_lm_head_params& p, sdllm_lm_head_plan* plan) {
  const LmPlan pl = lm_plan(p);
  const int t = pl.top;
  plan->rows_per_chunk = t == kShapeRows ? 256 : kShapeMax[t];
  plan->vocab_rows_per_tile = pl.bn[t]; plan->vocab_tiles = pl.ntile[t];
  plan->row_chunks = pl.nchunk;
  plan->workgroups = t != kShapeRows ? pl.ntile[t] : ((pl.ntile[t] + kNumXCDs - 1) / kNumXCDs) * pl.nchunk * kNumXCDs;
  plan->lds_bytes = (int32_t)lm_lds_bytes(t, pl.packed);
  plan->triples_per_position = pl.ntile_out;
}

size_t lm_head_workspace_bytes(const sdllm_lm_head_params& p) {
  return (size_t)p.B * p.K * lm_plan(p).ntile_out * sizeof(Partial);
}

size_t lm_head_packed_weight_bytes(int V, int Hd) {
  return (size_t)((V + 15) / 16) * (size_t)(Hd / 32) * 1024;
}

hipError_t launch_lm_head_pack_weight(int V, int Hd, long long ld_w, const void* weight, void* packed, hipStream_t stream) {
  const int NK = Hd / 32;
  const long long ntiles = (long long)((V + 15) / 16) * NK;
  const long long grid = (ntiles + kLmWaves - 1) / kLmWaves;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(lm_head_pack_kernel, dim3((unsigned)grid), dim3(kLmThreads), 0, stream,
                     (const uint16_t*)weight, ld_w, V, NK, ntiles, (u32x4*)packed);
  return hipGetLastError();
}

// One launch, or (r.hidden == nullptr: the preparation pass of sdllm_init) only the kernel's opt-in to its
// dynamic LDS size on the current device.
static hipError_t launch_kernel(void (*kernel)(LmHeadArgs), LdsOptIn& st, size_t lds, unsigned grid,
                                const LmHeadArgs& r, hipStream_t stream) {
  hipError_t e = ensure_lds_opt_in(reinterpret_cast<const void*>(kernel), lds, st);
  if (e != hipSuccess || r.hidden == nullptr) return e;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(kLmThreads), lds, stream, r);
  return hipGetLastError();
}

template <int TT>
static hipError_t launch_stream32(const LmHeadArgs& r, hipStream_t stream) {
  static LdsOptIn st;
  return launch_kernel(lm_head_stream_kernel<TT>, st, lm_lds_bytes(kShape32, 0), (unsigned)r.ntile, r, stream);
}
template <int TT>
static hipError_t launch_stream64(const LmHeadArgs& r, hipStream_t stream) {
  static LdsOptIn st;
  return launch_kernel(lm_head_stream64_kernel<TT>, st, lm_lds_bytes(kShape64, 0), (unsigned)r.ntile, r, stream);
}
template <int TT>
static hipError_t launch_packed32(const LmHeadArgs& r, hipStream_t stream) {
  static LdsOptIn st;
  return launch_kernel(lm_head_packed_kernel<TT>, st, 0, (unsigned)r.ntile, r, stream);
}
template <int TT, int RB, bool PACKED>
static hipError_t launch_dma(const LmHeadArgs& r, hipStream_t stream) {
  static LdsOptIn st;
  return launch_kernel(lm_head_dma_kernel<TT, RB, PACKED>, st, dma_lds_bytes(RB), (unsigned)r.ntile, r, stream);
}
template <int RB, bool PACKED>
static hipError_t launch_dma_tt(int tt, const LmHeadArgs& r, hipStream_t stream) {
  switch (tt) {                        // kDmTTs
    case 1: return launch_dma<1, RB, PACKED>(r, stream);
    case 2: return launch_dma<2, RB, PACKED>(r, stream);
    case 3: return launch_dma<3, RB, PACKED>(r, stream);
    case 4: return launch_dma<4, RB, PACKED>(r, stream);
    case 6: return launch_dma<6, RB, PACKED>(r, stream);
    case 8: return launch_dma<8, RB, PACKED>(r, stream);
    case 10: return launch_dma<10, RB, PACKED>(r, stream);
    case 16: return launch_dma<16, RB, PACKED>(r, stream);
  }
  return hipErrorInvalidValue;
}
static hipError_t launch_rows(const LmHeadArgs& r, hipStream_t stream) {
  static_assert(LmShape<256, 4, 4>::NST == 3 && LmShape<256, 4, 4>::BN == 256, "lm_lds_bytes, lm_plan");
  static LdsOptIn st[2];
  const unsigned grid = (unsigned)(((r.ntile + kNumXCDs - 1) / kNumXCDs) * r.nchunk * kNumXCDs);
  if (r.packed) return launch_kernel(lm_head_rows_kernel<256, 4, 4, true>, st[1], lm_lds_bytes(kShapeRows, 1), grid, r, stream);
  return launch_kernel(lm_head_rows_kernel<256, 4, 4, false>, st[0], lm_lds_bytes(kShapeRows, 0), grid, r, stream);
}

static hipError_t launch_shape(int shape, int tt, const LmHeadArgs& r, hipStream_t stream) {
  switch (shape) {
    case kShape32:
      if (r.packed) switch (tt) {      // kPkTTs
        case 1: return launch_packed32<1>(r, stream);
        case 2: return launch_packed32<2>(r, stream);
        case 4: return launch_packed32<4>(r, stream);
        case 6: return launch_packed32<6>(r, stream);
        case 8: return launch_packed32<8>(r, stream);
        case 10: return launch_packed32<10>(r, stream);
      } else switch (tt) {             // kStTTs
        case 2: return launch_stream32<2>(r, stream);
        case 4: return launch_stream32<4>(r, stream);
        case 8: return launch_stream32<8>(r, stream);
        case 12: return launch_stream32<12>(r, stream);
        case 16: return launch_stream32<16>(r, stream);
        case 20: return launch_stream32<20>(r, stream);
      }
      break;
    case kShape64:
      if (r.packed) return launch_dma_tt<1, true>(tt, r, stream);
      switch (tt) {                    // kSt2TTs
        case 2: return launch_stream64<2>(r, stream);
        case 4: return launch_stream64<4>(r, stream);
        case 8: return launch_stream64<8>(r, stream);
        case 10: return launch_stream64<10>(r, stream);
        case 12: return launch_stream64<12>(r, stream);
        case 16: return launch_stream64<16>(r, stream);
      }
      break;
    case kShape128:
      return r.packed ? launch_dma_tt<2, true>(tt, r, stream) : launch_dma_tt<2, false>(tt, r, stream);
    case kShapeRows: return launch_rows(r, stream);
  }
  return hipErrorInvalidValue;      // not reached: lm_plan picks from the same lists
}

// Every kernel shape and tile size the plan can pick, for both weight layouts: opt-ins only, nothing is launched.
hipError_t prepare_lm_head() {
  LmHeadArgs r{};
  r.hidden = nullptr; r.ntile = 1; r.nchunk = 1;
  hipError_t e = hipSuccess;
  for (int packed = 0; packed <= 1 && e == hipSuccess; ++packed) {
    r.packed = packed;
    if (packed) { for (int tt : kPkTTs) if (e == hipSuccess) e = launch_shape(kShape32, tt, r, nullptr); }
    else        { for (int tt : kStTTs) if (e == hipSuccess) e = launch_shape(kShape32, tt, r, nullptr); }
    if (packed) { for (int tt : kDmTTs) if (e == hipSuccess) e = launch_shape(kShape64, tt, r, nullptr); }
    else        { for (int tt : kSt2TTs) if (e == hipSuccess) e = launch_shape(kShape64, tt, r, nullptr); }
    for (int tt : kDmTTs) if (e == hipSuccess) e = launch_shape(kShape128, tt, r, nullptr);
    if (e == hipSuccess) e = launch_shape(kShapeRows, 1, r, nullptr);
  }
  return e;
}

hipError_t launch_lm_head_unmask(const sdllm_lm_head_params& p, const void* hidden, const void* weight,
                                 int32_t* tokens, uint8_t* masked, float* confidence, int32_t* n_committed,
                                 uint8_t* block_done, uint8_t* eos_seen, void* workspace, hipStream_t stream) {
  const LmPlan pl = lm_plan(p);
  LmHeadArgs r;
  r.hidden = (const uint16_t*)hidden; r.weight = (const uint16_t*)weight; r.masked = masked;
  r.partials = (Partial*)workspace;
  r.ld_h = p.ld_h; r.ld_w = p.ld_w;
  r.rows_total = p.B * p.K; r.V = p.V; r.Hd = p.Hd;
  r.nchunk = pl.nchunk; r.ntile_out = pl.ntile_out; r.packed = pl.packed;
  hipError_t e = hipSuccess;
  // every shape up to the one that B x K needs: the smaller ones take the call when few enough positions are
  // still masked (the later steps of a block); each launch exits unless the masked count is in its range
  for (int i = pl.first; i <= pl.top && e == hipSuccess; ++i) {
    r.ntile = pl.ntile[i];
    r.min_masked = i == pl.first ? 1 : kShapeMax[i - 1] + 1;
    r.max_masked = i == pl.top ? INT_MAX : kShapeMax[i];
    e = launch_shape(i, pl.tt[i], r, stream);
  }
  if (e != hipSuccess) return e;

  UnmaskArgs u;
  u.logits = nullptr; u.partials = (Partial*)workspace;
  u.tokens = tokens; u.masked = masked; u.confidence = confidence;
  u.n_committed = n_committed; u.block_done = block_done; u.eos_seen = eos_seen;
  u.ld = 0; u.V = p.V; u.nvec = 0; u.vec_per_split = 0;
  u.nsplit = pl.ntile_out; u.nsplit_p2 = 1; u.K = p.K;
  u.tau0 = p.tau0; u.alpha = p.alpha; u.r_extra_masked = p.r_extra_masked; u.r_extra_total = p.r_extra_total;
  u.eos_id = p.eos_id; u.tau_eos = p.tau_eos;
  return launch_unmask_commit(u, p.B, stream);
}

}  // namespace sdllm
