// Blockwise attention step for gfx950 (CDNA4): block_out, block_lse <- Attention(Q, K, V)
// of TokenRing's Algorithm 1 (Sec. 3.2), one Query chunk against one K/V chunk.
//
// Formulation.  Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// the A operand is a 32-key x 16-d slice of the K tile read from LDS, the B operand a
// 16-d x 32-query slice of Q^T held in registers for the whole kernel.  In the MFMA
// accumulator layout lane (q = lane%32, half = lane/32) then owns, for ONE query, the
// 16 keys {8g + 4*half + r} of a 32-key sub-tile: the softmax is in-lane.  The
// exponentiated sub-tile P^T, rounded to bf16, is already in the B-operand layout of the
// second product O^T = V^T P^T; its A operand (32 d x 16 keys of V^T) comes from the
// row-major V tile in LDS through the transposing read ds_read_b64_tr_b16, with the key
// order inside each 16-key step permuted to match the accumulator layout of P^T (a
// contraction index may be permuted freely as long as both operands agree).  The O^T
// accumulator again has one query per lane, so rescaling and the final 1/l need no
// cross-lane traffic.
//
// Pipeline.  A lone wave issues vector-ALU instructions far below the SIMD's rate and cannot
// hide its softmax behind another wave's MFMAs, so MFMA and softmax work are interleaved
// INSIDE every wave, one 32-key sub-tile apart: step j runs, as one instruction stream,
//     MFMA : O += V_{j-1}^T P_{j-1}      and      S_{j+1} = K_{j+1} Q^T
//     VALU : P_j = exp2((S_j - m_ref) * scale*log2e), row sums
// with no dependency between the two halves.  Two such waves per SIMD fill each other's
// gaps.  A workgroup has 8 waves of 32 query rows (256 rows); K/V tiles of 16 KiB (64 keys
// = two sub-tiles at D = 128, 128 keys = four at D = 64) go straight from global memory into
// 4-deep LDS rings (global_load_lds), the K tile with a 16-byte XOR swizzle and the V tile
// with a 32-byte XOR swizzle that make the ds_read_b128 and the transposing reads
// bank-conflict free.  One workgroup barrier per tile hands ring slots over.
#include <type_traits>

#include <atomic>

#include "tr_internal.h"

namespace tr {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kBM = kWaves * 32;  // query rows per workgroup
// keys per LDS tile: 16 KiB of K (and of V) either way, so a tile is 2 sub-tiles of 32 keys at
// D = 128 and 4 at D = 64, where a sub-tile carries half the MFMA work per barrier otherwise
template <int D>
constexpr int tile_keys() { return D == 64 ? 128 : 64; }
constexpr int kRing = 4;          // LDS ring depth (tiles) of K and of V
constexpr int kEpiBf16 = 0, kEpiF32 = 1, kEpiMerge = 2;

// Exchange between the two 32-lane halves of a wave with v_permlane32_swap, which swaps the
// upper half of its first operand with the lower half of its second: fed (x, x) it leaves
// x[lane%32] in the first and x[32 + lane%32] in the second register, in every lane.
// Written as inline asm: at -O3 the compiler folds the second result of the corresponding
// builtin into the first, which silently drops the other half's contribution.  The s_nop
// covers the VALU-write -> permlane-swap hazard the assembler does not see inside asm.
__device__ __forceinline__ void half_pair(float x, float& lo, float& hi) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  lo = a;
  hi = b;
}
__device__ __forceinline__ float half_swap_max(float x) {
  float lo, hi;
  half_pair(x, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float half_swap_sum(float x) {
  float lo, hi;
  half_pair(x, lo, hi);
  return lo + hi;
}

// Byte offset of 16-byte chunk c of row `row` inside a K tile (row-major, D bf16 per row).
template <int D>
__device__ __forceinline__ int k_lds_off(int row, int c) {
  constexpr int RB = 2 * D;             // row bytes
  constexpr int R2 = 256 / RB;          // rows per 256-byte bank line
  constexpr int NC = RB / 16;           // chunks per row
  return row * RB + ((c ^ ((row / R2) % NC)) << 4);
}
// Byte offset of 16-byte chunk c of row `row` inside a V tile: 32-byte slots XOR-swizzled
// by the row so that the four rows a transposing read touches fall on distinct banks.
template <int D>
__device__ __forceinline__ int v_lds_off(int row, int c) {
  constexpr int RB = 2 * D;
  int slot = c >> 1;
  int swz = (D == 128) ? ((row & 3) << 1) : (row & 2);
  return row * RB + ((slot ^ swz) << 5) + ((c & 1) << 4);
}

// Which (batch*head, query tile, block step) a workgroup computes.  The grid is three-dimensional
// - x: batch*head, y: query tile, z: block step of the launch - so the indices come from the
// hardware instead of integer divisions (a division costs ~40 dependent instructions and the
// decoding sits in front of every workgroup's first load).  Workgroups are dealt round-robin to
// the 8 XCDs in the order of their linear id, which is x-fastest, and the x extent is a multiple
// of 8 whenever xcd_map is set: XCD = blockIdx.x mod 8.  XCD x gets the K/V heads x, x+8, ... and
// all query heads and query tiles that read them, so a head's K/V stays in one L2.
__device__ __forceinline__ void decode_block(const AttnParams& p, int& qt, int& b, int& hq, int& hk, int& prob) {
  const int gq = p.gq, sh = p.gq_log2;   // query heads per K/V head; its log2, or -1 if not a power of two
  int bh = (int)blockIdx.x, qi = (int)blockIdx.y;
  if (p.xcd_map) {
    int x = bh & 7, hi = bh >> 3;
    if (p.xcd_map == 2) {   // x = XCD + 8 * query tile, y = head within the XCD
      qi = hi;
      hi = (int)blockIdx.y;
    }
    const int kvi = sh >= 0 ? hi >> sh : hi / gq;
    const int mem = sh >= 0 ? hi & (gq - 1) : hi % gq;
    bh = (kvi * 8 + x) * gq + mem;
  }
  b = p.B == 1 ? 0 : bh / p.Hq;
  hq = bh - b * p.Hq;
  hk = sh >= 0 ? hq >> sh : hq / gq;
  qt = p.n_qtiles - 1 - qi;  // late query tiles (most keys under a causal mask) first
  prob = (int)blockIdx.z;
}

typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// A pointer the compiler must keep in an SGPR pair (it is wave-uniform by construction).
__device__ __forceinline__ const __bf16* uniform_ptr(const __bf16* ptr) {
  const unsigned long long v = (unsigned long long)ptr;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (const __bf16*)(((unsigned long long)hi << 32) | lo);
}

// Workgroup barrier without the memory fence of __syncthreads(): the tile hand-off is
// ordered by explicit s_waitcnt vmcnt() on the direct-to-LDS loads instead.
__device__ __forceinline__ void wg_barrier() { __builtin_amdgcn_s_barrier(); }

template <int N>
using IC = std::integral_constant<int, N>;

// EPI selects the epilogue: kEpiBf16 / kEpiF32 store block_out and block_lse; kEpiMerge folds
// the block straight into fp32 accumulators with the Update of Sec. 3.1 (no block_out round trip).
template <int D, int EPI>
__global__ void __launch_bounds__(kThreads) block_attn_kernel(const AttnParams p) {
  constexpr int RB = 2 * D;
  constexpr int KS = D / 16;               // MFMA k-steps over the head dim
  constexpr int DB = D / 32;               // 32-wide d blocks of the output
  constexpr int CPR = D / 8;               // 16-byte chunks per row
  constexpr int BN = tile_keys<D>();       // keys per LDS tile
  constexpr int TILE_BYTES = BN * RB;
  constexpr int RPI = 1024 / RB;           // tile rows one wave-wide 16-byte load instruction covers
  constexpr int IPW = BN / RPI / kWaves;   // load instructions per wave, tile and tensor
  constexpr int NS = kRing;                // ring depth of the K and of the V tiles
  constexpr int SUB = 32;                  // keys per sub-tile (one MFMA row block)
  constexpr int NSUB = BN / SUB;           // sub-tiles (= steps) per tile
  static_assert(NSUB % 2 == 0, "the S / P register sets alternate with the step parity");
  static_assert(IPW >= 1, "tile too small for the workgroup");

  extern __shared__ __attribute__((aligned(1024))) char lds[];  // K ring | V ring

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in an SGPR
  const int ql = lane & 31, hf = lane >> 5;

  // which block step of the launch, batch, head and query tile this workgroup computes (wave-uniform)
  int qt, b, hq, hk, prob;
  decode_block(p, qt, b, hq, hk, prob);
  const AttnParams::Step sg = p.step[prob];
  const int64_t qseg = sg.q_seg, kseg = sg.k_seg;
  const bool causal = (p.causal_bits >> prob) & 1u;
  // A block step may attend a pair of K/V segments as one key range (the two segments a device of
  // the zigzag partition holds): keys 0 .. p.Sk-1 are segment kseg, keys p.Sk .. 2 p.Sk-1 segment
  // kseg2, which lies p.Sk positions later in the causal rule.  p.Sk is then a multiple of the
  // tile, so the tile stream changes segment between two tiles.
  const int kseg2 = sg.k_seg2;
  const int Sk = kseg2 >= 0 ? 2 * p.Sk : p.Sk;
  const int causal_off = kseg2 >= 0 ? p.Sk : p.causal_off;
  const int q0 = qt * kBM, qw0 = q0 + wave * 32;
  const int qrow = qw0 + ql;
  const int qrow_ld = min(qrow, p.Sq - 1);

  // Key range of this workgroup in tiles (needed to start the loads; the wave's own range follows below)
  const int q_last_wg = min(q0 + kBM, p.Sq) - 1;
  int kv_end = Sk;
  if (causal) kv_end = max(0, min(Sk, q_last_wg + causal_off + 1));
  const int n_tiles = (kv_end + BN - 1) / BN;

  const __bf16* kg = p.k + kseg * p.k_seg_elems + (int64_t)b * p.k_sb + (int64_t)hk * p.k_sh;
  const __bf16* vg = p.v + kseg * p.v_seg_elems + (int64_t)b * p.v_sb + (int64_t)hk * p.v_sh;

  // Direct global -> LDS staging (no VGPRs, no ds_write): one wave-wide instruction deposits
  // lane l's 16 bytes at lds_base + 16*l, i.e. RPI consecutive tile rows.  The swizzle is
  // applied on the global side: the lane that fills LDS position (row, pc) fetches the chunk
  // the swizzle maps there.  Addresses are a wave-uniform 64-bit tile base (SGPR pair) plus a
  // per-lane 32-bit byte offset that never changes, so issuing a tile costs no vector
  // arithmetic.  Rows past the end of the keys re-read the last key (they are masked later):
  // the last, possibly partial, tile has its own clamped offsets, and tiles beyond it (the
  // ring runs ahead of the loop) re-read the last tile.
  const int last_tile = (Sk - 1) / BN;
  unsigned k_off[IPW], v_off[IPW], k_off_last[IPW], v_off_last[IPW];
#pragma unroll
  for (int i = 0; i < IPW; i++) {
    const int row = (wave * IPW + i) * RPI + lane / CPR, pc = lane % CPR;
    const int kc = (pc ^ ((row / (256 / RB)) % CPR)) * 8;
    const int vswz = (D == 128) ? ((row & 3) << 1) : (row & 2);
    const int vc = ((((pc >> 1) ^ vswz) << 1) | (pc & 1)) * 8;
    const int row_last = max(0, min(row, Sk - 1 - last_tile * BN));
    k_off[i] = (unsigned)(((int64_t)row * p.k_ss + kc) * 2);
    v_off[i] = (unsigned)(((int64_t)row * p.v_ss + vc) * 2);
    k_off_last[i] = (unsigned)(((int64_t)row_last * p.k_ss + kc) * 2);
    v_off_last[i] = (unsigned)(((int64_t)row_last * p.v_ss + vc) * 2);
  }
  // Issued as inline asm: the compiler would otherwise treat every later LDS read as possibly
  // aliasing the in-flight load and drain vmcnt to 0 in front of it, serialising the pipeline;
  // here completion is waited for explicitly, one tile ahead of the first use.
  // The statement overwrites m0.  The compiler reserves m0 and sets it itself right before each of
  // its own uses (dynamic register indexing, LDS-direct forms), none of which this kernel
  // contains: every register-array index is a compile-time constant.  (m0 cannot be named in
  // the clobber list: it is a reserved register and the compiler rejects the promise.)
  const unsigned lds_base = (unsigned)(unsigned long)(lptr_t)lds;
  auto dma16 = [&](const __bf16* base, unsigned off, unsigned lds_off) __attribute__((always_inline)) {
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + lds_off);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0v), "v"(off), "s"(base) : "memory");
  };
  // Tiles are issued strictly in order, so the tile base is a running wave-uniform pointer that
  // stops advancing at the last tile (later issues re-read it with the clamped offsets).
  const __bf16* k_next = uniform_ptr(kg);
  const __bf16* v_next = uniform_ptr(vg);
  const int64_t k_tile_stride = (int64_t)BN * p.k_ss, v_tile_stride = (int64_t)BN * p.v_ss;
  int k_left = last_tile, v_left = last_tile;  // tiles still ahead of the pointer
  // with a segment pair: the pointer leaves the first segment when jump_left tiles are still ahead
  // (the counters run below zero when the ring issues past the last tile, so "never" is a value they cannot take)
  const int jump_left = kseg2 >= 0 ? last_tile + 1 - p.Sk / BN : 0x7fffffff;
  const int64_t k_jump = (int64_t)(kseg2 - (int)kseg - 1) * p.k_seg_elems, v_jump = (int64_t)(kseg2 - (int)kseg - 1) * p.v_seg_elems;
  auto issue_k = [&](int slot) __attribute__((always_inline)) {
    const bool last = k_left <= 0;
#pragma unroll
    for (int i = 0; i < IPW; i++)
      dma16(k_next, last ? k_off_last[i] : k_off[i], slot * TILE_BYTES + (wave * IPW + i) * 1024);
    k_next = uniform_ptr(k_next + (last ? 0 : k_tile_stride) + (k_left == jump_left ? k_jump : 0));
    k_left--;
  };
  auto issue_v = [&](int slot) __attribute__((always_inline)) {
    const bool last = v_left <= 0;
#pragma unroll
    for (int i = 0; i < IPW; i++)
      dma16(v_next, last ? v_off_last[i] : v_off[i], (NS + slot) * TILE_BYTES + (wave * IPW + i) * 1024);
    v_next = uniform_ptr(v_next + (last ? 0 : v_tile_stride) + (v_left == jump_left ? v_jump : 0));
    v_left--;
  };

  // ---- prologue: K_0..K_2, V_0, V_1 into the rings, then the Query fragments.  The loads go out
  // before the rest of the set-up (this wave's key range, LDS read addresses, cleared accumulators)
  // so that their latency, the longest wait of a workgroup's life, runs under that arithmetic.
  if (n_tiles > 0) {
    issue_k(0);
    issue_v(0);
    issue_k(1);
    issue_v(1);
    issue_k(2);
  }
  // Q^T fragments: lane (q, hf) holds Q[q][16*ks + 8*hf .. +7] for every k-step.
  bf16x8 qf[KS];
  {
    const __bf16* qp = p.q + qseg * p.q_seg_elems + (int64_t)b * p.q_sb + (int64_t)hq * p.q_sh + (int64_t)qrow_ld * p.q_ss;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * hf);
  }


  // Key range of this wave (in 32-key sub-tiles).
  int wave_kv_end = 0;
  if (qw0 < p.Sq) {
    wave_kv_end = Sk;
    if (causal) wave_kv_end = max(0, min(Sk, min(qw0 + 31, p.Sq - 1) + causal_off + 1));
  }
  const int jw = (wave_kv_end + SUB - 1) / SUB;  // sub-tiles this wave has visible keys in
  // wave-uniform loop bounds, forced into scalar registers so that every per-step test is one compare
  const int jw_first = __builtin_amdgcn_readfirstlane(jw);                            // last allowed step that opens a tile
  const int jw_in = __builtin_amdgcn_readfirstlane(min(jw, NSUB * n_tiles - 1));      // last allowed step inside a tile
  // a sub-tile starting at kstart needs masking iff kstart > kmask_from
  int kmask_from_v = Sk - SUB;
  if (causal) kmask_from_v = min(kmask_from_v, qw0 + causal_off - SUB + 1);
  const int kmask_from = __builtin_amdgcn_readfirstlane(kmask_from_v);

  // Per-lane LDS read offsets.
  // K operand: lane (key = ql, hf) reads chunk 2*ks + hf of row 32*kt + ql.
  // (All read addresses are LDS byte addresses with the ring base folded in, so that ring
  // slot and sub-tile offsets are instruction immediates.)
  unsigned k_rd[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) k_rd[ks] = lds_base + k_lds_off<D>(ql, 2 * ks + hf);
  // V^T operand through the transposing read: within each group of 16 lanes, lane i supplies
  // the address of row (i/4) of the 4-key group, 8-byte segment (i%4) of the 16 d's the
  // group covers, and receives the 4 keys of d = i.  (The V ring base is folded in.)
  unsigned v_rd[DB];
  {
    const int i16 = lane & 15, gq = (lane >> 4) & 1;
    const int row = 4 * hf + (i16 >> 2);
#pragma unroll
    for (int db = 0; db < DB; db++)
      v_rd[db] = lds_base + NS * TILE_BYTES + v_lds_off<D>(row, 4 * db + 2 * gq) + (i16 & 3) * 8;
  }

  f32x16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int i = 0; i < 16; i++) o_acc[db][i] = 0.f;
  // Largest sub-tile sum (16 weights of one row) the fast path accepts: 2^80.  The weights, their
  // bf16 roundings and the fp32 accumulators all carry an 8-bit exponent, so precision does not
  // depend on the magnitude; the cap only has to keep sums over a whole K/V chunk (up to 2^20 keys,
  // |v| up to 2^7) below 2^127.  A score must therefore exceed the reference by 55 (in natural
  // units) before the reference is moved: on all but pathological inputs that happens once, at
  // the row's first keys.
  constexpr float kSumCap = 0x1p80f;
  float m_ref = -INFINITY;  // exponent reference of this query, in raw (unscaled) score units
  float mc = 0.f;           // m_ref * c2 (0 while m_ref is -inf), kept alongside m_ref
  float l_run = 0.f;        // this lane's share of the running sum of exp
  float sum_cap = -1.f;     // largest sub-tile sum the fast path accepts; negative until m_ref is finite
  const float c2 = p.scale * 1.4426950408889634f;  // scale * log2(e)

  // ---- one step ---------------------------------------------------------------------
  // Step j (sub-tile j starts at key kstart) runs, as ONE interleaved instruction stream,
  //   MFMA : S_{j+1} = K_{j+1} Q^T   (NQK MFMAs, operands read from LDS by the PREVIOUS step)
  //          O += V_{j-1}^T P_{j-1}^T (NPV MFMAs, operands read from LDS during the QK half)
  //   LDS  : while the PV half runs, the K operands of step j+1 are read (into `pre`), so the
  //          read stream never stops at a step boundary or at a barrier (the tile they come
  //          from became visible a whole tile earlier)
  //   VALU : P_j = exp2((S_j - m_ref) * c2) and its row sums
  // QK goes first so that S_{j+1} is complete long before the next step's softmax reads it.
  //
  // P = exp2((s - m_ref) * scale*log2e) with an exponent reference m_ref that is NOT the
  // running maximum: any reference gives the same out = O/l and lse = m_ref*scale + ln l, so
  // the common path takes no row maximum.  Since P >= 0, a sub-tile sum <= kSumCap bounds
  // every P.  Only if some lane's sum exceeds the cap (or is NaN), or the reference is still
  // -inf, the slow path runs after the stream: row maximum, raise the reference, rescale l
  // and the O accumulators (which by then include P_{j-1}, consistently), redo the exponentials.
  // Row sums use the unrounded fp32 P: summing the bf16-rounded weights would cost up to
  // 2^-8 relative in l, more than the 1e-3 budget of lse for rows that see only a few keys.
  //
  // The stream is written out in the order it should issue - per MFMA: one operand's LDS
  // reads, the MFMA, and a slice of the softmax whose three dependent stages (fma, exp2,
  // add/convert) are staggered across consecutive slices - and pinned with sched_barrier.
  constexpr int NPV = 2 * DB, NQK = KS;
  static_assert(NPV == NQK, "the two halves of a step carry the same number of MFMAs");
  typedef const s16x4 __attribute__((address_space(3)))* lds_tr_ptr;
  typedef const bf16x8 __attribute__((address_space(3)))* lds_b128_ptr;
  auto load_k = [&](int ks, unsigned k_imm) __attribute__((always_inline)) -> bf16x8 {
    return *(lds_b128_ptr)(unsigned long)(k_rd[ks] + k_imm);
  };
  auto load_v = [&](int i, unsigned v_imm) __attribute__((always_inline)) -> bf16x8 {
    const int t = i / DB, db = i % DB;
    const unsigned a = v_rd[db] + v_imm + 16 * t * RB;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lds_tr_ptr)(unsigned long)a);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(lds_tr_ptr)(unsigned long)(a + 8 * RB));
    const bf16x4 lo_b = __builtin_bit_cast(bf16x4, lo), hi_b = __builtin_bit_cast(bf16x4, hi);
    return __builtin_shufflevector(lo_b, hi_b, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  bf16x8 pre[NQK];  // K operands of the next step's QK half, read one step ahead

  auto step = [&](int kstart, auto first_c, auto v_imm_c, auto k_imm_next_c, f32x16& s_in, f32x16& s_out,
                  bf16x8 (&p_in)[2], bf16x8 (&p_out)[2], auto inner_c) __attribute__((always_inline)) {
    constexpr bool FIRST = decltype(first_c)::value != 0;   // no previous sub-tile: QK half only
    constexpr bool INNER = decltype(inner_c)::value != 0;   // every key of the sub-tile is visible to every row: no mask test
    constexpr int n_mfma = FIRST ? NQK : NQK + NPV;
    constexpr int EPM = 16 / n_mfma;  // softmax elements handled per MFMA slice
    static_assert(16 % n_mfma == 0, "softmax elements must divide evenly over the MFMAs");
    constexpr unsigned v_imm = decltype(v_imm_c)::value, k_imm_next = decltype(k_imm_next_c)::value;

    if (!INNER && kstart > kmask_from) {  // some key of the sub-tile is past Sk or above this wave's first diagonal
      int limit = Sk - 1;
      if (causal) limit = min(limit, qrow + causal_off);
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const int key = kstart + 8 * (i >> 2) + 4 * hf + (i & 3);
        if (key > limit) s_in[i] = -INFINITY;
      }
    }

    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] = 0.f;
    bf16x8 pv_ops[NPV], nxt[NQK];
    float tq[16], ex[16];
    unsigned pw[8];
    float ps0 = 0.f, ps1 = 0.f;
    // Softmax element group g (EPM elements) passes stage A (fma) in slice g-2, stage B (exp2) in
    // slice g-1 and stage C (sum, convert) in slice g, so the stream ends with the last MFMA
    // and nothing but the sum check is left behind it.  The convert is opaque to the compiler,
    // which would otherwise sink all of them behind the slow-path branch.
    auto stage_a = [&](int g) __attribute__((always_inline)) {
#pragma unroll
      for (int k = 0; k < EPM; k++) tq[g * EPM + k] = __builtin_fmaf(s_in[g * EPM + k], c2, -mc);
    };
    auto stage_b = [&](int g) __attribute__((always_inline)) {
#pragma unroll
      for (int k = 0; k < EPM; k++) ex[g * EPM + k] = __builtin_amdgcn_exp2f(tq[g * EPM + k]);
    };
    auto stage_c = [&](int g) __attribute__((always_inline)) {
#pragma unroll
      for (int k = 0; k < EPM; k++) {
        const int e = g * EPM + k;
        if (e & 1) {
          ps1 += ex[e];
          asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pw[e >> 1]) : "v"(ex[e - 1]), "v"(ex[e]));
        } else {
          ps0 += ex[e];
        }
      }
    };
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < n_mfma; i++) {
      if (i < NQK) {
        if (FIRST) nxt[i] = load_k(i, k_imm_next);
        else pv_ops[i] = load_v(i, v_imm);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pre[i], qf[i], acc, 0, 0, 0);
      } else {
        const int j = i - NQK;
        nxt[j] = load_k(j, k_imm_next);
        o_acc[j % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pv_ops[j], p_in[j / DB], o_acc[j % DB], 0, 0, 0);
      }
      if (i == 0) {
        __builtin_amdgcn_sched_barrier(0);  // the first MFMA issues before any softmax work
        stage_a(0);
        stage_b(0);
        stage_a(1);
      }
      if (i + 1 < n_mfma) stage_b(i + 1);
      if (i + 2 < n_mfma) stage_a(i + 2);
      stage_c(i);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int h = 0; h < 2; h++) p_out[h] = __builtin_bit_cast(bf16x8, u32x4{pw[4 * h], pw[4 * h + 1], pw[4 * h + 2], pw[4 * h + 3]});
    float psum = ps0 + ps1;

    if (__any(!(psum <= sum_cap))) {   // sum_cap < 0 while m_ref is -inf, so that case is included
      float tmax = s_in[0];
#pragma unroll
      for (int i = 1; i < 16; i++) tmax = fmaxf(tmax, s_in[i]);
      tmax = half_swap_max(tmax);
      const float m_new = fmaxf(m_ref, tmax);
      const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c2);  // m_ref = -inf -> 0; equal -> 1
      const float a = (m_new == -INFINITY) ? 0.f : alpha;                 // (-inf) - (-inf) would be NaN
      l_run *= a;
#pragma unroll
      for (int db = 0; db < DB; db++)
#pragma unroll
        for (int i = 0; i < 16; i++) o_acc[db][i] *= a;
      m_ref = m_new;
      mc = (m_ref == -INFINITY) ? 0.f : m_ref * c2;
      sum_cap = (m_ref == -INFINITY) ? -1.f : kSumCap;
      const float mc2 = mc;
      float q0s = 0.f, q1s = 0.f;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[i], c2, -mc2));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_in[i + 1], c2, -mc2));
        p_out[i >> 3][i & 7] = (__bf16)p0;
        p_out[i >> 3][(i & 7) + 1] = (__bf16)p1;
        q0s += p0;
        q1s += p1;
      }
      psum = q0s + q1s;
    }
    l_run += psum;
    s_out = acc;
#pragma unroll
    for (int i = 0; i < NQK; i++) pre[i] = nxt[i];
  };

  // Tiles that are certain to lie before the last tile of the K/V segment (and not at the end of
  // the first segment of a pair) need neither the choice between the two offset sets nor the
  // end-of-stream and change-of-segment tests.
  auto issue_k_inner = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IPW; i++) dma16(k_next, k_off[i], slot * TILE_BYTES + (wave * IPW + i) * 1024);
    k_next = uniform_ptr(k_next + k_tile_stride);
    k_left--;
  };
  auto issue_v_inner = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IPW; i++) dma16(v_next, v_off[i], (NS + slot) * TILE_BYTES + (wave * IPW + i) * 1024);
    v_next = uniform_ptr(v_next + v_tile_stride);
    v_left--;
  };

#pragma unroll
  for (int ks = 0; ks < KS; ks++) asm volatile("" ::"v"(qf[ks]));  // Q is in registers before the loop
  __builtin_amdgcn_s_waitcnt(0);
  wg_barrier();  // B_0

  // Ring protocol.  Sub-tile j = NSUB*u + kt lives in tile u.  Step j reads the V operands of
  // sub-tile j-1 and the K operands of sub-tile j+2, so K_u is read in steps NSUB*u-2 ..
  // NSUB*(u+1)-3 and V_u in steps NSUB*u+1 .. NSUB*(u+1).  Barrier B_u sits in front of step
  // NSUB*u.  Right after B_w every wave issues the loads of K_{w+3} and V_{w+2} into the slots
  // K_{w-1} and V_{w-2} vacated (all waves are past step NSUB*w-1); they are first read two
  // tiles later, so each wave waits for its share (all but the newest 2*IPW loads, in order)
  // right before B_{w+2}.
  // S and P alternate between two register sets: even steps read sA / pB and write sB / pA,
  // odd steps the other way round, so no step has to copy its results.
  f32x16 sA, sB;
  bf16x8 pA[2], pB[2];
  constexpr unsigned SUBB = SUB * RB;  // bytes of one sub-tile inside a tile
  // Step NSUB*u + kt of the tile in ring slot `su` (previous tile in sp, next in sn).
  auto tile_step = [&](int u, auto su_c, auto kt_c, auto inner_c) __attribute__((always_inline)) {
    constexpr int su = decltype(su_c)::value, kt = decltype(kt_c)::value;
    constexpr bool INNER = decltype(inner_c)::value != 0;   // the step certainly runs and needs no mask
    constexpr int sp = (su + NS - 1) % NS, sn = (su + 1) % NS;
    constexpr unsigned v_imm = kt == 0 ? sp * TILE_BYTES + (NSUB - 1) * SUBB : su * TILE_BYTES + (kt - 1) * SUBB;
    constexpr unsigned k_imm = kt + 2 < NSUB ? su * TILE_BYTES + (kt + 2) * SUBB : sn * TILE_BYTES + (kt + 2 - NSUB) * SUBB;
    const int j = NSUB * u + kt;
    if (INNER || j <= (kt == 0 ? jw_first : jw_in)) {
      if (kt % 2 == 0) step(j * SUB, IC<0>{}, IC<(int)v_imm>{}, IC<(int)k_imm>{}, sA, sB, pB, pA, inner_c);
      else step(j * SUB, IC<0>{}, IC<(int)v_imm>{}, IC<(int)k_imm>{}, sB, sA, pA, pB, inner_c);
    }
  };
  if (n_tiles > 0) {
    issue_k(3 % NS);
    issue_v(2 % NS);
    if (jw > 0) {
      // S_0 = K_0[0:32] Q^T, plain (nothing to overlap with yet); operands of step 0 (sub-tile 1)
#pragma unroll
      for (int i = 0; i < 16; i++) sA[i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_k(ks, 0), qf[ks], sA, 0, 0, 0);
#pragma unroll
      for (int ks = 0; ks < KS; ks++) pre[ks] = load_k(ks, SUBB);
      // step 0: S_1 alongside the softmax of sub-tile 0 (no PV yet); prefetch the K operands of sub-tile 2
      constexpr unsigned k_imm0 = 2 < NSUB ? 2 * SUBB : 1 * TILE_BYTES;
      step(0, IC<1>{}, IC<0>{}, IC<(int)k_imm0>{}, sA, sB, pB, pA, IC<0>{});
      // the other steps of tile 0 (tiles 0 and 1 sit in ring slots 0 and 1)
      tile_step(0, IC<0>{}, IC<1>{}, IC<0>{});
      if constexpr (NSUB > 2) {
        tile_step(0, IC<0>{}, IC<2>{}, IC<0>{});
        tile_step(0, IC<0>{}, IC<3>{}, IC<0>{});
      }
    }
  }
  // tiles u = 1 .. n_tiles: steps NSUB*u .. NSUB*u + NSUB-1 (the last tile index only has its first
  // step, which folds in the PV product of the final sub-tile; its softmax sees only masked keys)
  auto tile_body = [&](int u, auto slot_c, auto inner_c) __attribute__((always_inline)) {   // slot_c = u % NS
    constexpr int su = decltype(slot_c)::value;
    constexpr bool INNER = decltype(inner_c)::value != 0;
    __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * IPW));  // vmcnt only
    wg_barrier();                                    // B_u
    if (INNER) {
      issue_k_inner((su + 3) % NS);   // K_{u+3}
      issue_v_inner((su + 2) % NS);   // V_{u+2}
    } else {
      issue_k((su + 3) % NS);
      issue_v((su + 2) % NS);
    }
    tile_step(u, slot_c, IC<0>{}, inner_c);
    tile_step(u, slot_c, IC<1>{}, inner_c);
    if constexpr (NSUB > 2) {
      tile_step(u, slot_c, IC<2>{}, inner_c);
      tile_step(u, slot_c, IC<3>{}, inner_c);
    }
  };
  static_assert(NSUB == 2 || NSUB == 4, "tile_body spells out 2 or 4 steps");
  // Inner tiles: every step of the tile runs in this wave without masking (all its keys are visible
  // to all of the wave's rows and lie inside the K/V segment) and the tiles it puts on their way
  // lie before the segment's last tile.  They take a tile body without the per-step tests; the
  // remaining tiles take the general one.  Both bodies hold the same barrier and the same number
  // of loads, so the waves of a workgroup may disagree about where the inner tiles end.
  const int j_inner = min(jw_in, kmask_from >= 0 ? kmask_from / SUB : -1) - (NSUB - 1);   // last step of the tile must pass both tests
  int u_inner = j_inner < 0 ? -1 : j_inner / NSUB;
  u_inner = __builtin_amdgcn_readfirstlane(min(u_inner, last_tile - 4));   // loads issued in tile u reach tile u + 3
  // tiles 1 .. 3 (tile 0 was the prologue)
  if (1 <= n_tiles) tile_body(1, IC<1 % NS>{}, IC<0>{});
  if (2 <= n_tiles) tile_body(2, IC<2 % NS>{}, IC<0>{});
  if (3 <= n_tiles) tile_body(3, IC<3 % NS>{}, IC<0>{});
  // Groups of NS tiles: first the groups of inner tiles, then general ones to the end.  With a pair
  // of segments the sequence runs twice: the groups whose loads (K_{u0+3} .. K_{u0+6}, V_{u0+2} ..
  // V_{u0+5}) include the last tile of the first segment, after which the stream changes segment,
  // take the general bodies, and the inner ones resume behind them.
  const int jump_tile = kseg2 >= 0 ? p.Sk / BN - 1 : 0x40000000;
  int u0 = NS;
  for (int half = 0; half < 2; half++) {
    const int inner_end = half == 0 ? min(u_inner, jump_tile - 4) : u_inner;
    const int general_end = half == 0 ? min(n_tiles, jump_tile - 2) : n_tiles;
    for (; u0 + NS - 1 <= inner_end; u0 += NS) {
      tile_body(u0, IC<0>{}, IC<1>{});
      tile_body(u0 + 1, IC<1 % NS>{}, IC<1>{});
      tile_body(u0 + 2, IC<2 % NS>{}, IC<1>{});
      tile_body(u0 + 3, IC<3 % NS>{}, IC<1>{});
    }
    for (; u0 <= general_end; u0 += NS) {
      tile_body(u0, IC<0>{}, IC<0>{});
      if (u0 + 1 <= n_tiles) tile_body(u0 + 1, IC<1 % NS>{}, IC<0>{});
      if (u0 + 2 <= n_tiles) tile_body(u0 + 2, IC<2 % NS>{}, IC<0>{});
      if (u0 + 3 <= n_tiles) tile_body(u0 + 3, IC<3 % NS>{}, IC<0>{});
    }
  }
  __builtin_amdgcn_s_waitcnt(0);  // no LDS write of this workgroup may still be in flight at exit

  // ---- epilogue: normalise, then store (or merge) with fully coalesced global accesses.
  // In the accumulator layout a lane holds 4-float pieces of ONE row, 32 bytes apart from its
  // neighbour's; each wave therefore transposes its 32 x D tile through a private, chunk-
  // swizzled LDS region (the rings are dead by now) and reads it back row-major, one 16-byte
  // chunk per lane, so that every global row is touched as one contiguous segment.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();  // every wave is done with the K/V rings and none of its loads is still landing
  constexpr int ROWB = 4 * D;                 // bytes of one fp32 output row
  constexpr int CPRF = D / 4;                 // 16-byte chunks per fp32 row = lanes per row when reading back
  constexpr int RPI_OUT = 64 / CPRF;          // rows one wave-wide access covers
  char* const my = lds + wave * (32 * ROWB);
  float* const my_w = reinterpret_cast<float*>(lds + kWaves * 32 * ROWB) + wave * 32;   // Update weight of each of the wave's rows
  int* const my_mode = reinterpret_cast<int*>(lds + kWaves * 32 * ROWB) + (kWaves + wave) * 32;   // and its case
  const float l_tot = half_swap_sum(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse_blk = l_tot > 0.f ? m_ref * p.scale + logf(l_tot) : -INFINITY;
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const int c = 8 * db + 2 * g + hf;  // 16-byte chunk of d = 32*db + 8*g + 4*hf
      f32x4 o;
#pragma unroll
      for (int r = 0; r < 4; r++) o[r] = o_acc[db][4 * g + r] * inv;
      *reinterpret_cast<f32x4*>(my + ql * ROWB + ((c ^ (ql & 15)) << 4)) = o;
    }
  if (EPI != kEpiMerge) __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the wave's own LDS writes are visible to all its lanes
  if (EPI != kEpiMerge && hf == 0 && qrow < p.Sq)
    p.lse[qseg * p.l_seg_elems + (int64_t)b * p.l_sb + (int64_t)hq * p.l_sh + (int64_t)qrow * p.l_ss] = lse_blk;
  const int rr = lane / CPRF, cc = lane % CPRF;
  constexpr int NIT = 32 / RPI_OUT;
  const int64_t o_bh = qseg * p.o_seg_elems + (int64_t)b * p.o_sb + (int64_t)hq * p.o_sh + 4 * cc;
  const int64_t l_bh = qseg * p.l_seg_elems + (int64_t)b * p.l_sb + (int64_t)hq * p.l_sh;
  if (EPI == kEpiMerge) {
    // Out, Lse <- Update(block_out, block_lse) on the accumulators p.out / p.lse.  All of the
    // wave's accumulator rows are fetched first (the O registers are free by now), so their
    // latencies overlap instead of each load waiting behind the previous row's store.  Rows
    // past Sq fetch the last valid row and are never stored.  The accumulator is touched once
    // per launch, so it is read and written past the caches (non-temporal).
    float* const acc_out = reinterpret_cast<float*>(p.out);
    f32x4 x[NIT];
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      const int grow = min(qw0 + it * RPI_OUT + rr, p.Sq - 1);
      x[it] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(acc_out + o_bh + (int64_t)grow * p.o_ss));
    }
    // The Update of a row is planned once, by the lanes that own the row in the accumulator layout
    // (its two exponentials and its logarithm would otherwise be evaluated in every lane that
    // blends a chunk of the row, 16 times per wave at D = 128), while the accumulator pieces are
    // on their way.  The same lane reads the row's old lse and writes the new one.
    {
      const int64_t l_at = l_bh + (int64_t)min(qrow, p.Sq - 1) * p.l_ss;
      const UpdatePlan plq = plan_update(p.lse[l_at], lse_blk);
      if (hf == 0) {
        my_w[ql] = plq.w;
        my_mode[ql] = plq.mode;
        if (qrow < p.Sq) p.lse[l_at] = plq.new_lse;
      }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the wave's own LDS writes are visible to all its lanes
    // All LDS reads of the wave's rows go out first (block piece, weight and case of its row), then
    // the pieces are blended and stored; the row address advances by a fixed step.
    f32x4 ov[NIT];
    UpdatePlan pl[NIT];
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      const int r = it * RPI_OUT + rr;
      ov[it] = *reinterpret_cast<const f32x4*>(my + r * ROWB + ((cc ^ (r & 15)) << 4));
      pl[it].w = my_w[r];
      pl[it].mode = my_mode[r];
      pl[it].new_lse = 0.f;
    }
    float* dst = acc_out + o_bh + (int64_t)(qw0 + rr) * p.o_ss;
    const int64_t dst_step = (int64_t)RPI_OUT * p.o_ss;
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      if (qw0 + it * RPI_OUT + rr < p.Sq) __builtin_nontemporal_store(apply_update(pl[it], x[it], ov[it]), reinterpret_cast<f32x4*>(dst));
      dst += dst_step;
    }
  } else if (EPI == kEpiF32) {
    f32x4 ov[NIT];
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      const int r = it * RPI_OUT + rr;
      ov[it] = *reinterpret_cast<const f32x4*>(my + r * ROWB + ((cc ^ (r & 15)) << 4));
    }
    float* dst = reinterpret_cast<float*>(p.out) + o_bh + (int64_t)(qw0 + rr) * p.o_ss;
    const int64_t dst_step = (int64_t)RPI_OUT * p.o_ss;
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      if (qw0 + it * RPI_OUT + rr < p.Sq) *reinterpret_cast<f32x4*>(dst) = ov[it];
      dst += dst_step;
    }
  } else {
    // bf16 rows are half as long: a lane converts two neighbouring chunks and stores 16 bytes
    constexpr int LPR = D / 8;          // lanes per bf16 row
    constexpr int RPI_B = 64 / LPR;     // rows one wave-wide store covers
    constexpr int NIT_B = 32 / RPI_B;
    const int rb = lane / LPR, cb = lane % LPR;
    const int64_t ob_bh = qseg * p.o_seg_elems + (int64_t)b * p.o_sb + (int64_t)hq * p.o_sh + 8 * cb;
    f32x4 o0[NIT_B], o1[NIT_B];
#pragma unroll
    for (int it = 0; it < NIT_B; it++) {
      const int r = it * RPI_B + rb;
      o0[it] = *reinterpret_cast<const f32x4*>(my + r * ROWB + (((2 * cb) ^ (r & 15)) << 4));
      o1[it] = *reinterpret_cast<const f32x4*>(my + r * ROWB + (((2 * cb + 1) ^ (r & 15)) << 4));
    }
    __bf16* dst = reinterpret_cast<__bf16*>(p.out) + ob_bh + (int64_t)(qw0 + rb) * p.o_ss;
    const int64_t dst_step = (int64_t)RPI_B * p.o_ss;
#pragma unroll
    for (int it = 0; it < NIT_B; it++) {
      bf16x8 ob;
#pragma unroll
      for (int k = 0; k < 4; k++) {
        ob[k] = (__bf16)o0[it][k];
        ob[4 + k] = (__bf16)o1[it][k];
      }
      if (qw0 + it * RPI_B + rb < p.Sq) *reinterpret_cast<bf16x8*>(dst) = ob;
      dst += dst_step;
    }
  }
}

template <int D, int EPI>
hipError_t launch_one(const AttnParams& p, dim3 grid, hipStream_t stream) {
  // K/V rings; the epilogue reuses them for kWaves private 32 x D fp32 tiles plus 32 lse each
  constexpr int ring_bytes = 2 * kRing * tile_keys<D>() * 2 * D;
  constexpr int epi_bytes = kWaves * 32 * 4 * D + 2 * kWaves * 32 * 4;
  constexpr int lds_bytes = ring_bytes > epi_bytes ? ring_bytes : epi_bytes;
  static_assert(lds_bytes <= 160 * 1024, "LDS budget of one CU exceeded");
  // Raising the dynamic-LDS limit is a per-function, per-device setting: done once for each
  // device this process launches on (the flags are atomics, a repeated set is harmless).
  constexpr int kMaxDevices = 64;
  static std::atomic<bool> attr_set[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices || !attr_set[dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&block_attn_kernel<D, EPI>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices) attr_set[dev].store(true, std::memory_order_release);
  }
  return launch_kernel(block_attn_kernel<D, EPI>, grid, dim3(kThreads), lds_bytes, stream, p);
}

}  // namespace

hipError_t launch_block_attn(const AttnParams& p, int D, int epilogue, hipStream_t stream) {
  const int64_t nbh = (int64_t)p.B * p.Hq;
  if (nbh * p.n_qtiles * p.n_prob == 0) return hipSuccess;
  if (p.n_qtiles > 65535 || p.n_prob > 65535) return hipErrorInvalidValue;   // grid y / z limits
  dim3 grid((unsigned)nbh, (unsigned)p.n_qtiles, (unsigned)p.n_prob);
  if (p.xcd_map == 2) grid = dim3(8u * (unsigned)p.n_qtiles, (unsigned)(nbh / 8), (unsigned)p.n_prob);
  if (D == 128) {
    if (epilogue == kEpiBf16) return launch_one<128, kEpiBf16>(p, grid, stream);
    if (epilogue == kEpiF32) return launch_one<128, kEpiF32>(p, grid, stream);
    return launch_one<128, kEpiMerge>(p, grid, stream);
  }
  if (epilogue == kEpiBf16) return launch_one<64, kEpiBf16>(p, grid, stream);
  if (epilogue == kEpiF32) return launch_one<64, kEpiF32>(p, grid, stream);
  return launch_one<64, kEpiMerge>(p, grid, stream);
}

int attn_rows_per_block() { return kBM; }

}  // namespace tr
