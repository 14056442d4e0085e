// Blockwise attention step for gfx950 (CDNA4): block_out, block_lse <- Attention(Q, K, V)
// of TokenRing's Algorithm 1 (Sec. 3.2), one Query chunk against one K/V chunk.
//
// Formulation.  Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// the A operand is a 32-key x 16-d slice of the K tile read from LDS, the B operand a
// 16-d x 32-query slice of Q^T held in registers for the whole kernel.  In the MFMA
// accumulator layout lane (q = lane%32, half = lane/32) then owns, for ONE query, the
// 16 keys {8g + 4*half + r}: the softmax row reductions are in-lane, plus a single
// cross-half exchange (v_permlane32_swap) for the running max.  The exponentiated tile
// P^T, rounded to bf16, is already in the B-operand layout of the second product
// O^T = V^T P^T; its A operand (32 d x 16 keys of V^T) comes from the row-major V tile in
// LDS through the transposing read ds_read_b64_tr_b16, with the key order inside each
// 16-key step permuted to match the accumulator layout of P^T (a contraction index may be
// permuted freely as long as both operands agree).  The O^T accumulator again has one
// query per lane, so rescaling and the final 1/l need no cross-lane traffic.
//
// Work split.  A workgroup has 8 waves (two per SIMD, so one wave's softmax VALU work
// overlaps the other's MFMAs); each wave owns 32 query rows, the workgroup 256.  K/V
// tiles of 64 keys are staged through double-buffered LDS, the K tile with a 16-byte XOR
// swizzle and the V tile with a 32-byte XOR swizzle that make the ds_read_b128 and the
// transposing reads bank-conflict free.
#include <type_traits>

#include "tr_internal.h"

namespace tr {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kBM = kWaves * 32;  // query rows per workgroup
constexpr int kBN = 64;           // keys per LDS tile

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

__device__ __forceinline__ void decode_block(const AttnParams& p, int bid, int& qt, int& bh) {
  const int nbh = p.B * p.Hq;
  int qt_rank;
  if (p.xcd_map) {
    // Workgroups are dealt round-robin to the 8 XCDs; give XCD x the K/V heads x, x+8, ...
    // and all query heads / query tiles that read them, so a head's K/V stays in one L2.
    const int G = p.Hq / p.Hkv;
    const int x = bid & 7, slot = bid >> 3;
    const int per_xcd = nbh >> 3;
    qt_rank = slot / per_xcd;
    const int hi = slot % per_xcd;
    const int kv = (hi / G) * 8 + x;
    bh = kv * G + hi % G;
  } else {
    qt_rank = bid / nbh;
    bh = bid % nbh;
  }
  qt = p.n_qtiles - 1 - qt_rank;  // late query tiles (most keys under a causal mask) first
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

template <int D, bool OUT_F32>
__global__ void __launch_bounds__(kThreads) block_attn_kernel(const AttnParams p) {
  constexpr int RB = 2 * D;
  constexpr int KS = D / 16;               // MFMA k-steps over the head dim
  constexpr int DB = D / 32;               // 32-wide d blocks of the output
  constexpr int CPR = D / 8;               // 16-byte chunks per row
  constexpr int TILE_BYTES = kBN * RB;
  constexpr int RPI = 1024 / RB;           // tile rows one wave-wide 16-byte load instruction covers
  constexpr int IPW = kBN / RPI / kWaves;  // load instructions per wave, tile and tensor
  constexpr int NS = 3;                    // ring depth of the K and of the V tiles
  static_assert(IPW >= 1, "tile too small for the workgroup");

  extern __shared__ __attribute__((aligned(1024))) char lds[];  // K ring | V ring

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in an SGPR
  const int ql = lane & 31, hf = lane >> 5;
  const int grp = wave >> 2;  // waves w and w+4 share a SIMD; the two groups run half a period apart

  int qt, bh;
  decode_block(p, blockIdx.x, qt, bh);
  const int b = bh / p.Hq, hq = bh % p.Hq, hk = hq / (p.Hq / p.Hkv);
  const int q0 = qt * kBM, qw0 = q0 + wave * 32;
  const int qrow = qw0 + ql;
  const int qrow_ld = min(qrow, p.Sq - 1);

  // Q^T fragments: lane (q, hf) holds Q[q][16*ks + 8*hf .. +7] for every k-step.
  bf16x8 qf[KS];
  {
    const __bf16* qp = p.q + (int64_t)b * p.q_sb + (int64_t)hq * p.q_sh + (int64_t)qrow_ld * p.q_ss;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * hf);
  }

  // Key range of this workgroup and of this wave.
  const int q_last_wg = min(q0 + kBM, p.Sq) - 1;
  int kv_end = p.Sk;
  if (p.causal) kv_end = max(0, min(p.Sk, q_last_wg + p.causal_off + 1));
  const int n_tiles = (kv_end + kBN - 1) / kBN;
  int wave_kv_end = 0;
  if (qw0 < p.Sq) {
    wave_kv_end = p.Sk;
    if (p.causal) wave_kv_end = max(0, min(p.Sk, min(qw0 + 31, p.Sq - 1) + p.causal_off + 1));
  }

  const __bf16* kg = p.k + (int64_t)b * p.k_sb + (int64_t)hk * p.k_sh;
  const __bf16* vg = p.v + (int64_t)b * p.v_sb + (int64_t)hk * p.v_sh;

  // Direct global -> LDS staging (no VGPRs, no ds_write): one wave-wide instruction deposits
  // lane l's 16 bytes at lds_base + 16*l, i.e. RPI consecutive tile rows.  The swizzle is
  // applied on the global side: the lane that fills LDS position (row, pc) fetches the chunk
  // the swizzle maps there.  Addresses are a wave-uniform 64-bit tile base (SGPR pair) plus a
  // per-lane 32-bit byte offset that never changes, so issuing a tile costs no vector
  // arithmetic.  Rows past the end of the keys re-read the last key (they are masked later):
  // the last, possibly partial, tile has its own clamped offsets, and tiles beyond it (the
  // ring runs ahead of the loop) re-read the last tile.
  const int last_tile = (p.Sk - 1) / kBN;
  unsigned k_off[IPW], v_off[IPW], k_off_last[IPW], v_off_last[IPW];
#pragma unroll
  for (int i = 0; i < IPW; i++) {
    const int row = (wave * IPW + i) * RPI + lane / CPR, pc = lane % CPR;
    const int kc = (pc ^ ((row / (256 / RB)) % CPR)) * 8;
    const int vswz = (D == 128) ? ((row & 3) << 1) : (row & 2);
    const int vc = ((((pc >> 1) ^ vswz) << 1) | (pc & 1)) * 8;
    const int row_last = max(0, min(row, p.Sk - 1 - last_tile * kBN));
    k_off[i] = (unsigned)(((int64_t)row * p.k_ss + kc) * 2);
    v_off[i] = (unsigned)(((int64_t)row * p.v_ss + vc) * 2);
    k_off_last[i] = (unsigned)(((int64_t)row_last * p.k_ss + kc) * 2);
    v_off_last[i] = (unsigned)(((int64_t)row_last * p.v_ss + vc) * 2);
  }
  // Issued as inline asm: the compiler would otherwise treat every later LDS read as possibly
  // aliasing the in-flight load and drain vmcnt to 0 in front of it, serialising the pipeline;
  // here completion is waited for explicitly, one ring slot ahead of its use.
  const unsigned lds_base = (unsigned)(unsigned long)(lptr_t)lds;
  auto dma16 = [&](const __bf16* base, unsigned off, unsigned lds_off) __attribute__((always_inline)) {
    const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + lds_off);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0v), "v"(off), "s"(base) : "memory");
  };
  auto issue_k = [&](int tile, int slot) __attribute__((always_inline)) {
    const int t = min(tile, last_tile);
    const __bf16* base = uniform_ptr(kg + (int64_t)t * kBN * p.k_ss);
#pragma unroll
    for (int i = 0; i < IPW; i++)
      dma16(base, t == last_tile ? k_off_last[i] : k_off[i], slot * TILE_BYTES + (wave * IPW + i) * 1024);
  };
  auto issue_v = [&](int tile, int slot) __attribute__((always_inline)) {
    const int t = min(tile, last_tile);
    const __bf16* base = uniform_ptr(vg + (int64_t)t * kBN * p.v_ss);
#pragma unroll
    for (int i = 0; i < IPW; i++)
      dma16(base, t == last_tile ? v_off_last[i] : v_off[i], (NS + slot) * TILE_BYTES + (wave * IPW + i) * 1024);
  };

  // Per-lane LDS read offsets.
  // K operand: lane (key = ql, hf) reads chunk 2*ks + hf of row 32*kt + ql.
  int k_rd[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) k_rd[ks] = k_lds_off<D>(ql, 2 * ks + hf);
  // V^T operand through the transposing read: within each group of 16 lanes, lane i supplies
  // the address of row (i/4) of the 4-key group, 8-byte segment (i%4) of the 16 d's the
  // group covers, and receives the 4 keys of d = i.
  int v_rd[DB];
  {
    const int i16 = lane & 15, gq = (lane >> 4) & 1;
    const int row = 4 * hf + (i16 >> 2);
#pragma unroll
    for (int db = 0; db < DB; db++) v_rd[db] = NS * TILE_BYTES + v_lds_off<D>(row, 4 * db + 2 * gq) + (i16 & 3) * 8;
  }

  f32x16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int i = 0; i < 16; i++) o_acc[db][i] = 0.f;
  float m_ref = -INFINITY;  // exponent reference of this query, in raw (unscaled) score units
  float l_run = 0.f;        // this lane's share of the running sum of exp
  const float c2 = p.scale * 1.4426950408889634f;  // scale * log2(e)

  f32x16 s[2];       // S^T of the tile the next softmax consumes
  bf16x8 pb[2][2];   // P^T of the tile the next PV product consumes

  // The X phase as one software-pipelined MFMA stream.  Operand i is, for i < NPV, the V^T
  // fragment (kt, t, db) of the PV product (two transposing 64-bit LDS reads) and, for
  // i >= NPV, the K fragment (ks, kt) of the next tile's QK^T (one 128-bit LDS read).  Reads
  // run PF operands ahead of the MFMAs that consume them so that LDS latency is covered by
  // matrix work; sched_group_barrier pins that interleaving in the instruction scheduler.
  constexpr int NPV = 4 * DB, NQK = 2 * KS, PF = 6;
  auto load_op = [&](int i, const char* vb, const char* kb) __attribute__((always_inline)) -> bf16x8 {
    if (i < NPV) {
      const int kt = i / (2 * DB), t = (i / DB) % 2, db = i % DB;
      const char* vp = vb + (32 * kt + 16 * t) * RB + v_rd[db];
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(vp + 8 * RB));
      const bf16x4 lo_b = __builtin_bit_cast(bf16x4, lo), hi_b = __builtin_bit_cast(bf16x4, hi);
      return __builtin_shufflevector(lo_b, hi_b, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    const int j = i - NPV, ks = j / 2, kt = j % 2;
    return *reinterpret_cast<const bf16x8*>(kb + kt * 32 * RB + k_rd[ks]);
  };
  auto do_mfma = [&](int i, bf16x8 a) __attribute__((always_inline)) {
    if (i < NPV) {
      const int kt = i / (2 * DB), t = (i / DB) % 2, db = i % DB;
      o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kt][t], o_acc[db], 0, 0, 0);
    } else {
      const int j = i - NPV, ks = j / 2, kt = j % 2;
      s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kt], 0, 0, 0);
    }
  };
  // ops [first, last) of the stream: PV only, QK only, or both back to back
  auto mfma_stream = [&](auto first_c, auto last_c, auto v_slot_c, auto k_slot_c) __attribute__((always_inline)) {
    constexpr int first = decltype(first_c)::value, last = decltype(last_c)::value;
    // ring slots are compile-time so that every LDS read offset is an instruction immediate
    const char* vb = lds + decltype(v_slot_c)::value * TILE_BYTES;  // v_rd already includes the V ring base
    const char* kb = lds + decltype(k_slot_c)::value * TILE_BYTES;
    if (last > NPV) {
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int i = 0; i < 16; i++) s[kt][i] = 0.f;
    }
    bf16x8 ops[NPV + NQK];
#pragma unroll
    for (int i = first; i < first + PF && i < last; i++) ops[i] = load_op(i, vb, kb);
#pragma unroll
    for (int i = first; i < last; i++) {
      if (i + PF < last) ops[i + PF] = load_op(i + PF, vb, kb);
      do_mfma(i, ops[i]);
    }
    // scheduling pipeline: prologue reads, then per MFMA the reads issued PF operands ahead
#pragma unroll
    for (int i = first; i < first + PF && i < last; i++) {
      if (i < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
#pragma unroll
    for (int i = first; i < last; i++) {
      if (i + PF < last) {
        if (i + PF < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
  };
  using std::integral_constant;
  using C0 = integral_constant<int, 0>;
  auto qk = [&](auto k_slot_c) __attribute__((always_inline)) { mfma_stream(integral_constant<int, NPV>{}, integral_constant<int, NPV + NQK>{}, C0{}, k_slot_c); };
  auto pv_qk = [&](auto v_slot_c, auto k_slot_c) __attribute__((always_inline)) {
    mfma_stream(C0{}, integral_constant<int, NPV + NQK>{}, v_slot_c, k_slot_c);
  };
  // Online softmax of s (tile starting at key kstart): fills pb, updates m_ref, l_run, O.
  // P = exp2((s - m_ref) * scale*log2e) with an exponent reference m_ref that is NOT the
  // running maximum: any reference gives the same out = O/l and lse = m_ref*scale + ln l, so
  // the common path takes no row maximum at all.  It exponentiates against the current
  // reference and sums; since P >= 0, a tile sum <= kSumCap bounds every P of the tile.  Only
  // if some lane's sum exceeds the cap (or is NaN from inf - inf), or the reference is still
  // -inf, the slow path runs: take the row maximum, raise the reference, rescale l and the
  // O accumulators, and redo the exponentials.  Row sums use the unrounded fp32 P: summing
  // the bf16-rounded weights would cost up to 2^-9 relative in l, more than the 1e-3 budget of
  // lse for rows that see only a few keys.
  constexpr float kSumCap = 65536.f;
  auto softmax = [&](int kstart) __attribute__((always_inline)) {
    const bool need_mask = (kstart + kBN > p.Sk) || (p.causal && (kstart + kBN - 1 > qw0 + p.causal_off));
    if (need_mask) {
      int limit = p.Sk - 1;
      if (p.causal) limit = min(limit, qrow + p.causal_off);
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
          const int key = kstart + 32 * kt + 8 * (i >> 2) + 4 * hf + (i & 3);
          if (key > limit) s[kt][i] = -INFINITY;
        }
    }
    auto exp_tile = [&]() __attribute__((always_inline)) -> float {
      const float mc = (m_ref == -INFINITY) ? 0.f : m_ref * c2;
      float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][i], c2, -mc));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][i + 1], c2, -mc));
          pb[kt][i >> 3][i & 7] = (__bf16)p0;
          pb[kt][i >> 3][(i & 7) + 1] = (__bf16)p1;
          ps0 += p0;
          ps1 += p1;
        }
      return ps0 + ps1;
    };
    float psum = exp_tile();
    if (__any(!(psum <= kSumCap) || m_ref == -INFINITY)) {
      float tmax = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int i = 0; i < 16; i++) tmax = fmaxf(tmax, s[kt][i]);
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
      psum = exp_tile();
    }
    l_run += psum;
  };

  // ---- prologue: K_0, K_1, K_2, V_0, V_1 into the rings; S_0 = K_0 Q^T
  if (n_tiles > 0) {
    issue_k(0, 0);
    issue_v(0, 0);
    issue_k(1, 1);
    issue_v(1, 1);
    issue_k(2, 2);
  }
#pragma unroll
  for (int ks = 0; ks < KS; ks++) asm volatile("" ::"v"(qf[ks]));  // Q is in registers before the loop
  __builtin_amdgcn_s_waitcnt(0);
  wg_barrier();
  if (0 < wave_kv_end) qk(C0{});
  if (grp == 1) wg_barrier();  // group 1 runs one phase behind group 0

  // Steady state, two phases per tile separated by workgroup barriers:
  //   Y(u): softmax of S_u (VALU)            X(u): O += V_u P_u, then S_{u+1} = K_{u+1} Q^T (MFMA)
  // Group 0 is in X while group 1 is in Y and vice versa, so each SIMD always has one wave
  // feeding the MFMA pipe and one doing VALU work.  At the start of group 0's X(u) (= group
  // 1's Y(u)) every wave issues the loads of K_{u+3} and V_{u+2} into the ring slots that
  // K_u and V_{u-1} just vacated; they are waited for (in order, all but the newest 2*IPW)
  // right before the barrier that precedes their first use two tiles later.
  auto tile_step = [&](int u, auto vs_c) __attribute__((always_inline)) {   // vs_c = u % NS: ring slot of V_u; K_{u+1} sits in the next one
    constexpr int vs = decltype(vs_c)::value, ks = (vs + 1) % NS;
    constexpr int ld_k_slot = vs, ld_v_slot = (vs + 2) % NS;  // slots of K_{u+3} (was K_u) and V_{u+2} (was V_{u-1})
    const bool act = u * kBN < wave_kv_end;
    // ---- Y(u)
    if (grp == 1) {
      issue_k(u + 3, ld_k_slot);
      issue_v(u + 2, ld_v_slot);
    }
    if (act) softmax(u * kBN);
    if (grp == 0) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * IPW) /* vmcnt only */);
    wg_barrier();
    // ---- X(u)
    if (grp == 0) {
      issue_k(u + 3, ld_k_slot);
      issue_v(u + 2, ld_v_slot);
    }
    // One code path only: when tile u+1 is not needed by this wave (or does not exist) the QK
    // half still runs on whatever the ring slot holds and its result is never used.  Separate
    // PV-only / PV+QK branches would make the compiler keep two copies of the O accumulators.
    if (act) pv_qk(integral_constant<int, vs>{}, integral_constant<int, ks>{});
    if (grp == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * IPW));
    wg_barrier();
  };
  for (int u = 0; u < n_tiles; u += NS) {
    tile_step(u, integral_constant<int, 0>{});
    if (u + 1 < n_tiles) tile_step(u + 1, integral_constant<int, 1>{});
    if (u + 2 < n_tiles) tile_step(u + 2, integral_constant<int, 2>{});
  }
  if (grp == 0) wg_barrier();
  __builtin_amdgcn_s_waitcnt(0);  // no LDS write of this workgroup may still be in flight at exit

  // ---- epilogue: normalise, write block_out and block_lse
  const float l_tot = half_swap_sum(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (qrow < p.Sq) {
    if (hf == 0) {
      const float lse = l_tot > 0.f ? m_ref * p.scale + logf(l_tot) : -INFINITY;
      p.lse[(int64_t)b * p.l_sb + (int64_t)hq * p.l_sh + (int64_t)qrow * p.l_ss] = lse;
    }
    const int64_t obase = (int64_t)b * p.o_sb + (int64_t)hq * p.o_sh + (int64_t)qrow * p.o_ss;
#pragma unroll
    for (int db = 0; db < DB; db++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const int d0 = 32 * db + 8 * g + 4 * hf;
        f32x4 o;
#pragma unroll
        for (int r = 0; r < 4; r++) o[r] = o_acc[db][4 * g + r] * inv;
        if (OUT_F32) {
          *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + obase + d0) = o;
        } else {
          bf16x4 ob;
#pragma unroll
          for (int r = 0; r < 4; r++) ob[r] = (__bf16)o[r];
          *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p.out) + obase + d0) = ob;
        }
      }
  }
}

template <int D, bool OUT_F32>
hipError_t launch_one(const AttnParams& p, dim3 grid, hipStream_t stream) {
  constexpr int lds_bytes = 2 * 3 * kBN * 2 * D;
  static bool attr_set = false;  // raising the dynamic-LDS limit is a per-function, per-process setting
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&block_attn_kernel<D, OUT_F32>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((block_attn_kernel<D, OUT_F32>), grid, dim3(kThreads), lds_bytes, stream, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_block_attn(const AttnParams& p, int D, bool out_f32, hipStream_t stream) {
  const int64_t nblocks = (int64_t)p.n_qtiles * p.B * p.Hq;
  if (nblocks == 0) return hipSuccess;
  dim3 grid((unsigned)nblocks);
  if (D == 128) return out_f32 ? launch_one<128, true>(p, grid, stream) : launch_one<128, false>(p, grid, stream);
  return out_f32 ? launch_one<64, true>(p, grid, stream) : launch_one<64, false>(p, grid, stream);
}

int attn_rows_per_block() { return kBM; }

}  // namespace tr
