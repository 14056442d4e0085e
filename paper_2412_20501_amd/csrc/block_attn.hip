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

template <int D, bool OUT_F32>
__global__ void __launch_bounds__(kThreads) block_attn_kernel(const AttnParams p) {
  constexpr int RB = 2 * D;
  constexpr int KS = D / 16;               // MFMA k-steps over the head dim
  constexpr int DB = D / 32;               // 32-wide d blocks of the output
  constexpr int CPR = D / 8;               // 16-byte chunks per row
  constexpr int CH = kBN * CPR / kThreads; // chunks each thread stages per tile and tensor
  constexpr int TILE_BYTES = kBN * RB;
  static_assert(CH >= 1, "tile too small for the workgroup");

  __shared__ __attribute__((aligned(256))) char lds[4 * TILE_BYTES];  // K0 K1 V0 V1
  char* const k_lds = lds;
  char* const v_lds = lds + 2 * TILE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ql = lane & 31, hf = lane >> 5;

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

  // Staging: thread handles chunks tid, tid + 512, ... of the tile.
  bf16x8 kreg[CH], vreg[CH];
  auto load_tile = [&](int tile) {
#pragma unroll
    for (int i = 0; i < CH; i++) {
      const int cidx = tid + kThreads * i;
      const int row = cidx / CPR, c = cidx % CPR;
      const int key = min(tile * kBN + row, p.Sk - 1);
      kreg[i] = *reinterpret_cast<const bf16x8*>(kg + (int64_t)key * p.k_ss + c * 8);
      vreg[i] = *reinterpret_cast<const bf16x8*>(vg + (int64_t)key * p.v_ss + c * 8);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CH; i++) {
      const int cidx = tid + kThreads * i;
      const int row = cidx / CPR, c = cidx % CPR;
      *reinterpret_cast<bf16x8*>(k_lds + buf * TILE_BYTES + k_lds_off<D>(row, c)) = kreg[i];
      *reinterpret_cast<bf16x8*>(v_lds + buf * TILE_BYTES + v_lds_off<D>(row, c)) = vreg[i];
    }
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
    for (int db = 0; db < DB; db++) v_rd[db] = v_lds_off<D>(row, 4 * db + 2 * gq) + (i16 & 3) * 8;
  }

  f32x16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int i = 0; i < 16; i++) o_acc[db][i] = 0.f;
  float m_run = -INFINITY;  // running max of the raw (unscaled) scores of this query
  float l_run = 0.f;        // this lane's share of the running sum of exp
  const float c2 = p.scale * 1.4426950408889634f;  // scale * log2(e)

  if (n_tiles > 0) {
    load_tile(0);
    store_tile(0);
  }
  __syncthreads();

  for (int tile = 0; tile < n_tiles; tile++) {
    const int buf = tile & 1;
    const bool has_next = tile + 1 < n_tiles;
    if (has_next) load_tile(tile + 1);

    const int kstart = tile * kBN;
    if (kstart < wave_kv_end) {
      // ---- S^T = K Q^T
      f32x16 s[2];
#pragma unroll
      for (int kt = 0; kt < 2; kt++) {
#pragma unroll
        for (int i = 0; i < 16; i++) s[kt][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(k_lds + buf * TILE_BYTES + kt * 32 * RB + k_rd[ks]);
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kt], 0, 0, 0);
        }
      }
      // ---- mask (only tiles that cross the causal boundary or the end of the keys)
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
      // ---- online softmax
      float tmax = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int i = 0; i < 16; i++) tmax = fmaxf(tmax, s[kt][i]);
      tmax = half_swap_max(tmax);
      const float m_new = fmaxf(m_run, tmax);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float mc = m_safe * c2;
      const float alpha = __builtin_amdgcn_exp2f(m_run * c2 - mc);
      float psum = 0.f;
      bf16x8 pb[2][2];
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
          const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][i], c2, -mc));
          psum += pe;
          pb[kt][i >> 3][i & 7] = (__bf16)pe;
        }
      l_run = l_run * alpha + psum;
      m_run = m_new;
      if (__any(alpha != 1.f)) {
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
          for (int i = 0; i < 16; i++) o_acc[db][i] *= alpha;
      }
      // ---- O^T += V^T P^T
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int t = 0; t < 2; t++)
#pragma unroll
          for (int db = 0; db < DB; db++) {
            const char* vp = v_lds + buf * TILE_BYTES + (32 * kt + 16 * t) * RB + v_rd[db];
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(vp));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(vp + 8 * RB));
            const bf16x4 lo_b = __builtin_bit_cast(bf16x4, lo), hi_b = __builtin_bit_cast(bf16x4, hi);
            const bf16x8 a = __builtin_shufflevector(lo_b, hi_b, 0, 1, 2, 3, 4, 5, 6, 7);
            o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kt][t], o_acc[db], 0, 0, 0);
          }
    }

    if (has_next) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: normalise, write block_out and block_lse
  const float l_tot = half_swap_sum(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (qrow < p.Sq) {
    if (hf == 0) {
      const float lse = l_tot > 0.f ? m_run * p.scale + logf(l_tot) : -INFINITY;
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

}  // namespace

hipError_t launch_block_attn(const AttnParams& p, int D, bool out_f32, hipStream_t stream) {
  const int64_t nblocks = (int64_t)p.n_qtiles * p.B * p.Hq;
  if (nblocks == 0) return hipSuccess;
  dim3 grid((unsigned)nblocks), block(kThreads);
  if (D == 128) {
    if (out_f32) hipLaunchKernelGGL((block_attn_kernel<128, true>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((block_attn_kernel<128, false>), grid, block, 0, stream, p);
  } else {
    if (out_f32) hipLaunchKernelGGL((block_attn_kernel<64, true>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((block_attn_kernel<64, false>), grid, block, 0, stream, p);
  }
  return hipGetLastError();
}

int attn_rows_per_block() { return kBM; }

}  // namespace tr
