// Internal declarations shared by the translation units of libtokenring (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "tokenring.h"

namespace tr {

constexpr int kAttnGroupMax = 32;  // block steps one attention launch can carry

// Arguments of the block-attention kernel: raw pointers, element strides, sizes.
struct AttnParams {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  void* out;    // bf16 or fp32, [B,Hq,Sq,D]
  float* lse;   // [B,Hq,Sq]
  int64_t q_sb, q_sh, q_ss;
  int64_t k_sb, k_sh, k_ss;
  int64_t v_sb, v_sh, v_ss;
  int64_t o_sb, o_sh, o_ss;
  int64_t l_sb, l_sh, l_ss;
  int B, Hq, Hkv, Sq, Sk;
  int causal;     // 0: every key visible; 1: key c visible to query r iff c <= r + causal_off
  int causal_off; // q_pos0 - k_pos0, clamped so that r + causal_off cannot overflow
  float scale;    // softmax scale (natural units)
  int n_qtiles;   // ceil(Sq / rows per workgroup)
  int xcd_map;    // 1: place all query tiles of a K/V head on one XCD (grid x = batch*head, y = query tile); 2: the same with grid x = XCD + 8 * query tile, y = head within the XCD
  int gq;         // query heads per K/V head (Hq / Hkv)
  int gq_log2;    // log2(gq) if gq is a power of two, else -1
  // Several independent block steps of equal shape in one launch (the steps different "devices"
  // run in the same iteration of a schedule): problem g = blockIdx.z works on the
  // Query segment step[g].q_seg (q, out, lse advanced by q_seg * *_seg elements) and the K/V
  // segment step[g].k_seg, with the causal rule iff bit g of causal_bits is set.  k_seg2 >= 0 appends
  // a second K/V segment to the key range of step g (keys Sk .. 2 Sk - 1, lying Sk positions after
  // the first in the causal rule: with the bit set, query r sees key c iff c <= r + Sk); Sk must
  // then be a multiple of 128.  n_prob = 1 with step[0] = {0, 0, -1} and causal_bits = causal is
  // the plain single step.  (One 16-byte record per step: the workgroup fetches it with a single
  // scalar load at a wave-uniform offset; arrays of 16-bit entries would be read through the
  // vector memory path, a round trip to the memory-side caches in front of the first K/V load.)
  int n_prob;
  int blocks_per_prob;
  unsigned causal_bits;
  int64_t q_seg_elems, k_seg_elems, v_seg_elems, o_seg_elems, l_seg_elems;
  struct Step { int q_seg, k_seg, k_seg2, pad; } step[kAttnGroupMax];
};

// Arguments of the merge kernel.
struct MergeParams {
  float* acc_out;
  float* acc_lse;
  const void* blk_out;  // fp32 or bf16
  const float* blk_lse;
  int64_t ao_sb, ao_sh, ao_ss;
  int64_t al_sb, al_sh, al_ss;
  int64_t bo_sb, bo_sh, bo_ss;
  int64_t bl_sb, bl_sh, bl_ss;
  int B, H, S, D;
  int contiguous;  // 1: all four tensors are dense [B*H*S, D] / [B*H*S]
  int stream_acc;  // 1: the caller knows the accumulator is not touched again soon (access past the caches)
};

// Arguments of the n-ary merge kernel: up to kMergeNMax partial results with common strides.
constexpr int kMergeNMax = 16;
struct MergeNParams {
  float* out;        // fp32 [B,H,S,D], written (read as one more partial if accumulate)
  float* lse;        // fp32 [B,H,S]
  const void* blk_out[kMergeNMax];   // fp32 or bf16
  const float* blk_lse[kMergeNMax];
  int64_t o_sb, o_sh, o_ss;
  int64_t l_sb, l_sh, l_ss;
  int64_t bo_sb, bo_sh, bo_ss;
  int64_t bl_sb, bl_sh, bl_ss;
  int B, H, S, D;
  int n;           // number of partials
  int accumulate;  // 1: the old contents of out / lse take part as a further partial
  int contiguous;  // 1: every tensor is dense [B*H*S, D] / [B*H*S]
};

// Launchers (defined next to their kernels). They only enqueue; errors come back as hipError_t.
// epilogue: 0 = bf16 block_out, 1 = fp32 block_out, 2 = merge into the fp32 accumulators p.out / p.lse
hipError_t launch_block_attn(const AttnParams& p, int D, int epilogue, hipStream_t stream);
hipError_t launch_merge(const MergeParams& p, bool blk_bf16, hipStream_t stream);
hipError_t launch_merge_n(const MergeNParams& p, bool blk_bf16, hipStream_t stream);
int attn_rows_per_block();  // query rows one attention workgroup covers

// Events armed by tr_time_next_kernel for the calling thread; the next launch consumes them.
struct TimingEvents { hipEvent_t start, stop; };
TimingEvents take_timing_events();

#if defined(__HIPCC__)
// Every kernel of the library is launched through here.  With armed events the dispatch itself
// carries them, so they hold the kernel's own begin and end timestamps (no queue gaps).
template <typename Kernel, typename... Args>
inline hipError_t launch_kernel(Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, Args... args) {
  const TimingEvents ev = take_timing_events();
  if (ev.start != nullptr || ev.stop != nullptr) hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, ev.start, ev.stop, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
  return hipGetLastError();
}
#endif

#if defined(__HIPCC__)
// The Update of Sec. 3.1 for one row, shared by the merge kernel and the fused attention
// epilogue:  lse' = max + log1p(exp(-|lse - block_lse|)),  w = exp(block_lse - lse')
// (= sigmoid(block_lse - lse)),  out' = out + w (block_out - out).  The identity element
// (out = 0, lse = -inf) on either side is handled exactly and never produces NaN.
typedef float tr_f32x4 __attribute__((ext_vector_type(4)));
struct UpdatePlan {
  int mode;  // 0: blend with weight w; 1: both empty -> 0; 2: empty accumulator -> block; 3: empty block -> keep
  float w, new_lse;
};
__device__ __forceinline__ UpdatePlan plan_update(float lse_acc, float lse_blk) {
  UpdatePlan r;
  const float m = fmaxf(lse_acc, lse_blk);
  r.mode = 0;
  r.w = 0.f;
  if (m == -INFINITY) { r.mode = 1; r.new_lse = -INFINITY; }
  else if (lse_acc == -INFINITY) { r.mode = 2; r.new_lse = lse_blk; }   // the accumulator's out may be uninitialised
  else if (lse_blk == -INFINITY) { r.mode = 3; r.new_lse = lse_acc; }
  else {
    r.new_lse = m + log1pf(expf(-fabsf(lse_acc - lse_blk)));
    r.w = expf(lse_blk - r.new_lse);
  }
  return r;
}
// Branch-free: the blend is evaluated for every lane and bit masks made from the plan's case pick
// the result among blend, block, accumulator and zero, so whatever NaN or Inf an uninitialised
// side holds never reaches it and no lane waits for another's case.
__device__ __forceinline__ tr_f32x4 apply_update(const UpdatePlan& pl, tr_f32x4 acc, tr_f32x4 blk) {
  const unsigned m_blend = pl.mode == 0 ? 0xffffffffu : 0u;
  const unsigned m_blk = pl.mode == 2 ? 0xffffffffu : 0u;
  const unsigned m_acc = pl.mode == 3 ? 0xffffffffu : 0u;
  tr_f32x4 o;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const float a = acc[i], y = blk[i];   // scalars: a bit cast must not be applied to a vector element directly
    const float blend = __builtin_fmaf(pl.w, y - a, a);
    const unsigned bits = (m_blend & __builtin_bit_cast(unsigned, blend)) | (m_blk & __builtin_bit_cast(unsigned, y)) |
                          (m_acc & __builtin_bit_cast(unsigned, a));
    o[i] = __builtin_bit_cast(float, bits);
  }
  return o;
}
#endif

}  // namespace tr
