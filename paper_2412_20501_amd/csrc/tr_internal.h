// Internal declarations shared by the translation units of libtokenring (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tokenring.h"

namespace tr {

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
  int xcd_map;    // 1: place all query tiles of a K/V head on one XCD
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
};

// Launchers (defined next to their kernels). They only enqueue; errors come back as hipError_t.
hipError_t launch_block_attn(const AttnParams& p, int D, bool out_f32, hipStream_t stream);
hipError_t launch_merge(const MergeParams& p, bool blk_bf16, hipStream_t stream);
int attn_rows_per_block();  // query rows one attention workgroup covers

}  // namespace tr
