// The Update step of TokenRing (the two equations of Sec. 3.1), in place on fp32 accumulators:
//   out <- out - sigmoid(block_lse - lse) * (out - block_out)
//   lse <- lse - ln(sigmoid(lse - block_lse))
// evaluated as lse' = max(lse, block_lse) + log1p(exp(-|lse - block_lse|)) and
// w = exp(block_lse - lse') = sigmoid(block_lse - lse), out' = out + w (block_out - out),
// which is the same function wherever the printed form is finite and keeps the identity
// element (out = 0, lse = -inf) exact on either side.
//
// Pure streaming kernel: per output element it reads 2 values and writes 1, a few flops.
#include "tr_internal.h"

namespace tr {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int kMergeThreads = 256;

// One row is always handled inside a single wavefront: `tpr` (a power of two <= 64) threads
// share a row and stride over its columns.  Every thread of the row reads the old lse before
// thread 0 of the row overwrites it, which program order within one wave guarantees.
// Neighbouring thread groups take neighbouring rows, so a wave touches one contiguous span of
// each stream.  (Giving a group several rows, near or far apart, measured slower.)
template <bool BLK_BF16>
__global__ void __launch_bounds__(kMergeThreads) merge_kernel(const MergeParams p, int64_t n_rows, int tpr_log2) {
  const int64_t gtid = (int64_t)blockIdx.x * kMergeThreads + threadIdx.x;
  const int64_t row = gtid >> tpr_log2;
  const int tpr = 1 << tpr_log2;
  const int t = (int)(gtid & (tpr - 1));
  if (row >= n_rows) return;

  int64_t ao, al, bo, bl;
  if (p.contiguous) {
    ao = row * p.D; bo = ao; al = row; bl = row;
  } else {
    const int64_t s = row % p.S, bh = row / p.S;
    const int64_t h = bh % p.H, b = bh / p.H;
    ao = b * p.ao_sb + h * p.ao_sh + s * p.ao_ss;
    al = b * p.al_sb + h * p.al_sh + s * p.al_ss;
    bo = b * p.bo_sb + h * p.bo_sh + s * p.bo_ss;
    bl = b * p.bl_sb + h * p.bl_sh + s * p.bl_ss;
  }
  const UpdatePlan plan = plan_update(p.acc_lse[al], p.blk_lse[bl]);

  for (int col = t * 4; col < p.D; col += tpr * 4) {
    const f32x4 x = *reinterpret_cast<const f32x4*>(p.acc_out + ao + col);
    f32x4 y;
    if (BLK_BF16) {
      const bf16x4 yb = __builtin_nontemporal_load(reinterpret_cast<const bf16x4*>(reinterpret_cast<const __bf16*>(p.blk_out) + bo + col));
#pragma unroll
      for (int i = 0; i < 4; i++) y[i] = (float)yb[i];
    } else {
      y = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.blk_out) + bo + col));
    }
    *reinterpret_cast<f32x4*>(p.acc_out + ao + col) = apply_update(plan, x, y);
  }
  if (t == 0) p.acc_lse[al] = plan.new_lse;
}

}  // namespace

hipError_t launch_merge(const MergeParams& p, bool blk_bf16, hipStream_t stream) {
  const int64_t n_rows = (int64_t)p.B * p.H * p.S;
  if (n_rows == 0 || p.D == 0) return hipSuccess;
  int tpr_log2 = 0;
  while ((1 << tpr_log2) < p.D / 4 && tpr_log2 < 6) tpr_log2++;
  const int64_t n_threads = n_rows << tpr_log2;
  const int64_t nblocks = (n_threads + kMergeThreads - 1) / kMergeThreads;
  dim3 grid((unsigned)nblocks), block(kMergeThreads);
  if (blk_bf16) return launch_kernel(merge_kernel<true>, grid, block, 0, stream, p, n_rows, tpr_log2);
  return launch_kernel(merge_kernel<false>, grid, block, 0, stream, p, n_rows, tpr_log2);
}

}  // namespace tr
