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
// Each thread group works on kRows rows (n_groups apart, so that neighbouring groups stay on
// neighbouring rows) and issues all their loads before the first dependent instruction, to
// keep enough bytes in flight per CU.
#ifndef TR_MERGE_ROWS
#define TR_MERGE_ROWS 2
#endif
#ifndef TR_MERGE_NT_STORE
#define TR_MERGE_NT_STORE 0
#endif
constexpr int kRows = TR_MERGE_ROWS;

template <bool BLK_BF16>
__global__ void __launch_bounds__(kMergeThreads) merge_kernel(const MergeParams p, int64_t n_rows, int64_t n_groups, int tpr_log2) {
  const int64_t gtid = (int64_t)blockIdx.x * kMergeThreads + threadIdx.x;
  const int64_t group = gtid >> tpr_log2;
  const int tpr = 1 << tpr_log2;
  const int t = (int)(gtid & (tpr - 1));
  if (group >= n_groups) return;

  int64_t ao[kRows], al[kRows], bo[kRows], bl[kRows];
  bool live[kRows];
  float a[kRows], bb[kRows];
#pragma unroll
  for (int r = 0; r < kRows; r++) {
    const int64_t row = group + r * n_groups;
    live[r] = row < n_rows;
    const int64_t rr = live[r] ? row : 0;
    if (p.contiguous) {
      ao[r] = rr * p.D; bo[r] = ao[r]; al[r] = rr; bl[r] = rr;
    } else {
      const int64_t s = rr % p.S, bh = rr / p.S;
      const int64_t h = bh % p.H, b = bh / p.H;
      ao[r] = b * p.ao_sb + h * p.ao_sh + s * p.ao_ss;
      al[r] = b * p.al_sb + h * p.al_sh + s * p.al_ss;
      bo[r] = b * p.bo_sb + h * p.bo_sh + s * p.bo_ss;
      bl[r] = b * p.bl_sb + h * p.bl_sh + s * p.bl_ss;
    }
    a[r] = p.acc_lse[al[r]];
    bb[r] = p.blk_lse[bl[r]];
  }

  for (int col = t * 4; col < p.D; col += tpr * 4) {
    f32x4 x[kRows], y[kRows];
#pragma unroll
    for (int r = 0; r < kRows; r++) {
      x[r] = *reinterpret_cast<const f32x4*>(p.acc_out + ao[r] + col);
      if (BLK_BF16) {
        const bf16x4 yb = __builtin_nontemporal_load(reinterpret_cast<const bf16x4*>(reinterpret_cast<const __bf16*>(p.blk_out) + bo[r] + col));
#pragma unroll
        for (int i = 0; i < 4; i++) y[r][i] = (float)yb[i];
      } else {
        y[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.blk_out) + bo[r] + col));
      }
    }
#pragma unroll
    for (int r = 0; r < kRows; r++) {
      if (!live[r]) continue;
      const f32x4 o = apply_update(plan_update(a[r], bb[r]), x[r], y[r]);
      f32x4* dst = reinterpret_cast<f32x4*>(p.acc_out + ao[r] + col);
#if TR_MERGE_NT_STORE
      __builtin_nontemporal_store(o, dst);
#else
      *dst = o;
#endif
    }
  }
  if (t == 0) {
#pragma unroll
    for (int r = 0; r < kRows; r++)
      if (live[r]) p.acc_lse[al[r]] = plan_update(a[r], bb[r]).new_lse;
  }
}

}  // namespace

hipError_t launch_merge(const MergeParams& p, bool blk_bf16, hipStream_t stream) {
  const int64_t n_rows = (int64_t)p.B * p.H * p.S;
  if (n_rows == 0 || p.D == 0) return hipSuccess;
  int tpr_log2 = 0;
  while ((1 << tpr_log2) < p.D / 4 && tpr_log2 < 6) tpr_log2++;
  const int64_t n_groups = (n_rows + kRows - 1) / kRows;
  const int64_t n_threads = n_groups << tpr_log2;
  const int64_t nblocks = (n_threads + kMergeThreads - 1) / kMergeThreads;
  dim3 grid((unsigned)nblocks), block(kMergeThreads);
  if (blk_bf16) hipLaunchKernelGGL((merge_kernel<true>), grid, block, 0, stream, p, n_rows, n_groups, tpr_log2);
  else hipLaunchKernelGGL((merge_kernel<false>), grid, block, 0, stream, p, n_rows, n_groups, tpr_log2);
  return hipGetLastError();
}

}  // namespace tr
