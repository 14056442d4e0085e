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

constexpr int kMergeThreads = 512;

// Accumulators beyond this size cannot stay in the chip's 256 MiB memory-side cache between two
// Updates, so they are read and written past the caches (non-temporal): measured on the 512 MiB
// merge-only workload, 5.8 -> 6.5 TB/s.  A smaller accumulator that is updated again soon (one
// device's Out between two iterations of Algorithm 1) is served from that cache and keeps the
// ordinary policy, which is the faster one there.
constexpr int64_t kStreamAccBytes = (int64_t)128 << 20;

// One row is always handled inside a single wavefront: `tpr` (a power of two <= 64) threads
// share a row; a thread takes the 16-byte column chunks t and t + tpr (then t + 2 tpr, ... for
// long rows), both loads of a pair issued before the first store, so the lse arithmetic of a
// row (two exponentials and a logarithm per thread) is spread over 32 bytes of every stream.
// Every thread of the row reads the old lse before thread 0 of the row overwrites it, which
// program order within one wave guarantees.  Neighbouring thread groups take neighbouring
// rows, so a wave touches one contiguous span of each stream.  (Giving a group several rows,
// near or far apart, measured slower; so did one or four chunks per thread.)
template <bool BLK_BF16, bool STREAM_ACC>
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

  auto load_acc = [&](int col) __attribute__((always_inline)) -> f32x4 {
    const f32x4* src = reinterpret_cast<const f32x4*>(p.acc_out + ao + col);
    return STREAM_ACC ? __builtin_nontemporal_load(src) : *src;
  };
  auto load_blk = [&](int col) __attribute__((always_inline)) -> f32x4 {
    if (BLK_BF16) {
      const bf16x4 yb = __builtin_nontemporal_load(reinterpret_cast<const bf16x4*>(reinterpret_cast<const __bf16*>(p.blk_out) + bo + col));
      return f32x4{(float)yb[0], (float)yb[1], (float)yb[2], (float)yb[3]};
    }
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.blk_out) + bo + col));
  };
  auto store_acc = [&](int col, f32x4 val) __attribute__((always_inline)) {
    f32x4* dst = reinterpret_cast<f32x4*>(p.acc_out + ao + col);
    if (STREAM_ACC) __builtin_nontemporal_store(val, dst);
    else *dst = val;
  };
  for (int col = t * 4; col < p.D; col += tpr * 8) {
    const int col2 = col + tpr * 4;
    const bool two = col2 < p.D;
    const f32x4 x0 = load_acc(col), y0 = load_blk(col);
    f32x4 x1 = x0, y1 = y0;
    if (two) { x1 = load_acc(col2); y1 = load_blk(col2); }
    store_acc(col, apply_update(plan, x0, y0));
    if (two) store_acc(col2, apply_update(plan, x1, y1));
  }
  if (t == 0) p.acc_lse[al] = plan.new_lse;
}

// n-ary form of the same Update: all partials of a row are combined in one pass,
//   lse = m + ln sum_i exp(lse_i - m),  out = sum_i exp(lse_i - lse) out_i,  m = max_i lse_i,
// which is what folding the Update of Sec. 3.1 over the partials gives (the Update is
// associative and commutative up to rounding), with every partial read exactly once and the
// result written once: (n + 1) streams instead of the 3n of n pairwise calls.  Partials with
// lse = -inf carry weight 0 and their out is never used (it may be uninitialised); if all are
// empty the result is the identity element (0, -inf).  Same row-to-thread mapping as above.
template <bool BLK_BF16, int N>
__global__ void __launch_bounds__(kMergeThreads) merge_n_kernel(const MergeNParams p, int64_t n_rows, int tpr_log2) {
  const int64_t gtid = (int64_t)blockIdx.x * kMergeThreads + threadIdx.x;
  const int64_t row = gtid >> tpr_log2;
  const int tpr = 1 << tpr_log2;
  const int t = (int)(gtid & (tpr - 1));
  if (row >= n_rows) return;

  int64_t oo, ol, bo, bl;
  if (p.contiguous) {
    oo = row * p.D; bo = oo; ol = row; bl = row;
  } else {
    const int64_t s = row % p.S, bh = row / p.S;
    const int64_t h = bh % p.H, b = bh / p.H;
    oo = b * p.o_sb + h * p.o_sh + s * p.o_ss;
    ol = b * p.l_sb + h * p.l_sh + s * p.l_ss;
    bo = b * p.bo_sb + h * p.bo_sh + s * p.bo_ss;
    bl = b * p.bl_sb + h * p.bl_sh + s * p.bl_ss;
  }
  float l[N];
#pragma unroll
  for (int i = 0; i < N; i++) l[i] = p.blk_lse[i][bl];
  const float l_old = p.accumulate ? p.lse[ol] : -INFINITY;
  float m = l_old;
#pragma unroll
  for (int i = 0; i < N; i++) m = fmaxf(m, l[i]);
  // weights relative to the maximum, then normalised; m = -inf means every partial is empty
  float w[N], w_old = 0.f, denom = 0.f;
  const bool any = m != -INFINITY;
#pragma unroll
  for (int i = 0; i < N; i++) {
    w[i] = any ? expf(l[i] - m) : 0.f;
    denom += w[i];
  }
  if (p.accumulate) {
    w_old = any ? expf(l_old - m) : 0.f;
    denom += w_old;
  }
  const float inv = any ? 1.f / denom : 0.f;
  const float new_lse = any ? m + logf(denom) : -INFINITY;

  for (int col = t * 4; col < p.D; col += tpr * 4) {
    f32x4 y[N];
#pragma unroll
    for (int i = 0; i < N; i++) {
      if (BLK_BF16) {
        const bf16x4 yb = __builtin_nontemporal_load(reinterpret_cast<const bf16x4*>(reinterpret_cast<const __bf16*>(p.blk_out[i]) + bo + col));
#pragma unroll
        for (int e = 0; e < 4; e++) y[i][e] = (float)yb[e];
      } else {
        y[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.blk_out[i]) + bo + col));
      }
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (p.accumulate && w_old != 0.f) {
      const f32x4 x = *reinterpret_cast<const f32x4*>(p.out + oo + col);
#pragma unroll
      for (int e = 0; e < 4; e++) acc[e] = w_old * x[e];
    }
#pragma unroll
    for (int i = 0; i < N; i++) {
      if (w[i] != 0.f) {   // a weight of exactly 0 must also silence NaN/Inf garbage of an empty partial
#pragma unroll
        for (int e = 0; e < 4; e++) acc[e] = __builtin_fmaf(w[i], y[i][e], acc[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; e++) acc[e] *= inv;
    // the result is streamed past the caches (measured +5-7 % on the 8-ary merge)
    __builtin_nontemporal_store(acc, reinterpret_cast<f32x4*>(p.out + oo + col));
  }
  if (t == 0) p.lse[ol] = new_lse;
}

template <bool BLK_BF16, int N>
hipError_t launch_merge_n_fixed(const MergeNParams& p, dim3 grid, int64_t n_rows, int tpr_log2, hipStream_t stream) {
  return launch_kernel(merge_n_kernel<BLK_BF16, N>, grid, dim3(kMergeThreads), 0, stream, p, n_rows, tpr_log2);
}

template <bool BLK_BF16>
hipError_t launch_merge_n_typed(const MergeNParams& p, dim3 grid, int64_t n_rows, int tpr_log2, hipStream_t stream) {
  switch (p.n) {
#define TR_CASE(N) case N: return launch_merge_n_fixed<BLK_BF16, N>(p, grid, n_rows, tpr_log2, stream);
    TR_CASE(1) TR_CASE(2) TR_CASE(3) TR_CASE(4) TR_CASE(5) TR_CASE(6) TR_CASE(7) TR_CASE(8)
    TR_CASE(9) TR_CASE(10) TR_CASE(11) TR_CASE(12) TR_CASE(13) TR_CASE(14) TR_CASE(15) TR_CASE(16)
#undef TR_CASE
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_merge_n(const MergeNParams& p, bool blk_bf16, hipStream_t stream) {
  const int64_t n_rows = (int64_t)p.B * p.H * p.S;
  if (n_rows == 0 || p.D == 0) return hipSuccess;
  int tpr_log2 = 0;
  while ((1 << tpr_log2) < p.D / 4 && tpr_log2 < 6) tpr_log2++;
  const int64_t n_threads = n_rows << tpr_log2;
  const int64_t nblocks = (n_threads + kMergeThreads - 1) / kMergeThreads;
  dim3 grid((unsigned)nblocks);
  return blk_bf16 ? launch_merge_n_typed<true>(p, grid, n_rows, tpr_log2, stream)
                  : launch_merge_n_typed<false>(p, grid, n_rows, tpr_log2, stream);
}

hipError_t launch_merge(const MergeParams& p, bool blk_bf16, hipStream_t stream) {
  const int64_t n_rows = (int64_t)p.B * p.H * p.S;
  if (n_rows == 0 || p.D == 0) return hipSuccess;
  // threads per row: half the row's 16-byte chunks (two chunks per thread), a power of two, at most a wave
  int tpr_log2 = 0;
  while ((1 << tpr_log2) < p.D / 8 && tpr_log2 < 6) tpr_log2++;
  const int64_t n_threads = n_rows << tpr_log2;
  const int64_t nblocks = (n_threads + kMergeThreads - 1) / kMergeThreads;
  dim3 grid((unsigned)nblocks), block(kMergeThreads);
  const bool stream_acc = p.stream_acc || n_rows * p.D * 4 > kStreamAccBytes;
  if (blk_bf16) {
    if (stream_acc) return launch_kernel(merge_kernel<true, true>, grid, block, 0, stream, p, n_rows, tpr_log2);
    return launch_kernel(merge_kernel<true, false>, grid, block, 0, stream, p, n_rows, tpr_log2);
  }
  if (stream_acc) return launch_kernel(merge_kernel<false, true>, grid, block, 0, stream, p, n_rows, tpr_log2);
  return launch_kernel(merge_kernel<false, false>, grid, block, 0, stream, p, n_rows, tpr_log2);
}

}  // namespace tr
