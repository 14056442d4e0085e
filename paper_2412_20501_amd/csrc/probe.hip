// Measurement aid, not a step of the method: a kernel that does nothing but issue dense bf16
// MFMAs on caller-supplied operands, on every CU, so that a benchmark can measure on the spot
// what the matrix cores sustain for a given operand distribution (the chip lowers its clock
// under dense MFMA load, and by how much depends on how much the operand bits toggle).
#include "tr_internal.h"

namespace tr {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 512;  // 8 waves per CU, two per SIMD, like the attention kernel
constexpr int kProbeOps = 8;        // operand pairs rotated through

// IDLE > 0 puts every wave to sleep for 64 * IDLE cycles after each 8 MFMAs, which lowers the
// duty cycle of the MFMA pipe without adding any other work.
template <int IDLE>
__global__ void __launch_bounds__(kProbeThreads) mfma_probe_kernel(const bf16x8* ops, float* sink, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[kProbeOps], b[kProbeOps];
#pragma unroll
  for (int i = 0; i < kProbeOps; i++) {
    a[i] = ops[i * 64 + lane];
    b[i] = ops[(kProbeOps + i) * 64 + lane];
  }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < kProbeOps; i += 4) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i + 3], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i + 1], b[i + 2], c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i + 2], b[i + 1], c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i + 3], b[i], c3, 0, 0, 0);
    }
    if (IDLE > 0) __builtin_amdgcn_s_sleep(IDLE);
  }
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < 16; v++) s += c0[v] + c1[v] + c2[v] + c3[v];
  if (s == 12345.678f) sink[0] = s;  // keeps the accumulators live; practically never true
}

}  // namespace

hipError_t launch_mfma_probe(const void* operands, float* sink, int iters, int idle, int n_blocks, hipStream_t stream) {
  const dim3 grid((unsigned)n_blocks), block(kProbeThreads);
  const bf16x8* ops = static_cast<const bf16x8*>(operands);
  switch (idle) {
    case 0: return launch_kernel(mfma_probe_kernel<0>, grid, block, 0, stream, ops, sink, iters);
    case 1: return launch_kernel(mfma_probe_kernel<1>, grid, block, 0, stream, ops, sink, iters);
    case 2: return launch_kernel(mfma_probe_kernel<2>, grid, block, 0, stream, ops, sink, iters);
    case 4: return launch_kernel(mfma_probe_kernel<4>, grid, block, 0, stream, ops, sink, iters);
    case 8: return launch_kernel(mfma_probe_kernel<8>, grid, block, 0, stream, ops, sink, iters);
    default: return hipErrorInvalidValue;
  }
}

int mfma_probe_threads() { return kProbeThreads; }
int mfma_probe_operand_bytes() { return 2 * kProbeOps * 64 * 16; }

}  // namespace tr
