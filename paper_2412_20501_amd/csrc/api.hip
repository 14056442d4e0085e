// C ABI of libtokenring: argument validation, descriptor -> kernel-parameter marshalling,
// and the host loop that replays TokenRing's Algorithm 1 on one GPU.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <vector>

#include "tr_internal.h"

namespace {

thread_local char g_err[512] = "";
thread_local tr::TimingEvents g_timing = {nullptr, nullptr};

tr_status fail(tr_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

int64_t elem_bytes(int32_t dtype) { return dtype == TR_BF16 ? 2 : 4; }

// Number of elements from ptr to one past the last addressed element of the view.
int64_t extent_elems(const tr_tensor* t) {
  if (t->B == 0 || t->H == 0 || t->S == 0 || t->D == 0) return 0;
  return (t->B - 1) * t->stride_b + (t->H - 1) * t->stride_h + (t->S - 1) * t->stride_s + t->D;
}

bool overlaps(const tr_tensor* a, const tr_tensor* b) {
  const int64_t ea = extent_elems(a) * elem_bytes(a->dtype), eb = extent_elems(b) * elem_bytes(b->dtype);
  if (ea == 0 || eb == 0) return false;
  const uintptr_t a0 = (uintptr_t)a->ptr, b0 = (uintptr_t)b->ptr;
  return a0 < b0 + (uintptr_t)eb && b0 < a0 + (uintptr_t)ea;
}

// Common checks of one descriptor. `row_align` = required multiple (in elements) of the strides
// and byte alignment of the pointer for vector access.
tr_status check_tensor(const char* name, const tr_tensor* t, bool allow_bf16, bool allow_f32, int row_align_bytes) {
  if (!t) return fail(TR_ERR_NULL, "%s: descriptor is NULL", name);
  if (t->dtype != TR_BF16 && t->dtype != TR_F32) return fail(TR_ERR_DTYPE, "%s: unknown dtype %d", name, (int)t->dtype);
  if ((t->dtype == TR_BF16 && !allow_bf16) || (t->dtype == TR_F32 && !allow_f32))
    return fail(TR_ERR_DTYPE, "%s: dtype %s not supported for this argument", name, t->dtype == TR_BF16 ? "bf16" : "fp32");
  if (t->B < 0 || t->H < 0 || t->S < 0 || t->D < 0) return fail(TR_ERR_SHAPE, "%s: negative dimension", name);
  if (t->B > INT32_MAX || t->H > INT32_MAX || t->S > (1 << 30) || t->D > INT32_MAX)
    return fail(TR_ERR_SHAPE, "%s: dimension too large", name);
  const bool empty = extent_elems(t) == 0;
  if (!empty && !t->ptr) return fail(TR_ERR_NULL, "%s: data pointer is NULL", name);
  if (t->stride_b < 0 || t->stride_h < 0 || t->stride_s < 0) return fail(TR_ERR_STRIDE, "%s: negative stride", name);
  if (!empty) {
    if (t->S > 1 && t->stride_s < t->D) return fail(TR_ERR_STRIDE, "%s: stride_s %lld smaller than D %lld", name, (long long)t->stride_s, (long long)t->D);
    const int64_t eb = elem_bytes(t->dtype);
    if (row_align_bytes > 1) {
      if (((uintptr_t)t->ptr) % row_align_bytes) return fail(TR_ERR_STRIDE, "%s: pointer not %d-byte aligned", name, row_align_bytes);
      if ((t->stride_b * eb) % row_align_bytes || (t->stride_h * eb) % row_align_bytes || (t->stride_s * eb) % row_align_bytes)
        return fail(TR_ERR_STRIDE, "%s: strides must be multiples of %d bytes", name, row_align_bytes);
    }
  }
  return TR_OK;
}

// A tensor the kernels write must not address one element through two index tuples (a zero or
// too small stride on a dimension larger than 1): rows are updated by different waves, so an
// overlapping view would race.  Sufficient test: ordered by stride, every dimension must step
// over the whole extent of the dimensions inside it.
tr_status check_written(const char* name, const tr_tensor* t) {
  if (extent_elems(t) == 0) return TR_OK;
  int64_t size[3] = {t->B, t->H, t->S}, stride[3] = {t->stride_b, t->stride_h, t->stride_s};
  for (int i = 0; i < 3; i++)
    for (int j = i + 1; j < 3; j++)
      if (stride[j] < stride[i]) {
        const int64_t a = size[i], b = stride[i];
        size[i] = size[j]; stride[i] = stride[j];
        size[j] = a; stride[j] = b;
      }
  int64_t inner = t->D;
  for (int i = 0; i < 3; i++) {
    if (size[i] <= 1) continue;
    if (stride[i] < inner) return fail(TR_ERR_STRIDE, "%s: a written tensor must not overlap itself (stride %lld < %lld elements inside it)", name, (long long)stride[i], (long long)inner);
    inner = stride[i] * (size[i] - 1) + inner;
  }
  return TR_OK;
}

// One block step of a schedule: Query segment qs attends K/V segment ks (equal segments of S),
// or, with ks2 >= 0, the pair of K/V segments ks and ks2 as one key range.
struct RingStep {
  int qs, ks;
  int ks2 = -1;
};

// Several block steps of one shape for a single launch: the tensors handed to attn_common are
// the views of segment 0 (length seg_len along S); step i works on Query segment steps[i].qs
// and K/V segment steps[i].ks, masked diagonally iff `causal` and both are equal; a step with a
// second K/V segment is masked iff that one equals the Query segment (the first lies before it).
struct StepGroup {
  const RingStep* steps;
  int n;
  int64_t seg_len;
  bool causal;
};

// fuse_update: out/lse are fp32 accumulators and the block is merged into them by the kernel's epilogue
tr_status attn_common(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int causal, int64_t off64, float scale,
                      const tr_tensor* out, const tr_tensor* lse, void* stream, bool fuse_update = false,
                      const StepGroup* group = nullptr) {
  tr_status st;
  if ((st = check_tensor("q", q, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("k", k, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("v", v, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("out", out, !fuse_update, true, 16)) != TR_OK) return st;
  if ((st = check_tensor("lse", lse, false, true, 4)) != TR_OK) return st;
  if ((st = check_written("out", out)) != TR_OK || (st = check_written("lse", lse)) != TR_OK) return st;
  if (q->D != 64 && q->D != 128) return fail(TR_ERR_SHAPE, "head dim %lld not supported (64 or 128)", (long long)q->D);
  if (k->D != q->D || v->D != q->D || out->D != q->D) return fail(TR_ERR_SHAPE, "head dims of q, k, v, out differ");
  if (lse->D != 1) return fail(TR_ERR_SHAPE, "lse must have D = 1");
  if (k->B != q->B || v->B != q->B || out->B != q->B || lse->B != q->B) return fail(TR_ERR_SHAPE, "batch sizes differ");
  if (k->H != v->H || k->S != v->S) return fail(TR_ERR_SHAPE, "k and v shapes differ");
  if (out->H != q->H || lse->H != q->H || out->S != q->S || lse->S != q->S) return fail(TR_ERR_SHAPE, "out/lse shape does not match q");
  if (q->H > 0 && (k->H <= 0 || q->H % k->H)) return fail(TR_ERR_SHAPE, "query heads %lld not a multiple of K/V heads %lld", (long long)q->H, (long long)k->H);
  if (!(scale > 0.f) || !isfinite(scale)) return fail(TR_ERR_UNSUPPORTED, "scale must be finite and > 0");
  if (overlaps(out, q) || overlaps(out, k) || overlaps(out, v) || overlaps(lse, q) || overlaps(lse, k) || overlaps(lse, v) || overlaps(out, lse))
    return fail(TR_ERR_ALIAS, "outputs overlap inputs or each other");
  if ((int64_t)q->B * q->H > (1 << 24)) return fail(TR_ERR_SHAPE, "too many (batch, head) pairs");
  // the K/V staging addresses a 64-key tile with 32-bit byte offsets from the tile base
  if (k->stride_s > ((int64_t)1 << 24) || v->stride_s > ((int64_t)1 << 24))
    return fail(TR_ERR_STRIDE, "stride_s of k and v must not exceed 2^24 elements");

  tr::AttnParams p;
  memset(&p, 0, sizeof(p));
  p.q = (const __bf16*)q->ptr; p.k = (const __bf16*)k->ptr; p.v = (const __bf16*)v->ptr;
  p.out = out->ptr; p.lse = (float*)lse->ptr;
  p.q_sb = q->stride_b; p.q_sh = q->stride_h; p.q_ss = q->stride_s;
  p.k_sb = k->stride_b; p.k_sh = k->stride_h; p.k_ss = k->stride_s;
  p.v_sb = v->stride_b; p.v_sh = v->stride_h; p.v_ss = v->stride_s;
  p.o_sb = out->stride_b; p.o_sh = out->stride_h; p.o_ss = out->stride_s;
  p.l_sb = lse->stride_b; p.l_sh = lse->stride_h; p.l_ss = lse->stride_s;
  p.B = (int)q->B; p.Hq = (int)q->H; p.Hkv = (int)k->H; p.Sq = (int)q->S; p.Sk = (int)k->S;
  p.causal = causal ? 1 : 0;
  const int64_t lim = (int64_t)1 << 30;
  p.causal_off = (int)(off64 > lim ? lim : (off64 < -lim ? -lim : off64));
  p.scale = scale;
  const int bm = tr::attn_rows_per_block();
  p.n_qtiles = (p.Sq + bm - 1) / bm;
  p.xcd_map = (p.B * p.Hkv) % 8 == 0 && (int64_t)p.n_qtiles * p.B * p.Hq >= 8;
  p.gq = p.Hkv > 0 ? p.Hq / p.Hkv : 1;
  p.gq_log2 = -1;
  for (int sh = 0; sh < 31; sh++)
    if (p.gq == (1 << sh)) p.gq_log2 = sh;
  if (p.n_qtiles > 65535) return fail(TR_ERR_SHAPE, "Sq too long for one launch (at most 65535 query tiles of %d rows)", bm);
  p.n_prob = 1;
  for (int i = 0; i < tr::kAttnGroupMax; i++) p.step[i].k_seg2 = -1;
  p.blocks_per_prob = p.n_qtiles * p.B * p.Hq;
  p.causal_bits = p.causal ? 1u : 0u;
  if (group) {
    if (group->n < 1 || group->n > tr::kAttnGroupMax) return fail(TR_ERR_SHAPE, "internal: %d steps in one launch", group->n);
    p.n_prob = group->n;
    p.causal = 0; p.causal_off = 0; p.causal_bits = 0;
    p.q_seg_elems = group->seg_len * q->stride_s; p.k_seg_elems = group->seg_len * k->stride_s;
    p.v_seg_elems = group->seg_len * v->stride_s; p.o_seg_elems = group->seg_len * out->stride_s;
    p.l_seg_elems = group->seg_len * lse->stride_s;
    // Workgroups are dispatched step by step, so the steps go in longest first: a launch then ends
    // on its short steps and the tail in which some compute units are idle is as short as possible.
    const RingStep* order[tr::kAttnGroupMax];
    auto cost = [&](const RingStep& s) { return (s.ks2 >= 0 ? 4 : 2) - ((group->causal && (s.ks2 >= 0 ? s.ks2 : s.ks) == s.qs) ? 1 : 0); };
    for (int i = 0; i < group->n; i++) order[i] = group->steps + i;
    std::stable_sort(order, order + group->n, [&](const RingStep* a, const RingStep* b) { return cost(*a) > cost(*b); });
    for (int i = 0; i < group->n; i++) {
      const RingStep& s = *order[i];
      if (s.ks2 >= 0 && (group->seg_len % 128 || s.ks2 <= s.ks)) return fail(TR_ERR_SHAPE, "internal: segment pair on segments of %lld keys", (long long)group->seg_len);
      p.step[i].q_seg = s.qs;
      p.step[i].k_seg = s.ks;
      p.step[i].k_seg2 = s.ks2;
      if (group->causal && (s.ks2 >= 0 ? s.ks2 : s.ks) == s.qs) p.causal_bits |= 1u << i;
    }
  }
  if ((int64_t)p.blocks_per_prob * p.n_prob >= ((int64_t)1 << 31)) return fail(TR_ERR_SHAPE, "too many workgroups for one launch");
  // Without a causal step in the launch all query tiles cost the same, and an XCD may finish the
  // query tiles of one head before it starts the next: half as many heads' K/V are then live in
  // its L2 at a time.  (Under a causal mask that order would bunch the heavy tiles.)
  if (p.xcd_map && p.causal_bits == 0 && (int64_t)p.B * p.Hq / 8 <= 65535) p.xcd_map = 2;
  if (p.B == 0 || p.Hq == 0 || p.Sq == 0) return TR_OK;
  const int epilogue = fuse_update ? 2 : (out->dtype == TR_F32 ? 1 : 0);
  const hipError_t e = tr::launch_block_attn(p, (int)q->D, epilogue, (hipStream_t)stream);
  if (e != hipSuccess) return fail(TR_ERR_HIP, "block attention launch failed: %s", hipGetErrorString(e));
  return TR_OK;
}

// View of chunk `c` (of length C along S) of a tensor.
tr_tensor chunk_view(const tr_tensor* t, int64_t c, int64_t C) {
  tr_tensor r = *t;
  r.ptr = (char*)t->ptr + c * C * t->stride_s * elem_bytes(t->dtype);
  r.S = C;
  return r;
}

inline int pmod(int a, int n) { return ((a % n) + n) % n; }

// Execution order of the block steps, all "devices" replayed in turn, and the number of equal
// segments the sequence is cut into.  Under the causal rule a step whose K/V segment lies
// after its Query segment is dropped (the caller masks ks == qs diagonally).
//   TokenRing (Algorithm 1): iteration i, device j (holds K_j, V_j) works on Query chunk (j-i) mod n.
//   Ring Attention (Sec. 2.1): device j keeps Q_j; at iteration i it holds K/V chunk (j-i) mod n.
//   Zigzag (Sec. 3.3.2): 2n segments, device g owns segments g and 2n-1-g of Q, K and V; the
//     Query pair circulates as in Algorithm 1.
//   Hybrid (Sec. 3.3.3): n = nodes * n_inner devices; K/V travel between nodes as in Ring
//     Attention (outer step t), Algorithm 1 runs among the n_inner devices of each node.
int build_schedule(int schedule, int n, int n_inner, bool causal, std::vector<RingStep>& steps, bool pair_kv = false) {
  steps.clear();
  auto add = [&](int qs, int ks) {
    if (!causal || ks <= qs) steps.push_back({qs, ks});
  };
  switch (schedule) {
    case TR_SCHED_TOKENRING:
      for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) add(pmod(j - i, n), j);
      return n;
    case TR_SCHED_RING_ATTENTION:
      for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) add(j, pmod(j - i, n));
      return n;
    case TR_SCHED_ZIGZAG:
      // Within an iteration the devices work concurrently, each on up to three segment pairs of
      // its own Query pair; they are emitted slot by slot (every device's first pair, then every
      // device's second, ...) so that pairs on distinct Query segments are adjacent and can share
      // a launch.  The order of the blocks each Query segment receives is unaffected.
      // pair_kv: when a Query segment meets both K/V segments of the device (always its later
      // segment), the two become one block step over the device's whole K/V; a device then has at
      // most two steps per iteration, on its two Query segments.
      for (int i = 0; i < n; i++) {
        for (int slot = 0; slot < 4; slot++) {
          for (int j = 0; j < n; j++) {
            const int c = pmod(j - i, n);
            const int qseg[2] = {c, 2 * n - 1 - c}, kseg[2] = {j, 2 * n - 1 - j};
            RingStep dev[4];
            int kept = 0;
            for (int a = 0; a < 2; a++)
              for (int b = 0; b < 2; b++) {
                if (kseg[b] > qseg[a]) continue;
                if (pair_kv && b == 1 && kept > 0 && dev[kept - 1].qs == qseg[a] && dev[kept - 1].ks2 < 0) dev[kept - 1].ks2 = kseg[b];
                else dev[kept++] = {qseg[a], kseg[b]};
              }
            if (slot < kept) steps.push_back(dev[slot]);
          }
        }
      }
      return 2 * n;
    case TR_SCHED_HYBRID: {
      const int nodes = n / n_inner;
      for (int t = 0; t < nodes; t++)
        for (int i = 0; i < n_inner; i++)
          for (int nd = 0; nd < nodes; nd++)
            for (int pp = 0; pp < n_inner; pp++) add(nd * n_inner + pmod(pp - i, n_inner), pmod(nd - t, nodes) * n_inner + pp);
      return n;
    }
    default:
      return 0;
  }
}

// One launch of the fused forms: steps [begin, end) of the list; `merge` = the blocks are merged
// into accumulators that already hold a result (otherwise they are each segment's first block).
struct LaunchGroup { size_t begin, end; bool merge; };

// Splits the step list into launches.  Consecutive steps that touch distinct Query segments and
// are of one kind (first block of their segment, which is written, or a later block, which is
// merged) are independent of each other - they are what different devices compute at the same
// time - and share a launch (at most kAttnGroupMax steps).
std::vector<LaunchGroup> group_steps(const std::vector<RingStep>& steps, int n_seg) {
  std::vector<LaunchGroup> groups;
  std::vector<char> started((size_t)n_seg, 0);  // has this Query segment received its first block?
  std::vector<int> in_group((size_t)n_seg, -1); // index of the group that last used the segment
  size_t pos = 0;
  while (pos < steps.size()) {
    const int group_id = (int)groups.size();
    const bool merge = started[(size_t)steps[pos].qs] != 0;
    size_t end = pos;
    while (end < steps.size() && (int)(end - pos) < tr::kAttnGroupMax && (started[(size_t)steps[end].qs] != 0) == merge &&
           in_group[(size_t)steps[end].qs] != group_id) {
      in_group[(size_t)steps[end].qs] = group_id;
      end++;
    }
    for (size_t i = pos; i < end; i++) started[(size_t)steps[i].qs] = 1;
    groups.push_back({pos, end, merge});
    pos = end;
  }
  return groups;
}

// Runs the steps in order with the Update fused into the attention epilogue, one launch per group.
tr_status run_steps_fused(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, const tr_tensor* out, const tr_tensor* lse,
                          int n_seg, bool causal, float scale, const std::vector<RingStep>& steps, void* stream) {
  const int64_t C = q->S / n_seg;
  const tr_tensor q0 = chunk_view(q, 0, C), k0 = chunk_view(k, 0, C), v0 = chunk_view(v, 0, C);
  const tr_tensor o0 = chunk_view(out, 0, C), l0 = chunk_view(lse, 0, C);
  for (const LaunchGroup& grp : group_steps(steps, n_seg)) {
    const StepGroup g = {steps.data() + grp.begin, (int)(grp.end - grp.begin), C, causal};
    const tr_status st = attn_common(&q0, &k0, &v0, 0, 0, scale, &o0, &l0, stream, grp.merge, &g);
    if (st != TR_OK) return st;
  }
  return TR_OK;
}

constexpr size_t kWsAlign = 256;
size_t align_up(size_t x) { return (x + kWsAlign - 1) / kWsAlign * kWsAlign; }

// Block workspace of tr_ring_attn_noalloc: one block result (block_out + block_lse) of the
// two-kernel form, held in a device array of the library itself so that the call needs no
// allocation.  Every GPU the library runs on holds its own copy until the process ends.  In
// host code the array's name is only a handle: the device address is resolved once per device
// (with that device current) and kept in g_scratch_ptr; kernels only ever see that address.
__device__ __align__(256) static unsigned char scratch[TR_NOALLOC_SCRATCH_BYTES];
constexpr int kScratchMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kScratchMaxDevices];

tr_status scratch_of_current_device(void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(TR_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kScratchMaxDevices) return fail(TR_ERR_UNSUPPORTED, "device index %d beyond the %d devices supported", dev, kScratchMaxDevices);
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(TR_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // the same address from any thread that races here
  }
  *ptr_out = ptr;
  return TR_OK;
}

}  // namespace

namespace tr {
TimingEvents take_timing_events() {
  const TimingEvents ev = g_timing;
  g_timing = {nullptr, nullptr};
  return ev;
}
}  // namespace tr

extern "C" {

const char* tr_last_error(void) { return g_err; }

tr_status tr_time_next_kernel(void* start_event, void* stop_event) {
  g_err[0] = 0;
  g_timing.start = static_cast<hipEvent_t>(start_event);
  g_timing.stop = static_cast<hipEvent_t>(stop_event);
  return TR_OK;
}
#ifndef TR_SOURCE_HASH_STR
#define TR_SOURCE_HASH_STR "0000000000000000"
#endif
// The tagged string is also what the build script looks for inside the binary to decide whether
// the library was compiled from the sources on disk.
__attribute__((used)) static const char tr_source_hash_tag[] = "TR_SOURCE_HASH=" TR_SOURCE_HASH_STR;
const char* tr_version(void) { return "tokenring-gfx950 0.2 (sources " TR_SOURCE_HASH_STR ")"; }

tr_status tr_block_attn(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int mask_kind, float scale,
                        const tr_tensor* out, const tr_tensor* lse, void* hip_stream) {
  g_err[0] = 0;
  if (mask_kind != TR_MASK_NONE && mask_kind != TR_MASK_CAUSAL_DIAG) return fail(TR_ERR_UNSUPPORTED, "unknown mask kind %d", mask_kind);
  if (mask_kind == TR_MASK_CAUSAL_DIAG && q && k && q->S != k->S)
    return fail(TR_ERR_SHAPE, "the diagonal causal mask needs Sq == Sk (got %lld, %lld)", (long long)q->S, (long long)k->S);
  return attn_common(q, k, v, mask_kind == TR_MASK_CAUSAL_DIAG, 0, scale, out, lse, hip_stream);
}

tr_status tr_block_attn_causal_at(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int64_t q_pos0, int64_t k_pos0,
                                  float scale, const tr_tensor* out, const tr_tensor* lse, void* hip_stream) {
  g_err[0] = 0;
  if (q_pos0 < 0 || k_pos0 < 0) return fail(TR_ERR_SHAPE, "chunk positions must be >= 0");
  return attn_common(q, k, v, 1, q_pos0 - k_pos0, scale, out, lse, hip_stream);
}

tr_status tr_block_attn_merge(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int mask_kind, float scale,
                              const tr_tensor* out_acc, const tr_tensor* lse_acc, void* hip_stream) {
  g_err[0] = 0;
  if (mask_kind != TR_MASK_NONE && mask_kind != TR_MASK_CAUSAL_DIAG) return fail(TR_ERR_UNSUPPORTED, "unknown mask kind %d", mask_kind);
  if (mask_kind == TR_MASK_CAUSAL_DIAG && q && k && q->S != k->S)
    return fail(TR_ERR_SHAPE, "the diagonal causal mask needs Sq == Sk (got %lld, %lld)", (long long)q->S, (long long)k->S);
  return attn_common(q, k, v, mask_kind == TR_MASK_CAUSAL_DIAG, 0, scale, out_acc, lse_acc, hip_stream, true);
}

}  // extern "C"

namespace {
// acc_streams: the caller knows that the accumulator view is part of a larger tensor that is swept
// once between two Updates of this view (a ring replay over many Query chunks)
tr_status merge_common(const tr_tensor* out_acc, const tr_tensor* lse_acc, const tr_tensor* block_out, const tr_tensor* block_lse,
                       void* hip_stream, bool acc_streams) {
  tr_status st;
  if ((st = check_tensor("out_acc", out_acc, false, true, 16)) != TR_OK) return st;
  if ((st = check_tensor("lse_acc", lse_acc, false, true, 4)) != TR_OK) return st;
  if ((st = check_tensor("block_out", block_out, true, true, 8)) != TR_OK) return st;
  if ((st = check_tensor("block_lse", block_lse, false, true, 4)) != TR_OK) return st;
  if (block_out->dtype == TR_F32 && (st = check_tensor("block_out", block_out, true, true, 16)) != TR_OK) return st;
  if ((st = check_written("out_acc", out_acc)) != TR_OK || (st = check_written("lse_acc", lse_acc)) != TR_OK) return st;
  if (lse_acc->D != 1 || block_lse->D != 1) return fail(TR_ERR_SHAPE, "lse tensors must have D = 1");
  if (out_acc->D % 4) return fail(TR_ERR_SHAPE, "D = %lld must be a multiple of 4", (long long)out_acc->D);
  if (block_out->B != out_acc->B || block_out->H != out_acc->H || block_out->S != out_acc->S || block_out->D != out_acc->D)
    return fail(TR_ERR_SHAPE, "block_out shape does not match out_acc");
  if (lse_acc->B != out_acc->B || lse_acc->H != out_acc->H || lse_acc->S != out_acc->S) return fail(TR_ERR_SHAPE, "lse_acc shape does not match out_acc");
  if (block_lse->B != out_acc->B || block_lse->H != out_acc->H || block_lse->S != out_acc->S) return fail(TR_ERR_SHAPE, "block_lse shape does not match out_acc");
  if (overlaps(out_acc, block_out) || overlaps(out_acc, block_lse) || overlaps(lse_acc, block_out) || overlaps(lse_acc, block_lse) || overlaps(out_acc, lse_acc))
    return fail(TR_ERR_ALIAS, "accumulator and block tensors overlap");
  if ((int64_t)out_acc->B * out_acc->H * out_acc->S >= ((int64_t)1 << 32))
    return fail(TR_ERR_SHAPE, "too many elements for one launch");

  tr::MergeParams p;
  memset(&p, 0, sizeof(p));
  p.acc_out = (float*)out_acc->ptr; p.acc_lse = (float*)lse_acc->ptr;
  p.blk_out = block_out->ptr; p.blk_lse = (const float*)block_lse->ptr;
  p.ao_sb = out_acc->stride_b; p.ao_sh = out_acc->stride_h; p.ao_ss = out_acc->stride_s;
  p.al_sb = lse_acc->stride_b; p.al_sh = lse_acc->stride_h; p.al_ss = lse_acc->stride_s;
  p.bo_sb = block_out->stride_b; p.bo_sh = block_out->stride_h; p.bo_ss = block_out->stride_s;
  p.bl_sb = block_lse->stride_b; p.bl_sh = block_lse->stride_h; p.bl_ss = block_lse->stride_s;
  p.B = (int)out_acc->B; p.H = (int)out_acc->H; p.S = (int)out_acc->S; p.D = (int)out_acc->D;
  auto dense = [](const tr_tensor* t) {
    return t->stride_s == t->D && t->stride_h == t->S * t->D && t->stride_b == t->H * t->S * t->D;
  };
  p.contiguous = dense(out_acc) && dense(block_out) && dense(lse_acc) && dense(block_lse);
  p.stream_acc = acc_streams ? 1 : 0;
  if (p.B == 0 || p.H == 0 || p.S == 0 || p.D == 0) return TR_OK;
  const hipError_t e = tr::launch_merge(p, block_out->dtype == TR_BF16, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(TR_ERR_HIP, "merge launch failed: %s", hipGetErrorString(e));
  return TR_OK;
}
}  // namespace

extern "C" {

tr_status tr_merge(const tr_tensor* out_acc, const tr_tensor* lse_acc, const tr_tensor* block_out, const tr_tensor* block_lse,
                   void* hip_stream) {
  g_err[0] = 0;
  return merge_common(out_acc, lse_acc, block_out, block_lse, hip_stream, false);
}

tr_status tr_merge_n(const tr_tensor* out, const tr_tensor* lse, const tr_tensor* const* block_outs,
                     const tr_tensor* const* block_lses, int n, int accumulate, void* hip_stream) {
  g_err[0] = 0;
  tr_status st;
  if (!block_outs || !block_lses) return fail(TR_ERR_NULL, "the arrays of partial results must not be NULL");
  if (n < 1 || n > tr::kMergeNMax) return fail(TR_ERR_SHAPE, "n = %d partials out of range [1, %d]", n, tr::kMergeNMax);
  if ((st = check_tensor("out", out, false, true, 16)) != TR_OK) return st;
  if ((st = check_tensor("lse", lse, false, true, 4)) != TR_OK) return st;
  if ((st = check_written("out", out)) != TR_OK || (st = check_written("lse", lse)) != TR_OK) return st;
  if (lse->D != 1) return fail(TR_ERR_SHAPE, "lse tensors must have D = 1");
  if (out->D % 4) return fail(TR_ERR_SHAPE, "D = %lld must be a multiple of 4", (long long)out->D);
  if (lse->B != out->B || lse->H != out->H || lse->S != out->S) return fail(TR_ERR_SHAPE, "lse shape does not match out");
  if (overlaps(out, lse)) return fail(TR_ERR_ALIAS, "out and lse overlap");
  if ((int64_t)out->B * out->H * out->S >= ((int64_t)1 << 32)) return fail(TR_ERR_SHAPE, "too many elements for one launch");
  const tr_tensor* bo0 = block_outs[0];
  const tr_tensor* bl0 = block_lses[0];
  for (int i = 0; i < n; i++) {
    const tr_tensor* bo = block_outs[i];
    const tr_tensor* bl = block_lses[i];
    if ((st = check_tensor("block_out", bo, true, true, 8)) != TR_OK) return st;
    if (bo->dtype == TR_F32 && (st = check_tensor("block_out", bo, true, true, 16)) != TR_OK) return st;
    if ((st = check_tensor("block_lse", bl, false, true, 4)) != TR_OK) return st;
    if (bo->B != out->B || bo->H != out->H || bo->S != out->S || bo->D != out->D) return fail(TR_ERR_SHAPE, "block_out %d: shape does not match out", i);
    if (bl->B != out->B || bl->H != out->H || bl->S != out->S || bl->D != 1) return fail(TR_ERR_SHAPE, "block_lse %d: shape does not match lse", i);
    if (bo->dtype != bo0->dtype) return fail(TR_ERR_DTYPE, "block_out %d: all partials must have one dtype", i);
    if (bo->stride_b != bo0->stride_b || bo->stride_h != bo0->stride_h || bo->stride_s != bo0->stride_s ||
        bl->stride_b != bl0->stride_b || bl->stride_h != bl0->stride_h || bl->stride_s != bl0->stride_s)
      return fail(TR_ERR_STRIDE, "partial %d: all partials must share their strides", i);
    if (overlaps(out, bo) || overlaps(out, bl) || overlaps(lse, bo) || overlaps(lse, bl))
      return fail(TR_ERR_ALIAS, "partial %d overlaps the result tensors", i);
  }

  tr::MergeNParams p;
  memset(&p, 0, sizeof(p));
  p.out = (float*)out->ptr; p.lse = (float*)lse->ptr;
  for (int i = 0; i < n; i++) { p.blk_out[i] = block_outs[i]->ptr; p.blk_lse[i] = (const float*)block_lses[i]->ptr; }
  p.o_sb = out->stride_b; p.o_sh = out->stride_h; p.o_ss = out->stride_s;
  p.l_sb = lse->stride_b; p.l_sh = lse->stride_h; p.l_ss = lse->stride_s;
  p.bo_sb = bo0->stride_b; p.bo_sh = bo0->stride_h; p.bo_ss = bo0->stride_s;
  p.bl_sb = bl0->stride_b; p.bl_sh = bl0->stride_h; p.bl_ss = bl0->stride_s;
  p.B = (int)out->B; p.H = (int)out->H; p.S = (int)out->S; p.D = (int)out->D;
  p.n = n; p.accumulate = accumulate ? 1 : 0;
  auto dense = [](const tr_tensor* t) {
    return t->stride_s == t->D && t->stride_h == t->S * t->D && t->stride_b == t->H * t->S * t->D;
  };
  p.contiguous = dense(out) && dense(bo0) && dense(lse) && dense(bl0);
  if (p.B == 0 || p.H == 0 || p.S == 0 || p.D == 0) return TR_OK;
  const hipError_t e = tr::launch_merge_n(p, bo0->dtype == TR_BF16, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(TR_ERR_HIP, "n-ary merge launch failed: %s", hipGetErrorString(e));
  return TR_OK;
}

size_t tr_ring_attn_blocks_workspace_bytes(const tr_tensor* q, int n_chunks, int block_dtype) {
  if (!q || n_chunks < 1 || q->B < 0 || q->H < 0 || q->S < 0 || q->D < 0 || q->S % n_chunks) return 0;
  if (block_dtype != TR_F32 && block_dtype != TR_BF16) return 0;
  const size_t C = (size_t)(q->S / n_chunks);
  const size_t rows = (size_t)q->B * (size_t)q->H * C;
  return align_up(rows * (size_t)q->D * (size_t)elem_bytes(block_dtype)) + align_up(rows * 4);
}

size_t tr_ring_attn_workspace_bytes(const tr_tensor* q, int n_chunks) {
  return tr_ring_attn_blocks_workspace_bytes(q, n_chunks, TR_F32);
}

}  // extern "C"

namespace {

// Algorithm 1 on one device.  workspace == NULL: fused form.  Otherwise the two-kernel form, the
// block result passing through the workspace as block_dtype (fp32, or bf16 as a transport format).
tr_status ring_attn_impl(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int n_chunks, int causal,
                         const tr_tensor* out, const tr_tensor* lse, float scale, int block_dtype, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  if (!q || !k || !v || !out || !lse) return fail(TR_ERR_NULL, "a tensor descriptor is NULL");
  if (n_chunks < 1) return fail(TR_ERR_SHAPE, "n_chunks must be >= 1");
  if (q->S < 0 || q->S % n_chunks) return fail(TR_ERR_SHAPE, "sequence length %lld is not a multiple of n_chunks %d", (long long)q->S, n_chunks);
  if (k->S != q->S || v->S != q->S) return fail(TR_ERR_SHAPE, "q, k, v must have the same sequence length");
  if (out->dtype != TR_F32) return fail(TR_ERR_DTYPE, "out must be fp32 (it is the merge accumulator)");
  if (q->D > 0 && !(scale > 0.f)) scale = 1.0f / sqrtf((float)q->D);
  const int64_t C = q->S / n_chunks;

  // Validate every argument once through the single-step checks (chunk 0 views have the
  // same strides, dtypes and alignment class as all others).
  tr_status st;
  if ((st = check_tensor("q", q, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("k", k, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("v", v, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("out", out, false, true, 16)) != TR_OK) return st;
  if ((st = check_tensor("lse", lse, false, true, 4)) != TR_OK) return st;
  if ((st = check_written("out", out)) != TR_OK || (st = check_written("lse", lse)) != TR_OK) return st;
  if (out->B != q->B || out->H != q->H || out->S != q->S || out->D != q->D || lse->B != q->B || lse->H != q->H || lse->S != q->S || lse->D != 1)
    return fail(TR_ERR_SHAPE, "out/lse shape does not match q");

  const size_t need = tr_ring_attn_blocks_workspace_bytes(q, n_chunks, block_dtype);
  const size_t rows = (size_t)q->B * (size_t)q->H * (size_t)C;
  tr_tensor ws_out, ws_lse;
  memset(&ws_out, 0, sizeof(ws_out));
  const bool fused = workspace == nullptr;  // no workspace: the Update runs in the attention epilogue
  if (!fused && workspace_bytes == 0) return fail(TR_ERR_WORKSPACE, "workspace given with size 0 (need %zu bytes)", need);
  if (!fused && n_chunks > 1 && rows > 0) {
    if (((uintptr_t)workspace) % kWsAlign) return fail(TR_ERR_WORKSPACE, "workspace must be %zu-byte aligned", kWsAlign);
    if (workspace_bytes < need) return fail(TR_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, need);
    ws_out.ptr = workspace; ws_out.dtype = block_dtype;
    ws_out.B = q->B; ws_out.H = q->H; ws_out.S = C; ws_out.D = q->D;
    ws_out.stride_s = q->D; ws_out.stride_h = C * q->D; ws_out.stride_b = q->H * C * q->D;
    ws_lse = ws_out;
    ws_lse.ptr = (char*)workspace + align_up(rows * (size_t)q->D * (size_t)elem_bytes(block_dtype));
    ws_lse.dtype = TR_F32;
    ws_lse.D = 1; ws_lse.stride_s = 1; ws_lse.stride_h = C; ws_lse.stride_b = q->H * C;
    tr_tensor ws_all = ws_out;  // alias check of the whole workspace against the user tensors
    ws_all.dtype = TR_F32;
    ws_all.B = 1; ws_all.H = 1; ws_all.S = 1; ws_all.D = (int64_t)(need / 4);
    if (overlaps(&ws_all, q) || overlaps(&ws_all, k) || overlaps(&ws_all, v) || overlaps(&ws_all, out) || overlaps(&ws_all, lse))
      return fail(TR_ERR_ALIAS, "workspace overlaps a tensor argument");
  }

  if (overlaps(out, q) || overlaps(out, k) || overlaps(out, v) || overlaps(lse, q) || overlaps(lse, k) || overlaps(lse, v) || overlaps(out, lse))
    return fail(TR_ERR_ALIAS, "outputs overlap inputs or each other");
  if (n_chunks > 8192) return fail(TR_ERR_SHAPE, "n_chunks %d too large (at most 8192)", n_chunks);

  // Algorithm 1 replayed on one device: iteration i, "device" j, Query chunk c = (j - i) mod n.
  if (fused) {
    std::vector<RingStep> steps;
    build_schedule(TR_SCHED_TOKENRING, n_chunks, 1, causal != 0, steps);
    return run_steps_fused(q, k, v, out, lse, n_chunks, causal != 0, scale, steps, hip_stream);
  }
  // between two Updates of one Query chunk every other chunk's accumulator is touched: if all of them
  // together exceed the memory-side cache, none survives there and the Update streams past the caches
  const bool out_sweeps = (int64_t)q->B * q->H * q->S * q->D * 4 > ((int64_t)128 << 20);
  for (int i = 0; i < n_chunks; i++) {
    for (int j = 0; j < n_chunks; j++) {
      const int c = ((j - i) % n_chunks + n_chunks) % n_chunks;
      if (causal && j > c) continue;
      const tr_tensor qc = chunk_view(q, c, C), kj = chunk_view(k, j, C), vj = chunk_view(v, j, C);
      const tr_tensor oc = chunk_view(out, c, C), lc = chunk_view(lse, c, C);
      const int diag = causal && j == c;
      if (i == 0) {
        // first block of Query chunk c: it *is* the accumulator's initial value
        st = attn_common(&qc, &kj, &vj, diag, 0, scale, &oc, &lc, hip_stream);
        if (st != TR_OK) return st;
      } else {
        st = attn_common(&qc, &kj, &vj, diag, 0, scale, &ws_out, &ws_lse, hip_stream);
        if (st != TR_OK) return st;
        st = merge_common(&oc, &lc, &ws_out, &ws_lse, hip_stream, out_sweeps);
        if (st != TR_OK) return st;
      }
    }
  }
  return TR_OK;
}

}  // namespace

extern "C" {

tr_status tr_ring_attn(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int n_chunks, int causal,
                       const tr_tensor* out, const tr_tensor* lse, float scale, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  g_err[0] = 0;
  return ring_attn_impl(q, k, v, n_chunks, causal, out, lse, scale, TR_F32, workspace, workspace_bytes, hip_stream);
}

tr_status tr_ring_attn_blocks(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int n_chunks, int causal,
                              const tr_tensor* out, const tr_tensor* lse, float scale, int block_dtype, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  g_err[0] = 0;
  if (block_dtype != TR_F32 && block_dtype != TR_BF16) return fail(TR_ERR_DTYPE, "block_dtype %d is neither fp32 nor bf16", block_dtype);
  if (!workspace) return fail(TR_ERR_WORKSPACE, "the two-kernel form needs a workspace");
  return ring_attn_impl(q, k, v, n_chunks, causal, out, lse, scale, block_dtype, workspace, workspace_bytes, hip_stream);
}

tr_status tr_ring_attn_noalloc(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int n_chunks, int causal,
                               const tr_tensor* out, const tr_tensor* lse, float scale, void* hip_stream) {
  g_err[0] = 0;
  // size check first (needs no device): the block result of one step must fit the library's array
  const size_t need = tr_ring_attn_blocks_workspace_bytes(q, n_chunks, TR_F32);
  if (q && n_chunks >= 1 && q->S >= 0 && q->S % n_chunks == 0 && need > (size_t)TR_NOALLOC_SCRATCH_BYTES)
    return fail(TR_ERR_WORKSPACE, "tr_ring_attn_noalloc: one block result needs %zu bytes, the built-in scratch holds %zu "
                "(B * Hq * (S / n_chunks) * (D + 1) * 4 bytes must fit); use tr_ring_attn with a workspace", need,
                (size_t)TR_NOALLOC_SCRATCH_BYTES);
  if (!q || !k || !v || !out || !lse) return fail(TR_ERR_NULL, "a tensor descriptor is NULL");
  void* ws = nullptr;
  const tr_status st = scratch_of_current_device(&ws);
  if (st != TR_OK) return st;
  return ring_attn_impl(q, k, v, n_chunks, causal, out, lse, scale, TR_F32, ws, (size_t)TR_NOALLOC_SCRATCH_BYTES, hip_stream);
}

int64_t tr_schedule_steps(int schedule, int n_devices, int n_inner, int causal, int32_t* steps_out, int64_t capacity) {
  g_err[0] = 0;
  if (n_devices < 1 || n_devices > 4096) { fail(TR_ERR_SHAPE, "n_devices %d out of range [1, 4096]", n_devices); return -1; }
  if (schedule < TR_SCHED_TOKENRING || schedule > TR_SCHED_HYBRID) { fail(TR_ERR_UNSUPPORTED, "unknown schedule %d", schedule); return -1; }
  if (schedule == TR_SCHED_ZIGZAG && !causal) { fail(TR_ERR_UNSUPPORTED, "the zigzag partition only exists for the causal case"); return -1; }
  if (schedule == TR_SCHED_HYBRID && (n_inner < 1 || n_devices % n_inner)) {
    fail(TR_ERR_SHAPE, "hybrid schedule: n_inner %d must divide n_devices %d", n_inner, n_devices);
    return -1;
  }
  std::vector<RingStep> steps;
  const int n_seg = build_schedule(schedule, n_devices, n_inner, causal != 0, steps, true);
  const std::vector<LaunchGroup> groups = group_steps(steps, n_seg);
  int64_t n_out = 0;   // a step on a pair of K/V segments is reported as its two segment pairs
  for (size_t g = 0; g < groups.size(); g++)
    for (size_t i = groups[g].begin; i < groups[g].end; i++)
      for (int half = 0; half < (steps[i].ks2 >= 0 ? 2 : 1); half++, n_out++)
        if (steps_out && n_out < capacity) {
          steps_out[3 * n_out] = steps[i].qs;
          steps_out[3 * n_out + 1] = half ? steps[i].ks2 : steps[i].ks;
          steps_out[3 * n_out + 2] = (int32_t)g;
        }
  return n_out;
}

tr_status tr_ring_attn_sched(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v, int n_devices, int causal,
                             int schedule, int n_inner, const tr_tensor* out, const tr_tensor* lse, float scale,
                             void* hip_stream) {
  g_err[0] = 0;
  if (!q || !k || !v || !out || !lse) return fail(TR_ERR_NULL, "a tensor descriptor is NULL");
  if (n_devices < 1 || n_devices > 4096) return fail(TR_ERR_SHAPE, "n_devices %d out of range [1, 4096]", n_devices);
  if (schedule < TR_SCHED_TOKENRING || schedule > TR_SCHED_HYBRID) return fail(TR_ERR_UNSUPPORTED, "unknown schedule %d", schedule);
  if (schedule == TR_SCHED_ZIGZAG && !causal)
    return fail(TR_ERR_UNSUPPORTED, "the zigzag partition only exists for the causal case");
  if (schedule == TR_SCHED_HYBRID && (n_inner < 1 || n_devices % n_inner))
    return fail(TR_ERR_SHAPE, "hybrid schedule: n_inner %d must divide n_devices %d", n_inner, n_devices);
  const int n_seg = schedule == TR_SCHED_ZIGZAG ? 2 * n_devices : n_devices;
  if (q->S < 0 || q->S % n_seg) return fail(TR_ERR_SHAPE, "sequence length %lld is not a multiple of %d segments", (long long)q->S, n_seg);
  if (k->S != q->S || v->S != q->S) return fail(TR_ERR_SHAPE, "q, k, v must have the same sequence length");
  if (out->dtype != TR_F32) return fail(TR_ERR_DTYPE, "out must be fp32 (it is the merge accumulator)");
  if (q->D > 0 && !(scale > 0.f)) scale = 1.0f / sqrtf((float)q->D);
  tr_status st;
  if ((st = check_tensor("q", q, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("k", k, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("v", v, true, false, 16)) != TR_OK) return st;
  if ((st = check_tensor("out", out, false, true, 16)) != TR_OK) return st;
  if ((st = check_tensor("lse", lse, false, true, 4)) != TR_OK) return st;
  if ((st = check_written("out", out)) != TR_OK || (st = check_written("lse", lse)) != TR_OK) return st;
  if (out->B != q->B || out->H != q->H || out->S != q->S || out->D != q->D || lse->B != q->B || lse->H != q->H || lse->S != q->S || lse->D != 1)
    return fail(TR_ERR_SHAPE, "out/lse shape does not match q");

  if (overlaps(out, q) || overlaps(out, k) || overlaps(out, v) || overlaps(lse, q) || overlaps(lse, k) || overlaps(lse, v) || overlaps(out, lse))
    return fail(TR_ERR_ALIAS, "outputs overlap inputs or each other");
  std::vector<RingStep> steps;
  // segments that are whole K/V tiles of either head dim can be attended in pairs
  build_schedule(schedule, n_devices, n_inner, causal != 0, steps, (q->S / n_seg) % 128 == 0);
  return run_steps_fused(q, k, v, out, lse, n_seg, causal != 0, scale, steps, hip_stream);
}

}  // extern "C"
