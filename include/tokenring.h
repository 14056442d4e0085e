/*
 * tokenring.h - C ABI of the MI355X (gfx950) implementation of TokenRing's per-device
 * compute path: blockwise attention, the log-sum-exp Update (merge), and the ring
 * schedule of (Query chunk, K/V chunk) steps replayed on one GPU.
 *
 * Source of the operations: TokenRing (arXiv 2412.20501).
 *   - Attention(Q, K, V) -> block_out, block_lse : Algorithm 1 and Sec. 3.2
 *   - Update(block_out, block_lse) -> Out, Lse    : the two equations of Sec. 3.1
 *   - iteration order of the steps                : Algorithm 1, walk-through of Sec. 3.3.1
 *   - causal chunks                               : Sec. 3.3.2
 *
 * Conventions common to every call
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees or keeps device memory between calls.
 *   - Layout is [B, H, S, D] with D contiguous; strides are in elements.  lse tensors
 *     are [B, H, S] and use D = 1, stride_s = 1 normally.  (The paper's (N,H,D)/(H,N)
 *     layout can be passed through the strides.)
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work on
 *     it and return without synchronising.
 *   - A tensor a call writes (out, lse, out_acc, lse_acc) must not overlap itself: a stride of 0
 *     or one smaller than what lies inside it on a dimension larger than 1 is TR_ERR_STRIDE.
 *   - Every call validates its arguments first; on an error nothing is launched, the
 *     status is returned and tr_last_error() describes it.  No exception crosses the ABI.
 *   - Grouped-query attention: q.H must be a multiple of k.H; query head h reads K/V
 *     head h / (q.H / k.H).
 *   - lse is the natural-log log-sum-exp of the scaled scores.  A row with no allowed key
 *     has out = 0 and lse = -inf, which is also the identity element of tr_merge.
 */
#ifndef TOKENRING_H
#define TOKENRING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TR_OK = 0,
  TR_ERR_NULL = 1,        /* a required pointer is NULL                               */
  TR_ERR_DTYPE = 2,       /* dtype not supported for that argument                    */
  TR_ERR_SHAPE = 3,       /* shapes inconsistent or head dim unsupported              */
  TR_ERR_STRIDE = 4,      /* stride too small for the shape, or misaligned            */
  TR_ERR_ALIAS = 5,       /* accumulator and block tensors overlap                    */
  TR_ERR_UNSUPPORTED = 6, /* valid request this build cannot run                      */
  TR_ERR_WORKSPACE = 7,   /* workspace NULL, misaligned or too small                  */
  TR_ERR_HIP = 8          /* a HIP runtime call failed (launch error)                 */
} tr_status;

typedef enum { TR_BF16 = 0, TR_F32 = 1 } tr_dtype;

typedef enum {
  TR_MASK_NONE = 0,        /* every key is visible                                    */
  TR_MASK_CAUSAL_DIAG = 1  /* diagonal chunk: key index <= query index (needs Sq==Sk) */
} tr_mask_kind;

/* A strided view of device memory.  Element (b,h,s,d) is at
 * ptr + (b*stride_b + h*stride_h + s*stride_s + d) elements of `dtype`. */
typedef struct {
  void* ptr;      /* device pointer; 16-byte aligned for bf16 Q/K/V and all out tensors */
  int32_t dtype;  /* tr_dtype */
  int64_t B, H, S, D;
  int64_t stride_b, stride_h, stride_s;
} tr_tensor;

/*
 * One block step of Algorithm 1 (Sec. 3.2): block_out, block_lse <- Attention(Q, K, V).
 *   out[b,h,r,:] = sum_c softmax_c(scale * <q[b,h,r,:], k[b,g,c,:]>) v[b,g,c,:]
 *   lse[b,h,r]   = ln sum_c exp(scale * <q[b,h,r,:], k[b,g,c,:]>)
 * over the keys c the mask allows.
 *   q   [B,Hq,Sq,D] bf16      k, v [B,Hkv,Sk,D] bf16      D in {64, 128}
 *   out [B,Hq,Sq,D] bf16 or fp32 (written)                lse [B,Hq,Sq] fp32 (written)
 * Sq and Sk are arbitrary (0 allowed; Sk == 0 gives out = 0, lse = -inf).
 * Strides of q/k/v/out must be multiples of 8 elements (16-byte rows); stride_s of k and v at
 * most 2^24 elements.
 * Arithmetic: bf16 MFMA with fp32 accumulation, fp32 softmax, probabilities rounded to
 * bf16 before the PV product.
 */
tr_status tr_block_attn(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v,
                        int mask_kind, float scale,
                        const tr_tensor* out, const tr_tensor* lse, void* hip_stream);

/*
 * Block step with the causal rule at arbitrary chunk positions (Sec. 3.3.2; needed for
 * the zigzag partition where a chunk is not aligned with the diagonal): query row r sits
 * at sequence position q_pos0 + r, key c at k_pos0 + c, and key c is visible iff
 * k_pos0 + c <= q_pos0 + r.  Rows that see no key get out = 0, lse = -inf.
 * Same tensors as tr_block_attn; Sq and Sk need not be equal.
 */
tr_status tr_block_attn_causal_at(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v,
                                  int64_t q_pos0, int64_t k_pos0, float scale,
                                  const tr_tensor* out, const tr_tensor* lse, void* hip_stream);

/*
 * Block step fused with the Update (Algorithm 1's Attention followed by Update, Sec. 3.1-3.2):
 * the block result is never written out; the kernel's epilogue merges it straight into the
 * fp32 accumulators, exactly as tr_merge would (same arithmetic, same identity handling).
 *   q [B,Hq,Sq,D] bf16   k, v [B,Hkv,Sk,D] bf16   D in {64, 128}
 *   out_acc [B,Hq,Sq,D] fp32 (read + written)   lse_acc [B,Hq,Sq] fp32 (read + written)
 * Rows whose lse_acc is -inf are treated as empty: their out_acc need not be initialised.
 */
tr_status tr_block_attn_merge(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v,
                              int mask_kind, float scale,
                              const tr_tensor* out_acc, const tr_tensor* lse_acc, void* hip_stream);

/*
 * Out, Lse <- Update(block_out, block_lse), the two equations of Sec. 3.1, in place:
 *   out_acc <- out_acc - sigmoid(block_lse - lse_acc) * (out_acc - block_out)
 *   lse_acc <- lse_acc - ln(sigmoid(lse_acc - block_lse))
 * evaluated as lse' = max + ln(1 + exp(-|diff|)) and w = exp(block_lse - lse') so that the
 * identity element (out = 0, lse = -inf) on either side is exact and never yields NaN.
 *   out_acc   [B,H,S,D] fp32 (read + written)    lse_acc   [B,H,S] fp32 (read + written)
 *   block_out [B,H,S,D] fp32 or bf16 (read)      block_lse [B,H,S] fp32 (read)
 * D must be a multiple of 4 (fp32 and bf16 blocks alike); any S (0 allowed).
 * The accumulator tensors must not overlap the block tensors (TR_ERR_ALIAS).
 */
tr_status tr_merge(const tr_tensor* out_acc, const tr_tensor* lse_acc,
                   const tr_tensor* block_out, const tr_tensor* block_lse, void* hip_stream);

/*
 * The Update of Sec. 3.1 folded over n partial results in one pass (n-ary merge):
 *   lse = ln sum_i exp(block_lse_i),   out = sum_i exp(block_lse_i - lse) * block_out_i
 * (evaluated relative to the largest block_lse).  Because the Update is associative and
 * commutative this equals n pairwise tr_merge calls up to fp32 rounding, but every partial is
 * read once and the result written once.
 *   out [B,H,S,D] fp32, lse [B,H,S] fp32: written; with accumulate != 0 their old contents take
 *     part as one more partial (read + written), otherwise they need not be initialised.
 *   block_outs[i] [B,H,S,D] fp32 or bf16 (one dtype for all), block_lses[i] [B,H,S] fp32, i < n,
 *     1 <= n <= 16: host arrays of n descriptor pointers; all partials share their strides.
 * A partial row with lse = -inf has weight 0 and its out values are ignored; if every partial
 * of a row is empty the result is out = 0, lse = -inf.  D must be a multiple of 4.
 * The partials must not overlap out / lse (TR_ERR_ALIAS).
 */
tr_status tr_merge_n(const tr_tensor* out, const tr_tensor* lse,
                     const tr_tensor* const* block_outs, const tr_tensor* const* block_lses,
                     int n, int accumulate, void* hip_stream);

/*
 * The whole schedule of Algorithm 1 on one GPU, without communication: Q, K, V are split
 * into n_chunks chunks along S; for i in 0..n-1, for j in 0..n-1 the "device" j attends
 * Query chunk c = (j - i) mod n to its K_j, V_j and the block result is merged into
 * out[c], lse[c] with the Update above.  With causal != 0 (contiguous chunks, Sec. 3.3.2)
 * steps with j > c are skipped and j == c uses the diagonal mask.
 *   q [B,Hq,S,D] bf16   k, v [B,Hkv,S,D] bf16   out [B,Hq,S,D] fp32   lse [B,Hq,S] fp32
 *   S must be a multiple of n_chunks; n_chunks >= 1; scale <= 0 selects 1/sqrt(D).
 *   workspace == NULL (workspace_bytes ignored): every step after a Query chunk's first one
 *   runs as tr_block_attn_merge, i.e. the Update happens in the attention kernel's epilogue;
 *   consecutive steps on distinct Query chunks (what different devices do at the same time)
 *   share one kernel launch (tr_schedule_steps shows the grouping).
 *   workspace != NULL: the two-kernel form of Algorithm 1 - tr_block_attn writes one fp32
 *   block result (block_out, block_lse) into the workspace and tr_merge folds it into
 *   out/lse.  It needs at least tr_ring_attn_workspace_bytes(q, n_chunks) bytes, 256-byte
 *   aligned; its contents on return are unspecified.
 * Both forms apply the same Update arithmetic in the same order.  The first block of every
 * Query chunk is written straight into out/lse, so the caller need not initialise them.  All
 * launches go to `hip_stream` in a fixed order, hence the result is bitwise reproducible.
 */
tr_status tr_ring_attn(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v,
                       int n_chunks, int causal,
                       const tr_tensor* out, const tr_tensor* lse, float scale,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Algorithm 1 in its literal two-kernel form with a chosen format for the block result that
 * travels between the Attention and the Update (Sec. 3.1 notes the volume of block_out and
 * block_lse): block_dtype = TR_F32 is tr_ring_attn with a workspace; TR_BF16 halves block_out
 * (what a multi-device run would put on the wire) at the cost of one bf16 rounding (at most 2^-8
 * relative) of every block before it is merged.  block_lse stays fp32.  The workspace is
 * required, 256-byte aligned, at least tr_ring_attn_blocks_workspace_bytes(q, n_chunks,
 * block_dtype) bytes.  Everything else as in tr_ring_attn.
 */
tr_status tr_ring_attn_blocks(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v,
                              int n_chunks, int causal,
                              const tr_tensor* out, const tr_tensor* lse, float scale,
                              int block_dtype, void* workspace, size_t workspace_bytes, void* hip_stream);
size_t tr_ring_attn_blocks_workspace_bytes(const tr_tensor* q, int n_chunks, int block_dtype);

/*
 * tr_ring_attn in its two-kernel form for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The block result that
 * travels from tr_block_attn to tr_merge (fp32 block_out + block_lse of one step) lives in a
 * device array inside the library (TR_NOALLOC_SCRATCH_BYTES, held by every GPU the library runs on
 * until the process ends) instead of a caller workspace; the call allocates and frees nothing on
 * the device and calls no allocating library routine.  Limit: one block result,
 *   align256(B * Hq * (S / n_chunks) * D * 4) + align256(B * Hq * (S / n_chunks) * 4) bytes,
 * must fit the array; larger problems return TR_ERR_WORKSPACE (use tr_ring_attn with a workspace).
 * Arguments, checks, arithmetic and results are those of tr_ring_attn with a workspace (bitwise).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or threads) race and must be serialised by the caller.  Nothing in the array needs
 * clearing: every step overwrites the block result before the Update reads it.
 */
#define TR_NOALLOC_SCRATCH_BYTES (8 * 1024 * 1024 + 64 * 1024)
tr_status tr_ring_attn_noalloc(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v,
                               int n_chunks, int causal,
                               const tr_tensor* out, const tr_tensor* lse, float scale, void* hip_stream);

/* Order in which tr_ring_attn_sched runs the block steps (all "devices" replayed on one GPU). */
typedef enum {
  TR_SCHED_TOKENRING = 0,      /* Algorithm 1: Q circulates, device j keeps K_j, V_j              */
  TR_SCHED_RING_ATTENTION = 1, /* Sec. 2.1: K/V circulate, device j keeps Q_j                     */
  TR_SCHED_ZIGZAG = 2,         /* Sec. 3.3.2: 2n segments, device g owns g and 2n-1-g (causal)    */
  TR_SCHED_HYBRID = 3          /* Sec. 3.3.3: Ring Attention between nodes, Algorithm 1 inside    */
} tr_schedule;

/*
 * tr_ring_attn with a selectable schedule; the Update always runs in the attention epilogue
 * (no workspace).  The sequence is cut into n_devices equal chunks (2 * n_devices segments for
 * TR_SCHED_ZIGZAG, which requires causal != 0); S must be a multiple of that.
 *   TR_SCHED_TOKENRING      for i, for j: Q chunk (j-i) mod n  x  K/V chunk j       (bitwise equal to
 *                           tr_ring_attn with workspace == NULL)
 *   TR_SCHED_RING_ATTENTION for i, for j: Q chunk j  x  K/V chunk (j-i) mod n
 *   TR_SCHED_ZIGZAG         for i, for j: the Query pair {c, 2n-1-c}, c = (j-i) mod n, against the K/V pair
 *                           {j, 2n-1-j}; of the four segment pairs the causal rule keeps two full ones
 *                           (three on i == 0, two of them diagonal), so every (i, j) carries the same work.  When the
 *                           later Query segment meets both K/V segments of the device and the segment length is a
 *                           multiple of 128, the two are attended in ONE block step over the device's whole K/V (one
 *                           softmax over both, one Update), which leaves the result of Sec. 3.1's Update unchanged; an iteration is then
 *                           a single launch of at most two steps per device.  Otherwise the devices' pairs are issued
 *                           slot by slot (all first pairs, then all second, ...)
 *   TR_SCHED_HYBRID         n_devices = nodes x n_inner; for t < nodes, for i < n_inner, for node, for p:
 *                           Q chunk node*n_inner + (p-i) mod n_inner  x  K/V chunk ((node-t) mod nodes)*n_inner + p
 *                           (n_inner is ignored by the other schedules)
 * With causal != 0 a step whose K/V segment lies after its Query segment is dropped and equal
 * segments use the diagonal mask.  Every schedule reaches the same result up to fp32 rounding of
 * the merge order; each is bitwise reproducible.  Tensors, scale and stream as in tr_ring_attn.
 */
tr_status tr_ring_attn_sched(const tr_tensor* q, const tr_tensor* k, const tr_tensor* v,
                             int n_devices, int causal, int schedule, int n_inner,
                             const tr_tensor* out, const tr_tensor* lse, float scale, void* hip_stream);

/*
 * Host-only view of what tr_ring_attn_sched (and the fused tr_ring_attn, schedule
 * TR_SCHED_TOKENRING) will run: the block steps of a schedule in execution order.  Returns
 * the number of steps, or -1 on invalid arguments (tr_last_error() says why).  If steps_out
 * (HOST memory, 3 * capacity int32) is given, step i < capacity is written as
 *   steps_out[3i] = Query segment, steps_out[3i+1] = K/V segment, steps_out[3i+2] = index of
 *   the attention launch that carries the step
 * (steps of one launch touch distinct Query segments and run concurrently; launches run in
 * order).  Segments are n_devices equal chunks of S, 2 * n_devices for TR_SCHED_ZIGZAG; with
 * causal != 0 a step with equal segments is the diagonal-masked one.  For TR_SCHED_ZIGZAG the
 * list is the one for segment lengths that are multiples of 128: a block step over a pair of
 * K/V segments appears as its two (Query segment, K/V segment) entries, adjacent and in the
 * same launch, the only case of a Query segment occurring twice in a launch.  Touches no device.
 */
int64_t tr_schedule_steps(int schedule, int n_devices, int n_inner, int causal, int32_t* steps_out, int64_t capacity);

/* Bytes of workspace the two-kernel form of tr_ring_attn needs for these shapes (0 on invalid arguments). */
size_t tr_ring_attn_workspace_bytes(const tr_tensor* q, int n_chunks);

/*
 * Measurement aid (no operation of the paper): arms two hipEvent_t handles (either may be
 * NULL; both NULL disarms) for the calling thread.  The next kernel any entry point launches
 * from this thread carries them in its dispatch: start_event then holds the time the kernel
 * began executing and stop_event the time it finished, so hipEventElapsedTime(start, stop)
 * is the kernel's own duration without queueing gaps.  Only that one launch is timed
 * (tr_ring_attn: its first kernel); the events stay owned by the caller.  Always TR_OK.
 */
tr_status tr_time_next_kernel(void* start_event, void* stop_event);

/* Description of the last error on the calling thread ("" if none). Static storage. */
const char* tr_last_error(void);

/* Library version string, "tokenring-gfx950 <version> (sources <16 hex digits>)": the digits are a hash of
 * the kernel sources, headers and compiler flags the library was built from.  Static storage. */
const char* tr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TOKENRING_H */
