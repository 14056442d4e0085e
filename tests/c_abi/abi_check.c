/* Plain C99 client of the C ABI: the header must compile as C, the library must link from C,
 * and argument validation must work without any GPU call being made.  Exit code 0 = all good. */
#include <stdio.h>
#include <string.h>

#include "tokenring.h"

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, tr_last_error()); failures++; } } while (0)

int main(void) {
  tr_tensor q, k, v, out, lse;
  const tr_tensor* parts[1];
  memset(&q, 0, sizeof q);
  q.ptr = (void*)0x7f0000000000ull; q.dtype = TR_BF16; q.B = 1; q.H = 2; q.S = 64; q.D = 128;
  q.stride_s = 128; q.stride_h = 64 * 128; q.stride_b = 2 * 64 * 128;
  k = q; k.ptr = (void*)0x7f1000000000ull;
  v = q; v.ptr = (void*)0x7f2000000000ull;
  out = q; out.ptr = (void*)0x7f3000000000ull; out.dtype = TR_F32;
  lse = out; lse.ptr = (void*)0x7f4000000000ull; lse.D = 1; lse.stride_s = 1; lse.stride_h = 64; lse.stride_b = 128;

  EXPECT(strncmp(tr_version(), "tokenring-gfx950", 16) == 0);
  EXPECT(sizeof(tr_tensor) == 72);
  EXPECT(tr_block_attn(NULL, &k, &v, TR_MASK_NONE, 0.1f, &out, &lse, NULL) == TR_ERR_NULL);
  EXPECT(tr_block_attn(&q, &k, &v, 5, 0.1f, &out, &lse, NULL) == TR_ERR_UNSUPPORTED);
  EXPECT(strlen(tr_last_error()) > 0);
  EXPECT(tr_block_attn(&q, &k, &v, TR_MASK_NONE, -1.0f, &out, &lse, NULL) == TR_ERR_UNSUPPORTED);
  EXPECT(tr_block_attn_merge(&q, &k, &v, TR_MASK_NONE, 0.1f, &q, &lse, NULL) == TR_ERR_DTYPE);
  EXPECT(tr_merge(&out, &lse, &out, &lse, NULL) == TR_ERR_ALIAS);
  parts[0] = &out;
  EXPECT(tr_merge_n(&out, &lse, parts, parts, 0, 0, NULL) == TR_ERR_SHAPE);
  EXPECT(tr_ring_attn(&q, &k, &v, 3, 1, &out, &lse, 0.0f, NULL, 0, NULL) == TR_ERR_SHAPE);           /* 64 % 3 */
  EXPECT(tr_ring_attn_sched(&q, &k, &v, 4, 0, TR_SCHED_ZIGZAG, 1, &out, &lse, 0.0f, NULL) == TR_ERR_UNSUPPORTED);
  EXPECT(tr_ring_attn_blocks(&q, &k, &v, 4, 1, &out, &lse, 0.0f, TR_F32, NULL, 0, NULL) == TR_ERR_WORKSPACE);
  EXPECT(tr_ring_attn_workspace_bytes(&q, 4) == 2 * 16 * 128 * 4 + 256);   /* block_out, then block_lse rounded up to 256 B */
  EXPECT(tr_ring_attn_blocks_workspace_bytes(&q, 4, TR_BF16) == 2 * 16 * 128 * 2 + 256);
  EXPECT(tr_time_next_kernel(NULL, NULL) == TR_OK);
  if (failures == 0) printf("c abi ok\n");
  return failures;
}
