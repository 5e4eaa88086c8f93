/* A plain C program against the boundary header: the header must compile as C (not only as
 * C++), every entry point must link, and host-visible argument errors must come back as status
 * codes without any GPU work (every call below fails validation before it would touch a GPU). */
#include <stdio.h>
#include <string.h>
#include "parallelcomp.h"
#include "parallelcomp_bench.h"

#define EXPECT(expr, want)                                                        \
  do {                                                                            \
    int got_ = (expr);                                                            \
    if (got_ != (want)) {                                                         \
      printf("FAIL %s: got %d (%s), want %d\n", #expr, got_, pc_status_string(got_), (want)); \
      return 1;                                                                   \
    }                                                                             \
  } while (0)

int main(void) {
  pc_shape s;
  void* one = (void*)256;   /* never dereferenced */
  memset(&s, 0, sizeof s);
  s.n_chunks = 2; s.chunk_len = 64; s.query_len = 16; s.n_q_heads = 8; s.n_kv_heads = 2;
  s.head_dim = 128; s.obs_window = 8; s.rope_base = 1.0e4f; s.softmax_scale = 0.0f;
  if (strncmp(pc_version(), "parallelcomp", 12) != 0) { printf("FAIL version\n"); return 1; }
  if (pc_chunk_prefill_workspace_bytes(&s) == 0 || pc_chunk_query_scores_workspace_bytes(&s) == 0) {
    printf("FAIL workspace size\n"); return 1;
  }
  EXPECT(pc_chunk_prefill_attn(&s, NULL, one, one, NULL, one, (float*)one, NULL, NULL, NULL, one, 1u << 30, NULL), PC_ERR_NULL);
  EXPECT(pc_chunk_prefill_attn(&s, one, one, one, NULL, one, (float*)one, NULL, NULL, NULL, one, 16, NULL), PC_ERR_WORKSPACE);
  s.head_dim = 96;
  EXPECT(pc_chunk_query_scores(&s, one, one, NULL, (float*)one, NULL, one, 1u << 30, NULL), PC_ERR_SHAPE);
  s.head_dim = 128;
  EXPECT(pc_select_chunks_topk((const float*)one, 4, 5, (int32_t*)one, NULL, NULL), PC_ERR_SHAPE);
  EXPECT(pc_select_tokens_topk(NULL, NULL, 1, 1, 8, 2, (int32_t*)one, NULL), PC_ERR_NULL);
  EXPECT(pc_select_tokens_calibrated((const float*)one, NULL, 1, 1, 8, 2, 0.5f, 5, 4, NULL, (int32_t*)one, (int32_t*)one, NULL), PC_ERR_SHAPE);
  EXPECT(pc_chunk_queue_update((const float*)one, 0, 0, 2, (int32_t*)one, (float*)one, (int32_t*)one, (int32_t*)one, NULL), PC_ERR_SHAPE);
  EXPECT(pc_gather_kv(one, one, NULL, NULL, 1, 2, 8, 1, 1, 4, 128, one, one, NULL), PC_ERR_NULL);
  EXPECT(pc_gather_kv_amax(one, one, NULL, (const int32_t*)one, 1, 2, 8, 1, 1, 4, 96, one, one, (float*)one, (float*)one, NULL), PC_ERR_SHAPE);
  EXPECT(pc_parallel_attn(NULL, one, one, NULL, 0, NULL, NULL, 1, 1, 2, 64, 8, 2, 128, -1, 1.0e4f, 0.0f, one, NULL, one, 1u << 30, NULL), PC_ERR_NULL);
  EXPECT(pc_parallel_attn_static(one, one, one, NULL, 0, NULL, NULL, 1, 64, 2, 64, 8, 2, 128, -1, 1.0e4f, 0.0f, one, NULL, NULL), PC_ERR_UNSUPPORTED);
  EXPECT(pc_kv_append(one, one, 2, 1, 3, 3, 64, 2, 128, 10, 1.0e4f, one, one, (int32_t*)one, 0, NULL), PC_ERR_SHAPE);
  EXPECT(pc_kv_quantize_fp8(NULL, one, NULL, 0, 2, 3, 64, 2, 128, one, one, (float*)one, (float*)one, NULL), PC_ERR_NULL);
  EXPECT(pc_kv_quantize_fp8_amax(one, one, NULL, (const float*)one, NULL, 0, 1, 1, 4, 1, 128, one, one, (float*)one, (float*)one, NULL), PC_ERR_NULL);
  EXPECT(pc_parallel_attn_fp8(one, NULL, one, (const float*)one, (const float*)one, NULL, 0, NULL, NULL, NULL, 0, NULL, NULL, 1, 1, 2, 64, 8, 2, 128, -1, 1.0e4f, 0.0f, one, NULL, one, 1u << 30, NULL), PC_ERR_NULL);
  EXPECT(pc_chunk_self_information(one, (const int32_t*)one, 1, 1, 7, 0, (float*)one, (float*)one, NULL), PC_ERR_SHAPE);
  EXPECT(pc_copy_ceiling(2, one, one, 1024, NULL), PC_ERR_SHAPE);
  if (pc_parallel_attn_static_max_bytes() != PC_STATIC_SCRATCH_BYTES) { printf("FAIL static size\n"); return 1; }
  printf("c abi ok: %s\n", pc_version());
  return 0;
}
