/*
 * parallelcomp.h - C ABI of the MI355X (gfx950) ParallelComp hot path.
 *
 * One transformer layer of the paper's method (section 3.1):
 *   chunked local attention with chunk-local RoPE positions   (Eq. 1-2, "Parallel attention")
 *   cumulative query->key attention scores                     (Eq. 5-6, "Parallel KV cache eviction")
 *   chunk selection by a per-chunk score, fixed count          (Eq. 3-4 mechanics, "Chunk eviction")
 *   per-head token selection and KV compaction                 (Eq. 7)
 *   global attention of the query over all surviving KV        (Eq. 9-11, "Global attention")
 *
 * Conventions for every call
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or keeps them.  Scratch memory comes from the caller's workspace `ws`
 *     (device memory, 256-byte aligned), whose minimum size the matching *_workspace_bytes
 *     function returns; it may be reused between calls on the same stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work and return; they never synchronise with the host.
 *   - bf16 tensors are raw 16-bit patterns.  All layouts are row-major with the head
 *     dimension D innermost and contiguous.  Supported D: 64 and 128.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - RoPE pairs dimension i with i + D/2 and uses theta_i = rope_base^(-2i/D).
 *   - Return value: PC_OK or a negative pc_status.  Host-visible arguments are validated
 *     before any GPU work; nothing is launched when an error is returned.  The contents of
 *     device buffers are not validated, except that selection indices handed to pc_gather_kv
 *     that fall outside the source are read as rows of zeros instead of faulting.
 *   - No call throws or aborts across this boundary.
 */
#ifndef PARALLELCOMP_H
#define PARALLELCOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pc_status {
  PC_OK = 0,
  PC_ERR_NULL = -1,        /* a required pointer is NULL                                    */
  PC_ERR_SHAPE = -2,       /* a size is out of range or inconsistent                        */
  PC_ERR_WORKSPACE = -3,   /* ws is NULL, misaligned or smaller than *_workspace_bytes      */
  PC_ERR_HIP = -4,         /* a HIP call failed; see pc_last_hip_error()                    */
  PC_ERR_UNSUPPORTED = -5  /* valid request this build has no kernel for                    */
} pc_status;

/* Shape of a chunk batch (section 3.1): C sequences, each = [w context rows ; w_q query rows],
 * L = w + w_q, the position id of a row is its index in [0, L) and restarts in every chunk. */
typedef struct pc_shape {
  int32_t n_chunks;      /* C  >= 1                                                          */
  int32_t chunk_len;     /* w  >= 1                                                          */
  int32_t query_len;     /* w_q >= 0                                                         */
  int32_t n_q_heads;     /* H_q, multiple of n_kv_heads                                      */
  int32_t n_kv_heads;    /* H_kv                                                             */
  int32_t head_dim;      /* D in {64, 128}                                                   */
  int32_t obs_window;    /* w_obs: the last w_obs rows of each sequence vote; 1..L (1..w_q
                            when chunk_lens is given); w_obs = w_q is Eq. 6 as printed         */
  float   rope_base;     /* e.g. 1e4, 5e5                                                    */
  float   softmax_scale; /* 0 => 1/sqrt(D)                                                   */
} pc_shape;

/* ---- Eq. 1-2 (+ Eq. 5-6 when tok_score != NULL) --------------------------------------------
 * Local attention inside every chunk sequence, all chunks in one launch: rotate q and k at the
 * chunk-local positions, o = softmax(q' k'^T * scale, causal j <= r) v, lse = row logsumexp.
 *   q  [C, L, H_q, D]  bf16, before RoPE            k, v [C, L, H_kv, D] bf16, k before RoPE
 *   o  [C, L, H_q, D]  bf16 out                     lse  [C, H_q, L]     fp32 out (natural log)
 *   k_rope [C, L, H_kv, D] bf16 out, nullable: the rotated keys (the KV cache the later
 *          steps gather from); when NULL they are not written.
 *   tok_score [C, H_kv, w] fp32 out, nullable; chunk_score [C] fp32 out, nullable (needs
 *          tok_score): exactly what pc_chunk_query_scores writes, from the same launch queue.
 *   chunk_lens [C] int32 (device), nullable: ragged chunks ("at most w tokens" per chunk,
 *          sec. 3.1).  Chunk c then holds chunk_lens[c] <= w context rows (clamped to [0, w]) and
 *          its sequence is rows [0, chunk_lens[c] + w_q) of q[c], k[c], v[c]: the query rows
 *          follow the context directly, at positions chunk_lens[c] + t.  Rows behind a short
 *          sequence are padding: o and lse there are not written, tok_score of the missing
 *          tokens is 0, k_rope there is unspecified.  NULL => every chunk has w rows.
 * Arithmetic: bf16 MFMA products, fp32 softmax and accumulation.  The operands are the rotated
 * k rounded to bf16 (the cache's precision) and the rotated q multiplied by scale * log2(e) in
 * fp32 and then rounded to bf16, once; probabilities are rounded to bf16 for the second product.
 * Workspace: pc_chunk_prefill_workspace_bytes(shape). */
int pc_chunk_prefill_attn(const pc_shape* shape, const void* q, const void* k, const void* v,
                          const int32_t* chunk_lens, void* o, float* lse, void* k_rope, float* tok_score,
                          float* chunk_score, void* ws, size_t ws_bytes, void* stream);
size_t pc_chunk_prefill_workspace_bytes(const pc_shape* shape);

/* ---- Eq. 5-6 -------------------------------------------------------------------------------
 * Cumulative attention of the voting rows R = {L - w_obs, ..., L - 1} to every chunk key
 * (with chunk_lens, as in pc_chunk_prefill_attn: L = chunk_lens[c] + w_q and j < chunk_lens[c]):
 *   tok_score[c, g, j] = sum_{h in group g} sum_{r in R} P[c, h, r, j],  j < w
 *   chunk_score[c]     = sum_g sum_j tok_score[c, g, j]                    (nullable)
 * where P[c, h, r, :] is row r of Eq. 1 (softmax over all causal keys j <= r of the sequence,
 * query keys included).  q, k as in pc_chunk_prefill_attn (before RoPE).  The probability
 * block is never written to memory.  Logits are computed from split bf16 (hi + lo) operands
 * with fp32 accumulation, i.e. to about fp32 accuracy, so that selections are stable.
 * Workspace: pc_chunk_query_scores_workspace_bytes(shape). */
int pc_chunk_query_scores(const pc_shape* shape, const void* q, const void* k,
                          const int32_t* chunk_lens, float* tok_score, float* chunk_score,
                          void* ws, size_t ws_bytes, void* stream);
size_t pc_chunk_query_scores_workspace_bytes(const pc_shape* shape);

/* ---- Eq. 3 ----------------------------------------------------------------------------------
 * Self-information of the query tokens given each chunk, from the language model's logits:
 *   token_nll[c, t] = log sum_v exp(logits[c, t, v]) - logits[c, t, targets[t]]      (nats)
 *   info[c]         = sum_t token_nll[c, t] = -log P(X^q | X^c), or its negative if negate != 0
 *                     (so that pc_select_chunks_topk, which keeps the largest scores, keeps the
 *                     chunks of lowest self-information, as Eq. 4 asks)
 *   logits  [n_chunks, n_tokens, vocab] bf16 (device): row (c, t) = the logits that predict query
 *           token t after chunk c; producing them (the LM head) is the caller's business
 *   targets [n_tokens] int32 (device), clamped to [0, vocab);  token_nll [n_chunks, n_tokens] fp32
 *           out (also the scratch of the reduction: required);  info [n_chunks] fp32 out.
 * fp32 accumulation in a fixed order (deterministic).  vocab % 8 == 0, 8 <= vocab <= 2^24,
 * n_chunks * n_tokens < 2^31, logits 16-byte aligned.  No workspace. */
int pc_chunk_self_information(const void* logits, const int32_t* targets, int32_t n_chunks,
                              int32_t n_tokens, int32_t vocab, int32_t negate, float* token_nll,
                              float* info, void* stream);

/* ---- Eq. 3-4 mechanics ---------------------------------------------------------------------
 * Keep a fixed number of chunks: out_idx[0..k) = indices of the k largest chunk_score under
 * the total order (score descending, index ascending), in that rank order; out_score
 * (nullable) the matching scores.  NaN orders below every number.  1 <= k <= n <= 4096.
 * The score is the caller's choice (here: the query's attention mass on the chunk, larger is
 * better; the paper's self-information would be passed negated). */
int pc_select_chunks_topk(const float* chunk_score, int32_t n, int32_t k,
                          int32_t* out_idx, float* out_score, void* stream);

/* ---- sec. 3.1 "Chunk eviction": the fixed-size priority queue, a batch at a time -------------
 * The chunks are encoded in memory-sized batches and a fixed-size priority queue keeps the best
 * ones; only the chunks in the queue keep their compressed KV.  The queue lives on the device:
 *   queue_id    [capacity] int32  chunk ids in rank order (score descending, earlier chunk first
 *                                 on ties, NaN lowest); -1 = empty entry.  Fill with -1 to start.
 *   queue_score [capacity] fp32   their scores
 *   queue_slot  [capacity] int32  the KV slot (0 .. capacity-1) each entry owns
 * One call merges a batch: batch_score [n_batch] fp32 are the scores of the chunks with ids
 * chunk_id0 .. chunk_id0 + n_batch - 1 (ids grow from batch to batch).  After it the queue holds
 * the top `capacity` of all chunks seen so far, i.e. what pc_select_chunks_topk returns on the
 * whole prefix.  A chunk that stays keeps its slot; the entrants, in rank order, take the free
 * slots (never used, or freed by a chunk that left) in ascending order.
 *   slot_src [capacity] int32 out: slot_src[s] = index within this batch (0 .. n_batch-1) of the
 *     chunk that enters slot s, or -1 if slot s keeps its content.  Passed as chunk_idx (n_sel =
 *     capacity) to pc_select_tokens_topk / pc_select_tokens_calibrated and pc_gather_kv, it makes
 *     them process exactly the entrants, each into its own slot, with no host round trip.
 * 1 <= n_batch, capacity <= 1024.  One small workgroup; calls on one stream are ordered. */
int pc_chunk_queue_update(const float* batch_score, int32_t n_batch, int32_t chunk_id0,
                          int32_t capacity, int32_t* queue_id, float* queue_score,
                          int32_t* queue_slot, int32_t* slot_src, void* stream);

/* ---- Eq. 7 (index sets) --------------------------------------------------------------------
 * For every selected chunk s < n_sel and KV head g: the k tokens of
 * tok_score[chunk_idx[s], g, 0:chunk_len] that are largest under (score descending, index
 * ascending), written in ascending index order.
 *   tok_score [n_chunks_total, H_kv, chunk_len] fp32   chunk_idx [n_sel] int32, NULL => s;
 *             an entry chunk_idx[s] < 0 is skipped: out_idx[s] (and out_cnt[s]) stay as they are
 *   out_idx   [n_sel, H_kv, k] int32.        1 <= k <= chunk_len <= 32768.   No workspace. */
int pc_select_tokens_topk(const float* tok_score, const int32_t* chunk_idx, int32_t n_sel,
                          int32_t n_kv_heads, int32_t chunk_len, int32_t k,
                          int32_t* out_idx, void* stream);

/* ---- Eq. 8 then Eq. 7 (attention calibration + compression) ---------------------------------
 * As pc_select_tokens_topk, after evicting R_H: the tokens j of ONE position class
 * class_lo <= j < class_hi (the appendix's first 100 / last 100 / the rest) whose score is
 * strictly above lambda (a NaN score is not).  Of the remaining tokens the k best are kept, so
 * head (s, g) keeps out_cnt[s, g] = min(k, chunk_len - |R_H|) tokens:
 *   out_idx [n_sel, H_kv, k] int32 ascending, entries past out_cnt[s, g] are -1 (pc_gather_kv
 *   turns them into zero rows; pass out_cnt to pc_parallel_attn as per-head seg_len)
 *   out_cnt [n_sel, H_kv] int32.
 * chunk_lens [n_chunks_total] int32 (device, nullable): chunk c holds only chunk_lens[c] tokens
 * (ragged chunks); the missing ones are never kept, so out_cnt = min(k, chunk_lens[c] - |R_H|).
 * 0 <= class_lo <= class_hi <= chunk_len (an empty class gives Eq. 7), lambda not NaN
 * (+inf evicts nothing); otherwise as pc_select_tokens_topk.  No workspace. */
int pc_select_tokens_calibrated(const float* tok_score, const int32_t* chunk_idx, int32_t n_sel,
                                int32_t n_kv_heads, int32_t chunk_len, int32_t k, float lambda,
                                int32_t class_lo, int32_t class_hi, const int32_t* chunk_lens,
                                int32_t* out_idx, int32_t* out_cnt, void* stream);

/* ---- Eq. 7 (compressed KV cache) -----------------------------------------------------------
 * dst[b, s, g, t, :] = src[b, chunk_idx[b, s], tok_idx[b, s, g, t], g, :]  for K and V.
 *   k_src, v_src [batch, n_chunks, rows_per_chunk, H_kv, D] bf16 (a pure 16-bit copy)
 *   chunk_idx [batch, n_sel] int32, NULL => s      tok_idx [batch, n_sel, H_kv, k] int32
 *   k_dst, v_dst [batch, n_sel, H_kv, k, D].   Token indices outside the source (and chunk
 *   indices >= n_chunks) give zero rows; a segment with chunk_idx[b, s] < 0 is left untouched. */
int pc_gather_kv(const void* k_src, const void* v_src, const int32_t* chunk_idx,
                 const int32_t* tok_idx, int32_t batch, int32_t n_chunks,
                 int32_t rows_per_chunk, int32_t n_sel, int32_t n_kv_heads, int32_t k,
                 int32_t head_dim, void* k_dst, void* v_dst, void* stream);

/* ---- Eq. 9-11 ------------------------------------------------------------------------------
 * Global ("parallel") attention of n_q query rows over the concatenation of S compressed
 * segments and, optionally, the causal self segment of the query's own keys:
 *   out[b, t, h, :] = softmax over { kc[b, s, g, 0:seg_len[b,s]] for all s } U
 *                                  { k_self[b, 0..t, g] } of q . k * scale, times the values.
 * Computed as independent per-segment (and per-split) softmaxes merged exactly by logsumexp:
 *   LSE = log sum_p exp(lse_p),  out = sum_p exp(lse_p - LSE) o_p.
 *   q [B, n_q, H_q, D] bf16; if q_pos0 >= 0 it is rotated here at positions q_pos0 + t,
 *     if q_pos0 < 0 it is taken as already rotated.
 *   kc, vc [B, S, H_kv, k_t, D] bf16, keys already rotated (chunk-local positions kept)
 *   seg_len int32 valid rows per segment, NULL => k_t: [B, S] if seg_len_per_head = 0,
 *     [B, S, H_kv] (one length per KV head, as Eq. 8 leaves them) if seg_len_per_head = 1
 *   k_self, v_self [B, n_q, H_kv, D] bf16 rotated keys / values of the query rows, both NULL
 *     for no self segment (decode)
 *   out [B, n_q, H_q, D] bf16;  lse_out [B, H_q, n_q] fp32, nullable.
 * n_q * (H_q / H_kv) <= 16 runs the HBM-bound split-KV kernel (bf16 operands as given, scale
 * applied to the fp32 logits); larger n_q the MFMA tile kernel, whose query operand is the rotated
 * q times scale * log2(e), rounded to bf16 once when q_pos0 >= 0 (a q that arrives rotated,
 * q_pos0 < 0, is scaled and rounded a second time).
 * Workspace: pc_parallel_attn_workspace_bytes(...). */
int pc_parallel_attn(const void* q, const void* kc, const void* vc, const int32_t* seg_len,
                     int32_t seg_len_per_head, const void* k_self, const void* v_self, int32_t batch, int32_t n_q,
                     int32_t n_seg, int32_t k_t, int32_t n_q_heads, int32_t n_kv_heads,
                     int32_t head_dim, int32_t q_pos0, float rope_base, float softmax_scale,
                     void* out, float* lse_out, void* ws, size_t ws_bytes, void* stream);
size_t pc_parallel_attn_workspace_bytes(int32_t batch, int32_t n_q, int32_t n_seg, int32_t k_t,
                                        int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                        int32_t has_self);

/* ---- decoding stage (Eq. 9-11 token by token) ------------------------------------------------
 * Append the keys / values of n_new newly generated tokens to segment `seg` of the compacted
 * cache, behind the seg_len[b, seg] rows it holds (the growing tail: query block + generated
 * tokens), and add n_new to seg_len[b, seg] on the device.  pc_parallel_attn with that seg_len is
 * then one decode step over [compressed segments ; tail], the new token included.
 *   k_new, v_new [B, n_new, H_kv, D] bf16; k_new before RoPE if pos0 >= 0 (rotated here at
 *     positions pos0 + t, which continue behind the query block), already rotated if pos0 < 0
 *   kc, vc [B, n_seg, H_kv, k_t, D] bf16 in/out;  seg_len [B, n_seg] int32 (device) in/out, or
 *     [B, n_seg, H_kv] when seg_len_per_head != 0 (the layout pc_parallel_attn takes after
 *     pc_select_tokens_calibrated; every head of the tail then advances by the same n_new)
 * Rows that do not fit (seg_len + n_new > k_t) are dropped and seg_len saturates at k_t: size the
 * tail segment for the longest generation.  Calls on one stream are ordered; no workspace.
 * Errors: PC_ERR_NULL, PC_ERR_SHAPE (seg outside [0, n_seg), head_dim not 64 / 128, rope_base
 * <= 1 with pos0 >= 0), PC_ERR_HIP.  batch == 0 or n_new == 0 is a no-op. */
int pc_kv_append(const void* k_new, const void* v_new, int32_t batch, int32_t n_new, int32_t n_seg,
                 int32_t seg, int32_t k_t, int32_t n_kv_heads, int32_t head_dim, int32_t pos0,
                 float rope_base, void* kc, void* vc, int32_t* seg_len, int32_t seg_len_per_head,
                 void* stream);

/* ---- 8-bit compressed cache for the decoding stage (extension) -------------------------------
 * The paper leaves the precision of the cache open (its decoding stage, Eq. 9-11 with one query
 * row, reads the whole compressed cache per token: the ms/token column of its throughput table).
 * Storing the compressed segments in 8 bits halves those bytes.  Format: OCP 8-bit float E4M3
 * (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, largest magnitude 448, no infinities),
 * one fp32 scale per (sequence, segment, KV head) for K and one for V:
 *   scale = max |x| over the segment's valid rows / 448 (1 if that maximum is 0), in fp32
 *   code  = E4M3(x / scale), fp32 division, round to nearest (ties to the even code), saturating
 * pc_kv_quantize_fp8:
 *   kc, vc [B, S, H_kv, k_t, D] bf16 (finite values);  seg_len as in pc_parallel_attn, nullable
 *   k8, v8 [B, S, H_kv, ceil(k_t / 32) * 32 * D] uint8 out: the codes of a segment in blocks of
 *     32 keys laid out so that every load of the attention kernel reads 1 KiB of consecutive
 *     bytes and hands each lane its matrix-core operand bytes.  Keys behind seg_len or behind
 *     k_t carry code 0.
 *     K block = two 16-key tiles; a tile is D / 64 pieces of 1 KiB; piece i is 64 lanes x 16
 *     bytes, lane 16 kk + c (kk < 4, c < 16) holding the codes of values d = 64 i + 16 kk .. + 15
 *     of key c of the tile.
 *     V block (transposed) = D / 32 pieces of 1 KiB; piece q is 64 lanes x 16 bytes, lane
 *     16 g + m (g < 4, m < 16) holding [h][j] (h < 2, j < 8) = the code of value d = 32 q + 16 h
 *     + m of key 4 g + j (j < 4) or 16 + 4 g + (j - 4) (j >= 4) of the block.
 *   k_scale, v_scale [B, S, H_kv] fp32 out.   Pointers 16-byte aligned.  No workspace.
 *   B = 0 or S = 0 is a no-op (pointers are not looked at).
 * pc_parallel_attn_fp8: pc_parallel_attn over the 8-bit segments plus, optionally, one 16-bit tail
 * segment (the query block and the generated tokens, grown by pc_kv_append with n_seg = 1) and,
 * optionally, the causal self segment of the query rows:
 *   k_tail, v_tail [B, 1, H_kv, tail_cap, D] bf16 rotated, tail_len [B] int32 (device); all
 *     three NULL and tail_cap = 0 for no tail.  Every tail row is visible to every query row.
 *   k_self, v_self [B, n_q, H_kv, D] bf16 rotated keys / values of the query rows themselves
 *     (row t sees rows 0..t), both NULL for none: the prefill stage of Eq. 9-11, where the query
 *     block attends over the compressed cache and, causally, over itself.
 *   out = softmax over { dequantised segments } U { tail rows } U { self rows <= t } exactly as
 *   pc_parallel_attn computes it on the dequantised values code * scale.
 * n_q * H_q / H_kv <= 16 (the decoding stage) runs the split-KV kernel on the 8-bit codes (each
 * code is exact in bf16; the scales ride on the fp32 logits and probabilities).  More query rows
 * run the MFMA tile kernel: the segments are first widened to bf16 rows of code * scale (rounded
 * to bf16) in the workspace, then handled like a 16-bit cache.
 * Other arguments, errors and the workspace rule as pc_parallel_attn. */
/* One-read quantisation.  pc_kv_quantize_fp8 reads every segment twice (maximum, then codes).
 * pc_gather_kv_amax is pc_gather_kv that also leaves, per destination segment, the largest
 * |value| of its K rows and of its V rows (k_amax, v_amax [batch, n_sel, H_kv] fp32 out; a
 * segment with chunk_idx < 0 keeps its old maxima), taken while the rows are in flight; an
 * integer maximum, so the result does not depend on timing.  pc_kv_quantize_fp8_amax takes
 * those maxima ([B, S, H_kv], the maximum over the segment's valid rows: rows behind seg_len must
 * not exceed it, which holds for a cache the gather filled, whose missing rows are zero) and
 * writes the same codes and scales as pc_kv_quantize_fp8 from a single read of the segment. */
int pc_gather_kv_amax(const void* k_src, const void* v_src, const int32_t* chunk_idx,
                      const int32_t* tok_idx, int32_t batch, int32_t n_chunks,
                      int32_t rows_per_chunk, int32_t n_sel, int32_t n_kv_heads, int32_t k,
                      int32_t head_dim, void* k_dst, void* v_dst, float* k_amax, float* v_amax,
                      void* stream);
int pc_kv_quantize_fp8_amax(const void* kc, const void* vc, const float* k_amax, const float* v_amax,
                            const int32_t* seg_len, int32_t seg_len_per_head, int32_t batch,
                            int32_t n_seg, int32_t k_t, int32_t n_kv_heads, int32_t head_dim,
                            void* k8, void* v8, float* k_scale, float* v_scale, void* stream);
int pc_kv_quantize_fp8(const void* kc, const void* vc, const int32_t* seg_len,
                       int32_t seg_len_per_head, int32_t batch, int32_t n_seg, int32_t k_t,
                       int32_t n_kv_heads, int32_t head_dim, void* k8, void* v8, float* k_scale,
                       float* v_scale, void* stream);
int pc_parallel_attn_fp8(const void* q, const void* k8, const void* v8, const float* k_scale,
                         const float* v_scale, const int32_t* seg_len, int32_t seg_len_per_head,
                         const void* k_tail, const void* v_tail, const int32_t* tail_len,
                         int32_t tail_cap, const void* k_self, const void* v_self, int32_t batch,
                         int32_t n_q, int32_t n_seg, int32_t k_t, int32_t n_q_heads,
                         int32_t n_kv_heads, int32_t head_dim, int32_t q_pos0, float rope_base,
                         float softmax_scale, void* out, float* lse_out, void* ws, size_t ws_bytes,
                         void* stream);
size_t pc_parallel_attn_fp8_workspace_bytes(int32_t batch, int32_t n_q, int32_t n_seg, int32_t k_t,
                                            int32_t tail_cap, int32_t n_q_heads, int32_t n_kv_heads,
                                            int32_t head_dim, int32_t has_self);

/* ---- Eq. 9-11 for callers that cannot allocate ----------------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc:
 * pc_parallel_attn for few query rows (n_q * H_q / H_kv <= 16: the decoding stage), with the
 * scratch memory (rotated query + per-workgroup partial results) in a fixed array inside the
 * library instead of a caller workspace.  Calls no hipMalloc / hipFree / allocating routine.
 * Same arguments, arithmetic and results as pc_parallel_attn (the same kernels run), except:
 *   - no ws / ws_bytes;
 *   - PC_ERR_UNSUPPORTED when n_q * H_q / H_kv > 16 (the tile path's K/V images do not fit);
 *   - PC_ERR_WORKSPACE when the request needs more than PC_STATIC_SCRATCH_BYTES, i.e. when
 *     pc_parallel_attn_workspace_bytes(...) of the same shape exceeds it
 *     (the decode config, 16 sequences x 32 heads x 128, 2 partials per group, needs 0.63 MiB).
 * Each GPU holds one such array from the moment the library is loaded until the process ends;
 * its address is looked up on the first call on a device.  All calls on one GPU share the array:
 * calls whose kernels overlap on a GPU (different streams, several threads) race; calls on one
 * stream are ordered and safe.  Every byte the call reads from the array it has written first,
 * so the previous call's contents do not matter. */
#define PC_STATIC_SCRATCH_BYTES (4u << 20)
int pc_parallel_attn_static(const void* q, const void* kc, const void* vc, const int32_t* seg_len,
                            int32_t seg_len_per_head, const void* k_self, const void* v_self,
                            int32_t batch, int32_t n_q, int32_t n_seg, int32_t k_t,
                            int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t q_pos0,
                            float rope_base, float softmax_scale, void* out, float* lse_out,
                            void* stream);
size_t pc_parallel_attn_static_max_bytes(void);   /* = PC_STATIC_SCRATCH_BYTES */

/* ---- housekeeping -------------------------------------------------------------------------- */
const char* pc_status_string(int status);   /* static string, never NULL                       */
int         pc_last_hip_error(void);        /* hipError_t of the last PC_ERR_HIP on this thread */
const char* pc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PARALLELCOMP_H */
