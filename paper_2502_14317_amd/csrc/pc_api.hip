// C ABI of the ParallelComp library: argument validation, workspace carving, kernel dispatch.
// Every host-visible argument is checked before any GPU work is enqueued.
#include "pc_common.h"
#include <math.h>
#include <mutex>

static thread_local int g_last_hip_error = 0;
void pc_set_hip_error(int err) { g_last_hip_error = err; }

extern "C" int pc_last_hip_error(void) { return g_last_hip_error; }

extern "C" const char* pc_version(void) { return "parallelcomp-gfx950 0.1"; }

extern "C" const char* pc_status_string(int status) {
  switch (status) {
    case PC_OK: return "PC_OK";
    case PC_ERR_NULL: return "PC_ERR_NULL: a required pointer is NULL";
    case PC_ERR_SHAPE: return "PC_ERR_SHAPE: a size is out of range or inconsistent";
    case PC_ERR_WORKSPACE: return "PC_ERR_WORKSPACE: workspace missing, misaligned or too small";
    case PC_ERR_HIP: return "PC_ERR_HIP: a HIP call failed (see pc_last_hip_error)";
    case PC_ERR_UNSUPPORTED: return "PC_ERR_UNSUPPORTED: no kernel for this request";
    default: return "unknown pc_status";
  }
}

// ---------------------------------------------------------------------------- profiling
#define PC_PROF_MAX 4096
static bool g_prof_on = false;
static int g_prof_only = -1;          // kernel id to record, -1 = every kernel
static int g_prof_n = 0;
static int g_prof_created = 0;
static hipEvent_t g_prof_ev[PC_PROF_MAX][2];
static int g_prof_id[PC_PROF_MAX];

PcProfScope::PcProfScope(int kernel_id, hipStream_t stream) : slot(-1), st(stream) {
  if (!g_prof_on || g_prof_n >= PC_PROF_MAX) return;
  if (g_prof_only >= 0 && kernel_id != g_prof_only) return;
  if (g_prof_n >= g_prof_created) {
    if (hipEventCreate(&g_prof_ev[g_prof_n][0]) != hipSuccess) return;
    if (hipEventCreate(&g_prof_ev[g_prof_n][1]) != hipSuccess) return;
    g_prof_created = g_prof_n + 1;
  }
  slot = g_prof_n++;
  g_prof_id[slot] = kernel_id;
  (void)hipEventRecord(g_prof_ev[slot][0], st);
}
PcProfScope::~PcProfScope() {
  if (slot >= 0) (void)hipEventRecord(g_prof_ev[slot][1], st);
}

extern "C" int pc_profile_begin(void) { g_prof_n = 0; g_prof_only = -1; g_prof_on = true; return PC_OK; }
extern "C" int pc_profile_begin_kernel(int kernel_id) {
  if (kernel_id < 0 || kernel_id >= PC_KERNEL_COUNT) return PC_ERR_SHAPE;
  g_prof_n = 0; g_prof_only = kernel_id; g_prof_on = true;
  return PC_OK;
}
extern "C" int pc_profile_end(void) { g_prof_on = false; return PC_OK; }
extern "C" int pc_profile_count(void) { return g_prof_n; }
extern "C" int pc_profile_get(int i, int* kernel_id, float* ms) {
  if (!kernel_id || !ms) return PC_ERR_NULL;
  if (i < 0 || i >= g_prof_n) return PC_ERR_SHAPE;
  PC_HIP_TRY(hipEventSynchronize(g_prof_ev[i][1]));
  PC_HIP_TRY(hipEventElapsedTime(ms, g_prof_ev[i][0], g_prof_ev[i][1]));
  *kernel_id = g_prof_id[i];
  return PC_OK;
}
extern "C" const char* pc_kernel_name(int id) {
  static const char* names[PC_KERNEL_COUNT] = {
      "rope_table_kernel", "kv_prepass_kernel", "flash_fwd_kernel", "scores_kernel<1>",
      "scores_kernel<2>", "chunk_score_kernel", "select_chunks_kernel", "select_tokens_kernel",
      "gather_kv_kernel", "rope_q_kernel", "decode_attn_kernel", "merge_kernel",
      "self_info_rows_kernel", "kv_append_kernel", "scores_lse_kernel", "kv_quantize_fp8_kernel",
      "decode_attn_fp8_kernel", "scores_kernel<1>+kv_prepass", "chunk_queue_kernel",
      "fp8_to_rows_kernel"};
  return (id >= 0 && id < PC_KERNEL_COUNT) ? names[id] : "unknown";
}

static const size_t kAlign = 256;

static int check_shape(const pc_shape* s) {
  if (!s) return PC_ERR_NULL;
  if (s->n_chunks < 1 || s->chunk_len < 1 || s->query_len < 0) return PC_ERR_SHAPE;
  if (s->n_kv_heads < 1 || s->n_q_heads < 1 || s->n_q_heads % s->n_kv_heads != 0) return PC_ERR_SHAPE;
  if (s->head_dim != 64 && s->head_dim != 128) return PC_ERR_SHAPE;
  const long long L = (long long)s->chunk_len + s->query_len;
  if (L > (1 << 20) || s->n_chunks > (1 << 20) || s->n_q_heads > 1024) return PC_ERR_SHAPE;
  // kernels index (chunk, head, row) tuples and workgroups with 32-bit integers
  if ((long long)s->n_chunks * s->n_q_heads * ((L + 127) / 128) > 0x7fffffffLL / 8) return PC_ERR_SHAPE;
  if ((long long)s->n_chunks * L * s->n_q_heads > 0x7fffffffLL) return PC_ERR_SHAPE;
  if (!(s->rope_base > 1.0f) || !isfinite(s->rope_base)) return PC_ERR_SHAPE;
  if (!(s->softmax_scale >= 0.0f) || !isfinite(s->softmax_scale)) return PC_ERR_SHAPE;
  return PC_OK;
}

// The voting rows are the last w_obs rows of a sequence.  With ragged chunks a sequence may be
// as short as the query block alone, so the window must then fit the query block (Eq. 6 sums
// over query rows only); with full chunks it may reach into the context rows.
static int check_obs(const pc_shape* s, bool ragged) {
  const int L = s->chunk_len + s->query_len;
  if (s->obs_window < 1 || s->obs_window > (ragged ? s->query_len : L)) return PC_ERR_SHAPE;
  return PC_OK;
}

static float eff_scale(float scale, int head_dim) {
  return scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
}

struct PrefillWs {
  size_t table, v_img, k_img, ml, total;
  int Lp;
};

static PrefillWs prefill_ws_layout(const pc_shape* s) {
  PrefillWs w;
  const size_t L = (size_t)s->chunk_len + s->query_len;
  w.Lp = (int)((L + 63) / 64 * 64);
  size_t off = 0;
  w.table = off; off = pc_align_up(off + L * (s->head_dim / 2) * sizeof(float2), kAlign);
  const size_t img_bytes = (size_t)s->n_chunks * s->n_kv_heads * s->head_dim * w.Lp * 2;   // tile images
  w.v_img = off; off = pc_align_up(off + img_bytes, kAlign);
  w.k_img = off; off = pc_align_up(off + img_bytes, kAlign);
  w.ml = off;    off = pc_align_up(off + pc_scores_ml_bytes(s), kAlign);
  w.total = off;
  return w;
}

extern "C" size_t pc_chunk_prefill_workspace_bytes(const pc_shape* s) {
  if (check_shape(s) != PC_OK) return 0;
  pc_shape t = *s;
  // a call without scores ignores the window: size for any window the call could accept
  if (t.obs_window < 1) t.obs_window = 1;
  if (t.obs_window > t.chunk_len + t.query_len) t.obs_window = t.chunk_len + t.query_len;
  return prefill_ws_layout(&t).total;
}

extern "C" size_t pc_chunk_query_scores_workspace_bytes(const pc_shape* s) {
  if (check_shape(s) != PC_OK || check_obs(s, false) != PC_OK) return 0;
  const size_t L = (size_t)s->chunk_len + s->query_len;
  return pc_align_up(L * (s->head_dim / 2) * sizeof(float2), kAlign) +
         pc_align_up(pc_scores_ml_bytes(s), kAlign);
}

extern "C" int pc_chunk_prefill_attn(const pc_shape* s, const void* q, const void* k, const void* v,
                                     const int32_t* chunk_lens, void* o, float* lse, void* k_rope, float* tok_score,
                                     float* chunk_score, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(s);
  if (rc != PC_OK) return rc;
  if (!q || !k || !v || !o || !lse) return PC_ERR_NULL;
  if (chunk_score && !tok_score) return PC_ERR_NULL;
  // every kernel moves these tensors with 16-byte loads and stores
  if (!pc_aligned(q, 16) || !pc_aligned(k, 16) || !pc_aligned(v, 16) || !pc_aligned(o, 16) ||
      !pc_aligned(k_rope, 16))
    return PC_ERR_SHAPE;
  if (tok_score) {
    rc = check_obs(s, chunk_lens != nullptr);
    if (rc != PC_OK) return rc;
  }
  pc_shape t = *s;
  if (!tok_score) t.obs_window = 1;
  const PrefillWs w = prefill_ws_layout(&t);
  if (!ws || !pc_aligned(ws, kAlign) || ws_bytes < w.total) return PC_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)ws;
  float2* table = (float2*)(base + w.table);
  void* v_img = base + w.v_img;
  void* k_img = base + w.k_img;
  void* kr = k_rope;                                       // nullable: then only the images are written
  const int L = s->chunk_len + s->query_len, D = s->head_dim;

  rc = pc_launch_rope_table(table, L, D, s->rope_base, st);
  if (rc != PC_OK) return rc;
  if (tok_score) {
    // the first score pass reads and rotates every key anyway: it also writes the rotated keys
    // and the tile images (the keys are read from memory once for both jobs)
    const PcPrepassOut pre = {v, kr, k_img, v_img, w.Lp};
    rc = pc_launch_scores(s, q, k, chunk_lens, table, base + w.ml, tok_score, chunk_score, &pre, st);
  } else {
    rc = pc_launch_kv_prepass(k, v, table, kr, k_img, v_img, s->n_chunks, L, w.Lp, s->n_kv_heads, D, st);
  }
  if (rc != PC_OK) return rc;

  PcFlashArgs a = {};
  a.q = q; a.k_img = k_img; a.v_img = v_img; a.table = table; a.o = o; a.lse = lse;
  a.part_o = nullptr; a.part_lse = nullptr; a.part_len = nullptr;
  a.img_seq_stride = (long long)s->n_kv_heads * (w.Lp / 64); a.img_part_stride = 0;
  a.img_head_stride = w.Lp / 64;
  a.n_seq = s->n_chunks; a.n_rows = L; a.n_keys = L;
  a.n_q_heads = s->n_q_heads; a.n_kv_heads = s->n_kv_heads; a.head_dim = D;
  a.n_parts_grid = 1; a.n_parts_total = 1; a.part0 = 0;
  a.causal_offset = 0; a.q_pos0 = 0;
  a.seq_ctx = chunk_lens; a.seq_add = s->query_len;
  a.scale = eff_scale(s->softmax_scale, D);
  return pc_launch_flash(a, st);
}

extern "C" int pc_chunk_query_scores(const pc_shape* s, const void* q, const void* k,
                                     const int32_t* chunk_lens, float* tok_score, float* chunk_score, void* ws,
                                     size_t ws_bytes, void* stream) {
  int rc = check_shape(s);
  if (rc != PC_OK) return rc;
  rc = check_obs(s, chunk_lens != nullptr);
  if (rc != PC_OK) return rc;
  if (!q || !k || !tok_score) return PC_ERR_NULL;
  if (!pc_aligned(q, 16) || !pc_aligned(k, 16)) return PC_ERR_SHAPE;
  const size_t need = pc_chunk_query_scores_workspace_bytes(s);
  if (!ws || !pc_aligned(ws, kAlign) || ws_bytes < need) return PC_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int L = s->chunk_len + s->query_len;
  float2* table = (float2*)ws;
  void* ml = (char*)ws + pc_align_up((size_t)L * (s->head_dim / 2) * sizeof(float2), kAlign);
  rc = pc_launch_rope_table(table, L, s->head_dim, s->rope_base, st);
  if (rc != PC_OK) return rc;
  return pc_launch_scores(s, q, k, chunk_lens, table, ml, tok_score, chunk_score, nullptr, st);
}

extern "C" int pc_kv_append(const void* k_new, const void* v_new, int32_t batch, int32_t n_new,
                            int32_t n_seg, int32_t seg, int32_t k_t, int32_t n_kv_heads,
                            int32_t head_dim, int32_t pos0, float rope_base, void* kc, void* vc,
                            int32_t* seg_len, int32_t seg_len_per_head, void* stream) {
  if (!k_new || !v_new || !kc || !vc || !seg_len) return PC_ERR_NULL;
  if (batch < 0 || n_new < 0 || n_seg < 1 || seg < 0 || seg >= n_seg || k_t < 1 || n_kv_heads < 1)
    return PC_ERR_SHAPE;
  if (head_dim != 64 && head_dim != 128) return PC_ERR_SHAPE;
  if (pos0 >= 0 && (!(rope_base > 1.0f) || !isfinite(rope_base))) return PC_ERR_SHAPE;
  if (!pc_aligned(k_new, 2) || !pc_aligned(v_new, 2) || !pc_aligned(kc, 2) || !pc_aligned(vc, 2) ||
      !pc_aligned(seg_len, 4))
    return PC_ERR_SHAPE;
  if (batch == 0 || n_new == 0) return PC_OK;
  return pc_launch_kv_append(k_new, v_new, batch, n_new, n_seg, seg, k_t, n_kv_heads, head_dim,
                             pos0, rope_base, kc, vc, seg_len, seg_len_per_head != 0,
                             (hipStream_t)stream);
}

// ---------------------------------------------------------------------------- 8-bit cache
extern "C" int pc_kv_quantize_fp8(const void* kc, const void* vc, const int32_t* seg_len,
                                  int32_t seg_len_per_head, int32_t batch, int32_t n_seg,
                                  int32_t k_t, int32_t n_kv_heads, int32_t head_dim, void* k8,
                                  void* v8, float* k_scale, float* v_scale, void* stream) {
  if (batch < 0 || n_seg < 0 || k_t < 1 || n_kv_heads < 1) return PC_ERR_SHAPE;
  if (head_dim != 64 && head_dim != 128) return PC_ERR_SHAPE;
  if (seg_len_per_head != 0 && seg_len_per_head != 1) return PC_ERR_SHAPE;
  if (batch == 0 || n_seg == 0) return PC_OK;            // nothing to quantise
  if (!kc || !vc || !k8 || !v8 || !k_scale || !v_scale) return PC_ERR_NULL;
  if (!pc_aligned(kc, 16) || !pc_aligned(vc, 16) || !pc_aligned(k8, 16) || !pc_aligned(v8, 16))
    return PC_ERR_SHAPE;
  return pc_launch_kv_quantize_fp8(kc, vc, seg_len, seg_len_per_head,
                                   (long long)batch * n_seg * n_kv_heads, n_kv_heads, k_t, head_dim,
                                   nullptr, nullptr, k8, v8, k_scale, v_scale, (hipStream_t)stream);
}

extern "C" int pc_kv_quantize_fp8_amax(const void* kc, const void* vc, const float* k_amax,
                                       const float* v_amax, const int32_t* seg_len,
                                       int32_t seg_len_per_head, int32_t batch, int32_t n_seg,
                                       int32_t k_t, int32_t n_kv_heads, int32_t head_dim, void* k8,
                                       void* v8, float* k_scale, float* v_scale, void* stream) {
  if (batch < 0 || n_seg < 0 || k_t < 1 || n_kv_heads < 1) return PC_ERR_SHAPE;
  if (head_dim != 64 && head_dim != 128) return PC_ERR_SHAPE;
  if (seg_len_per_head != 0 && seg_len_per_head != 1) return PC_ERR_SHAPE;
  if (batch == 0 || n_seg == 0) return PC_OK;
  if (!kc || !vc || !k_amax || !v_amax || !k8 || !v8 || !k_scale || !v_scale) return PC_ERR_NULL;
  if (!pc_aligned(kc, 16) || !pc_aligned(vc, 16) || !pc_aligned(k8, 16) || !pc_aligned(v8, 16))
    return PC_ERR_SHAPE;
  return pc_launch_kv_quantize_fp8(kc, vc, seg_len, seg_len_per_head,
                                   (long long)batch * n_seg * n_kv_heads, n_kv_heads, k_t, head_dim,
                                   k_amax, v_amax, k8, v8, k_scale, v_scale, (hipStream_t)stream);
}

struct Par8Ws {
  size_t q_rot, part_o, part_lse, rows_k, rows_v, k_seg, v_seg, k_tail, v_tail, k_self, v_self, total;
  int n_parts, parts8, ktp, tcp, nqp;
  bool small;
};

static Par8Ws par8_ws_layout(int batch, int n_q, int n_seg, int k_t, int tail_cap, int n_q_heads,
                             int n_kv_heads, int D, int has_self) {
  Par8Ws w;
  w.small = (long long)n_q * (n_q_heads / n_kv_heads) <= 16;
  w.ktp = (k_t + 63) / 64 * 64; w.tcp = (tail_cap + 63) / 64 * 64; w.nqp = (n_q + 63) / 64 * 64;
  if (w.small) {
    w.parts8 = pc_decode_split(k_t, n_seg, (long long)batch * n_kv_heads).n_parts;
    w.n_parts = w.parts8;
    if (tail_cap > 0) w.n_parts += pc_decode_split(tail_cap, 1, (long long)batch * n_kv_heads).n_parts;
  } else {           // tile path: one partial per segment, one for the tail, one for the self segment
    w.parts8 = n_seg;
    w.n_parts = n_seg + (tail_cap > 0 ? 1 : 0) + (has_self ? 1 : 0);
  }
  size_t off = 0;
  const size_t rows = (size_t)batch * n_q * n_q_heads;
  w.q_rot = off;    off = pc_align_up(off + rows * D * 2, kAlign);
  w.part_o = off;   off = pc_align_up(off + rows * (size_t)w.n_parts * D * sizeof(float), kAlign);
  w.part_lse = off; off = pc_align_up(off + rows * (size_t)w.n_parts * sizeof(float), kAlign);
  w.rows_k = w.rows_v = w.k_seg = w.v_seg = w.k_tail = w.v_tail = w.k_self = w.v_self = off;
  if (!w.small) {
    // dequantised segments as bf16 rows, then the tile images of segments, tail and self segment
    const size_t seg_rows = (size_t)batch * n_seg * n_kv_heads * k_t * D * 2;
    const size_t seg_img = (size_t)batch * n_seg * n_kv_heads * D * w.ktp * 2;
    const size_t tail_img = (size_t)batch * n_kv_heads * D * w.tcp * 2;
    const size_t self_img = has_self ? (size_t)batch * n_kv_heads * D * w.nqp * 2 : 0;
    w.rows_k = off; off = pc_align_up(off + seg_rows, kAlign);
    w.rows_v = off; off = pc_align_up(off + seg_rows, kAlign);
    w.k_seg = off;  off = pc_align_up(off + seg_img, kAlign);
    w.v_seg = off;  off = pc_align_up(off + seg_img, kAlign);
    w.k_tail = off; off = pc_align_up(off + tail_img, kAlign);
    w.v_tail = off; off = pc_align_up(off + tail_img, kAlign);
    w.k_self = off; off = pc_align_up(off + self_img, kAlign);
    w.v_self = off; off = pc_align_up(off + self_img, kAlign);
  }
  w.total = off;
  return w;
}

static int check_par8(int batch, int n_q, int n_seg, int k_t, int tail_cap, int n_q_heads,
                      int n_kv_heads, int D) {
  if (batch < 1 || n_q < 1 || n_seg < 0 || k_t < 1 || tail_cap < 0) return PC_ERR_SHAPE;
  if (n_kv_heads < 1 || n_q_heads < 1 || n_q_heads % n_kv_heads != 0) return PC_ERR_SHAPE;
  if (D != 64 && D != 128) return PC_ERR_SHAPE;
  if (k_t > (1 << 24) || tail_cap > (1 << 24) || n_seg > (1 << 20) || batch > (1 << 20) || n_q > (1 << 20))
    return PC_ERR_SHAPE;
  const long long parts = (long long)n_seg + 2;
  if ((long long)batch * parts * n_kv_heads > 0x7fffffffLL / 64) return PC_ERR_SHAPE;
  if ((long long)batch * parts * n_q_heads * ((n_q + 127) / 128) > 0x7fffffffLL / 8) return PC_ERR_SHAPE;
  if ((long long)batch * n_q * n_q_heads > 0x7fffffffLL / 64) return PC_ERR_SHAPE;
  return PC_OK;
}

static int parallel_attn_fp8_tiles(const void* q, const void* k8, const void* v8, const float* k_scale,
                                   const float* v_scale, const int32_t* seg_len, int seg_len_per_head,
                                   const void* k_tail, const void* v_tail, const int32_t* tail_len,
                                   int tail_cap, const void* k_self, const void* v_self, int batch,
                                   int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads, int D,
                                   int q_pos0, float rope_base, float scale, void* out, float* lse_out,
                                   const Par8Ws& w, char* base, hipStream_t st);

extern "C" size_t pc_parallel_attn_fp8_workspace_bytes(int32_t batch, int32_t n_q, int32_t n_seg,
                                                       int32_t k_t, int32_t tail_cap,
                                                       int32_t n_q_heads, int32_t n_kv_heads,
                                                       int32_t head_dim, int32_t has_self) {
  if (check_par8(batch, n_q, n_seg, k_t, tail_cap, n_q_heads, n_kv_heads, head_dim) != PC_OK) return 0;
  return par8_ws_layout(batch, n_q, n_seg, k_t, tail_cap, n_q_heads, n_kv_heads, head_dim, has_self).total;
}

extern "C" int pc_parallel_attn_fp8(const void* q, const void* k8, const void* v8,
                                    const float* k_scale, const float* v_scale,
                                    const int32_t* seg_len, int32_t seg_len_per_head,
                                    const void* k_tail, const void* v_tail, const int32_t* tail_len,
                                    int32_t tail_cap, const void* k_self, const void* v_self,
                                    int32_t batch, int32_t n_q, int32_t n_seg,
                                    int32_t k_t, int32_t n_q_heads, int32_t n_kv_heads,
                                    int32_t head_dim, int32_t q_pos0, float rope_base,
                                    float softmax_scale, void* out, float* lse_out, void* ws,
                                    size_t ws_bytes, void* stream) {
  int rc = check_par8(batch, n_q, n_seg, k_t, tail_cap, n_q_heads, n_kv_heads, head_dim);
  if (rc != PC_OK) return rc;
  if (!q || !out) return PC_ERR_NULL;
  if (n_seg > 0 && (!k8 || !v8 || !k_scale || !v_scale)) return PC_ERR_NULL;
  if (tail_cap > 0 && (!k_tail || !v_tail || !tail_len)) return PC_ERR_NULL;
  if ((k_self == nullptr) != (v_self == nullptr)) return PC_ERR_NULL;
  const int has_self = k_self != nullptr;
  if (n_seg == 0 && tail_cap == 0 && !has_self) return PC_ERR_SHAPE;
  if (seg_len_per_head != 0 && seg_len_per_head != 1) return PC_ERR_SHAPE;
  if (q_pos0 >= 0 && (!(rope_base > 1.0f) || !isfinite(rope_base))) return PC_ERR_SHAPE;
  if (!(softmax_scale >= 0.0f) || !isfinite(softmax_scale)) return PC_ERR_SHAPE;
  if (n_seg > 0 && (!pc_aligned(k8, 16) || !pc_aligned(v8, 16))) return PC_ERR_SHAPE;
  if (!pc_aligned(q, 16) || !pc_aligned(out, 16) || !pc_aligned(k_tail, 16) || !pc_aligned(v_tail, 16) ||
      !pc_aligned(k_self, 16) || !pc_aligned(v_self, 16))
    return PC_ERR_SHAPE;
  const int D = head_dim;
  const Par8Ws w = par8_ws_layout(batch, n_q, n_seg, k_t, tail_cap, n_q_heads, n_kv_heads, D, has_self);
  if (!ws || !pc_aligned(ws, kAlign) || ws_bytes < w.total) return PC_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)ws;
  const float scale = eff_scale(softmax_scale, D);
  if (!w.small)
    return parallel_attn_fp8_tiles(q, k8, v8, k_scale, v_scale, seg_len, seg_len_per_head, k_tail, v_tail,
                                   tail_len, tail_cap, k_self, v_self, batch, n_q, n_seg, k_t, n_q_heads,
                                   n_kv_heads, D, q_pos0, rope_base, scale, out, lse_out, w, base, st);
  const void* q_rot = q;
  if (q_pos0 >= 0) {
    rc = pc_launch_rope_q(q, base + w.q_rot, (long long)batch * n_q * n_q_heads, n_q, n_q_heads, D,
                          q_pos0, rope_base, 1.0f, st);
    if (rc != PC_OK) return rc;
    q_rot = base + w.q_rot;
  }
  float* part_o = (float*)(base + w.part_o);
  float* part_lse = (float*)(base + w.part_lse);
  if (n_seg > 0) {
    rc = pc_launch_decode_fp8(q_rot, k8, v8, k_scale, v_scale, seg_len, seg_len_per_head, batch, n_q,
                              n_seg, k_t, n_q_heads, n_kv_heads, D, scale, part_o, part_lse,
                              w.n_parts, st);
    if (rc != PC_OK) return rc;
  }
  if (tail_cap > 0) {     // the 16-bit tail: one more segment of the split-KV kernel
    rc = pc_launch_decode(q_rot, k_tail, v_tail, tail_len, 0, batch, n_q, 1, tail_cap, n_q_heads,
                          n_kv_heads, D, scale, part_o, part_lse, w.n_parts, w.parts8, st);
    if (rc != PC_OK) return rc;
  }
  // the few-row causal self segment (if any) is evaluated inside the merge
  return pc_launch_merge(part_o, part_lse, q_rot, k_self, v_self, out, lse_out, batch, n_q,
                         n_q_heads, n_kv_heads, D, w.n_parts, scale, st);
}

extern "C" int pc_chunk_self_information(const void* logits, const int32_t* targets, int32_t n_chunks,
                                         int32_t n_tokens, int32_t vocab, int32_t negate,
                                         float* token_nll, float* info, void* stream) {
  if (!logits || !targets || !token_nll || !info) return PC_ERR_NULL;
  if (n_chunks < 1 || n_tokens < 1 || vocab < 8 || vocab > (1 << 24) || vocab % 8 != 0) return PC_ERR_SHAPE;
  if ((long long)n_chunks * n_tokens > 0x7fffffffLL || !pc_aligned(logits, 16)) return PC_ERR_SHAPE;
  return pc_launch_self_info(logits, targets, n_chunks, n_tokens, vocab, negate, token_nll, info,
                             (hipStream_t)stream);
}

extern "C" int pc_select_chunks_topk(const float* chunk_score, int32_t n, int32_t k,
                                     int32_t* out_idx, float* out_score, void* stream) {
  if (!chunk_score || !out_idx) return PC_ERR_NULL;
  if (n < 1 || n > 4096 || k < 1 || k > n) return PC_ERR_SHAPE;
  return pc_launch_select_chunks(chunk_score, n, k, out_idx, out_score, (hipStream_t)stream);
}

extern "C" int pc_chunk_queue_update(const float* batch_score, int32_t n_batch, int32_t chunk_id0,
                                     int32_t capacity, int32_t* queue_id, float* queue_score,
                                     int32_t* queue_slot, int32_t* slot_src, void* stream) {
  if (!batch_score || !queue_id || !queue_score || !queue_slot || !slot_src) return PC_ERR_NULL;
  if (n_batch < 1 || n_batch > 1024 || capacity < 1 || capacity > 1024 || chunk_id0 < 0) return PC_ERR_SHAPE;
  if ((long long)chunk_id0 + n_batch > 0x7fffffffLL) return PC_ERR_SHAPE;
  return pc_launch_chunk_queue(batch_score, n_batch, chunk_id0, capacity, queue_id, queue_score,
                               queue_slot, slot_src, (hipStream_t)stream);
}

extern "C" int pc_select_tokens_topk(const float* tok_score, const int32_t* chunk_idx, int32_t n_sel,
                                     int32_t n_kv_heads, int32_t chunk_len, int32_t k,
                                     int32_t* out_idx, void* stream) {
  if (!tok_score || !out_idx) return PC_ERR_NULL;
  if (n_sel < 0 || n_kv_heads < 1 || chunk_len < 1 || chunk_len > 32768 || k < 1 || k > chunk_len)
    return PC_ERR_SHAPE;
  if ((long long)n_sel * n_kv_heads > 0x7fffffffLL) return PC_ERR_SHAPE;
  if (n_sel == 0) return PC_OK;
  return pc_launch_select_tokens(tok_score, chunk_idx, n_sel, n_kv_heads, chunk_len, k, 0.f, 0, 0,
                                 nullptr, out_idx, nullptr, (hipStream_t)stream);
}

extern "C" int pc_select_tokens_calibrated(const float* tok_score, const int32_t* chunk_idx,
                                           int32_t n_sel, int32_t n_kv_heads, int32_t chunk_len,
                                           int32_t k, float lambda, int32_t class_lo,
                                           int32_t class_hi, const int32_t* chunk_lens,
                                           int32_t* out_idx, int32_t* out_cnt, void* stream) {
  if (!tok_score || !out_idx || !out_cnt) return PC_ERR_NULL;
  if (n_sel < 0 || n_kv_heads < 1 || chunk_len < 1 || chunk_len > 32768 || k < 1 || k > chunk_len)
    return PC_ERR_SHAPE;
  if ((long long)n_sel * n_kv_heads > 0x7fffffffLL) return PC_ERR_SHAPE;
  if (class_lo < 0 || class_hi < class_lo || class_hi > chunk_len || lambda != lambda) return PC_ERR_SHAPE;
  if (n_sel == 0) return PC_OK;
  return pc_launch_select_tokens(tok_score, chunk_idx, n_sel, n_kv_heads, chunk_len, k, lambda,
                                 class_lo, class_hi, chunk_lens, out_idx, out_cnt, (hipStream_t)stream);
}

extern "C" int pc_gather_kv(const void* k_src, const void* v_src, const int32_t* chunk_idx,
                            const int32_t* tok_idx, int32_t batch, int32_t n_chunks,
                            int32_t rows_per_chunk, int32_t n_sel, int32_t n_kv_heads, int32_t k,
                            int32_t head_dim, void* k_dst, void* v_dst, void* stream) {
  if (!k_src || !v_src || !tok_idx || !k_dst || !v_dst) return PC_ERR_NULL;
  if (batch < 0 || n_chunks < 1 || rows_per_chunk < 1 || n_sel < 0 || n_kv_heads < 1 || k < 0)
    return PC_ERR_SHAPE;
  if (head_dim != 64 && head_dim != 128) return PC_ERR_SHAPE;
  if (!pc_aligned(k_src, 16) || !pc_aligned(v_src, 16) || !pc_aligned(k_dst, 16) || !pc_aligned(v_dst, 16))
    return PC_ERR_SHAPE;
  return pc_launch_gather(k_src, v_src, chunk_idx, tok_idx, batch, n_chunks, rows_per_chunk, n_sel,
                          n_kv_heads, k, head_dim, k_dst, v_dst, nullptr, nullptr, (hipStream_t)stream);
}

extern "C" int pc_gather_kv_amax(const void* k_src, const void* v_src, const int32_t* chunk_idx,
                                 const int32_t* tok_idx, int32_t batch, int32_t n_chunks,
                                 int32_t rows_per_chunk, int32_t n_sel, int32_t n_kv_heads, int32_t k,
                                 int32_t head_dim, void* k_dst, void* v_dst, float* k_amax,
                                 float* v_amax, void* stream) {
  if (!k_src || !v_src || !tok_idx || !k_dst || !v_dst || !k_amax || !v_amax) return PC_ERR_NULL;
  if (batch < 0 || n_chunks < 1 || rows_per_chunk < 1 || n_sel < 0 || n_kv_heads < 1 || k < 1)
    return PC_ERR_SHAPE;
  if (head_dim != 64 && head_dim != 128) return PC_ERR_SHAPE;
  if (!pc_aligned(k_src, 16) || !pc_aligned(v_src, 16) || !pc_aligned(k_dst, 16) || !pc_aligned(v_dst, 16))
    return PC_ERR_SHAPE;
  return pc_launch_gather(k_src, v_src, chunk_idx, tok_idx, batch, n_chunks, rows_per_chunk, n_sel,
                          n_kv_heads, k, head_dim, k_dst, v_dst, k_amax, v_amax, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------- parallel attention
struct ParWs {
  size_t q_rot, part_o, part_lse, v_seg, k_seg, v_self, k_self, total;
  int n_parts, ktp, nqp;
  bool small;
};

static ParWs par_ws_layout(int batch, int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads,
                           int D, int has_self) {
  ParWs w;
  const int G = n_q_heads / n_kv_heads;
  w.small = (long long)n_q * G <= 16;
  w.ktp = (k_t + 63) / 64 * 64;
  w.nqp = (n_q + 63) / 64 * 64;
  if (w.small) {
    w.n_parts = pc_decode_split(k_t, n_seg, (long long)batch * n_kv_heads).n_parts;
  } else {
    w.n_parts = n_seg + (has_self ? 1 : 0);
  }
  size_t off = 0;
  const size_t rows = (size_t)batch * n_q * n_q_heads;
  w.q_rot = off;    off = pc_align_up(off + rows * D * 2, kAlign);
  w.part_o = off;   off = pc_align_up(off + rows * (size_t)w.n_parts * D * sizeof(float), kAlign);
  w.part_lse = off; off = pc_align_up(off + rows * (size_t)w.n_parts * sizeof(float), kAlign);
  w.v_seg = w.k_seg = w.v_self = w.k_self = off;
  if (!w.small) {   // tile images of the segments and of the self segment (K and V^T)
    const size_t seg_bytes = (size_t)batch * n_seg * n_kv_heads * D * w.ktp * 2;
    const size_t self_bytes = has_self ? (size_t)batch * n_kv_heads * D * w.nqp * 2 : 0;
    w.v_seg = off;  off = pc_align_up(off + seg_bytes, kAlign);
    w.k_seg = off;  off = pc_align_up(off + seg_bytes, kAlign);
    w.v_self = off; off = pc_align_up(off + self_bytes, kAlign);
    w.k_self = off; off = pc_align_up(off + self_bytes, kAlign);
  }
  w.total = off;
  return w;
}

static int check_par(int batch, int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads, int D) {
  if (batch < 1 || n_q < 1 || n_seg < 0 || k_t < 1) return PC_ERR_SHAPE;
  if (n_kv_heads < 1 || n_q_heads < 1 || n_q_heads % n_kv_heads != 0) return PC_ERR_SHAPE;
  if (D != 64 && D != 128) return PC_ERR_SHAPE;
  if (n_q > (1 << 20) || k_t > (1 << 24) || n_seg > (1 << 20) || batch > (1 << 20)) return PC_ERR_SHAPE;
  // kernels index (sequence, segment, head) tuples, partial rows and workgroups with 32-bit integers
  const long long parts = (long long)n_seg + 1;
  if ((long long)batch * parts * n_kv_heads > 0x7fffffffLL / 64) return PC_ERR_SHAPE;
  if ((long long)batch * parts * n_q_heads * ((n_q + 127) / 128) > 0x7fffffffLL / 8) return PC_ERR_SHAPE;
  if ((long long)batch * n_q * n_q_heads > 0x7fffffffLL / 64) return PC_ERR_SHAPE;
  return PC_OK;
}

extern "C" size_t pc_parallel_attn_workspace_bytes(int32_t batch, int32_t n_q, int32_t n_seg,
                                                   int32_t k_t, int32_t n_q_heads,
                                                   int32_t n_kv_heads, int32_t head_dim,
                                                   int32_t has_self) {
  if (check_par(batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim) != PC_OK) return 0;
  return par_ws_layout(batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim, has_self).total;
}

// Host-visible argument checks shared by pc_parallel_attn and its no-allocation variant.
static int check_par_args(const void* q, const void* kc, const void* vc, int32_t seg_len_per_head,
                          const void* k_self, const void* v_self, int32_t batch, int32_t n_q,
                          int32_t n_seg, int32_t k_t, int32_t n_q_heads, int32_t n_kv_heads,
                          int32_t head_dim, int32_t q_pos0, float rope_base, float softmax_scale,
                          const void* out) {
  int rc = check_par(batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim);
  if (rc != PC_OK) return rc;
  if (!q || !out) return PC_ERR_NULL;
  if (n_seg > 0 && (!kc || !vc)) return PC_ERR_NULL;
  if (seg_len_per_head != 0 && seg_len_per_head != 1) return PC_ERR_SHAPE;
  if ((k_self == nullptr) != (v_self == nullptr)) return PC_ERR_NULL;
  if (n_seg == 0 && k_self == nullptr) return PC_ERR_SHAPE;
  if (q_pos0 >= 0 && (!(rope_base > 1.0f) || !isfinite(rope_base))) return PC_ERR_SHAPE;
  if (!(softmax_scale >= 0.0f) || !isfinite(softmax_scale)) return PC_ERR_SHAPE;
  // 16-byte loads and stores on every tensor
  if (!pc_aligned(q, 16) || !pc_aligned(kc, 16) || !pc_aligned(vc, 16) || !pc_aligned(k_self, 16) ||
      !pc_aligned(v_self, 16) || !pc_aligned(out, 16))
    return PC_ERR_SHAPE;
  return PC_OK;
}

// Enqueues the kernels of Eq. 9-11 on a validated request; ws holds at least w.total bytes.
static int parallel_attn_run(const void* q, const void* kc, const void* vc, const int32_t* seg_len,
                             int32_t seg_len_per_head, const void* k_self, const void* v_self,
                             int32_t batch, int32_t n_q, int32_t n_seg, int32_t k_t,
                             int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                             int32_t q_pos0, float rope_base, float softmax_scale, void* out,
                             float* lse_out, const ParWs& w, void* ws, void* stream) {
  int rc;
  const int has_self = k_self != nullptr;
  const int D = head_dim;
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)ws;
  const float scale = eff_scale(softmax_scale, D);

  // Query operand.  Split-KV path: the rotated rows (the scale is applied to the fp32 logits).
  // Tile path: rotated and multiplied by scale * log2(e) before the one rounding to bf16, so the
  // matrix cores deliver logits in log2 units (rows that arrive already rotated, q_pos0 < 0, are
  // only scaled: their bf16 values are rounded a second time).
  const void* q_rot = q;
  if (q_pos0 >= 0 || !w.small) {
    rc = pc_launch_rope_q(q, base + w.q_rot, (long long)batch * n_q * n_q_heads, n_q, n_q_heads, D,
                          q_pos0, rope_base, w.small ? 1.0f : scale * 1.4426950408889634f, st);
    if (rc != PC_OK) return rc;
    q_rot = base + w.q_rot;
  }
  float* part_o = (float*)(base + w.part_o);
  float* part_lse = (float*)(base + w.part_lse);

  if (w.small) {
    if (n_seg > 0) {
      rc = pc_launch_decode(q_rot, kc, vc, seg_len, seg_len_per_head, batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads,
                            D, scale, part_o, part_lse, w.n_parts, 0, st);
      if (rc != PC_OK) return rc;
    }
    return pc_launch_merge(part_o, part_lse, q_rot, k_self, v_self, out, lse_out, batch, n_q,
                           n_q_heads, n_kv_heads, D, w.n_parts, scale, st);
  }

  // ---- many query rows: MFMA tile kernel per (segment), partials merged afterwards
  PcFlashArgs a = {};
  a.q = q_rot; a.table = nullptr; a.o = nullptr; a.lse = nullptr;
  a.part_o = part_o; a.part_lse = part_lse;
  a.n_seq = batch; a.n_rows = n_q; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads;
  a.head_dim = D; a.n_parts_total = w.n_parts; a.q_pos0 = 0; a.scale = scale;
  if (n_seg > 0) {
    // compacted K is already rotated: copy it into tile images next to those of V^T
    rc = pc_launch_kv_prepass(kc, vc, nullptr, nullptr, base + w.k_seg, base + w.v_seg,
                              batch * n_seg * n_kv_heads, k_t, w.ktp, 1, D, st);
    if (rc != PC_OK) return rc;
    a.k_img = base + w.k_seg; a.v_img = base + w.v_seg; a.part_len = seg_len;
    a.part_len_per_head = seg_len_per_head;
    a.img_seq_stride = (long long)n_seg * n_kv_heads * (w.ktp / 64);
    a.img_part_stride = (long long)n_kv_heads * (w.ktp / 64);
    a.img_head_stride = w.ktp / 64;
    a.n_keys = k_t; a.n_parts_grid = n_seg; a.part0 = 0; a.causal_offset = PC_NO_CAUSAL;
    rc = pc_launch_flash(a, st);
    if (rc != PC_OK) return rc;
  }
  if (has_self) {
    rc = pc_launch_kv_prepass(k_self, v_self, nullptr, nullptr, base + w.k_self, base + w.v_self,
                              batch, n_q, w.nqp, n_kv_heads, D, st);
    if (rc != PC_OK) return rc;
    a.k_img = base + w.k_self; a.v_img = base + w.v_self; a.part_len = nullptr;
    a.part_len_per_head = 0;
    a.img_seq_stride = (long long)n_kv_heads * (w.nqp / 64); a.img_part_stride = 0;
    a.img_head_stride = w.nqp / 64;
    a.n_keys = n_q; a.n_parts_grid = 1; a.part0 = n_seg; a.causal_offset = 0;
    rc = pc_launch_flash(a, st);
    if (rc != PC_OK) return rc;
  }
  return pc_launch_merge(part_o, part_lse, q_rot, nullptr, nullptr, out, lse_out, batch, n_q,
                         n_q_heads, n_kv_heads, D, w.n_parts, scale, st);
}

// Eq. 9-11 for a block of query rows over the 8-bit cache: the segments are widened to bf16 rows
// (code * scale, rounded to bf16) in the workspace, then everything runs through the tile kernel
// as for a 16-bit cache: one partial per segment, one for the 16-bit tail (all its rows
// visible), one for the causal self segment, merged by logsumexp.
static int parallel_attn_fp8_tiles(const void* q, const void* k8, const void* v8, const float* k_scale,
                                   const float* v_scale, const int32_t* seg_len, int seg_len_per_head,
                                   const void* k_tail, const void* v_tail, const int32_t* tail_len,
                                   int tail_cap, const void* k_self, const void* v_self, int batch,
                                   int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads, int D,
                                   int q_pos0, float rope_base, float scale, void* out, float* lse_out,
                                   const Par8Ws& w, char* base, hipStream_t st) {
  int rc = pc_launch_rope_q(q, base + w.q_rot, (long long)batch * n_q * n_q_heads, n_q, n_q_heads, D,
                            q_pos0, rope_base, scale * 1.4426950408889634f, st);
  if (rc != PC_OK) return rc;
  PcFlashArgs a = {};
  a.q = base + w.q_rot; a.table = nullptr; a.o = nullptr; a.lse = nullptr;
  a.part_o = (float*)(base + w.part_o); a.part_lse = (float*)(base + w.part_lse);
  a.n_seq = batch; a.n_rows = n_q; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads;
  a.head_dim = D; a.n_parts_total = w.n_parts; a.q_pos0 = 0; a.scale = scale;
  int part0 = 0;
  // groups of segments [batch, n, H_kv, cap, D] (bf16 rows): images, then one partial each
  auto segment_group = [&](const void* kc, const void* vc, const int32_t* len, int per_head, int n,
                           int cap, int capp, void* k_img, void* v_img) -> int {
    int r = pc_launch_kv_prepass(kc, vc, nullptr, nullptr, k_img, v_img, batch * n * n_kv_heads, cap, capp,
                                 1, D, st);
    if (r != PC_OK) return r;
    a.k_img = k_img; a.v_img = v_img; a.part_len = len; a.part_len_per_head = per_head;
    a.img_seq_stride = (long long)n * n_kv_heads * (capp / 64);
    a.img_part_stride = (long long)n_kv_heads * (capp / 64);
    a.img_head_stride = capp / 64;
    a.n_keys = cap; a.n_parts_grid = n; a.part0 = part0; a.causal_offset = PC_NO_CAUSAL;
    part0 += n;
    return pc_launch_flash(a, st);
  };
  if (n_seg > 0) {
    rc = pc_launch_fp8_to_rows(k8, v8, k_scale, v_scale, (long long)batch * n_seg * n_kv_heads, k_t, D,
                               base + w.rows_k, base + w.rows_v, st);
    if (rc != PC_OK) return rc;
    rc = segment_group(base + w.rows_k, base + w.rows_v, seg_len, seg_len_per_head, n_seg, k_t, w.ktp,
                       base + w.k_seg, base + w.v_seg);
    if (rc != PC_OK) return rc;
  }
  if (tail_cap > 0) {
    rc = segment_group(k_tail, v_tail, tail_len, 0, 1, tail_cap, w.tcp, base + w.k_tail, base + w.v_tail);
    if (rc != PC_OK) return rc;
  }
  if (k_self != nullptr) {
    rc = pc_launch_kv_prepass(k_self, v_self, nullptr, nullptr, base + w.k_self, base + w.v_self, batch, n_q,
                              w.nqp, n_kv_heads, D, st);
    if (rc != PC_OK) return rc;
    a.k_img = base + w.k_self; a.v_img = base + w.v_self; a.part_len = nullptr; a.part_len_per_head = 0;
    a.img_seq_stride = (long long)n_kv_heads * (w.nqp / 64); a.img_part_stride = 0;
    a.img_head_stride = w.nqp / 64;
    a.n_keys = n_q; a.n_parts_grid = 1; a.part0 = part0; a.causal_offset = 0;
    rc = pc_launch_flash(a, st);
    if (rc != PC_OK) return rc;
  }
  return pc_launch_merge(a.part_o, a.part_lse, a.q, nullptr, nullptr, out, lse_out, batch, n_q, n_q_heads,
                         n_kv_heads, D, w.n_parts, scale, st);
}

extern "C" int pc_parallel_attn(const void* q, const void* kc, const void* vc, const int32_t* seg_len,
                                int32_t seg_len_per_head, const void* k_self, const void* v_self, int32_t batch, int32_t n_q,
                                int32_t n_seg, int32_t k_t, int32_t n_q_heads, int32_t n_kv_heads,
                                int32_t head_dim, int32_t q_pos0, float rope_base,
                                float softmax_scale, void* out, float* lse_out, void* ws,
                                size_t ws_bytes, void* stream) {
  const int rc = check_par_args(q, kc, vc, seg_len_per_head, k_self, v_self, batch, n_q, n_seg, k_t,
                                n_q_heads, n_kv_heads, head_dim, q_pos0, rope_base, softmax_scale, out);
  if (rc != PC_OK) return rc;
  const ParWs w = par_ws_layout(batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim,
                                k_self != nullptr);
  if (!ws || !pc_aligned(ws, kAlign) || ws_bytes < w.total) return PC_ERR_WORKSPACE;
  return parallel_attn_run(q, kc, vc, seg_len, seg_len_per_head, k_self, v_self, batch, n_q, n_seg,
                           k_t, n_q_heads, n_kv_heads, head_dim, q_pos0, rope_base, softmax_scale,
                           out, lse_out, w, ws, stream);
}

// ---------------------------------------------------------------------------- no-allocation variant
// The scratch memory of pc_parallel_attn_static: one array per GPU, part of the loaded code
// object, alive until the process ends.  `scratch` names it in device code only; host code uses
// the per-device address that hipGetSymbolAddress returns (the array sits at a different address
// on every GPU).
static __device__ __align__(256) unsigned char scratch[PC_STATIC_SCRATCH_BYTES];

#define PC_MAX_DEVICES 64
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[PC_MAX_DEVICES];     // by device ordinal; nullptr = not resolved yet

// Address of `scratch` on the current device (resolved once per device, with that device current).
static int static_scratch(void** ptr) {
  int dev = -1;
  PC_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= PC_MAX_DEVICES) return PC_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    PC_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr || !pc_aligned(p, kAlign)) return PC_ERR_WORKSPACE;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return PC_OK;
}

extern "C" size_t pc_parallel_attn_static_max_bytes(void) { return PC_STATIC_SCRATCH_BYTES; }

extern "C" int pc_parallel_attn_static(const void* q, const void* kc, const void* vc,
                                       const int32_t* seg_len, int32_t seg_len_per_head,
                                       const void* k_self, const void* v_self, int32_t batch,
                                       int32_t n_q, int32_t n_seg, int32_t k_t, int32_t n_q_heads,
                                       int32_t n_kv_heads, int32_t head_dim, int32_t q_pos0,
                                       float rope_base, float softmax_scale, void* out,
                                       float* lse_out, void* stream) {
  int rc = check_par_args(q, kc, vc, seg_len_per_head, k_self, v_self, batch, n_q, n_seg, k_t,
                          n_q_heads, n_kv_heads, head_dim, q_pos0, rope_base, softmax_scale, out);
  if (rc != PC_OK) return rc;
  const ParWs w = par_ws_layout(batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim,
                                k_self != nullptr);
  if (!w.small) return PC_ERR_UNSUPPORTED;                  // the tile path needs K/V images: too large
  if (w.total > PC_STATIC_SCRATCH_BYTES) return PC_ERR_WORKSPACE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != PC_OK) return rc;
  // every byte of the scratch that the merge reads is written by this call's kernels first
  // (rotated q, one partial per workgroup), so nothing has to be cleared
  return parallel_attn_run(q, kc, vc, seg_len, seg_len_per_head, k_self, v_self, batch, n_q, n_seg,
                           k_t, n_q_heads, n_kv_heads, head_dim, q_pos0, rope_base, softmax_scale,
                           out, lse_out, w, ws, stream);
}
