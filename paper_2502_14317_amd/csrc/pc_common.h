// Internal helpers shared by the HIP translation units of the ParallelComp library (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "parallelcomp.h"
#include "parallelcomp_bench.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16-byte register quad

#define PC_WAVE 64

// ---------------------------------------------------------------- host-side error plumbing
void pc_set_hip_error(int err);
#define PC_HIP_TRY(expr)                                   \
  do {                                                     \
    hipError_t _e = (expr);                                \
    if (_e != hipSuccess) {                                \
      pc_set_hip_error((int)_e);                           \
      return PC_ERR_HIP;                                   \
    }                                                      \
  } while (0)
#define PC_LAUNCH_CHECK() PC_HIP_TRY(hipGetLastError())

// Brackets the kernel launches of one scope with HIP events when profiling is enabled.
struct PcProfScope {
  int slot;
  hipStream_t st;
  PcProfScope(int kernel_id, hipStream_t stream);
  ~PcProfScope();
};

// hipFuncAttributeMaxDynamicSharedMemorySize, set once per (kernel, device) instead of on every
// launch: `done` holds one bit per device ordinal (ordinals beyond 63 set it every time).
#include <atomic>
static inline int pc_raise_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  PC_HIP_TRY(hipGetDevice(&dev));
  const uint64_t bit = dev < 64 ? (1ull << dev) : 0ull;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return PC_OK;
  PC_HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  done.fetch_or(bit, std::memory_order_release);
  return PC_OK;
}

static inline size_t pc_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline bool pc_aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// ---------------------------------------------------------------- bf16 <-> fp32 (device)
__device__ __forceinline__ float bf16_lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; inputs are finite by contract (NaN keeps a NaN pattern)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
// two fp32 -> packed bf16 pair (round-to-nearest-even) in one v_cvt_pk_bf16_f32
typedef __bf16 pc_bf16x2 __attribute__((ext_vector_type(2)));
typedef float pc_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  pc_f32x2 v = {lo, hi};
  pc_bf16x2 r = __builtin_convertvector(v, pc_bf16x2);
  return *(uint32_t*)&r;
}

// 16-byte global load / store of data that is touched once (streamed): the non-temporal hint
// keeps it from displacing reusable lines in the caches
__device__ __forceinline__ uint4 pc_load_once(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void pc_store_once(uint4* p, uint4 x) {
  const u32x4 v = {x.x, x.y, x.z, x.w};
  __builtin_nontemporal_store(v, (u32x4*)p);
}
__device__ __forceinline__ u32x4 pc_load_once(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void pc_store_once(u32x4* p, u32x4 x) { __builtin_nontemporal_store(x, p); }

// Exchange between lane l and lane l ^ 32 without going through LDS: v_permlane32_swap leaves
// the low half's values in both halves of the first result and the high half's in the second.
__device__ __forceinline__ float pc_xhalf_max(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pc_xhalf_sum(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// fp32 score -> uint32 key whose unsigned order is the float order; NaN -> 0 (below everything),
// -0.0 and +0.0 map to the same key
__device__ __forceinline__ uint32_t pc_order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---------------------------------------------------------------- kernels' host launchers
// (each defined in its own translation unit; all arguments already validated)
int pc_launch_gather(const void* k_src, const void* v_src, const int32_t* chunk_idx,
                     const int32_t* tok_idx, int batch, int n_chunks, int rows, int n_sel,
                     int n_kv_heads, int k, int head_dim, void* k_dst, void* v_dst,
                     float* k_amax, float* v_amax, hipStream_t st);   // amax: both or neither
int pc_launch_select_chunks(const float* score, int n, int k, int32_t* out_idx, float* out_score,
                            hipStream_t st);
// cls_lo >= cls_hi: plain top-k (Eq. 7); else Eq. 8 first.  out_cnt may be nullptr.
int pc_launch_select_tokens(const float* tok_score, const int32_t* chunk_idx, int n_sel,
                            int n_kv_heads, int chunk_len, int k, float lambda, int cls_lo,
                            int cls_hi, const int32_t* chunk_lens, int32_t* out_idx,
                            int32_t* out_cnt, hipStream_t st);

int pc_launch_chunk_queue(const float* batch_score, int n_batch, int chunk_id0, int cap,
                          int32_t* queue_id, float* queue_score, int32_t* queue_slot,
                          int32_t* slot_src, hipStream_t st);

int pc_launch_rope_table(float2* table, int n_pos, int head_dim, float base, hipStream_t st);

// K/V pre-pass: K (rotated when a table is given; skipped when k == nullptr) -> k_rope (row-major,
// optional) and K tile images (optional); V -> V^T tile images.  Images: [n_seq][n_kv_heads][Lp / 64][64 * D].
int pc_launch_kv_prepass(const void* k, const void* v, const float2* table, void* k_rope,
                         void* k_img, void* v_img, int n_seq, int L, int Lp, int n_kv_heads,
                         int head_dim, hipStream_t st);

// Flash-style tile kernel.  A workgroup handles (sequence, query head, 128-row Q tile, part);
// a "part" is an independent key set (a compressed segment) with its own softmax.
struct PcFlashArgs {
  const void* q;            // [n_seq, n_rows, H_q, D] bf16
  const void* k_img;        // K tile images (rotated keys), image index = seq * img_seq_stride +
  const void* v_img;        //   part * img_part_stride + head * img_head_stride + tile; V^T likewise
  const float2* table;      // rope table (rotate q at q_pos0 + row, then scale), or nullptr: q is
                            //   already rotated AND already multiplied by scale * log2(e)
  void* o;                  // [n_seq, n_rows, H_q, D] bf16 (final output mode)
  float* lse;               // [n_seq, H_q, n_rows] or nullptr
  float* part_o;            // partial mode: [n_seq, n_parts_total, n_rows, H_q, D] fp32, else nullptr
  float* part_lse;          // [n_seq, n_parts_total, n_rows, H_q]
  const int32_t* part_len;  // [n_seq, n_parts_grid] (x [n_kv_heads] if part_len_per_head) valid keys per part, or nullptr (= n_keys)
  int part_len_per_head;
  const int32_t* seq_ctx;   // [n_seq] context rows per sequence or nullptr: sequence s has
  int seq_add;              //   min(seq_ctx[s], n_rows - seq_add) + seq_add rows (and keys)
  long long img_seq_stride, img_part_stride, img_head_stride;              // in tile images
  int n_seq, n_rows, n_keys, n_q_heads, n_kv_heads, head_dim;
  int n_parts_grid, n_parts_total, part0;
  int causal_offset;        // key j visible to row r iff j <= r + causal_offset; >= 2^29: no mask
  int q_pos0;
  float scale;
};
#define PC_NO_CAUSAL (1 << 29)
int pc_launch_flash(const PcFlashArgs& a, hipStream_t st);

int pc_launch_self_info(const void* logits, const int32_t* targets, int n_chunks, int n_tokens,
                        int vocab, int negate, float* token_nll, float* info, hipStream_t st);

size_t pc_scores_ml_bytes(const pc_shape* s);
// Pre-pass duties the first score pass can take over (it reads and rotates every key anyway):
// the rotated keys (k_rope, nullable), the K tile images and the V^T tile images of
// pc_launch_kv_prepass, Lp = L rounded up to 64.
struct PcPrepassOut { const void* v; void* k_rope; void* k_img; void* v_img; int Lp; };
int pc_launch_scores(const pc_shape* s, const void* q, const void* k, const int32_t* chunk_lens, const float2* table,
                     void* ml_ws, float* tok_score, float* chunk_score, const PcPrepassOut* pre,
                     hipStream_t st);

int pc_launch_rope_q(const void* q, void* q_rot, long long n_rows, int n_q, int n_heads, int D,
                     int pos0, float base, float mul, hipStream_t st);
// How the split-KV decode kernels cut the keys into workgroups (n_bg = batch * H_kv): the keys of
// a (sequence, KV head) group, all its segments laid end to end in blocks of 32 keys, are cut
// into n_parts equal runs of blocks, one workgroup (and one partial result) each.
struct PcDecodeSplit { int n_parts; };
PcDecodeSplit pc_decode_split(int k_t, int n_seg, long long n_bg);

// A wavefront's walk over its run of 32-key blocks.  The group's blocks are numbered through all
// segments (segment s has ceil(len_s / 32) of them); part `part` of n_parts takes blocks
// [NB part / n_parts, NB (part + 1) / n_parts), wavefront w of n_waves the w-th of n_waves equal
// runs of that.  Everything here is wavefront-uniform.
struct PcSegLens {
  const int32_t* seg_len;   // [B, S] ([B, S, H_kv] if per_head) or nullptr (= k_t)
  int per_head, n_seg, n_kv_heads, k_t, b, g;
  __device__ __forceinline__ int len(int s) const {
    if (!seg_len) return k_t;
    const int idx = per_head ? (b * n_seg + s) * n_kv_heads + g : b * n_seg + s;
    return min(max(seg_len[idx], 0), k_t);
  }
};
struct PcBlockCursor {
  int s, blk, n_blk, len, left;   // segment, block within it, its block count and length, blocks left in the run
  bool valid;
};
__device__ __forceinline__ PcBlockCursor pc_blocks_begin(const PcSegLens& L, int part, int n_parts,
                                                         int wave, int n_waves, int lane) {
  PcBlockCursor c; c.s = 0; c.blk = 0; c.n_blk = 0; c.len = 0; c.left = 0; c.valid = false;
  const int nb_full = (L.k_t + 31) / 32;
  long long total = 0;
  if (!L.seg_len) {
    total = (long long)L.n_seg * nb_full;
  } else {
    // lanes take a segment each, 64 segments per round
    for (int s0 = 0; s0 < L.n_seg; s0 += PC_WAVE) {
      int nb = s0 + lane < L.n_seg ? (L.len(s0 + lane) + 31) / 32 : 0;
#pragma unroll
      for (int off = PC_WAVE / 2; off > 0; off >>= 1) nb += __shfl_xor(nb, off);
      total += __builtin_amdgcn_readfirstlane(nb);
    }
  }
  const long long lo = total * part / n_parts, hi = total * (part + 1) / n_parts;
  const long long w_lo = lo + (hi - lo) * wave / n_waves, w_hi = lo + (hi - lo) * (wave + 1) / n_waves;
  if (w_lo >= w_hi) return c;
  c.left = (int)(w_hi - w_lo);
  if (!L.seg_len) {
    c.s = (int)(w_lo / nb_full); c.blk = (int)(w_lo % nb_full); c.n_blk = nb_full; c.len = L.k_t;
    c.valid = true;
    return c;
  }
  long long base = 0;
  for (int s0 = 0; s0 < L.n_seg; s0 += PC_WAVE) {
    const int len = s0 + lane < L.n_seg ? L.len(s0 + lane) : 0;
    const int nb = (len + 31) / 32;
    int incl = nb;                                            // inclusive prefix sum over the lanes
#pragma unroll
    for (int off = 1; off < PC_WAVE; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const long long rel = w_lo - base;                        // the run's first block, counted from this round's first segment
    const unsigned long long hit = __ballot(nb > 0 && incl - nb <= rel && rel < incl);
    if (hit) {
      const int src = __ffsll((long long)hit) - 1;
      c.s = s0 + src;
      c.blk = __builtin_amdgcn_readfirstlane((int)rel - __shfl(incl - nb, src));
      c.n_blk = __builtin_amdgcn_readfirstlane(__shfl(nb, src));
      c.len = __builtin_amdgcn_readfirstlane(__shfl(len, src));
      c.valid = true;
      return c;
    }
    base += __builtin_amdgcn_readfirstlane(__shfl(incl, PC_WAVE - 1));
  }
  return c;                                                   // not reached: w_lo < total
}
__device__ __forceinline__ PcBlockCursor pc_blocks_next(const PcSegLens& L, PcBlockCursor c) {
  if (--c.left <= 0) { c.valid = false; return c; }
  if (++c.blk < c.n_blk) return c;
  c.blk = 0;
  for (++c.s; c.s < L.n_seg; ++c.s) {                         // the next segment that has keys
    c.len = L.len(c.s);
    c.n_blk = (c.len + 31) / 32;
    if (c.n_blk > 0) return c;
  }
  c.valid = false;                                            // not reached: left counted real blocks
  return c;
}
int pc_launch_kv_append(const void* k_new, const void* v_new, int batch, int n_new, int n_seg,
                        int seg, int k_t, int n_kv_heads, int head_dim, int pos0, float base,
                        void* kc, void* vc, int32_t* seg_len, int seg_len_per_head,
                        hipStream_t st);
int pc_launch_decode(const void* q_rot, const void* kc, const void* vc, const int32_t* seg_len,
                     int seg_len_per_head, int batch, int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads,
                     int head_dim, float scale, float* part_o, float* part_lse, int n_parts, int part0,
                     hipStream_t st);
// k_amax, v_amax [n_segs] (both or neither): the largest |value| of every segment's valid rows,
// known beforehand (the gather leaves it): the kernel then reads the segment once
int pc_launch_kv_quantize_fp8(const void* kc, const void* vc, const int32_t* seg_len,
                              int seg_len_per_head, long long n_segs, int n_kv_heads, int k_t,
                              int head_dim, const float* k_amax, const float* v_amax, void* k8,
                              void* v8, float* k_scale, float* v_scale, hipStream_t st);
// 8-bit segments (32-key block layout of pc_kv_quantize_fp8) -> bf16 rows [n_segs, k_t, D] of
// code * scale (rounded to bf16), K and V
int pc_launch_fp8_to_rows(const void* k8, const void* v8, const float* k_scale, const float* v_scale,
                          long long n_segs, int k_t, int head_dim, void* k_rows, void* v_rows,
                          hipStream_t st);
int pc_launch_decode_fp8(const void* q_rot, const void* k8, const void* v8, const float* k_scale,
                         const float* v_scale, const int32_t* seg_len, int seg_len_per_head,
                         int batch, int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads,
                         int head_dim, float scale, float* part_o, float* part_lse, int n_parts,
                         hipStream_t st);
int pc_launch_merge(const float* part_o, const float* part_lse, const void* q_rot,
                    const void* k_self, const void* v_self, void* out, float* lse_out, int batch,
                    int n_q, int n_q_heads, int n_kv_heads, int head_dim, int n_parts, float scale,
                    hipStream_t st);
