// 8-bit compressed cache for the decoding stage (Eq. 9-11 with few query rows).
//
// The decode kernel reads every K / V byte once and is bound by HBM bandwidth, so storing the
// compressed segments in 8 bits halves its time.  Format: OCP 8-bit float E4M3 (1 sign, 4
// exponent bits with bias 7, 3 mantissa bits, largest magnitude 448, no infinities), one fp32
// scale per (sequence, segment, KV head) for K and one for V:
//   scale = max |x| over the segment's valid rows / 448   (1 if that maximum is 0)
//   code  = E4M3(x / scale), round to nearest even, saturating
// The paper leaves the cache precision open; this format is an extension of this library.
//
// kv_quantize_fp8_kernel   one workgroup per (sequence, segment, KV head, K or V): maximum,
//                          then codes; the second sweep reads the segment again (5 bytes per
//                          element in all), unless the caller hands in the maxima (the gather
//                          that fills the cache can leave them: 3 bytes per element).  Codes are
//                          written in 32-key blocks laid out for the matrix cores (below), V
//                          transposed.
// decode_attn_fp8_kernel   the split-KV kernel of decode_attn.hip on 8-bit operands: codes are
//                          widened in registers (every E4M3 value is exact in bf16), both
//                          products run on the 16x16x32 bf16 MFMA, the scales are folded into the
//                          logit scale and into the probabilities.  Every load instruction
//                          of a wavefront reads 1 KiB of consecutive bytes.
//
// K block layout.  A block of 32 keys x D codes is two 16-key tiles; a tile is D / 64 pieces of
// 1 KiB, piece i = 64 lanes x 16 bytes, lane 16 kk + c (kk < 4, c < 16) holding the codes of
// d = 64 i + 16 kk .. + 15 of key c of the tile: the A operand bytes of that lane for k-steps
// 2 i and 2 i + 1 of S^T = K Q^T (the query operand is permuted to the same d order).
//
// V block layout.  O^T[d, column] += V^T[d, key] P^T[key, column] wants, per lane, 8 keys of one
// d, and the probabilities a lane holds after the two 16-key logit tiles of a 32-key block are
// those of keys 4g..4g+3 and 16+4g..16+4g+3 (g = lane / 16).  So the codes of a block of 32 keys
// x D values are stored as D / 32 pieces of 1 KiB, piece q = 64 lanes x 16 bytes, lane (g, m)
// = 16 g + m holding [h][j]: h = 0, 1 -> d = 32 q + 16 h + m; j = 0..7 -> key 4 g + j (j < 4),
// 16 + 4 g + (j - 4) (j >= 4).  A piece is one fully coalesced 16-byte-per-lane load and gives
// two A operands.  A segment holds ceil(k_t / 32) blocks of K and of V; keys behind k_t or behind
// the segment's length carry code 0.
#include "pc_common.h"
#include <math.h>

#define PC_D8_WAVES 4
#define PC_D8_ITER_KEYS 32
#define PC_D8_LOG2E 1.4426950408889634f
#define PC_E4M3_MAX 448.0f


// ------------------------------------------------------------------------------------------
// Quantisation.  blockIdx.x = (b, s, g), blockIdx.y = 0 (K) or 1 (V).  The segment is read twice
// (maximum, then codes): 5 bytes of traffic per element.  1024 threads with 4 loads each in
// flight keep HBM busy (6.0 TB/s of actual traffic at the decode config); bounding the
// workgroups per CU so that the segments between the two sweeps would fit the last-level cache
// measured no gain.
#define PC_Q8_THREADS 1024
#define PC_Q8_UNROLL 4
__global__ __launch_bounds__(PC_Q8_THREADS) void kv_quantize_fp8_kernel(
    const uint16_t* __restrict__ kc, const uint16_t* __restrict__ vc,
    const int32_t* __restrict__ seg_len, int per_head, int n_kv_heads, int k_t, int D,
    const float* __restrict__ k_amax, const float* __restrict__ v_amax,
    uint8_t* __restrict__ k8, uint8_t* __restrict__ v8, float* __restrict__ k_scale,
    float* __restrict__ v_scale) {
  __shared__ uint32_t red[PC_Q8_THREADS / PC_WAVE];
  __shared__ __attribute__((aligned(16))) uint8_t tile[PC_Q8_THREADS * PC_Q8_UNROLL * 8];   // 32 KiB of codes, block layout
  const long long seg = blockIdx.x;
  const uint16_t* src = (blockIdx.y ? vc : kc) + seg * (long long)k_t * D;
  const int n_blk = (k_t + 31) / 32;
  uint8_t* dst = (blockIdx.y ? v8 : k8) + seg * (long long)n_blk * 32 * D;
  float* scale_out = blockIdx.y ? v_scale : k_scale;
  const int len = seg_len ? min(max(seg_len[per_head ? seg : seg / n_kv_heads], 0), k_t) : k_t;
  // 8-element groups: of the valid rows, and of all rows to write (whole 32-key blocks)
  const long long n_valid = (long long)len * D / 8;
  const long long n_all = (long long)n_blk * 32 * D / 8;
  const int gpr = D / 8;                                   // groups per row

  // largest magnitude: bf16 magnitudes order like their 15-bit patterns.  When the caller knows
  // it already (the gather leaves it), the first sweep is skipped and the segment is read once.
  const float* amax_in = blockIdx.y ? v_amax : k_amax;
  uint32_t amax = 0;
  for (long long i0 = 0; amax_in == nullptr && i0 < n_valid; i0 += PC_Q8_THREADS * PC_Q8_UNROLL) {
    uint4 x[PC_Q8_UNROLL];
#pragma unroll
    for (int u = 0; u < PC_Q8_UNROLL; ++u) {
      const long long i = i0 + u * PC_Q8_THREADS + threadIdx.x;
      x[u] = i < n_valid ? *(const uint4*)(src + 8 * i) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < PC_Q8_UNROLL; ++u) {
      const uint32_t w[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) amax = max(amax, max(w[e] & 0x7fffu, (w[e] >> 16) & 0x7fffu));
    }
  }
#pragma unroll
  for (int off = PC_WAVE / 2; off > 0; off >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, off));
  if (threadIdx.x % PC_WAVE == 0) red[threadIdx.x / PC_WAVE] = amax;
  __syncthreads();
  amax = 0;
#pragma unroll
  for (int w = 0; w < PC_Q8_THREADS / PC_WAVE; ++w) amax = max(amax, red[w]);
  const float fmax_ = amax_in ? fabsf(amax_in[seg]) : __uint_as_float(amax << 16);
  const float scale = fmax_ > 0.f ? fmax_ / PC_E4M3_MAX : 1.0f;
  if (threadIdx.x == 0) scale_out[seg] = scale;

  for (long long i0 = 0; i0 < n_all; i0 += PC_Q8_THREADS * PC_Q8_UNROLL) {
    uint4 x[PC_Q8_UNROLL];
#pragma unroll
    for (int u = 0; u < PC_Q8_UNROLL; ++u) {
      const long long i = i0 + u * PC_Q8_THREADS + threadIdx.x;
      x[u] = i < n_valid ? pc_load_once((const uint4*)(src + 8 * i)) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < PC_Q8_UNROLL; ++u) {
      const long long i = i0 + u * PC_Q8_THREADS + threadIdx.x;
      if (i >= n_all) continue;
      uint2 code = make_uint2(0u, 0u);              // rows behind the segment's length or behind k_t
      if (i < n_valid) {
        const uint32_t w[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
        float f[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          f[2 * e] = fminf(fmaxf(bf16_lo_to_f32(w[e]) / scale, -PC_E4M3_MAX), PC_E4M3_MAX);
          f[2 * e + 1] = fminf(fmaxf(bf16_hi_to_f32(w[e]) / scale, -PC_E4M3_MAX), PC_E4M3_MAX);
        }
        uint32_t c0 = 0, c1 = 0;
        c0 = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], c0, false);
        c0 = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], c0, true);
        c1 = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], c1, false);
        c1 = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], c1, true);
        code = make_uint2(c0, c1);
      }
      // group i = 8 values d0..d0+7 of one key: to its place in the block layout, in LDS
      const int il = (int)(i - i0);                         // group within this sweep step
      const int key_l = il / gpr, d0 = (il % gpr) * 8;      // key within the step's rows
      const int kib = key_l % 32, blk_l = key_l / 32;
      if (!blockIdx.y) {
        uint8_t* t = tile + blk_l * 32 * D + (kib / 16) * 16 * D + (d0 / 64) * 1024 +
                     (16 * ((d0 % 64) / 16) + kib % 16) * 16 + d0 % 16;
        *(uint2*)t = code;
      } else {
        const int g = (kib % 16) / 4, j = kib % 4 + 4 * (kib / 16);
        uint8_t* t = tile + blk_l * 32 * D + (d0 / 32) * 1024 + g * 256 + ((d0 % 32) / 16) * 8 + j;
        const int m0 = d0 % 16;                               // m = m0 .. m0 + 7
#pragma unroll
        for (int e = 0; e < 8; ++e)
          t[(m0 + e) * 16] = (uint8_t)(((e < 4 ? code.x : code.y) >> (8 * (e % 4))) & 0xffu);
      }
    }
    // a sweep step covers whole blocks (its rows are a multiple of 32): copy them out
    __syncthreads();
    const long long step_bytes = min((long long)PC_Q8_THREADS * PC_Q8_UNROLL * 8, (n_all - i0) * 8);
    for (long long o = 16LL * threadIdx.x; o < step_bytes; o += 16LL * PC_Q8_THREADS)
      pc_store_once((uint4*)(dst + i0 * 8 + o), *(const uint4*)(tile + o));
    __syncthreads();
  }
}

int pc_launch_kv_quantize_fp8(const void* kc, const void* vc, const int32_t* seg_len,
                              int seg_len_per_head, long long n_segs, int n_kv_heads, int k_t,
                              int head_dim, const float* k_amax, const float* v_amax, void* k8,
                              void* v8, float* k_scale, float* v_scale, hipStream_t st) {
  if (n_segs == 0) return PC_OK;
  if (n_segs > 0x7fffffffLL) return PC_ERR_SHAPE;
  PcProfScope prof(PC_KERNEL_KV_QUANTIZE, st);
  hipLaunchKernelGGL(kv_quantize_fp8_kernel, dim3((unsigned)n_segs, 2), dim3(PC_Q8_THREADS), 0, st,
                     (const uint16_t*)kc, (const uint16_t*)vc, seg_len, seg_len_per_head, n_kv_heads,
                     k_t, head_dim, k_amax, v_amax, (uint8_t*)k8, (uint8_t*)v8, k_scale, v_scale);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
struct PcDecode8Args {
  const uint16_t* q;      // rotated queries [B, n_q, H_q, D] bf16
  const uint8_t* k8;      // [B, S, H_kv, ceil(k_t / 32) * 32 * D] E4M3 codes in 32-key blocks
  const uint8_t* v8;      // the same size, transposed blocks
  const float* k_scale;   // [B, S, H_kv]
  const float* v_scale;
  const int32_t* seg_len; // [B, S] ([B, S, H_kv] if seg_len_per_head) or nullptr
  int seg_len_per_head;
  float* part_o;          // [B, P, n_q, H_q, D]
  float* part_lse;        // [B, P, n_q, H_q]
  int n_q, n_seg, k_t, n_q_heads, n_kv_heads, n_parts;
  int parts_grid;         // workgroups (partials) per (sequence, KV head) in this launch
  float scale_log2;       // softmax scale * log2(e)
};

// four E4M3 codes of one 32-bit word -> two packed bf16 pairs (exact: every E4M3 value is a bf16
// value), one conversion instruction per pair (the scaled form with scale 1)
typedef __bf16 pc_bf2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void pc_e4m3x4_to_bf16(uint32_t w, uint32_t& lo, uint32_t& hi) {
  const pc_bf2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
  const pc_bf2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);
  lo = *(const uint32_t*)&a;
  hi = *(const uint32_t*)&b;
}

// ------------------------------------------------------------------------------------------
// Widening of 8-bit segments to bf16 rows (for the tile kernel, which takes the query block over
// the 8-bit cache through the same path as a 16-bit cache): value = code * scale, rounded to bf16.
// One workgroup per (segment, 32-key block, K or V); a thread takes one 16-byte piece of the block
// (the layouts are those of kv_quantize_fp8_kernel above).
__global__ __launch_bounds__(256) void fp8_to_rows_kernel(
    const uint8_t* __restrict__ k8, const uint8_t* __restrict__ v8, const float* __restrict__ k_scale,
    const float* __restrict__ v_scale, int k_t, int D, uint16_t* __restrict__ k_rows,
    uint16_t* __restrict__ v_rows) {
  const long long seg = blockIdx.x;
  const int blk = blockIdx.y, is_v = blockIdx.z;
  const int n_blk = (k_t + 31) / 32;
  const int p = threadIdx.x;                              // 16-byte piece of the block
  if (p >= 32 * D / 16) return;
  const uint8_t* src = (is_v ? v8 : k8) + (seg * n_blk + blk) * 32LL * D + 16 * p;
  uint16_t* dst = (is_v ? v_rows : k_rows) + seg * (long long)k_t * D;
  const float scale = (is_v ? v_scale : k_scale)[seg];
  const uint4 raw = *(const uint4*)src;
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
  float f[16];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    uint32_t lo, hi;
    pc_e4m3x4_to_bf16(w[e], lo, hi);
    f[4 * e] = bf16_lo_to_f32(lo) * scale; f[4 * e + 1] = bf16_hi_to_f32(lo) * scale;
    f[4 * e + 2] = bf16_lo_to_f32(hi) * scale; f[4 * e + 3] = bf16_hi_to_f32(hi) * scale;
  }
  const int lane = p % 64, piece = p / 64;
  if (!is_v) {
    // piece = tile * (D / 64) + i; lane 16 kk + c: values d = 64 i + 16 kk .. + 15 of key c of the tile
    const int tile = piece / (D / 64), i = piece % (D / 64), kk = lane / 16, c = lane % 16;
    const int key = 32 * blk + 16 * tile + c;
    if (key < k_t) {
      uint32_t o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = pack_bf16x2(f[2 * e], f[2 * e + 1]);
      uint4* d4 = (uint4*)(dst + (long long)key * D + 64 * i + 16 * kk);
      d4[0] = make_uint4(o[0], o[1], o[2], o[3]);
      d4[1] = make_uint4(o[4], o[5], o[6], o[7]);
    }
  } else {
    // piece q; lane 16 g + m holds [h][j]: value d = 32 q + 16 h + m of key 4 g + j (j < 4) or
    // 16 + 4 g + (j - 4)
    const int g = lane / 16, m = lane % 16;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int key = 32 * blk + (j < 4 ? 4 * g + j : 16 + 4 * g + (j - 4));
        if (key < k_t) dst[(long long)key * D + 32 * piece + 16 * h + m] = (uint16_t)f32_to_bf16_bits(f[8 * h + j]);
      }
  }
}

int pc_launch_fp8_to_rows(const void* k8, const void* v8, const float* k_scale, const float* v_scale,
                          long long n_segs, int k_t, int head_dim, void* k_rows, void* v_rows,
                          hipStream_t st) {
  if (n_segs == 0) return PC_OK;
  const int n_blk = (k_t + 31) / 32;
  if (n_segs > 0x7fffffffLL || n_blk > 65535) return PC_ERR_SHAPE;
  PcProfScope prof(PC_KERNEL_FP8_TO_ROWS, st);
  hipLaunchKernelGGL(fp8_to_rows_kernel, dim3((unsigned)n_segs, n_blk, 2), dim3(256), 0, st,
                     (const uint8_t*)k8, (const uint8_t*)v8, k_scale, v_scale, k_t, head_dim,
                     (uint16_t*)k_rows, (uint16_t*)v_rows);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

template <int D, int NQ>
__global__ __launch_bounds__(PC_D8_WAVES * PC_WAVE) void decode_attn_fp8_kernel(PcDecode8Args a) {
  constexpr int KSTEPS = D / 32;            // MFMA k-steps; a lane owns 8 KSTEPS = D / 4 bytes of each of its K rows
  constexpr int KQ = D / 64;                // 16-byte loads per lane and 16-key block
  constexpr int VLOADS = D / 32;            // 1 KiB pieces of a V block: one 16-byte load per lane each
  constexpr int MB = D / 16;                // 16-row blocks of O^T
  constexpr int KBLK = PC_D8_ITER_KEYS / 16;
  static_assert(KBLK == 2, "the V block layout assumes two 16-key logit tiles per block");

  __shared__ float red_o[PC_D8_WAVES][NQ][D];
  __shared__ float red_m[PC_D8_WAVES][NQ], red_l[PC_D8_WAVES][NQ];

  const int G = a.n_q_heads / a.n_kv_heads;
  const int n_cols = a.n_q * G;             // valid query columns (<= NQ)
  const int lane = threadIdx.x % PC_WAVE, wave = threadIdx.x / PC_WAVE;
  const int kk = lane / 16, c16 = lane % 16;

  int bid = blockIdx.x;
  const int part = bid % a.parts_grid; bid /= a.parts_grid;
  const int g = bid % a.n_kv_heads;    bid /= a.n_kv_heads;
  const int b = bid;

  // A wavefront streams its run of 32-key blocks, through segment boundaries, under one running
  // softmax (one partial per workgroup).  A cursor names the next block: where it is, the
  // segment's base pointers and its scales (K: folded into the logit scale; V: applied to the
  // probabilities that multiply the codes, not to the row sum).
  struct Cursor { PcBlockCursor at; const uint8_t* k; const uint8_t* v; float k_sc, v_sc; bool valid; };
  const long long seg_bytes = (long long)((a.k_t + 31) / 32) * 32 * D;
  PcSegLens lens;
  lens.seg_len = a.seg_len; lens.per_head = a.seg_len_per_head; lens.n_seg = a.n_seg;
  lens.n_kv_heads = a.n_kv_heads; lens.k_t = a.k_t; lens.b = b; lens.g = g;
  auto place = [&](const PcBlockCursor& at) {
    Cursor c; c.at = at; c.valid = at.valid; c.k = nullptr; c.v = nullptr; c.k_sc = 0.f; c.v_sc = 0.f;
    if (at.valid) {
      const long long seg_id = ((long long)b * a.n_seg + at.s) * a.n_kv_heads + g;
      c.k = a.k8 + seg_id * seg_bytes; c.v = a.v8 + seg_id * seg_bytes;
      c.k_sc = a.k_scale[seg_id] * a.scale_log2;           // logits in log2 units
      c.v_sc = a.v_scale[seg_id];
    }
    return c;
  };
  auto next = [&](const Cursor& c) { return place(pc_blocks_next(lens, c.at)); };

  // B operand: column c16 = (t, head-in-group); k-step j of lane group kk covers
  // d = 64 (j / 2) + 16 kk + 8 (j % 2) .. + 7, the d order of the K block layout
  bf16x8 bq[KSTEPS];
  {
    const bool valid = c16 < n_cols;
    const int t = valid ? c16 / G : 0, hg = valid ? c16 % G : 0;
    const uint16_t* qrow = a.q + (((long long)b * a.n_q + t) * a.n_q_heads + g * G + hg) * D;
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j) {
      uint4 raw = valid ? *(const uint4*)(qrow + 64 * (j / 2) + 16 * kk + 8 * (j % 2)) : make_uint4(0, 0, 0, 0);
      bq[j] = *(bf16x8*)&raw;
    }
  }

  float m_run = -INFINITY, l_run = 0.f;     // of column c16 (this lane's share of the sum)
  // O^T: row block mb, register r = value d = 16 mb + 4 kk + r of column c16
  floatx4 o_acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) o_acc[mb] = floatx4{0.f, 0.f, 0.f, 0.f};

  // three register buffers: the loads of two iterations (2 x 8 KiB per wavefront) stay in flight
  uint4 kbuf[3][KBLK][KQ], vbuf[3][VLOADS];
  auto issue_loads = [&](int buf, const Cursor& c) {
    // the block's pieces: key0 is a multiple of 32, and whole blocks exist up to ceil(k_t / 32)
    const long long blk_off = (long long)c.at.blk * 32 * D + 16 * lane;
    const uint8_t* kblk = c.k + blk_off;
    const uint8_t* vblk = c.v + blk_off;
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi)
#pragma unroll
      for (int i = 0; i < KQ; ++i)
        kbuf[buf][bi][i] = pc_load_once((const uint4*)(kblk + bi * 16 * D + 1024 * i));
#pragma unroll
    for (int i = 0; i < VLOADS; ++i)
      vbuf[buf][i] = pc_load_once((const uint4*)(vblk + 1024 * i));
  };

  auto consume = [&](int buf, const Cursor& cur) {
    const int key0 = 32 * cur.at.blk, w_end = cur.at.len;
    const float k_sc = cur.k_sc, v_sc = cur.v_sc;
    floatx4 acc[KBLK];
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi) {
      acc[bi] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < KSTEPS; ++j) {
        // k-step j: words 2 (j % 2), 2 (j % 2) + 1 of the lane's load j / 2
        const uint4 raw = kbuf[buf][bi][j / 2];
        const uint32_t w0 = (j % 2) ? raw.z : raw.x, w1 = (j % 2) ? raw.w : raw.y;
        u32x4 kb16;
        uint32_t lo, hi;
        pc_e4m3x4_to_bf16(w0, lo, hi); kb16[0] = lo; kb16[1] = hi;
        pc_e4m3x4_to_bf16(w1, lo, hi); kb16[2] = lo; kb16[3] = hi;
        acc[bi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8*)&kb16, bq[j], acc[bi], 0, 0, 0);
      }
    }
    float sv[KBLK][4];
    float bmax = -INFINITY;
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int key = key0 + 16 * bi + 4 * kk + j;
        sv[bi][j] = (key < w_end) ? acc[bi][j] * k_sc : -INFINITY;
        bmax = fmaxf(bmax, sv[bi][j]);
      }
    bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
    const float m_new = fmaxf(m_run, bmax);          // finite: every block holds a valid key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // arguments <= 0: the bare instruction
    m_run = m_new;
    float psum = 0.f;
    // P^T as the B operand: this lane's 8 probabilities are k-slice kk of column c16, in the
    // key order of the V block layout; the V scale rides on them (not on the row sum)
    u32x4 pb;
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi)
#pragma unroll
      for (int j = 0; j < 4; j += 2) {
        const float p0 = __builtin_amdgcn_exp2f(sv[bi][j] - m_new);
        const float p1 = __builtin_amdgcn_exp2f(sv[bi][j + 1] - m_new);
        psum += p0 + p1;
        pb[2 * bi + j / 2] = pack_bf16x2(p0 * v_sc, p1 * v_sc);
      }
    l_run = l_run * alpha + psum;
    if (__any(alpha != 1.0f)) {                      // some column's maximum grew (rare after the first keys)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) o_acc[mb][r] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < VLOADS; ++i) {
      const uint4 raw = vbuf[buf][i];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t w0 = h ? raw.z : raw.x, w1 = h ? raw.w : raw.y;
        u32x4 va;
        uint32_t lo, hi;
        pc_e4m3x4_to_bf16(w0, lo, hi); va[0] = lo; va[1] = hi;
        pc_e4m3x4_to_bf16(w1, lo, hi); va[2] = lo; va[3] = hi;
        o_acc[2 * i + h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8*)&va, *(bf16x8*)&pb, o_acc[2 * i + h], 0, 0, 0);
      }
    }
  };

  // three register buffers: the loads of two blocks (2 x 8 KiB per wavefront) stay in flight
  Cursor c0 = place(pc_blocks_begin(lens, part, a.parts_grid, __builtin_amdgcn_readfirstlane(wave),
                                    PC_D8_WAVES, lane));
  if (c0.valid) {
    Cursor c1 = next(c0);
    issue_loads(0, c0);
    if (c1.valid) issue_loads(1, c1);
    auto iter = [&](int cur_buf, int fill_buf) __attribute__((always_inline)) {
      // c0 = block to consume (in cur_buf), c1 = the block after it (already in flight)
      Cursor c2 = c1.valid ? next(c1) : c1;
      if (c2.valid) issue_loads(fill_buf, c2);
      consume(cur_buf, c0);
      c0 = c1; c1 = c2;
    };
    while (true) {
      iter(0, 2); if (!c0.valid) break;
      iter(1, 0); if (!c0.valid) break;
      iter(2, 1); if (!c0.valid) break;
    }
  }

  // ---- wavefront totals: sum the per-lane shares
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (kk == 0 && c16 < NQ) { red_m[wave][c16] = m_run; red_l[wave][c16] = l_run; }
  if (c16 < NQ) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 4; ++r) red_o[wave][c16][16 * mb + 4 * kk + r] = o_acc[mb][r];
  }
  __syncthreads();

  // ---- merge the 4 wavefronts, write one partial per workgroup (values scaled back)
  for (int idx = threadIdx.x; idx < n_cols * D; idx += blockDim.x) {
    const int n = idx / D, d = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < PC_D8_WAVES; ++w) M = fmaxf(M, red_m[w][n]);
    float num = 0.f, den = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int w = 0; w < PC_D8_WAVES; ++w) {
        const float sc = exp2f(red_m[w][n] - M);
        num += sc * red_o[w][n][d];
        den += sc * red_l[w][n];
      }
    }
    const int t = n / G, hg = n % G;
    const long long row = (((long long)b * a.n_parts + part) * a.n_q + t) * a.n_q_heads + g * G + hg;
    a.part_o[row * D + d] = (den > 0.f) ? num / den : 0.f;
    if (d == 0) a.part_lse[row] = (den > 0.f) ? (M + log2f(den)) * 0.6931471805599453f : -INFINITY;
  }
}

template <int D>
static int launch_decode8_d(const PcDecode8Args& a, int batch, int nq_pad, hipStream_t st) {
  const long long blocks = (long long)batch * a.n_kv_heads * a.parts_grid;
  if (blocks == 0) return PC_OK;
  if (blocks > 0x7fffffffLL) return PC_ERR_SHAPE;
  dim3 grid((unsigned)blocks), block(PC_D8_WAVES * PC_WAVE);
  PcProfScope prof(PC_KERNEL_DECODE_FP8, st);
  if (nq_pad == 4) hipLaunchKernelGGL((decode_attn_fp8_kernel<D, 4>), grid, block, 0, st, a);
  else if (nq_pad == 8) hipLaunchKernelGGL((decode_attn_fp8_kernel<D, 8>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((decode_attn_fp8_kernel<D, 16>), grid, block, 0, st, a);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

int pc_launch_decode_fp8(const void* q_rot, const void* k8, const void* v8, const float* k_scale,
                         const float* v_scale, const int32_t* seg_len, int seg_len_per_head,
                         int batch, int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads,
                         int head_dim, float scale, float* part_o, float* part_lse, int n_parts,
                         hipStream_t st) {
  PcDecode8Args a;
  a.q = (const uint16_t*)q_rot; a.k8 = (const uint8_t*)k8; a.v8 = (const uint8_t*)v8;
  a.k_scale = k_scale; a.v_scale = v_scale;
  a.seg_len = seg_len; a.seg_len_per_head = seg_len_per_head; a.part_o = part_o; a.part_lse = part_lse;
  a.n_q = n_q; a.n_seg = n_seg; a.k_t = k_t; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads;
  a.parts_grid = pc_decode_split(k_t, n_seg, (long long)batch * n_kv_heads).n_parts;
  a.n_parts = n_parts;
  a.scale_log2 = scale * PC_D8_LOG2E;
  const int cols = n_q * (n_q_heads / n_kv_heads);
  if (cols > 16) return PC_ERR_UNSUPPORTED;               // the columns of one 16x16x32 MFMA
  const int nq_pad = cols <= 4 ? 4 : (cols <= 8 ? 8 : 16);
  return head_dim == 128 ? launch_decode8_d<128>(a, batch, nq_pad, st)
                         : launch_decode8_d<64>(a, batch, nq_pad, st);
}
