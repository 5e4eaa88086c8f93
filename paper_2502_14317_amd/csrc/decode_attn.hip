// Parallel (global) attention for few query rows: the HBM-bound split-KV kernel and the exact
// logsumexp merge (Eq. 9-11: one softmax over [K^1 .. K^S, K^q], evaluated as independent
// per-piece softmaxes that are merged by LSE = log sum exp(lse_p), o = sum exp(lse_p - LSE) o_p).
//
// Every K/V byte is read exactly once, so the kernel is bound by HBM bandwidth.  Design:
//   * the keys of a (sequence, KV head) group, all its segments end to end in blocks of 32, are
//     cut into equal runs, one workgroup (4 wavefronts) each, so that the launch has one
//     workgroup per CU where the shapes allow (long runs, equal work, no ragged last round);
//     a wavefront owns a contiguous quarter of the run and streams it 32 keys at a time with
//     16-byte loads, the next 32 keys already in flight while the current ones are used;
//   * the query columns of one KV group (n_q * G <= 16) form the N side of a 16x16x32 bf16
//     MFMA: S^T = K Q^T, so the lane that owns a column owns its running max and sum;
//   * P V runs on the vector ALUs in the layout the V loads arrive in (D across lanes), with
//     the probabilities broadcast through a small per-wavefront LDS tile;
//   * partial (o, lse) per workgroup go to the workspace; a second kernel merges them.
#include "pc_common.h"
#include <math.h>

#define PC_DEC_WAVES 4
#define PC_DEC_ITER_KEYS 32
#define PC_DEC_LOG2E 1.4426950408889634f

#define PC_WAVE_LDS_SYNC()                                   \
  do {                                                       \
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   \
    __builtin_amdgcn_wave_barrier();                         \
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");   \
  } while (0)

struct PcDecodeArgs {
  const uint16_t* q;      // rotated queries [B, n_q, H_q, D]
  const uint16_t* kc;     // [B, S, H_kv, k_t, D]
  const uint16_t* vc;
  const int32_t* seg_len; // [B, S] ([B, S, H_kv] if seg_len_per_head) or nullptr
  int seg_len_per_head;
  float* part_o;          // [B, P, n_q, H_q, D]
  float* part_lse;        // [B, P, n_q, H_q]
  int n_q, n_seg, k_t, n_q_heads, n_kv_heads, n_parts;
  int parts_grid;         // workgroups (partials) per (sequence, KV head) in this launch
  int part0;              // index of this launch's first partial among the n_parts
  float scale_log2;       // softmax scale * log2(e)
};

template <int D, int NQ>
__global__ __launch_bounds__(PC_DEC_WAVES * PC_WAVE) void decode_attn_kernel(PcDecodeArgs a) {
  constexpr int KSTEPS = D / 32;            // MFMA k-steps over the head dimension
  constexpr int LPR = D / 8;                // lanes per V row (16-byte pieces)
  constexpr int RPI = PC_WAVE / LPR;        // V rows per load instruction
  constexpr int VLOADS = PC_DEC_ITER_KEYS / RPI;
  constexpr int KBLK = PC_DEC_ITER_KEYS / 16;

  __shared__ float p_lds[PC_DEC_WAVES][PC_DEC_ITER_KEYS][NQ];
  __shared__ float alpha_lds[PC_DEC_WAVES][NQ];
  __shared__ float red_o[PC_DEC_WAVES][NQ][D];
  __shared__ float red_m[PC_DEC_WAVES][NQ], red_l[PC_DEC_WAVES][NQ];

  const int G = a.n_q_heads / a.n_kv_heads;
  const int n_cols = a.n_q * G;             // valid query columns (<= NQ)
  const int lane = threadIdx.x % PC_WAVE, wave = threadIdx.x / PC_WAVE;
  const int kk = lane / 16, c16 = lane % 16;

  int bid = blockIdx.x;
  const int part = bid % a.parts_grid; bid /= a.parts_grid;
  const int g = bid % a.n_kv_heads;    bid /= a.n_kv_heads;
  const int b = bid;

  // A wavefront streams its run of 32-key blocks, through segment boundaries; the running
  // softmax carries over (same query columns, same KV head), so a workgroup leaves one partial.
  // A cursor names the next block: where it is, plus the segment's base pointers.
  struct Cursor { PcBlockCursor at; int key0; const uint16_t* k; const uint16_t* v; bool valid; };
  PcSegLens lens;
  lens.seg_len = a.seg_len; lens.per_head = a.seg_len_per_head; lens.n_seg = a.n_seg;
  lens.n_kv_heads = a.n_kv_heads; lens.k_t = a.k_t; lens.b = b; lens.g = g;
  auto place = [&](const PcBlockCursor& at) {
    Cursor c; c.at = at; c.valid = at.valid; c.key0 = 32 * at.blk; c.k = nullptr; c.v = nullptr;
    if (at.valid) {
      const long long seg_base = ((((long long)b * a.n_seg + at.s) * a.n_kv_heads + g) * a.k_t) * D;
      c.k = a.kc + seg_base; c.v = a.vc + seg_base;
    }
    return c;
  };
  auto next = [&](const Cursor& c) { return place(pc_blocks_next(lens, c.at)); };

  // B operand: column c16 = (t, head-in-group); lane holds d = 32*ks + 8*kk .. +7
  bf16x8 bq[KSTEPS];
  {
    const bool valid = c16 < n_cols;
    const int t = valid ? c16 / G : 0, hg = valid ? c16 % G : 0;
    const uint16_t* qrow = a.q + (((long long)b * a.n_q + t) * a.n_q_heads + g * G + hg) * D;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      uint4 raw = valid ? *(const uint4*)(qrow + 32 * ks + 8 * kk) : make_uint4(0, 0, 0, 0);
      bq[ks] = *(bf16x8*)&raw;
    }
  }

  float m_run = -INFINITY, l_run = 0.f;     // of column c16 (this lane's share of the sum)
  float o_acc[NQ][8];
#pragma unroll
  for (int n = 0; n < NQ; ++n)
#pragma unroll
    for (int e = 0; e < 8; ++e) o_acc[n][e] = 0.f;

  const int v_row = lane / LPR, v_piece = lane % LPR;

  uint4 kbuf[2][KBLK][KSTEPS], vbuf[2][VLOADS];
  auto issue_loads = [&](int buf, const Cursor& c) {
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi) {
      const int row = min(c.key0 + 16 * bi + c16, c.at.len - 1);
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks)
        kbuf[buf][bi][ks] = pc_load_once((const uint4*)(c.k + (long long)row * D + 32 * ks + 8 * kk));
    }
#pragma unroll
    for (int i = 0; i < VLOADS; ++i) {
      const int row = min(c.key0 + RPI * i + v_row, c.at.len - 1);
      vbuf[buf][i] = pc_load_once((const uint4*)(c.v + (long long)row * D + 8 * v_piece));
    }
  };

  auto consume = [&](int buf, const Cursor& cur) {
    const int key0 = cur.key0, w_end = cur.at.len;
    // S^T block: keys x columns
    floatx4 acc[KBLK];
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi) {
      acc[bi] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks)
        acc[bi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8*)&kbuf[buf][bi][ks], bq[ks],
                                                          acc[bi], 0, 0, 0);
    }
    float sv[KBLK][4];
    float bmax = -INFINITY;
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int key = key0 + 16 * bi + 4 * kk + j;
        sv[bi][j] = (key < w_end) ? acc[bi][j] * a.scale_log2 : -INFINITY;
        bmax = fmaxf(bmax, sv[bi][j]);
      }
    bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
    const float m_new = fmaxf(m_run, bmax);          // finite: every block holds a valid key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // arguments <= 0: the bare instruction
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int bi = 0; bi < KBLK; ++bi)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float p = __builtin_amdgcn_exp2f(sv[bi][j] - m_new);
        psum += p;
        if (c16 < NQ) p_lds[wave][16 * bi + 4 * kk + j][c16] = p;
      }
    l_run = l_run * alpha + psum;
    const bool moved = __any(alpha != 1.0f);         // some column's maximum grew (rare after the first keys)
    if (moved && kk == 0 && c16 < NQ) alpha_lds[wave][c16] = alpha;
    PC_WAVE_LDS_SYNC();
    // rescale (only when a maximum moved), then o[n][:] += p[key][n] * v[key][:]
    if (moved) {
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        const float al = alpha_lds[wave][n];
#pragma unroll
        for (int e = 0; e < 8; ++e) o_acc[n][e] *= al;
      }
    }
#pragma unroll
    for (int i = 0; i < VLOADS; ++i) {
      const int key_local = RPI * i + v_row;
      const uint4 raw = vbuf[buf][i];
      float vf[8];
      vf[0] = bf16_lo_to_f32(raw.x); vf[1] = bf16_hi_to_f32(raw.x);
      vf[2] = bf16_lo_to_f32(raw.y); vf[3] = bf16_hi_to_f32(raw.y);
      vf[4] = bf16_lo_to_f32(raw.z); vf[5] = bf16_hi_to_f32(raw.z);
      vf[6] = bf16_lo_to_f32(raw.w); vf[7] = bf16_hi_to_f32(raw.w);
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        const float p = p_lds[wave][key_local][n];    // 0 for masked keys
#pragma unroll
        for (int e = 0; e < 8; ++e) o_acc[n][e] = fmaf(p, vf[e], o_acc[n][e]);
      }
    }
    PC_WAVE_LDS_SYNC();
  };

  Cursor cur = place(pc_blocks_begin(lens, part, a.parts_grid, __builtin_amdgcn_readfirstlane(wave),
                                     PC_DEC_WAVES, lane));
  if (cur.valid) {
    issue_loads(0, cur);
    while (true) {
      Cursor nx = next(cur);
      if (nx.valid) issue_loads(1, nx);
      consume(0, cur);
      if (!nx.valid) break;
      cur = nx;
      nx = next(cur);
      if (nx.valid) issue_loads(0, nx);
      consume(1, cur);
      if (!nx.valid) break;
      cur = nx;
    }
  }

  // ---- wavefront totals: sum the per-lane shares
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
#pragma unroll
  for (int n = 0; n < NQ; ++n)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x = o_acc[n][e];
#pragma unroll
      for (int off = LPR; off < PC_WAVE; off <<= 1) x += __shfl_xor(x, off);
      o_acc[n][e] = x;
    }
  if (kk == 0 && c16 < NQ) { red_m[wave][c16] = m_run; red_l[wave][c16] = l_run; }
  if (v_row == 0) {
#pragma unroll
    for (int n = 0; n < NQ; ++n)
#pragma unroll
      for (int e = 0; e < 8; ++e) red_o[wave][n][8 * v_piece + e] = o_acc[n][e];
  }
  __syncthreads();

  // ---- merge the 4 wavefronts, write one partial per workgroup
  const int part_out = a.part0 + part;
  for (int idx = threadIdx.x; idx < n_cols * D; idx += blockDim.x) {
    const int n = idx / D, d = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < PC_DEC_WAVES; ++w) M = fmaxf(M, red_m[w][n]);
    float num = 0.f, den = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int w = 0; w < PC_DEC_WAVES; ++w) {
        const float sc = exp2f(red_m[w][n] - M);
        num += sc * red_o[w][n][d];
        den += sc * red_l[w][n];
      }
    }
    const int t = n / G, hg = n % G;
    const long long row = (((long long)b * a.n_parts + part_out) * a.n_q + t) * a.n_q_heads + g * G + hg;
    a.part_o[row * D + d] = (den > 0.f) ? num / den : 0.f;
    if (d == 0) a.part_lse[row] = (den > 0.f) ? (M + log2f(den)) * 0.6931471805599453f : -INFINITY;
  }
}

// ------------------------------------------------------------------------------------------
// Merge of partials (+ the causal self segment for the few-row path).  One workgroup of D
// threads per (b, t, h).  lse values are natural logarithms.
struct PcMergeArgs {
  const float* part_o;     // [B, P, n_q, H_q, D]
  const float* part_lse;   // [B, P, n_q, H_q]
  const uint16_t* q;       // rotated q, used only with the self segment
  const uint16_t* k_self;  // [B, n_q, H_kv, D] or nullptr
  const uint16_t* v_self;
  uint16_t* out;           // [B, n_q, H_q, D]
  float* lse_out;          // [B, H_q, n_q] or nullptr
  int n_q, n_q_heads, n_kv_heads, n_parts;
  float scale;
};

#define PC_MERGE_MAX_LDS_PARTS 1024      // weights of up to this many partials are kept in LDS

template <int D>
__global__ __launch_bounds__(D) void merge_kernel(PcMergeArgs a) {
  __shared__ float red[D / PC_WAVE + 1];
  __shared__ float self_s[16];
  __shared__ float wgt_lds[PC_MERGE_MAX_LDS_PARTS];
  const int d = threadIdx.x;
  int bid = blockIdx.x;
  const int h = bid % a.n_q_heads; bid /= a.n_q_heads;
  const int t = bid % a.n_q;       bid /= a.n_q;
  const int b = bid;
  const int G = a.n_q_heads / a.n_kv_heads, g = h / G;
  // partial p of this (b, t, h): row = row0 + p * row_stride
  const long long row0 = ((long long)b * a.n_parts * a.n_q + t) * a.n_q_heads + h;
  const long long row_stride = (long long)a.n_q * a.n_q_heads;
  const bool in_lds = a.n_parts <= PC_MERGE_MAX_LDS_PARTS;

  // the partials' logsumexps, one per thread and round (independent loads), and their maximum
  float M = -INFINITY;
  for (int p = d; p < a.n_parts; p += D) {
    const float l = a.part_lse[row0 + p * row_stride];
    if (in_lds) wgt_lds[p] = l;
    M = fmaxf(M, l);
  }
#pragma unroll
  for (int off = PC_WAVE / 2; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
  if (d % PC_WAVE == 0) red[d / PC_WAVE] = M;
  __syncthreads();
  M = red[0];
#pragma unroll
  for (int w = 1; w < D / PC_WAVE; ++w) M = fmaxf(M, red[w]);
  __syncthreads();                                           // red is reused below

  // self segment (only launched with n_q <= 16): logits of keys 0..t
  const bool has_self = a.k_self != nullptr;
  if (has_self) {
    const float qd = bf16_bits_to_f32(a.q[(((long long)b * a.n_q + t) * a.n_q_heads + h) * D + d]);
    for (int j = 0; j <= t; ++j) {
      float x = qd * bf16_bits_to_f32(a.k_self[(((long long)b * a.n_q + j) * a.n_kv_heads + g) * D + d]);
#pragma unroll
      for (int off = PC_WAVE / 2; off > 0; off >>= 1) x += __shfl_xor(x, off);
      if (d % PC_WAVE == 0) red[d / PC_WAVE] = x;
      __syncthreads();
      if (d == 0) {
        float tot = 0.f;
        for (int w = 0; w < D / PC_WAVE; ++w) tot += red[w];
        self_s[j] = tot * a.scale;
      }
      __syncthreads();
    }
    for (int j = 0; j <= t; ++j) M = fmaxf(M, self_s[j]);
  }
  float num = 0.f, den = 0.f;
  if (M > -INFINITY) {
    // weights exp(lse_p - M): computed once per partial and kept in LDS; every thread then sums
    // them in the same (partial) order, so all threads hold the same denominator
    if (in_lds) {
      for (int p = d; p < a.n_parts; p += D) wgt_lds[p] = expf(wgt_lds[p] - M);
      __syncthreads();
    }
    constexpr int U = 8;                                     // independent loads in flight per thread
    for (int p0 = 0; p0 < a.n_parts; p0 += U) {
      float w[U], x[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int p = min(p0 + u, a.n_parts - 1);
        w[u] = in_lds ? wgt_lds[p] : expf(a.part_lse[row0 + p * row_stride] - M);
        x[u] = a.part_o[(row0 + p * row_stride) * D + d];
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (p0 + u < a.n_parts) { num += w[u] * x[u]; den += w[u]; }
    }
    if (has_self) {
      for (int j = 0; j <= t; ++j) {
        const float wgt = expf(self_s[j] - M);
        num += wgt * bf16_bits_to_f32(a.v_self[(((long long)b * a.n_q + j) * a.n_kv_heads + g) * D + d]);
        den += wgt;
      }
    }
  }
  const long long orow = ((long long)b * a.n_q + t) * a.n_q_heads + h;
  a.out[orow * D + d] = (uint16_t)f32_to_bf16_bits(den > 0.f ? num / den : 0.f);
  if (a.lse_out && d == 0)
    a.lse_out[((long long)b * a.n_q_heads + h) * a.n_q + t] = den > 0.f ? M + logf(den) : -INFINITY;
}

// ------------------------------------------------------------------------------------------
// Rotate the query rows of the global attention at positions pos0 + t (fp64 angles; pos0 < 0:
// the rows are already rotated) and multiply them by `mul` before the one rounding to bf16 (the
// tile kernel wants its query operand scaled by softmax scale x log2(e); 1 for the split-KV kernel).
__global__ void rope_q_kernel(const uint16_t* __restrict__ q, uint16_t* __restrict__ q_rot,
                              long long n_pairs, int n_q, int n_heads, int D, int pos0,
                              double log_base, double mul) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pairs) return;
  const int half = D / 2;
  const int i = (int)(idx % half);
  const long long row = idx / half;                       // (b, t, h)
  const int t = (int)((row / n_heads) % n_q);
  double sn = 0.0, cs = 1.0;
  if (pos0 >= 0) {
    const double theta = exp(-2.0 * (double)i / (double)D * log_base);
    sincos((double)(pos0 + t) * theta, &sn, &cs);
  }
  const double x1 = bf16_bits_to_f32(q[row * D + i]), x2 = bf16_bits_to_f32(q[row * D + i + half]);
  q_rot[row * D + i] = (uint16_t)f32_to_bf16_bits((float)((x1 * cs - x2 * sn) * mul));
  q_rot[row * D + i + half] = (uint16_t)f32_to_bf16_bits((float)((x2 * cs + x1 * sn) * mul));
}

int pc_launch_rope_q(const void* q, void* q_rot, long long n_rows, int n_q, int n_heads, int D,
                     int pos0, float base, float mul, hipStream_t st) {
  const long long n_pairs = n_rows * (D / 2);
  if (n_pairs == 0) return PC_OK;
  PcProfScope prof(PC_KERNEL_ROPE_Q, st);
  hipLaunchKernelGGL(rope_q_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, st,
                     (const uint16_t*)q, (uint16_t*)q_rot, n_pairs, n_q, n_heads, D, pos0,
                     log((double)(pos0 >= 0 ? base : 2.0f)), (double)mul);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
// Decoding stage: append the K / V rows of newly generated tokens to one segment of the
// compacted cache (the growing tail behind the query block).  One workgroup per sequence: it
// reads the segment's length(s), writes the rows behind them (K rotated at pos0 + t when
// pos0 >= 0, fp64 angles) and, after a barrier that orders every read of a length before its
// update, stores the new length(s), all on the device, so a decode loop needs no host round
// trip.  Rows that would not fit the segment's capacity are dropped.
__global__ __launch_bounds__(256) void kv_append_kernel(
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new, int n_new, int n_seg,
    int seg, int k_t, int n_kv_heads, int D, int pos0, double log_base, uint16_t* __restrict__ kc,
    uint16_t* __restrict__ vc, int32_t* __restrict__ seg_len, int per_head) {
  const int b = blockIdx.x;
  const int half = D / 2;
  const long long len_base = per_head ? ((long long)b * n_seg + seg) * n_kv_heads
                                      : (long long)b * n_seg + seg;
  const long long items = (long long)n_new * n_kv_heads * half;
  for (long long it = threadIdx.x; it < items; it += blockDim.x) {
    const int i = (int)(it % half);
    const int g = (int)((it / half) % n_kv_heads);
    const int t = (int)(it / ((long long)half * n_kv_heads));
    const int len = min(max(seg_len[len_base + (per_head ? g : 0)], 0), k_t);
    if (len + t >= k_t) continue;                          // no room left in this head's segment
    const long long src = (((long long)b * n_new + t) * n_kv_heads + g) * D;
    const long long dst = ((((long long)b * n_seg + seg) * n_kv_heads + g) * k_t + len + t) * D;
    const uint16_t a1 = k_new[src + i], a2 = k_new[src + i + half];
    if (pos0 >= 0) {
      const double theta = exp(-2.0 * (double)i / (double)D * log_base);
      double sn, cs;
      sincos((double)(pos0 + t) * theta, &sn, &cs);
      const float x1 = bf16_bits_to_f32(a1), x2 = bf16_bits_to_f32(a2);
      kc[dst + i] = (uint16_t)f32_to_bf16_bits((float)(x1 * cs - x2 * sn));
      kc[dst + i + half] = (uint16_t)f32_to_bf16_bits((float)(x2 * cs + x1 * sn));
    } else {
      kc[dst + i] = a1; kc[dst + i + half] = a2;
    }
    vc[dst + i] = v_new[src + i]; vc[dst + i + half] = v_new[src + i + half];
  }
  __syncthreads();                                         // every length has been read
  const int n_len = per_head ? n_kv_heads : 1;
  for (int g = threadIdx.x; g < n_len; g += blockDim.x) {
    const int len = min(max(seg_len[len_base + g], 0), k_t);
    seg_len[len_base + g] = len + min(n_new, k_t - len);
  }
}

int pc_launch_kv_append(const void* k_new, const void* v_new, int batch, int n_new, int n_seg,
                        int seg, int k_t, int n_kv_heads, int head_dim, int pos0, float base,
                        void* kc, void* vc, int32_t* seg_len, int seg_len_per_head, hipStream_t st) {
  PcProfScope prof(PC_KERNEL_KV_APPEND, st);
  hipLaunchKernelGGL(kv_append_kernel, dim3(batch), dim3(256), 0, st, (const uint16_t*)k_new,
                     (const uint16_t*)v_new, n_new, n_seg, seg, k_t, n_kv_heads, head_dim, pos0,
                     log((double)(pos0 >= 0 ? base : 2.0f)), (uint16_t*)kc, (uint16_t*)vc, seg_len,
                     seg_len_per_head);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

template <int D>
static int launch_decode_d(const PcDecodeArgs& a, int batch, int nq_pad, hipStream_t st) {
  const long long blocks = (long long)batch * a.n_kv_heads * a.parts_grid;
  if (blocks == 0) return PC_OK;
  if (blocks > 0x7fffffffLL) return PC_ERR_SHAPE;
  dim3 grid((unsigned)blocks), block(PC_DEC_WAVES * PC_WAVE);
  PcProfScope prof(PC_KERNEL_DECODE, st);
  if (nq_pad == 4) hipLaunchKernelGGL((decode_attn_kernel<D, 4>), grid, block, 0, st, a);
  else if (nq_pad == 8) hipLaunchKernelGGL((decode_attn_kernel<D, 8>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((decode_attn_kernel<D, 16>), grid, block, 0, st, a);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

PcDecodeSplit pc_decode_split(int k_t, int n_seg, long long n_bg) {
  // Workgroups (partials) per (sequence, KV head) group.  Measured at the decode config (128
  // groups of 32 x 2048 keys, bf16): 256 workgroups, one per CU, each streaming half of a
  // group's keys, reach 89 % of the HBM peak; 512 and 1024
  // workgroups (the same bytes in shorter runs, two workgroups per CU at a time) 81 %.  Fewer
  // concurrent streams with longer runs are kinder to the memory system than more occupancy, and
  // a launch of exactly one round has no ragged end.  So: the number of parts that minimises
  // rounds / parts (the time of the slowest CU in units of one group's work), each round count
  // weighted by the bandwidth fraction measured for it; every wavefront keeps at least one
  // 32-key block at full lengths; at most 64 parts (the merge reads them all).
  const int n_cu = 256;                                    // MI355X
  const long long blocks_full = (long long)n_seg * ((k_t + 31) / 32);
  const long long p_cap = blocks_full / PC_DEC_WAVES;
  const int p_max = (int)(p_cap < 1 ? 1 : (p_cap > 64 ? 64 : p_cap));
  PcDecodeSplit d;
  d.n_parts = n_seg > 0 ? 1 : 0;                           // no segments: no launch, no partial
  if (n_seg <= 0) return d;
  double best = 0.0;
  for (int p = 1; p <= p_max; ++p) {
    const long long rounds = (n_bg * p + n_cu - 1) / n_cu;
    const double cost = (double)rounds / p / (rounds == 1 ? 0.89 : 0.81);
    if (p == 1 || cost < best * (1.0 - 1e-9)) { best = cost; d.n_parts = p; }
  }
  return d;
}

int pc_launch_decode(const void* q_rot, const void* kc, const void* vc, const int32_t* seg_len,
                     int seg_len_per_head, int batch, int n_q, int n_seg, int k_t, int n_q_heads, int n_kv_heads,
                     int head_dim, float scale, float* part_o, float* part_lse, int n_parts,
                     int part0, hipStream_t st) {
  PcDecodeArgs a;
  a.part0 = part0;
  a.q = (const uint16_t*)q_rot; a.kc = (const uint16_t*)kc; a.vc = (const uint16_t*)vc;
  a.seg_len = seg_len; a.seg_len_per_head = seg_len_per_head; a.part_o = part_o; a.part_lse = part_lse;
  a.n_q = n_q; a.n_seg = n_seg; a.k_t = k_t; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads;
  a.parts_grid = pc_decode_split(k_t, n_seg, (long long)batch * n_kv_heads).n_parts;
  a.n_parts = n_parts;
  a.scale_log2 = scale * PC_DEC_LOG2E;
  const int cols = n_q * (n_q_heads / n_kv_heads);
  const int nq_pad = cols <= 4 ? 4 : (cols <= 8 ? 8 : 16);
  return head_dim == 128 ? launch_decode_d<128>(a, batch, nq_pad, st)
                         : launch_decode_d<64>(a, batch, nq_pad, st);
}

int pc_launch_merge(const float* part_o, const float* part_lse, const void* q_rot,
                    const void* k_self, const void* v_self, void* out, float* lse_out, int batch,
                    int n_q, int n_q_heads, int n_kv_heads, int head_dim, int n_parts, float scale,
                    hipStream_t st) {
  PcMergeArgs a;
  a.part_o = part_o; a.part_lse = part_lse; a.q = (const uint16_t*)q_rot;
  a.k_self = (const uint16_t*)k_self; a.v_self = (const uint16_t*)v_self;
  a.out = (uint16_t*)out; a.lse_out = lse_out;
  a.n_q = n_q; a.n_q_heads = n_q_heads; a.n_kv_heads = n_kv_heads; a.n_parts = n_parts;
  a.scale = scale;
  const long long blocks = (long long)batch * n_q * n_q_heads;
  if (blocks == 0) return PC_OK;
  if (blocks > 0x7fffffffLL) return PC_ERR_SHAPE;
  PcProfScope prof(PC_KERNEL_MERGE, st);
  if (head_dim == 128) hipLaunchKernelGGL(merge_kernel<128>, dim3((unsigned)blocks), dim3(128), 0, st, a);
  else hipLaunchKernelGGL(merge_kernel<64>, dim3((unsigned)blocks), dim3(64), 0, st, a);
  PC_LAUNCH_CHECK();
  return PC_OK;
}
