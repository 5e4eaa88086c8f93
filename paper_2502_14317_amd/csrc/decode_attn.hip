// Parallel (global) attention for few query rows: the HBM-bound split-KV kernel and the exact
// logsumexp merge (Eq. 9-11: one softmax over [K^1 .. K^S, K^q], evaluated as independent
// per-piece softmaxes that are merged by LSE = log sum exp(lse_p), o = sum exp(lse_p - LSE) o_p).
//
// Every K/V byte is read exactly once, so the kernel is bound by HBM bandwidth.  Design:
//   * one workgroup (4 wavefronts) per (sequence, KV head, segment, split); a wavefront owns a
//     contiguous run of keys and streams them 32 at a time with 16-byte loads, the next 32
//     keys already in flight while the current ones are used;
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
  int n_q, n_seg, k_t, n_q_heads, n_kv_heads, n_split, keys_per_wg, n_parts;
  int seg_per_wg;         // consecutive segments streamed by one workgroup (1 if n_split > 1)
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

  const int n_sgroups = (a.n_seg + a.seg_per_wg - 1) / a.seg_per_wg;
  int bid = blockIdx.x;
  const int split = bid % a.n_split; bid /= a.n_split;
  const int sg = bid % n_sgroups;    bid /= n_sgroups;
  const int g = bid % a.n_kv_heads;  bid /= a.n_kv_heads;
  const int b = bid;
  const int s_first = sg * a.seg_per_wg, s_last = min(a.n_seg, s_first + a.seg_per_wg);

  // A wavefront streams its quarter of the workgroup's key range of every segment of the group,
  // one segment after the other; the running softmax carries over (same query columns, same KV
  // head), so a workgroup leaves one partial for all its segments.  A cursor names the next
  // 32-key block: segment, first key, the segment's base pointers, length and range end.
  struct Cursor { int s, key0, len, w_end; const uint16_t* k; const uint16_t* v; bool valid; };
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // wavefront-uniform: cursors live in scalar registers
  const int per_wave = a.keys_per_wg / PC_DEC_WAVES;      // multiple of PC_DEC_ITER_KEYS
  auto seek = [&](int s) {                                 // first segment >= s with keys for this wavefront
    Cursor c; c.valid = false; c.s = s; c.key0 = 0; c.len = 0; c.w_end = 0; c.k = nullptr; c.v = nullptr;
    for (; s < s_last; ++s) {
      const int len_idx = a.seg_len_per_head ? (b * a.n_seg + s) * a.n_kv_heads + g : b * a.n_seg + s;
      const int len = a.seg_len ? min(max(a.seg_len[len_idx], 0), a.k_t) : a.k_t;
      const int wg_begin = split * a.keys_per_wg;
      const int wg_end = min(len, wg_begin + a.keys_per_wg);
      const int w_begin = wg_begin + wave_u * per_wave;
      const int w_end = min(wg_end, w_begin + per_wave);
      if (w_begin < w_end) {
        const long long seg_base = ((((long long)b * a.n_seg + s) * a.n_kv_heads + g) * a.k_t) * D;
        c.valid = true; c.s = s; c.key0 = w_begin; c.len = len; c.w_end = w_end;
        c.k = a.kc + seg_base; c.v = a.vc + seg_base;
        break;
      }
    }
    return c;
  };
  auto next = [&](const Cursor& c) {
    Cursor n = c;
    n.key0 += PC_DEC_ITER_KEYS;
    if (n.key0 >= c.w_end) n = seek(c.s + 1);
    return n;
  };

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
      const int row = min(c.key0 + 16 * bi + c16, c.len - 1);
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks)
        kbuf[buf][bi][ks] = pc_load_once((const uint4*)(c.k + (long long)row * D + 32 * ks + 8 * kk));
    }
#pragma unroll
    for (int i = 0; i < VLOADS; ++i) {
      const int row = min(c.key0 + RPI * i + v_row, c.len - 1);
      vbuf[buf][i] = pc_load_once((const uint4*)(c.v + (long long)row * D + 8 * v_piece));
    }
  };

  auto consume = [&](int buf, const Cursor& cur) {
    const int key0 = cur.key0, w_end = cur.w_end;
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

  Cursor cur = seek(s_first);
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
  const int part = a.part0 + sg * a.n_split + split;
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
    const long long row = (((long long)b * a.n_parts + part) * a.n_q + t) * a.n_q_heads + g * G + hg;
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
// Rotate the query rows of the global attention at positions pos0 + t (fp64 angles).
__global__ void rope_q_kernel(const uint16_t* __restrict__ q, uint16_t* __restrict__ q_rot,
                              long long n_pairs, int n_q, int n_heads, int D, int pos0,
                              double log_base) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pairs) return;
  const int half = D / 2;
  const int i = (int)(idx % half);
  const long long row = idx / half;                       // (b, t, h)
  const int t = (int)((row / n_heads) % n_q);
  const double theta = exp(-2.0 * (double)i / (double)D * log_base);
  double sn, cs;
  sincos((double)(pos0 + t) * theta, &sn, &cs);
  const float x1 = bf16_bits_to_f32(q[row * D + i]), x2 = bf16_bits_to_f32(q[row * D + i + half]);
  q_rot[row * D + i] = (uint16_t)f32_to_bf16_bits((float)(x1 * cs - x2 * sn));
  q_rot[row * D + i + half] = (uint16_t)f32_to_bf16_bits((float)(x2 * cs + x1 * sn));
}

int pc_launch_rope_q(const void* q, void* q_rot, long long n_rows, int n_q, int n_heads, int D,
                     int pos0, float base, hipStream_t st) {
  const long long n_pairs = n_rows * (D / 2);
  if (n_pairs == 0) return PC_OK;
  PcProfScope prof(PC_KERNEL_ROPE_Q, st);
  hipLaunchKernelGGL(rope_q_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, st,
                     (const uint16_t*)q, (uint16_t*)q_rot, n_pairs, n_q, n_heads, D, pos0,
                     log((double)base));
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
  const long long blocks = (long long)batch * a.n_kv_heads * ((a.n_seg + a.seg_per_wg - 1) / a.seg_per_wg) * a.n_split;
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
  // A workgroup streams up to 2048 keys of one (sequence, KV head, segment): the longer its run,
  // the smaller the share of its start-up and of its partial result (at the decode config 256 /
  // 1024 / 2048 keys per workgroup reach 68 / 75 / 80.5 % of the HBM peak).  Short segments use
  // one workgroup each, and the runs are halved while the launch would have fewer than four
  // workgroups per CU of a 256-CU part.  Where a segment fits one workgroup, a workgroup takes
  // one, two or four consecutive segments under one running softmax (one partial for all of
  // them): at the decode config 1 / 2 / 4 segments per workgroup reach 76 / 80 / 83 % on one machine.
  PcDecodeSplit d;
  const long long n_groups = n_bg * n_seg;
  int kpw = 2048;
  while (kpw > PC_DEC_WAVES * PC_DEC_ITER_KEYS && kpw / 2 >= k_t) kpw /= 2;
  while (kpw > PC_DEC_WAVES * PC_DEC_ITER_KEYS && n_groups * ((k_t + kpw - 1) / kpw) < 1024) kpw /= 2;
  d.keys_per_wg = kpw;
  d.n_split = (k_t + kpw - 1) / kpw;
  d.seg_per_wg = 1;
  if (d.n_split == 1) {
    // Pick 1, 2 or 4 segments per workgroup by a makespan estimate in units of one segment: the
    // full workgroups run in rounds of 512 (resident workgroups of a 256-CU part, 2 per CU),
    // the workgroups that take the n_seg % spw left-over segments of every (sequence, KV head)
    // in rounds after them; each term is divided by the bandwidth fraction measured at that
    // run length.  A ragged last round of full workgroups costs a whole round, a round of
    // left-overs only its own length, so e.g. 32 + 1 segments still run four to a workgroup.
    const double eff[3] = {0.76, 0.80, 0.83};
    double best = 0.0;
    for (int i = 0; i < 3; ++i) {
      const int spw = 1 << i;
      const long long n_full = n_bg * (n_seg / spw);
      const int rem = n_seg % spw;
      const double cost = (double)((n_full + 511) / 512) * spw / eff[i] +
                          (rem ? (double)((n_bg + 511) / 512) * rem / eff[rem > 1] : 0.0);
      if (i == 0 || cost < best) { best = cost; d.seg_per_wg = spw; }
    }
  }
  d.n_parts = ((n_seg + d.seg_per_wg - 1) / d.seg_per_wg) * d.n_split;
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
  const PcDecodeSplit sp = pc_decode_split(k_t, n_seg, (long long)batch * n_kv_heads);
  a.keys_per_wg = sp.keys_per_wg; a.n_split = sp.n_split; a.seg_per_wg = sp.seg_per_wg;
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
