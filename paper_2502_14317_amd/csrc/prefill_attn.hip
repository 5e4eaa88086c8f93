// Chunk-batched causal local attention (Eq. 1-2) with chunk-local RoPE, for gfx950.
//
// Three kernels:
//   rope_table_kernel   cos/sin of position * theta_i, computed in fp64, stored fp32
//   kv_prepass_kernel   K -> rotated K (bf16, the KV cache later steps gather from);
//                       V -> V^T [seq, H_kv, D, Lp] so that the P.V product finds its
//                       contraction index (keys) contiguous, as the MFMA operand layout needs
//   flash_fwd_kernel    online-softmax attention on 32x32x16 bf16 MFMA
//
// flash_fwd_kernel computes S^T = K Q^T and O^T = V^T P^T.  In the MFMA result layout a lane
// then owns ONE query (column) and holds many keys (rows) in its registers, so the row max
// and row sum are in-register reductions plus one exchange between lane l and l+32, the
// rescale factor of O is a per-lane scalar, and P^T in registers is already the B operand
// of the second product (after rounding to bf16).  K rows are fed to the first MFMA in a
// permuted order (bits 2 and 3 of the row index swapped) so that the 8 probabilities a lane
// holds for one k-step belong to 8 consecutive keys, i.e. one 16-byte LDS read of V^T.
//
// Workgroup: 8 wavefronts x 32 query rows = 256 rows of one (sequence, query head); key tiles
// of 64 staged in LDS (K: [64][D], V^T: [D][64], padded rows, double buffered).  Two
// wavefronts share a SIMD, so one wavefront's softmax (vector ALU, exp) overlaps the other's
// MFMA.  Causal structure: a Q tile only visits key tiles up to its diagonal, the mask is
// applied on diagonal tiles only, and row blocks are paired (i, 7 - i) per SIMD for balance.
// Workgroups are ordered so that one XCD works on one (sequence, KV head) at a time (its K/V
// stay in that XCD's L2) and takes the long (late) Q tiles first.
#include "pc_common.h"
#include <math.h>

#define PC_FA_WAVES 8
#define PC_FA_THREADS (PC_FA_WAVES * PC_WAVE)
#define PC_FA_BM (PC_FA_WAVES * 32)
#define PC_FA_BN 64
#define PC_LOG2E 1.4426950408889634f
#define PC_LN2 0.6931471805599453f

// ------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float2* __restrict__ table, int n_pos, int D, double log_base) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int half = D / 2;
  if (idx >= n_pos * half) return;
  const int p = idx / half, i = idx % half;
  const double theta = exp(-2.0 * (double)i / (double)D * log_base);
  double sn, cs;
  sincos((double)p * theta, &sn, &cs);
  table[idx] = make_float2((float)cs, (float)sn);
}

int pc_launch_rope_table(float2* table, int n_pos, int head_dim, float base, hipStream_t st) {
  const int n = n_pos * (head_dim / 2);
  PcProfScope prof(PC_KERNEL_ROPE_TABLE, st);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, table, n_pos,
                     head_dim, log((double)base));
  PC_LAUNCH_CHECK();
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
// One workgroup per (sequence, KV head, 64-row tile).
template <int D>
__global__ __launch_bounds__(256) void kv_prepass_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const float2* __restrict__ table, uint16_t* __restrict__ k_rope, uint16_t* __restrict__ v_t,
    int L, int Lp, int n_kv_heads) {
  constexpr int HALF = D / 2;
  constexpr int VSTRIDE = D + 2;                  // bf16 elements, odd number of dwords
  __shared__ uint16_t v_lds[64 * VSTRIDE];
  const int seq = blockIdx.x, g = blockIdx.y, tile = blockIdx.z;
  const int row0 = tile * 64;
  const long long seq_base = (long long)seq * L;

  // ---- K: rotate pairs (i, i + D/2); a thread handles 8 consecutive i of one row
  constexpr int K_ITEMS = 64 * (HALF / 8);
  for (int it = threadIdx.x; k != nullptr && it < K_ITEMS; it += 256) {
    const int r = it / (HALF / 8), i0 = (it % (HALF / 8)) * 8;
    const int row = row0 + r;
    if (row < L) {
      const long long off = ((seq_base + row) * n_kv_heads + g) * D;
      const uint4 a = *(const uint4*)(k + off + i0);
      const uint4 b = *(const uint4*)(k + off + HALF + i0);
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
      uint32_t ra[4], rb[4];
      const float2* cs = table + (long long)row * HALF + i0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float2 c0 = cs[2 * e], c1 = cs[2 * e + 1];
        const float x1l = bf16_lo_to_f32(aw[e]), x1h = bf16_hi_to_f32(aw[e]);
        const float x2l = bf16_lo_to_f32(bw[e]), x2h = bf16_hi_to_f32(bw[e]);
        ra[e] = pack_bf16x2(x1l * c0.x - x2l * c0.y, x1h * c1.x - x2h * c1.y);
        rb[e] = pack_bf16x2(x2l * c0.x + x1l * c0.y, x2h * c1.x + x1h * c1.y);
      }
      *(uint4*)(k_rope + off + i0) = make_uint4(ra[0], ra[1], ra[2], ra[3]);
      *(uint4*)(k_rope + off + HALF + i0) = make_uint4(rb[0], rb[1], rb[2], rb[3]);
    }
  }

  // ---- V: 64 x D tile -> LDS -> D x 64 tile of V^T (zero beyond row L)
  constexpr int V_ITEMS = 64 * (D / 8);
  for (int it = threadIdx.x; it < V_ITEMS; it += 256) {
    const int r = it / (D / 8), c8 = (it % (D / 8)) * 8;
    const int row = row0 + r;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (row < L) x = *(const uint4*)(v + ((seq_base + row) * n_kv_heads + g) * D + c8);
    uint32_t* dst = (uint32_t*)(v_lds + r * VSTRIDE + c8);   // 4-byte aligned: VSTRIDE, c8 even
    dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
  }
  __syncthreads();
  constexpr int T_ITEMS = D * 8;                  // (d, group of 8 keys)
  for (int it = threadIdx.x; it < T_ITEMS; it += 256) {
    const int d = it / 8, r8 = (it % 8) * 8;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t lo = v_lds[(r8 + 2 * e) * VSTRIDE + d];
      const uint32_t hi = v_lds[(r8 + 2 * e + 1) * VSTRIDE + d];
      w[e] = lo | (hi << 16);
    }
    const long long off = (((long long)seq * n_kv_heads + g) * D + d) * Lp + row0 + r8;
    *(uint4*)(v_t + off) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

int pc_launch_kv_prepass(const void* k, const void* v, const float2* table, void* k_rope,
                         void* v_t, int n_seq, int L, int Lp, int n_kv_heads, int head_dim,
                         hipStream_t st) {
  dim3 grid(n_seq, n_kv_heads, Lp / 64), block(256);
  PcProfScope prof(PC_KERNEL_KV_PREPASS, st);
  if (head_dim == 128)
    hipLaunchKernelGGL(kv_prepass_kernel<128>, grid, block, 0, st, (const uint16_t*)k,
                       (const uint16_t*)v, table, (uint16_t*)k_rope, (uint16_t*)v_t, L, Lp,
                       n_kv_heads);
  else
    hipLaunchKernelGGL(kv_prepass_kernel<64>, grid, block, 0, st, (const uint16_t*)k,
                       (const uint16_t*)v, table, (uint16_t*)k_rope, (uint16_t*)v_t, L, Lp,
                       n_kv_heads);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
template <int D>
struct FlashSmem {
  static constexpr int KSTRIDE = D + 8;            // bf16 elements per K row (16 B pad)
  static constexpr int VSTRIDE = PC_FA_BN + 8;     // bf16 elements per V^T row (16 B pad)
  static constexpr int K_ELEMS = PC_FA_BN * KSTRIDE;
  static constexpr int V_ELEMS = D * VSTRIDE;
  static constexpr int BYTES = 2 * (K_ELEMS + V_ELEMS) * 2;
};

// row index of the first MFMA's A operand -> key within a 32-key block (swap bits 2 and 3)
__device__ __forceinline__ int pc_key_of_row(int m) {
  return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1);
}

template <int D, bool ROPE_Q, bool PARTIAL>
__global__ __launch_bounds__(PC_FA_THREADS) void flash_fwd_kernel(PcFlashArgs a) {
  using SM = FlashSmem<D>;
  constexpr int KS = D / 16;        // k-steps of the first product (over head_dim)
  constexpr int DB = D / 32;        // 32-row blocks of O^T (over head_dim)
  constexpr int HALF = D / 2;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  auto k_lds = [&](int buf) { return smem + buf * SM::K_ELEMS; };
  auto v_lds = [&](int buf) { return smem + 2 * SM::K_ELEMS + buf * SM::V_ELEMS; };

  // ---- which (sequence, head, Q tile): one XCD (blockIdx % 8) works through whole
  //      (sequence, KV head) groups, heavy Q tiles first, the group's query heads adjacent
  const int G = a.n_q_heads / a.n_kv_heads;
  const int n_qt = (a.n_rows + PC_FA_BM - 1) / PC_FA_BM;
  const int per_group = G * n_qt * a.n_parts_grid;
  const int xcd = blockIdx.x % 8, j = blockIdx.x / 8;
  const int cg = (j / per_group) * 8 + xcd;
  if (cg >= a.n_seq * a.n_kv_heads) return;
  int within = j % per_group;
  const int part = within % a.n_parts_grid; within /= a.n_parts_grid;
  const int qt = n_qt - 1 - within / G;
  const int hg = within % G;
  const int seq = cg / a.n_kv_heads, g = cg % a.n_kv_heads;
  const int h = g * G + hg;

  const int tid = threadIdx.x, lane = tid % PC_WAVE, wave = tid / PC_WAVE;
  const int hf = lane / 32, n = lane % 32;
  const int rb = wave < 4 ? wave : 11 - wave;     // row blocks (i, 7 - i) share a SIMD
  const int row0_wg = qt * PC_FA_BM;
  const int row0 = row0_wg + 32 * rb;             // first query row of this wavefront
  const int my_row = row0 + n;
  const int ld_row = min(my_row, a.n_rows - 1);

  // ---- keys of this workgroup: [0, key_end) of the part
  const int key_begin = 0;
  const int n_valid = a.part_len ? min(max(a.part_len[seq * a.n_parts_grid + part], 0), a.n_keys)
                                 : a.n_keys;
  int key_end = n_valid;
  if (a.causal_offset < PC_NO_CAUSAL) key_end = min(key_end, row0_wg + PC_FA_BM + a.causal_offset);
  const int n_tiles = (key_end - key_begin + PC_FA_BN - 1) / PC_FA_BN;

  const uint16_t* kbase = (const uint16_t*)a.k + seq * a.k_seq_stride + part * a.k_part_stride +
                          g * a.k_head_stride;
  const uint16_t* vtbase = (const uint16_t*)a.v_t + seq * a.vt_seq_stride +
                           part * a.vt_part_stride + g * a.vt_head_stride;

  // ---- Q^T as B operand: lane holds query n, d = 16*ks + 8*hf .. +7
  bf16x8 bq[KS];
  {
    const uint16_t* qrow = (const uint16_t*)a.q + (((long long)seq * a.n_rows + ld_row) * a.n_q_heads + h) * D;
    if (ROPE_Q) {
      const float2* cs = a.table + (long long)(a.q_pos0 + ld_row) * HALF;
#pragma unroll
      for (int ks = 0; ks < KS / 2; ++ks) {
        const int i0 = 16 * ks + 8 * hf;          // pair index of the first half
        const uint4 x1 = *(const uint4*)(qrow + i0);
        const uint4 x2 = *(const uint4*)(qrow + HALF + i0);
        const uint32_t aw[4] = {x1.x, x1.y, x1.z, x1.w}, bw[4] = {x2.x, x2.y, x2.z, x2.w};
        uint32_t ra[4], rbv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float2 c0 = cs[i0 + 2 * e], c1 = cs[i0 + 2 * e + 1];
          const float x1l = bf16_lo_to_f32(aw[e]), x1h = bf16_hi_to_f32(aw[e]);
          const float x2l = bf16_lo_to_f32(bw[e]), x2h = bf16_hi_to_f32(bw[e]);
          ra[e] = pack_bf16x2(x1l * c0.x - x2l * c0.y, x1h * c1.x - x2h * c1.y);
          rbv[e] = pack_bf16x2(x2l * c0.x + x1l * c0.y, x2h * c1.x + x1h * c1.y);
        }
        uint4 pa = make_uint4(ra[0], ra[1], ra[2], ra[3]), pb = make_uint4(rbv[0], rbv[1], rbv[2], rbv[3]);
        bq[ks] = *(bf16x8*)&pa;
        bq[ks + KS / 2] = *(bf16x8*)&pb;
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 x = *(const uint4*)(qrow + 16 * ks + 8 * hf);
        bq[ks] = *(bf16x8*)&x;
      }
    }
  }

  // ---- cooperative tile loads: global -> registers -> LDS (16-byte pieces)
  constexpr int K_LD = (PC_FA_BN * D / 8) / PC_FA_THREADS;
  constexpr int V_LD = (D * PC_FA_BN / 8) / PC_FA_THREADS;
  u32x4 kreg[K_LD], vreg[V_LD];
  int k_ld_row[K_LD], k_ld_c8[K_LD], v_ld_d[V_LD], v_ld_c8[V_LD];
#pragma unroll
  for (int i = 0; i < K_LD; ++i) {
    const int piece = tid + i * PC_FA_THREADS;
    k_ld_row[i] = piece / (D / 8);
    k_ld_c8[i] = (piece % (D / 8)) * 8;
  }
#pragma unroll
  for (int i = 0; i < V_LD; ++i) {
    const int piece = tid + i * PC_FA_THREADS;
    v_ld_d[i] = piece / (PC_FA_BN / 8);
    v_ld_c8[i] = (piece % (PC_FA_BN / 8)) * 8;
  }
#define PC_FA_LOAD_TILE(T)                                                                    \
  {                                                                                           \
    const int key0_ = key_begin + (T) * PC_FA_BN;                                             \
    _Pragma("unroll") for (int i = 0; i < K_LD; ++i) {                                        \
      const int key_ = min(key0_ + k_ld_row[i], a.n_keys - 1);                                \
      kreg[i] = *(const u32x4*)(kbase + (long long)key_ * a.k_row_stride + k_ld_c8[i]);       \
    }                                                                                         \
    _Pragma("unroll") for (int i = 0; i < V_LD; ++i)                                          \
      vreg[i] = *(const u32x4*)(vtbase + (long long)v_ld_d[i] * a.vt_d_stride + key0_ + v_ld_c8[i]); \
  }
#define PC_FA_STORE_TILE(BUF)                                                                 \
  {                                                                                           \
    _Pragma("unroll") for (int i = 0; i < K_LD; ++i)                                          \
      *(u32x4*)(k_lds(BUF) + k_ld_row[i] * SM::KSTRIDE + k_ld_c8[i]) = kreg[i];               \
    _Pragma("unroll") for (int i = 0; i < V_LD; ++i)                                          \
      *(u32x4*)(v_lds(BUF) + v_ld_d[i] * SM::VSTRIDE + v_ld_c8[i]) = vreg[i];                 \
  }

  floatx16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c_log2 = a.scale * PC_LOG2E;
  const int krow = pc_key_of_row(n);               // LDS row this lane feeds into MFMA row n
  const int max_key = min(my_row + a.causal_offset, n_valid - 1);     // last visible key of my query
  const int wave_max_key = min(row0 + 31 + a.causal_offset, n_valid - 1);
  const int wave_min_vis = min(row0 + a.causal_offset, n_valid - 1); // visible to every row of the wave

  if (n_tiles > 0) {
    PC_FA_LOAD_TILE(0);
    PC_FA_STORE_TILE(0);
  }
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int buf = t & 1;
    if (t + 1 < n_tiles) PC_FA_LOAD_TILE(t + 1);
    const int key0 = key_begin + t * PC_FA_BN;
    if (key0 <= wave_max_key) {
      // ---- S^T = K Q^T for two 32-key blocks
      floatx16 s_acc[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[kb][r] = 0.f;
        const uint16_t* kp = k_lds(buf) + (32 * kb + krow) * SM::KSTRIDE + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 ka = *(const bf16x8*)(kp + 16 * ks);
          s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, bq[ks], s_acc[kb], 0, 0, 0);
        }
      }
      // register r of block kb at lane half hf is key key0 + 32kb + 16(r/8) + 8hf + (r%8)
      if (key0 + PC_FA_BN - 1 > wave_min_vis) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + 32 * kb + 16 * (r / 8) + 8 * hf + (r % 8);
            if (key > max_key) s_acc[kb][r] = -INFINITY;
          }
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s_acc[kb][r]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32)) * c_log2;
      // Lazy rescale: the reference m_run only moves when some row's tile maximum exceeds it by
      // more than 2^8; until then p = exp2(s - m_run) <= 256 and O, l stay in the old scale.
      if (__any(tmax > m_run + 8.0f)) {
        const float m_new = fmaxf(m_run, tmax);
        const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
      }
      // rows with no visible key yet keep m = -inf; use 0 as the reference to avoid inf - inf
      const float neg_ref = (m_run == -INFINITY) ? 0.f : -m_run;
      float psum = 0.f;
      bf16x8 pb[4];                                // B operands: [kb][k-step] -> index 2kb + ts
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
          uint32_t pk[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][8 * ts + 2 * e], c_log2, neg_ref));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][8 * ts + 2 * e + 1], c_log2, neg_ref));
            psum += p0 + p1;
            pk[e] = pack_bf16x2(p0, p1);
          }
          uint4 pv = make_uint4(pk[0], pk[1], pk[2], pk[3]);
          pb[2 * kb + ts] = *(bf16x8*)&pv;
        }
      l_run += psum;
      // ---- O^T += V^T P^T
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const uint16_t* vp = v_lds(buf) + (32 * db + n) * SM::VSTRIDE + 8 * hf;
#pragma unroll
        for (int ksp = 0; ksp < 4; ++ksp) {
          const bf16x8 va = *(const bf16x8*)(vp + 16 * ksp);
          o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[ksp], o_acc[db], 0, 0, 0);
        }
      }
    }
    if (t + 1 < n_tiles) PC_FA_STORE_TILE(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane halves hold disjoint key subsets of the same query
  l_run += __shfl_xor(l_run, 32);
  const float inv_l = l_run > 0.f ? 1.f / l_run : 0.f;
  const float lse = l_run > 0.f ? m_run * PC_LN2 + logf(l_run) : -INFINITY;
  if (my_row < a.n_rows) {
    if (PARTIAL) {
      const long long prow = ((((long long)seq * a.n_parts_total + a.part0 + part) * a.n_rows) + my_row) * a.n_q_heads + h;
      float* po = a.part_o + prow * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float4 x = make_float4(o_acc[db][4 * i] * inv_l, o_acc[db][4 * i + 1] * inv_l,
                                 o_acc[db][4 * i + 2] * inv_l, o_acc[db][4 * i + 3] * inv_l);
          *(float4*)(po + 32 * db + 8 * i + 4 * hf) = x;
        }
      if (hf == 0) a.part_lse[prow] = lse;
    } else {
      uint16_t* orow = (uint16_t*)a.o + (((long long)seq * a.n_rows + my_row) * a.n_q_heads + h) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          uint2 x;
          x.x = pack_bf16x2(o_acc[db][4 * i] * inv_l, o_acc[db][4 * i + 1] * inv_l);
          x.y = pack_bf16x2(o_acc[db][4 * i + 2] * inv_l, o_acc[db][4 * i + 3] * inv_l);
          *(uint2*)(orow + 32 * db + 8 * i + 4 * hf) = x;
        }
      if (hf == 0 && a.lse) a.lse[((long long)seq * a.n_q_heads + h) * a.n_rows + my_row] = lse;
    }
  }
}

template <int D, bool ROPE_Q, bool PARTIAL>
static int launch_flash_t(const PcFlashArgs& a, hipStream_t st) {
  using SM = FlashSmem<D>;
  auto kern = flash_fwd_kernel<D, ROPE_Q, PARTIAL>;
  PC_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 SM::BYTES));
  const int G = a.n_q_heads / a.n_kv_heads;
  const int n_qt = (a.n_rows + PC_FA_BM - 1) / PC_FA_BM;
  const long long per_group = (long long)G * n_qt * a.n_parts_grid;
  const long long groups = (long long)a.n_seq * a.n_kv_heads;
  const long long blocks = (groups + 7) / 8 * per_group * 8;
  if (blocks == 0) return PC_OK;
  if (blocks > 0x7fffffffLL) return PC_ERR_SHAPE;
  PcProfScope prof(PC_KERNEL_FLASH, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(PC_FA_THREADS), SM::BYTES, st, a);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

int pc_launch_flash(const PcFlashArgs& a, hipStream_t st) {
  const bool rope = a.table != nullptr, partial = a.part_o != nullptr;
  if (a.head_dim == 128) {
    if (rope) return partial ? launch_flash_t<128, true, true>(a, st) : launch_flash_t<128, true, false>(a, st);
    return partial ? launch_flash_t<128, false, true>(a, st) : launch_flash_t<128, false, false>(a, st);
  }
  if (rope) return partial ? launch_flash_t<64, true, true>(a, st) : launch_flash_t<64, true, false>(a, st);
  return partial ? launch_flash_t<64, false, true>(a, st) : launch_flash_t<64, false, false>(a, st);
}
