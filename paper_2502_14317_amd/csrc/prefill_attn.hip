// Chunk-batched causal local attention (Eq. 1-2) with chunk-local RoPE, for gfx950.
//
// Three kernels:
//   rope_table_kernel   cos/sin of position * theta_i, computed in fp64, stored fp32
//   kv_prepass_kernel   K -> rotated K (bf16, the KV cache later steps gather from) and K tile
//                       images; V -> V^T tile images (the layouts the tile kernel copies to LDS)
//   flash_fwd_kernel    online-softmax attention on 32x32x16 bf16 MFMA
//
// flash_fwd_kernel computes S^T = K Q^T and O^T = V^T P^T.  In the MFMA result layout a lane
// then owns ONE query (column) and holds many keys (rows) in its registers, so the row max
// and row sum are in-register reductions plus one exchange between lane l and l+32, the
// rescale factor of O is a per-lane scalar, and P^T in registers is already the B operand
// of the second product (after rounding to bf16).  K rows are fed to the first MFMA in a
// permuted order (bits 2 and 3 of the row index swapped) so that the 8 probabilities a lane
// holds for one k-step belong to 8 consecutive keys, i.e. one 16-byte granule of V^T.
//
// Workgroup: 4 wavefronts x 32 query rows = 128 rows of one (sequence, query head), one
// wavefront per SIMD, at most 256 registers and 80 KiB of LDS, so that two workgroups share a
// CU: the second wavefront of every SIMD belongs to an independent workgroup and fills the
// issue slots the first one leaves (a single wavefront cannot keep the matrix pipe busy: its
// own vector-ALU, LDS and barrier time is exposed).  Key tiles of 64 are copied into LDS by
// direct global->LDS loads (K double-, V^T triple-buffered).  Causal structure: a Q tile only
// visits key tiles up to its diagonal and the mask is applied on diagonal tiles only.
// Workgroups are ordered so that one XCD works on one (sequence, KV head) at a time (its K/V
// stay in that XCD's L2) and takes the long (late) Q tiles first.
#include "pc_common.h"
#include <math.h>
#include <type_traits>

#define PC_FA_NB 1                   // 32-row blocks per wavefront
#define PC_FA_WAVES 4                // wavefronts per workgroup (one per SIMD); two workgroups share a CU
#define PC_FA_THREADS (PC_FA_WAVES * PC_WAVE)
#define PC_FA_BM (PC_FA_WAVES * 32 * PC_FA_NB)   // query rows per workgroup
#define PC_FA_BN 64                  // keys per tile
#define PC_LOG2E 1.4426950408889634f
// orders a wavefront's own LDS writes before its own later LDS reads (no other wavefront involved)
#define PC_FA_WAVE_LDS_SYNC()                                \
  do {                                                       \
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   \
    __builtin_amdgcn_wave_barrier();                         \
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");   \
  } while (0)
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
// Tile images.  flash_fwd_kernel copies whole 64-key tiles of K and V^T into LDS with contiguous
// 1 KiB loads, so this pre-pass writes both in the exact byte order the MFMA operand reads want,
// 16-byte granules (8 bf16) stored granule-column by granule-column:
//   K image   [16 * D / 128 .. i.e. D/8 columns][64 keys]:   granule (c, r) = K[key r][8c .. 8c+7]
//   V^T image [8 columns][D rows]:                           granule (c, d) = V[keys 8c .. 8c+7][d]
// The 16 lanes an LDS read serves together then touch 256 consecutive bytes (no bank conflict,
// no swizzle), and every operand address is one per-lane base plus an immediate offset.
// Images of one (sequence, KV head) are consecutive: [n_seq][n_kv_heads][Lp / 64][64 * D].
// Keys past the end of a sequence are zero in both images.
// One workgroup per (sequence, KV head, 64-row tile).
template <int D>
__global__ __launch_bounds__(256) void kv_prepass_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const float2* __restrict__ table, uint16_t* __restrict__ k_rope, uint16_t* __restrict__ k_img,
    uint16_t* __restrict__ v_img, int L, int Lp, int n_kv_heads) {
  constexpr int HALF = D / 2;
  constexpr int VSTRIDE = D + 2;                  // bf16 elements, odd number of dwords
  __shared__ uint16_t v_lds[64 * VSTRIDE];
  const int seq = blockIdx.x, g = blockIdx.y, tile = blockIdx.z;
  const int row0 = tile * 64;
  const long long seq_base = (long long)seq * L;
  const long long img = (((long long)seq * n_kv_heads + g) * (Lp / 64) + tile) * (64 * D);

  // ---- K: rotate pairs (i, i + D/2) when a table is given; a thread handles 8 consecutive i of one row
  constexpr int K_ITEMS = 64 * (HALF / 8);
  for (int it = threadIdx.x; k != nullptr && it < K_ITEMS; it += 256) {
    const int r = it / (HALF / 8), i0 = (it % (HALF / 8)) * 8;
    const int row = row0 + r;
    uint4 oa = make_uint4(0, 0, 0, 0), ob = make_uint4(0, 0, 0, 0);
    if (row < L) {
      const long long off = ((seq_base + row) * n_kv_heads + g) * D;
      const uint4 a = pc_load_once((const uint4*)(k + off + i0));
      const uint4 b = pc_load_once((const uint4*)(k + off + HALF + i0));
      if (table != nullptr) {
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
        oa = make_uint4(ra[0], ra[1], ra[2], ra[3]);
        ob = make_uint4(rb[0], rb[1], rb[2], rb[3]);
      } else {
        oa = a; ob = b;
      }
      if (k_rope != nullptr) {
        pc_store_once((uint4*)(k_rope + off + i0), oa);
        pc_store_once((uint4*)(k_rope + off + HALF + i0), ob);
      }
    }
    if (k_img != nullptr) {
      pc_store_once((uint4*)(k_img + img + ((i0 / 8) * 64 + r) * 8), oa);
      pc_store_once((uint4*)(k_img + img + (((HALF + i0) / 8) * 64 + r) * 8), ob);
    }
  }

  // ---- V: 64 x D tile -> LDS -> V^T image (zero beyond row L)
  constexpr int V_ITEMS = 64 * (D / 8);
  for (int it = threadIdx.x; it < V_ITEMS; it += 256) {
    const int r = it / (D / 8), c8 = (it % (D / 8)) * 8;
    const int row = row0 + r;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (row < L) x = pc_load_once((const uint4*)(v + ((seq_base + row) * n_kv_heads + g) * D + c8));
    uint32_t* dst = (uint32_t*)(v_lds + r * VSTRIDE + c8);   // 4-byte aligned: VSTRIDE, c8 even
    dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
  }
  __syncthreads();
  constexpr int T_ITEMS = 8 * D;                  // (granule column = group of 8 keys, d)
  for (int it = threadIdx.x; it < T_ITEMS; it += 256) {
    const int c = it / D, d = it % D;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t lo = v_lds[(8 * c + 2 * e) * VSTRIDE + d];
      const uint32_t hi = v_lds[(8 * c + 2 * e + 1) * VSTRIDE + d];
      w[e] = lo | (hi << 16);
    }
    pc_store_once((uint4*)(v_img + img + (c * D + d) * 8), make_uint4(w[0], w[1], w[2], w[3]));
  }
}

int pc_launch_kv_prepass(const void* k, const void* v, const float2* table, void* k_rope,
                         void* k_img, void* v_img, int n_seq, int L, int Lp, int n_kv_heads,
                         int head_dim, hipStream_t st) {
  if (n_kv_heads > 65535 || Lp / 64 > 65535) return PC_ERR_SHAPE;       // grid limits
  dim3 grid(n_seq, n_kv_heads, Lp / 64), block(256);
  PcProfScope prof(PC_KERNEL_KV_PREPASS, st);
  if (head_dim == 128)
    hipLaunchKernelGGL(kv_prepass_kernel<128>, grid, block, 0, st, (const uint16_t*)k,
                       (const uint16_t*)v, table, (uint16_t*)k_rope, (uint16_t*)k_img,
                       (uint16_t*)v_img, L, Lp, n_kv_heads);
  else
    hipLaunchKernelGGL(kv_prepass_kernel<64>, grid, block, 0, st, (const uint16_t*)k,
                       (const uint16_t*)v, table, (uint16_t*)k_rope, (uint16_t*)k_img,
                       (uint16_t*)v_img, L, Lp, n_kv_heads);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
template <int D>
struct FlashSmem {
  static constexpr int KBUF = 2;                   // K tile t lives in buffer t % 2
  static constexpr int VBUF = 3;                   // V^T tile t in buffer t % 3 (read one period early)
  static constexpr int K_ELEMS = PC_FA_BN * D;
  static constexpr int V_ELEMS = D * PC_FA_BN;
  static constexpr int BYTES = (KBUF * K_ELEMS + VBUF * V_ELEMS) * 2;
};

// row index of the first MFMA's A operand -> key within a 32-key block (swap bits 2 and 3)
__device__ __forceinline__ int pc_key_of_row(int m) {
  return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1);
}

template <int D, bool ROPE_Q, bool PARTIAL>
__global__ __launch_bounds__(PC_FA_THREADS, 2) void flash_fwd_kernel(PcFlashArgs a) {
  using SM = FlashSmem<D>;
  constexpr int KS = D / 16;        // k-steps of the first product (over head_dim)
  constexpr int DB = D / 32;        // 32-row blocks of O^T (over head_dim)
  constexpr int HALF = D / 2;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  auto k_lds = [&](int t) __attribute__((always_inline)) { return smem + (t % SM::KBUF) * SM::K_ELEMS; };
  auto v_lds = [&](int t) __attribute__((always_inline)) {
    return smem + SM::KBUF * SM::K_ELEMS + (t % SM::VBUF) * SM::V_ELEMS;
  };

  // ---- which (sequence, head, Q tile): one XCD (blockIdx % 8) works through whole
  //      (sequence, KV head) groups, heavy Q tiles first, the group's query heads adjacent
  const int G = a.n_q_heads / a.n_kv_heads;
  const int n_qt = (a.n_rows + PC_FA_BM - 1) / PC_FA_BM;
  const int per_group = G * n_qt * a.n_parts_grid;
  const int xcd = blockIdx.x % 8, jb = blockIdx.x / 8;
  const int cg = (jb / per_group) * 8 + xcd;
  if (cg >= a.n_seq * a.n_kv_heads) return;
  int within = jb % per_group;
  const int part = within % a.n_parts_grid; within /= a.n_parts_grid;
  const int qt = n_qt - 1 - within / G;
  const int hg = within % G;
  const int seq = cg / a.n_kv_heads, g = cg % a.n_kv_heads;
  const int h = g * G + hg;

  const int tid = threadIdx.x, lane = tid % PC_WAVE, wave = tid / PC_WAVE;
  const int hf = lane / 32, n = lane % 32;
  const int row0_wg = qt * PC_FA_BM;
  // rows (= keys) of this sequence: a short chunk is [its context rows ; the query rows]
  const int seq_rows = a.seq_ctx ? min(max(a.seq_ctx[seq], 0), a.n_rows - a.seq_add) + a.seq_add : a.n_rows;
  if (row0_wg >= seq_rows) return;                 // a Q tile of padding rows (uniform over the workgroup)
  constexpr int NB = PC_FA_NB;
  const int row0 = row0_wg + 32 * NB * wave;      // first query row of this wavefront
  int my_row[NB], max_key[NB];

  // ---- keys of this workgroup: [0, key_end) of the part
  const int len_idx = a.part_len_per_head ? (seq * a.n_parts_grid + part) * a.n_kv_heads + g
                                          : seq * a.n_parts_grid + part;
  const int n_valid = a.part_len ? min(max(a.part_len[len_idx], 0), a.n_keys)
                                 : (a.seq_ctx ? min(a.n_keys, seq_rows) : a.n_keys);
  int key_end = n_valid;
  if (a.causal_offset < PC_NO_CAUSAL) key_end = min(key_end, row0_wg + PC_FA_BM + a.causal_offset);
  const int T = (key_end + PC_FA_BN - 1) / PC_FA_BN;          // 64-key tiles
  // steps of 32 keys: steps [0, J0) are visible to every row of the workgroup (no mask)
  const int J0 = (min(row0_wg + a.causal_offset, n_valid - 1) + 1) / 32;

  // tile images of this (sequence, part, KV head): consecutive 64-key tiles of 64 * D elements
  const long long img0 = (seq * a.img_seq_stride + part * a.img_part_stride + g * a.img_head_stride) * (64LL * D);
  const uint16_t* kbase = (const uint16_t*)a.k_img + img0;
  const uint16_t* vbase = (const uint16_t*)a.v_img + img0;

  // ---- Q^T as B operand, NB 32-row blocks: lane holds query n of each, d = 16*ks + 8*hf .. +7.
  //      The softmax scale and log2(e) are folded into Q before its rounding to bf16, so the
  //      first product yields logits in log2 units and the exponent needs no multiply.
  const float c_log2 = a.scale * PC_LOG2E;
  bf16x8 bq[NB][KS];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    my_row[nb] = row0 + 32 * nb + n;
    max_key[nb] = min(my_row[nb] + a.causal_offset, n_valid - 1);
    const int ld_row = min(my_row[nb], seq_rows - 1);
    const uint16_t* qrow = (const uint16_t*)a.q + (((long long)seq * a.n_rows + ld_row) * a.n_q_heads + h) * D;
    if (ROPE_Q) {
      // The wavefront's 32 query rows and their (cos, sin) table rows are fetched with
      // coalesced loads (a load instruction covers whole rows, 1 KiB contiguous where the rows
      // are adjacent) and handed to the lanes that own them through a private, XOR-swizzled
      // LDS area in the tile buffers, which are still unused at this point.  A gather straight
      // into the operand layout (every lane its own row) would touch 32 to 64 cache lines per
      // instruction and costs several microseconds per workgroup.
      constexpr int PPR = D / 8;                  // 16-byte pieces per query row (and per table half row)
      constexpr int RPL = PC_WAVE / PPR;          // rows per load instruction
      constexpr int NLD = 32 / RPL;               // load instructions per 32 rows
      constexpr int KS_HALF = D / 64;             // ks iterations served by one half of a table row
      static_assert(NB == 1, "staging area is sized for one row block per wavefront");
      uint16_t* st_q = smem + wave * (2 * 32 * D);            // 32 rows x D bf16
      uint16_t* st_t = st_q + 32 * D;                         // 32 half rows of the table (D bytes x 2)
      const int l_row = lane / PPR, l_piece = lane % PPR;
      u32x4 rq[NLD], rt[2][NLD];
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int r = RPL * i + l_row;
        const int grow = min(row0 + 32 * nb + r, seq_rows - 1);
        rq[i] = pc_load_once((const u32x4*)((const uint16_t*)a.q + (((long long)seq * a.n_rows + grow) * a.n_q_heads + h) * D + 8 * l_piece));
        const char* trow = (const char*)(a.table + (long long)(a.q_pos0 + grow) * HALF);
        rt[0][i] = *(const u32x4*)(trow + 16 * l_piece);
        rt[1][i] = *(const u32x4*)(trow + 2 * D + 16 * l_piece);
      }
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int r = RPL * i + l_row;
        *(u32x4*)(st_q + (r * PPR + (l_piece ^ (r % PPR))) * 8) = rq[i];
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
          const int r = RPL * i + l_row;
          *(u32x4*)(st_t + (r * PPR + (l_piece ^ (r % PPR))) * 8) = rt[half][i];
        }
        PC_FA_WAVE_LDS_SYNC();
#pragma unroll
        for (int kh = 0; kh < KS_HALF; ++kh) {
          const int ks = half * KS_HALF + kh;
          const int pq = 2 * ks + hf;                         // piece of the row's first half; + PPR / 2: second half
          const u32x4 x1 = *(const u32x4*)(st_q + (n * PPR + (pq ^ (n % PPR))) * 8);
          const u32x4 x2 = *(const u32x4*)(st_q + (n * PPR + ((pq + PPR / 2) ^ (n % PPR))) * 8);
          u32x4 ra, rbv;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int pt = 8 * kh + 4 * hf + e;               // piece e of the lane's 64 bytes of (cos, sin)
            const u32x4 cw = *(const u32x4*)(st_t + (n * PPR + (pt ^ (n % PPR))) * 8);
            const float2 c0 = make_float2(__uint_as_float(cw[0]), __uint_as_float(cw[1]));
            const float2 c1 = make_float2(__uint_as_float(cw[2]), __uint_as_float(cw[3]));
            const float x1l = bf16_lo_to_f32(x1[e]), x1h = bf16_hi_to_f32(x1[e]);
            const float x2l = bf16_lo_to_f32(x2[e]), x2h = bf16_hi_to_f32(x2[e]);
            ra[e] = pack_bf16x2((x1l * c0.x - x2l * c0.y) * c_log2, (x1h * c1.x - x2h * c1.y) * c_log2);
            rbv[e] = pack_bf16x2((x2l * c0.x + x1l * c0.y) * c_log2, (x2h * c1.x + x1h * c1.y) * c_log2);
          }
          bq[nb][ks] = *(bf16x8*)&ra;
          bq[nb][ks + KS / 2] = *(bf16x8*)&rbv;
        }
        PC_FA_WAVE_LDS_SYNC();                                // the table area is rewritten / the tiles move in
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        // already rotated and scaled by the caller (rounded to bf16 once, there)
        const u32x4 x = *(const u32x4*)(qrow + 16 * ks + 8 * hf);
        bq[nb][ks] = *(bf16x8*)&x;
      }
    }
  }

  // ---- cooperative tile loads, straight from global memory into LDS: a tile image is copied
  //      as it is, wavefront w issuing instruction i for its 1 KiB block WAVES i + w.  Loads go
  //      through buffer descriptors (descriptor base + scalar offset + one constant per-lane
  //      offset, no 64-bit vector arithmetic per load).
  constexpr int WAVES = PC_FA_WAVES;
  constexpr int T_LD = D / 8 / WAVES;              // load instructions per wavefront per tile
  constexpr int IMG_BYTES = 64 * D * 2;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  typedef __attribute__((address_space(3))) void* lptr_t;
  const int n_img = (a.n_keys + 63) / 64;
  const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kbase, 0, n_img * IMG_BYTES, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)vbase, 0, n_img * IMG_BYTES, 0x00020000);
  const int ld_goff = 1024 * wave_s + 16 * lane;
  auto load_k_i = [&](int t, int i) __attribute__((always_inline)) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (lptr_t)(k_lds(t) + 512 * (WAVES * i + wave_s)), 16,
                                             ld_goff, t * IMG_BYTES + 1024 * WAVES * i, 0, 0);
  };
  auto load_v_i = [&](int t, int i) __attribute__((always_inline)) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (lptr_t)(v_lds(t) + 512 * (WAVES * i + wave_s)), 16,
                                             ld_goff, t * IMG_BYTES + 1024 * WAVES * i, 0, 0);
  };
  auto load_k = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < T_LD; ++i) load_k_i(t, i);
  };
  auto load_v = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < T_LD; ++i) load_v_i(t, i);
  };
  // s_waitcnt vmcnt(N): N newest loads of this wavefront may still be in flight
#define PC_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14))

  floatx16 o_acc[NB][DB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[nb][db][r] = 0.f;
  // Softmax state per row: reference m_run (log2 units), row sum l_run, and -m_run replicated
  // over an accumulator tile: it is the C operand of the first MFMA of every S^T, so S^T comes
  // out of the matrix pipe already relative to the reference.
  float m_run[NB], l_run[NB];
  floatx16 negm[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m_run[nb] = 0.f; l_run[nb] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[nb][r] = 0.f;
  }
  const int krow = pc_key_of_row(n);               // LDS row this lane feeds into MFMA row n

  // A step is 32 keys.  Step j reads K rows / V^T columns 32 (j & 1) .. + 31 of tile j >> 1.
  // S^T of step j lives in s_buf[j & 1], its probabilities P^T (bf16) in p_buf[j & 1].
  floatx16 s_buf[2][NB];                           // [step parity][row block]
  u32x4 p_buf[2][NB][2];                            // [step parity][row block][16-key k-step], bf16 pairs

  // Per-lane element offsets of the MFMA A operands inside a tile image: K granule
  // (2 ks + hf, 32 (j & 1) + krow), V^T granule (4 (j & 1) + 2 ts + hf, 32 db + n).  Everything
  // but the lane's own part is a compile-time offset of the LDS read.
  int k_base = (hf * 64 + krow) * 8;
  int v_base = (hf * D + n) * 8;

  // MFMA A operands, read from LDS one region ahead of their use
  bf16x8 ka[KS], va[2][DB];                        // K rows of a step; V^T [16-key k-step][d block]
  using no_mask = std::integral_constant<bool, false>;
  using with_mask = std::integral_constant<bool, true>;
  using yes = std::integral_constant<bool, true>;
  using no = std::integral_constant<bool, false>;

  // One step of the software pipeline, j = the step whose softmax runs now.  A region is NM
  // slices of [one MFMA, at most one LDS operand read, a few vector-ALU instructions], and the
  // compiler may not move instructions across a slice boundary, so the three pipes are fed
  // evenly by construction instead of by the scheduler's heuristics:
  //   region 1:  MFMA  O^T += V^T(j-1) P^T(j-1)     LDS  K(j+1) operands
  //              VALU  row maxima of S^T(j), reference update, first part of P^T(j)
  //   (rare)     rescale O after the reference of some row moved
  //   region 2:  MFMA  S^T(j+1) = K(j+1) Q^T        LDS  V^T(j) operands
  //              VALU  rest of P^T(j) = exp2(S^T(j) - m)
  // Register r of a row block at lane half hf is key 32 j + 16 (r / 8) + 8 hf + (r % 8).
  // Lazy rescale: the reference m_run of a row only moves when the step maximum exceeds it by
  // more than 2^8; until then p = exp2(s - m_run) <= 256 and O, l keep their scale.  The P V
  // products of step j - 1 (old reference) are all issued in region 1, so O is rescaled after it.
  // has_pv / has_qk are compile-time: the first step has no previous P V, the last no next K Q^T.
  // Steps that lie wholly above a wavefront's rows on the diagonal: those inside the loop are
  // not skipped, their logits are masked to -inf and add exact zeros (straight-line code keeps
  // the register allocation of the loop tight); the ones at the very end (the last period and
  // the last step) are left out per wavefront, see the end of the main loop.
  constexpr int NM = NB * KS;                      // MFMAs per region (= 2 NB DB)
  constexpr int MAX_SL = NM / 4;                   // slices of region 1 that take the row maxima
  constexpr int NG = 16 * NB + 1;                  // probability groups per step
  // groups placed in region 1: the share of its free slices among all slices that take groups
  constexpr int G1 = NG * (NM - MAX_SL - 1) / (2 * NM - MAX_SL - 1);
  auto step = [&](auto mask_tag, auto has_pv, auto has_qk, auto has_ld, int j, int t_ld, floatx16(&s_cur)[NB],
                  floatx16(&s_next)[NB], u32x4(&p_cur)[NB][2],
                  const u32x4(&p_prev)[NB][2]) __attribute__((always_inline)) {
    constexpr bool MASK = decltype(mask_tag)::value;
    constexpr bool PV = decltype(has_pv)::value, QK = decltype(has_qk)::value, LD = decltype(has_ld)::value;
    const uint16_t* kp = k_lds((j + 1) >> 1) + 32 * 8 * ((j + 1) & 1) + k_base;   // this lane's granule of column hf
    const uint16_t* vp = v_lds(j >> 1) + 4 * (j & 1) * D * 8 + v_base;
    float t[NB], alpha[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { t[nb] = 0.f; alpha[nb] = 1.f; }
    bool grow_any = false;
    // probability e (0..31: row block e / 16, register e % 16) of this step
    // The probabilities of a step go through two stages, one stage per group: group g takes
    // the exp2 of element g and the sum / bf16 pack of element g - 1, so no instruction waits on
    // the one issued just before it.  Element e is register e % 16 of row block e / 16.  Opaque
    // uses pin each group to the slice it is written in: without them the compiler sinks this
    // (side-effect-free) arithmetic past slice boundaries.
    float pr[16 * NB];
    auto prob_group = [&](int g) __attribute__((always_inline)) {
      if (g >= 1 && g - 1 < 16 * NB) {
        const int e = g - 1, nb = e / 16, r = e % 16;
        l_run[nb] += pr[e];
        asm volatile("" : "+v"(l_run[nb]));
        if (r % 2 == 1) {
          uint32_t w = pack_bf16x2(pr[e - 1], pr[e]);
          asm volatile("" : "+v"(w));
          p_cur[nb][r / 8][(r % 8) / 2] = w;
        }
      }
      if (g < 16 * NB) {
        pr[g] = __builtin_amdgcn_exp2f(s_cur[g / 16][g % 16]);
        asm volatile("" : "+v"(pr[g]));
      }
    };
    // ---------------- region 1
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      if (PV) {
        const int ts = i / (NB * DB), db = (i / NB) % DB, nb = i % NB;
        o_acc[nb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            va[ts][db], *(const bf16x8*)&p_prev[nb][ts], o_acc[nb][db], 0, 0, 0);
      }
      if (QK && i < KS) ka[i] = *(const bf16x8*)(kp + 2 * i * 64 * 8);
      if (LD && i >= NM - 2 * T_LD) {               // one tile-load instruction per slice
        const int li = i - (NM - 2 * T_LD);
        if (li < T_LD) load_k_i(t_ld, li);
        else load_v_i(t_ld, li - T_LD);
      }
      if (MASK && i == 0) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = 32 * j + 16 * (r / 8) + 8 * hf + (r % 8);
            if (key > max_key[nb]) s_cur[nb][r] = -INFINITY;
          }
      }
      if (i < MAX_SL) {
        // the 8 links of each row block's maximum chain, 8 / MAX_SL per slice
#pragma unroll
        for (int q = i * (8 / MAX_SL); q < (i + 1) * (8 / MAX_SL); ++q)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            if (q == 0) t[nb] = fmaxf(fmaxf(s_cur[nb][0], s_cur[nb][1]), s_cur[nb][2]);
            else if (q < 7) t[nb] = fmaxf(fmaxf(t[nb], s_cur[nb][2 * q + 1]), s_cur[nb][2 * q + 2]);
            else t[nb] = fmaxf(t[nb], s_cur[nb][15]);
          }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+v"(t[nb]));
      }
      if (i == MAX_SL) {
        // Does any row's maximum leave the window of its reference?  S^T is already relative
        // to the reference, so the test is a compare with a constant; everything else is rare.
        bool grow = !PV;                            // the first step sets the reference exactly
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) grow |= t[nb] > 8.0f;
        grow_any = __any(grow);
        if (grow_any) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const float tm = pc_xhalf_max(t[nb]);   // both lane halves hold keys of the same row
            const bool gr = PV ? tm > 8.0f : tm != -INFINITY;
            const float delta = gr ? tm : 0.f;
            alpha[nb] = PV ? __builtin_amdgcn_exp2f(-delta) : 1.0f;   // nothing accumulated before the first step
            m_run[nb] += delta;
            l_run[nb] *= alpha[nb];
#pragma unroll
            for (int r = 0; r < 16; ++r) { negm[nb][r] = -m_run[nb]; s_cur[nb][r] -= delta; }
          }
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+v"(l_run[nb]));
      }
#pragma unroll
      for (int g = 0; g < G1; ++g)
        if (MAX_SL + 1 + g * (NM - MAX_SL - 1) / G1 == i) prob_group(g);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (grow_any) {
      // O sits in the accumulation registers; walk it one 16-register block at a time so this
      // rare path needs only a handful of temporaries
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
          for (int r = 0; r < 16; ++r) o_acc[nb][db][r] *= alpha[nb];
          __builtin_amdgcn_sched_barrier(0);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---------------- region 2
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      if (QK) {
        const int ks = i / NB, nb = i % NB;
        s_next[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], bq[nb][ks], ks == 0 ? negm[nb] : s_next[nb], 0, 0, 0);
      }
      if (i < KS) {
        const int ts = i / DB, db = i % DB;
        va[ts][db] = *(const bf16x8*)(vp + 2 * ts * D * 8 + 32 * db * 8);
      }
#pragma unroll
      for (int g = G1; g < NG; ++g)
        if ((g - G1) * NM / (NG - G1) == i) prob_group(g);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // first S^T of a workgroup: operands of step 0, then the product
  auto first_qk = [&](floatx16(&s)[NB]) __attribute__((always_inline)) {
    const uint16_t* kp = k_lds(0) + k_base;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ka[ks] = *(const bf16x8*)(kp + 2 * ks * 64 * 8);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[nb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], bq[nb][ks], s[nb], 0, 0, 0);
  };
  // trailing O^T += V^T(j) P^T(j) of the last step
  auto last_pv = [&](const u32x4(&p)[NB][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int ts = 0; ts < 2; ++ts)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          o_acc[nb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ts][db], *(const bf16x8*)&p[nb][ts], o_acc[nb][db], 0, 0, 0);
  };

  if (T > 0) {
    // ---- prologue: tiles 0 and 1 must have landed before the first step; tiles 2, 3 stay in flight
    if (ROPE_Q) __syncthreads();                   // every wavefront has left its staging area
    load_k(0);
    load_v(0);
    load_k(min(1, T - 1));
    load_v(min(1, T - 1));
    PC_WAIT_VMCNT(0);
    __syncthreads();
    first_qk(s_buf[0]);
    step(with_mask{}, no{}, yes{}, no{}, 0, 0, s_buf[0], s_buf[1], p_buf[0], p_buf[1]);

    // One period = two steps.  Period p runs steps 2p+1 and 2p+2: it reads K tile p + 1 and the
    // V^T tiles p and p + 1 (the latter only its first half, for the next period's first step).
    // After its barrier it issues the loads of K(p + 4) and V(p + 4), one instruction per slice
    // of its first step, into the buffers that held K(p) and V(p - 1), both last read before
    // that barrier.  Tiles are first read three periods after their loads were issued, so before
    // a barrier a wavefront only waits for the loads it issued two periods earlier (the two
    // newest batches may stay in flight).  Past the last tile the loads repeat tile T - 1 into
    // buffers nobody reads again, which keeps the loop free of branches.
    auto period = [&](auto mask_tag, int p) __attribute__((always_inline)) {
      // Opaque no-ops on the address seeds: they stop the compiler from hoisting a dozen
      // loop-invariant per-lane addresses out of the loop into registers the loop cannot spare;
      // recomputing them costs a few vector-ALU instructions per period.
      asm volatile("" : "+v"(k_base), "+v"(v_base));
      PC_WAIT_VMCNT(0);
      __syncthreads();
      const int t_ld = min(p + 2, T - 1);
      step(mask_tag, yes{}, yes{}, yes{}, 2 * p + 1, t_ld, s_buf[1], s_buf[0], p_buf[1], p_buf[0]);
      step(mask_tag, yes{}, yes{}, no{}, 2 * p + 2, 0, s_buf[0], s_buf[1], p_buf[0], p_buf[1]);
    };
    const int n_plain = min(T - 1, max(0, (J0 - 1) / 2));   // periods whose steps need no mask
    // Last step with a key visible to any row of this wavefront.  On the diagonal the steps
    // behind it hold only masked keys: the wavefront keeps the workgroup's barrier count but
    // leaves their arithmetic out (the tile loads of the last period only repeat tile T - 1).
    const int j_need = __builtin_amdgcn_readfirstlane(
        min(row0 + 32 * NB - 1 + a.causal_offset, n_valid - 1) >> 5);
    const bool skip_last_period = T >= 2 && j_need < 2 * T - 3;
    const int n_periods = skip_last_period ? T - 2 : T - 1;
    int p = 0;
    for (; p < min(n_plain, n_periods); ++p) period(no_mask{}, p);
    for (; p < n_periods; ++p) period(with_mask{}, p);
    if (skip_last_period) {
      PC_WAIT_VMCNT(0);
      __syncthreads();                                       // the barrier of period T - 2
    }
    // ---- last period: step 2T-1 and the trailing P V
    PC_WAIT_VMCNT(0);
    __syncthreads();
    if (j_need >= 2 * T - 1) {
      step(with_mask{}, yes{}, no{}, no{}, 2 * T - 1, 0, s_buf[1], s_buf[0], p_buf[1], p_buf[0]);
      last_pv(p_buf[1]);
    } else {
      last_pv(p_buf[0]);                                     // P V of the last step that ran (an even one)
    }
  }

  // ---- epilogue: lane halves hold disjoint key subsets of the same query
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const float l = pc_xhalf_sum(l_run[nb]);
    const float inv_l = l > 0.f ? 1.f / l : 0.f;
    const float lse = l > 0.f ? m_run[nb] * PC_LN2 + logf(l) : -INFINITY;
    if (PARTIAL) {
      if (my_row[nb] < seq_rows) {
        const long long prow = ((((long long)seq * a.n_parts_total + a.part0 + part) * a.n_rows) + my_row[nb]) * a.n_q_heads + h;
        float* po = a.part_o + prow * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            floatx4 x = {o_acc[nb][db][4 * i] * inv_l, o_acc[nb][db][4 * i + 1] * inv_l,
                         o_acc[nb][db][4 * i + 2] * inv_l, o_acc[nb][db][4 * i + 3] * inv_l};
            *(floatx4*)(po + 32 * db + 8 * i + 4 * hf) = x;
          }
        if (hf == 0) a.part_lse[prow] = lse;
      }
    } else {
      // The lane that owns a query holds its output row in 8-byte pieces; stored from there,
      // an instruction would touch 32 rows.  The rows go through a swizzled staging area in the
      // K buffers (nobody reads K after the last barrier: the last step has no next S^T) and
      // leave as whole 16-byte-per-lane rows, 1 KiB per instruction where rows are adjacent.
      constexpr int PPR = D / 8, RPL = PC_WAVE / PPR, NLD = 32 / RPL;
      static_assert(NB == 1 && PC_FA_WAVES * 32 * D <= SM::KBUF * SM::K_ELEMS, "staging area is the K buffers");
      uint16_t* st_o = smem + wave * (32 * D);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          uint2 x;
          x.x = pack_bf16x2(o_acc[nb][db][4 * i] * inv_l, o_acc[nb][db][4 * i + 1] * inv_l);
          x.y = pack_bf16x2(o_acc[nb][db][4 * i + 2] * inv_l, o_acc[nb][db][4 * i + 3] * inv_l);
          const int p = 4 * db + i;                             // 16-byte piece of the row; half hf of it
          *(uint2*)(st_o + (n * PPR + (p ^ (n % PPR))) * 8 + 4 * hf) = x;
        }
      PC_FA_WAVE_LDS_SYNC();
      const int l_row = lane / PPR, l_piece = lane % PPR;
#pragma unroll
      for (int k = 0; k < NLD; ++k) {
        const int r = RPL * k + l_row;
        const u32x4 x = *(const u32x4*)(st_o + (r * PPR + (l_piece ^ (r % PPR))) * 8);
        const int grow = row0 + 32 * nb + r;
        if (grow < seq_rows)
          pc_store_once((u32x4*)((uint16_t*)a.o + (((long long)seq * a.n_rows + grow) * a.n_q_heads + h) * D + 8 * l_piece), x);
      }
      if (my_row[nb] < seq_rows && hf == 0 && a.lse)
        a.lse[((long long)seq * a.n_q_heads + h) * a.n_rows + my_row[nb]] = lse;
    }
  }
}

template <int D, bool ROPE_Q, bool PARTIAL>
static int launch_flash_t(const PcFlashArgs& a, hipStream_t st) {
  using SM = FlashSmem<D>;
  auto kern = flash_fwd_kernel<D, ROPE_Q, PARTIAL>;
  static std::atomic<uint64_t> raised{0};          // one per instantiation of this launcher
  const int lds_rc = pc_raise_dynamic_lds((const void*)kern, SM::BYTES, raised);
  if (lds_rc != PC_OK) return lds_rc;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int n_qt = (a.n_rows + PC_FA_BM - 1) / PC_FA_BM;
  const long long per_group = (long long)G * n_qt * a.n_parts_grid;
  const long long groups = (long long)a.n_seq * a.n_kv_heads;
  const long long blocks = (groups + 7) / 8 * per_group * 8;
  if (blocks == 0) return PC_OK;
  if (blocks > 0x7fffffffLL) return PC_ERR_SHAPE;
  // tile loads address one (sequence, part, head) region with 32-bit byte offsets
  if (((long long)a.n_keys + 63) / 64 * 64 * D * 2 >= 0x7fffffffLL) return PC_ERR_SHAPE;
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
