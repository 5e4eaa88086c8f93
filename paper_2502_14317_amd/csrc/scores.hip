// Cumulative query->key attention scores (Eq. 5-6):
//   tok_score[c, g, j] = sum over the query heads h of KV group g and over the voting rows r
//                        (the last w_obs rows of the chunk sequence) of P[c, h, r, j],  j < w,
// where P[c, h, r, :] is the causal softmax row of Eq. 1 over ALL keys of the sequence.
// The probability block [H_q, w_obs, L] is never written to memory: it is recomputed.
//
// Accuracy.  The scores decide which tokens are kept, so logits are computed to about fp32
// accuracy although they run on the bf16 matrix cores: q and k are rotated in fp32 and split
// into bf16 hi + lo parts, and q.k = hi.hi + hi.lo + lo.hi (three MFMAs; the lo.lo term is
// below 2^-16 relative).
//
// Two passes over the keys, both fully parallel over key blocks of 256 to 1024 keys (the largest
// block that still leaves every CU several workgroups: a workgroup's start-up, rotating and
// splitting its query columns, is then spread over more keys):
//   pass 1  (S^T = K Q^T, a lane owns a voting row)  per-block running max / sum of every
//           voting row -> workspace [c, g, key block, column] (m, l)
//   between the passes a small kernel combines the blocks' (m, l) into the row logsumexp
//   pass 2  (S = Q K^T, a lane owns a key)           recompute the logits, p = exp2(s - lse)
//           and sum p over the columns (voting rows x heads of the group) for each key
//           -> tok_score
// Pass 2 also leaves the sum of its tok_score block; a last kernel adds those per chunk in a
// fixed order (deterministic) -> chunk_score.
//
// Fused K/V pre-pass.  Inside pc_chunk_prefill_attn pass 1 takes over the work of
// kv_prepass_kernel (switched on by its output pointers): it already reads every key row once and rotates it in
// fp32, and the bf16 "hi" half of the split IS the rotated key rounded to bf16, so in its first
// round over the columns it also writes the rotated keys (row-major cache) and the K tile images,
// and moves V through LDS into the V^T tile images.  The keys are then read from HBM once for
// both jobs, and rotated once.
//
// Any number of voting rows: the (row, head) columns of a KV group are handled in rounds of 128
// (4 blocks of 32), the key tiles being re-read (from the caches) in every round.
#include "pc_common.h"
#include <math.h>

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define PC_SC_THREADS 256
#define PC_SC_WAVES 4
#define PC_SC_KB 256        // keys per workgroup: the smallest block (sizes the workspace)
#define PC_SC_KB_MAX 1024   // the largest
#define PC_SC_TILE 64       // keys staged in LDS at a time
#define PC_SC_LOG2E 1.4426950408889634f

struct PcScoreArgs {
  const uint16_t* q;       // [C, L, H_q, D] before RoPE
  const uint16_t* k;       // [C, L, H_kv, D] before RoPE
  const int32_t* chunk_lens; // [C] context rows per chunk or nullptr (= w)
  const float2* table;     // [L, D/2] (cos, sin)
  float2* ml;              // workspace [C, H_kv, n_kb, n_cols] (max in log2 units, sum)
  float* lse2;             // workspace [C, H_kv, n_cols] row logsumexp in log2 units
  float* tok_score;        // [C, H_kv, w]
  int L, w, w_obs, n_q_heads, n_kv_heads, n_kb, n_cols;
  int kb_keys;             // keys per workgroup: 256, 512 or 1024 (at most 512 when WPC == 4)
  float scale_log2;        // softmax scale x log2(e), folded into the query operand
  float* blk_sum;          // workspace [C, H_kv, n_kb]: sum of each pass-2 block's tok_score
  // pre-pass duties of pass 1 (all nullptr: off): V rows in, rotated keys / K images / V^T images out
  const uint16_t* v;       // [C, L, H_kv, D]
  uint16_t* k_rope;        // [C, L, H_kv, D] or nullptr
  uint16_t* k_img;         // tile images [C][H_kv][Lp / 64][64 * D]
  uint16_t* v_img;
  int Lp;                  // L rounded up to 64
};

// (x0, x1) -> packed bf16 pair of the values and packed bf16 pair of the rounding remainders
// (both roundings to nearest-even, in hardware; inputs are finite by contract)
__device__ __forceinline__ void split_bf16x2(float x0, float x1, uint32_t& hi, uint32_t& lo) {
  hi = pack_bf16x2(x0, x1);
  lo = pack_bf16x2(x0 - bf16_lo_to_f32(hi), x1 - bf16_hi_to_f32(hi));
}

// WPC = wavefronts per block of 32 columns.  With 4 or more column blocks (a GQA group of 4
// heads x 32 voting rows) a wavefront owns a column block and takes both 32-key halves of every
// 64-key tile (WPC = 1).  With fewer column blocks the wavefronts of a block share its keys
// instead of idling: WPC = 2 splits the halves of a 64-key tile, WPC = 4 (one column block, e.g.
// MHA with 32 voting rows) the four 32-key quarters of a 128-key tile.
template <int D, int PASS, int WPC>
__global__ __launch_bounds__(PC_SC_THREADS, 2) void scores_kernel(PcScoreArgs a) {
  // The pre-pass duties ride on pass 1 and are switched at run time (a.v_img != nullptr), so the
  // standalone score call and the fused one execute the same code and give the same bits.
  constexpr bool PRE = PASS == 1;
  constexpr int KS = D / 16, HALF = D / 2, KSTRIDE = D + 8;
  constexpr int TILE = WPC == 4 ? 2 * PC_SC_TILE : PC_SC_TILE;   // keys staged in LDS at a time
  constexpr int NSUB = TILE / 32;                                // 32-key sub-blocks per tile
  constexpr int CB_PER_ROUND = PC_SC_WAVES / WPC;
  __shared__ __attribute__((aligned(16))) uint16_t k_hi[TILE * KSTRIDE];
  __shared__ __attribute__((aligned(16))) uint16_t k_lo[TILE * KSTRIDE];
  constexpr int KB_CAP = WPC == 4 ? PC_SC_KB_MAX / 2 : PC_SC_KB_MAX;   // LDS: two workgroups per CU
  __shared__ float tok_part[PC_SC_WAVES][PASS == 2 ? KB_CAP : 1];
  __shared__ float2 ml_part[PC_SC_WAVES][32];

  const int c = blockIdx.x, g = blockIdx.y, kblock = blockIdx.z;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int tid = threadIdx.x, lane = tid % PC_WAVE, wave = tid / PC_WAVE;
  const int hf = lane / 32, n = lane % 32;
  const int n_cb = (a.n_cols + 31) / 32;
  // a short chunk is [len context rows ; the query rows]: its voting rows end at len + w_q
  const int ctx_len = a.chunk_lens ? min(max(a.chunk_lens[c], 0), a.w) : a.w;
  const int first_obs = ctx_len + (a.L - a.w) - a.w_obs;
  const long long ml_base = (((long long)c * a.n_kv_heads + g) * a.n_kb) * a.n_cols;

  const float* lse2 = a.lse2 + ((long long)c * a.n_kv_heads + g) * a.n_cols;

  // pass 2: every wavefront accumulates its columns' share of the keys' sums in its own LDS row
  if (PASS == 2)
    for (int i = lane; i < a.kb_keys; i += PC_WAVE) tok_part[wave][i] = 0.f;

  const int n_rounds = (n_cb + CB_PER_ROUND - 1) / CB_PER_ROUND;
  const int kb0 = wave % WPC;                      // this wavefront's first sub-block of a tile
  for (int round = 0; round < n_rounds; ++round) {
    const int cb = round * CB_PER_ROUND + wave / WPC;
    const bool active = cb < n_cb;
    // ---- this lane's column as an MFMA operand: rotate at the row's position, split hi/lo
    const int col = min(32 * cb + n, a.n_cols - 1);
    const int hg = col / a.w_obs, qrow_idx = first_obs + col % a.w_obs;
    bf16x8 qhi[KS], qlo[KS];
    if (active) {
      const uint16_t* qrow = a.q + (((long long)c * a.L + qrow_idx) * a.n_q_heads + g * G + hg) * D;
      const float2* cs = a.table + (long long)qrow_idx * HALF;
#pragma unroll
      for (int ks = 0; ks < KS / 2; ++ks) {
        const int i0 = 16 * ks + 8 * hf;
        const uint4 x1 = *(const uint4*)(qrow + i0);
        const uint4 x2 = *(const uint4*)(qrow + HALF + i0);
        const uint32_t aw[4] = {x1.x, x1.y, x1.z, x1.w}, bw[4] = {x2.x, x2.y, x2.z, x2.w};
        uint32_t h1[4], l1[4], h2[4], l2[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float2 c0 = cs[i0 + 2 * e], c1 = cs[i0 + 2 * e + 1];
          const float x1l = bf16_lo_to_f32(aw[e]), x1h = bf16_hi_to_f32(aw[e]);
          const float x2l = bf16_lo_to_f32(bw[e]), x2h = bf16_hi_to_f32(bw[e]);
          // logits come out of the matrix cores in log2 units: the scale rides on q
          split_bf16x2((x1l * c0.x - x2l * c0.y) * a.scale_log2, (x1h * c1.x - x2h * c1.y) * a.scale_log2, h1[e], l1[e]);
          split_bf16x2((x2l * c0.x + x1l * c0.y) * a.scale_log2, (x2h * c1.x + x1h * c1.y) * a.scale_log2, h2[e], l2[e]);
        }
        uint4 t;
        t = make_uint4(h1[0], h1[1], h1[2], h1[3]); qhi[ks] = *(bf16x8*)&t;
        t = make_uint4(l1[0], l1[1], l1[2], l1[3]); qlo[ks] = *(bf16x8*)&t;
        t = make_uint4(h2[0], h2[1], h2[2], h2[3]); qhi[ks + KS / 2] = *(bf16x8*)&t;
        t = make_uint4(l2[0], l2[1], l2[2], l2[3]); qlo[ks + KS / 2] = *(bf16x8*)&t;
      }
    }
    // pass 1: this lane's voting row (column) and its running statistics
    const int my_qrow = qrow_idx;
    float m_run = -INFINITY, l_run = 0.f;
    // pass 2: the voting rows / logsumexp of the 16 result registers (rows of S)
    float lse_r[16];
    int qrow_r[16];
    if (PASS == 2) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int cc = 32 * cb + 8 * (r / 4) + 4 * hf + (r % 4);
        const bool ok = active && cc < a.n_cols;
        lse_r[r] = ok ? lse2[cc] : INFINITY;                // exp2(-inf) = 0 for padding columns
        qrow_r[r] = ok ? first_obs + cc % a.w_obs : -1;
      }
    }

    // K tile staging, split in two so that the loads of tile t + 1 are in flight while the
    // matrix cores work on tile t: fetch (global -> registers), stage (rotate in fp32, split
    // hi / lo, registers -> LDS).  A thread always handles the same 8 rotation pairs, of rows
    // RP apart, so it reads (cos, sin) from the table once, for its first row, and turns them by
    // the constant angle of RP rows from item to item (one complex multiplication per pair in
    // fp32, at most kb_keys / RP - 1 <= 31 in a chain: ~1e-7 relative per link).
    constexpr int ITEMS = TILE * (HALF / 8) / PC_SC_THREADS;           // per thread and tile
    constexpr int RP = PC_SC_THREADS / (HALF / 8);                     // rows between a thread's items
    static_assert(ITEMS >= 1 && TILE * (HALF / 8) % PC_SC_THREADS == 0, "tile / thread mismatch");
    const int st_r0 = tid / (HALF / 8), st_i0 = (tid % (HALF / 8)) * 8;
    uint4 pf_x1[ITEMS], pf_x2[ITEMS];
    float2 cs_cur[8], cs_step[8];
    {
      const float4* c4 = (const float4*)(a.table + (long long)min(kblock * a.kb_keys + st_r0, a.L - 1) * HALF + st_i0);
      const float4* s4 = (const float4*)(a.table + (long long)min(RP, a.L - 1) * HALF + st_i0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float4 cv = c4[e], sv4 = s4[e];
        cs_cur[2 * e] = make_float2(cv.x, cv.y); cs_cur[2 * e + 1] = make_float2(cv.z, cv.w);
        cs_step[2 * e] = make_float2(sv4.x, sv4.y); cs_step[2 * e + 1] = make_float2(sv4.z, sv4.w);
      }
    }
    // pre-pass duties run in the first round only (every round stages the same keys)
    const bool pre = PRE && round == 0 && a.v_img != nullptr;
    // V: a thread takes 8 consecutive keys x 4 values (eight 8-byte loads), transposes them in
    // registers and stores four 16-byte granules of the V^T image, (8 keys, d) each
    constexpr int V_ALL = (TILE / 8) * (D / 4);                        // such items per tile
    constexpr int V_ITEMS = (V_ALL + PC_SC_THREADS - 1) / PC_SC_THREADS;
    u32x2 pf_v[PRE ? V_ITEMS : 1][8];
    const long long img_cg = ((long long)c * a.n_kv_heads + g) * (a.Lp / 64);   // first tile image of (c, g)
    auto fetch = [&](int key0) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < ITEMS; ++u) {
        const int row = min(key0 + st_r0 + u * RP, a.L - 1);
        const uint16_t* krow = a.k + (((long long)c * a.L + row) * a.n_kv_heads + g) * D;
        pf_x1[u] = pc_load_once((const uint4*)(krow + st_i0));
        pf_x2[u] = pc_load_once((const uint4*)(krow + HALF + st_i0));
      }
      if (pre) {
#pragma unroll
        for (int u = 0; u < V_ITEMS; ++u) {
          const int it = tid + u * PC_SC_THREADS;
          const int row0 = key0 + 8 * (it / (D / 4)), d4 = (it % (D / 4)) * 4;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            pf_v[u][j] = u32x2{0u, 0u};                                // rows past the sequence: zeros in the image
            if (it < V_ALL && row0 + j < a.L)
              pf_v[u][j] = __builtin_nontemporal_load(
                  (const u32x2*)(a.v + (((long long)c * a.L + row0 + j) * a.n_kv_heads + g) * D + d4));
          }
        }
      }
    };
    auto stage = [&](int key0) __attribute__((always_inline)) {
      if (pre) {
        // V^T tile images: granule (c8, d) = V[keys 8 c8 .. 8 c8 + 7][d]; word e of a granule pairs
        // the values of keys 2 e and 2 e + 1 (one byte permute per word)
#pragma unroll
        for (int u = 0; u < V_ITEMS; ++u) {
          const int it = tid + u * PC_SC_THREADS;
          const int row0 = key0 + 8 * (it / (D / 4)), d4 = (it % (D / 4)) * 4;
          if (it < V_ALL && row0 < a.Lp) {
            uint16_t* img = a.v_img + (img_cg + row0 / 64) * (64LL * D) + (((row0 % 64) / 8) * D + d4) * 8;
            uint4 gr[4];
            uint32_t* gw = (uint32_t*)gr;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const u32x2 r0 = pf_v[u][2 * e], r1 = pf_v[u][2 * e + 1];
              gw[0 * 4 + e] = __builtin_amdgcn_perm(r1.x, r0.x, 0x05040100u);   // d4 + 0: low halves
              gw[1 * 4 + e] = __builtin_amdgcn_perm(r1.x, r0.x, 0x07060302u);   // d4 + 1: high halves
              gw[2 * 4 + e] = __builtin_amdgcn_perm(r1.y, r0.y, 0x05040100u);   // d4 + 2
              gw[3 * 4 + e] = __builtin_amdgcn_perm(r1.y, r0.y, 0x07060302u);   // d4 + 3
            }
            // ordinary stores: an instruction writes 16 bytes of every 64 a lane owns, and the
            // last-level cache merges the four pieces of a line (with the streaming hint they
            // reached memory as partial lines: 2.4 times slower)
#pragma unroll
            for (int dd = 0; dd < 4; ++dd) *(uint4*)(img + dd * 8) = gr[dd];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < ITEMS; ++u) {
        const int r = st_r0 + u * RP, i0 = st_i0;
        const uint32_t aw[4] = {pf_x1[u].x, pf_x1[u].y, pf_x1[u].z, pf_x1[u].w};
        const uint32_t bw[4] = {pf_x2[u].x, pf_x2[u].y, pf_x2[u].z, pf_x2[u].w};
        uint32_t h1[4], l1[4], h2[4], l2[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float2 c0 = cs_cur[2 * e], c1 = cs_cur[2 * e + 1];
          const float x1l = bf16_lo_to_f32(aw[e]), x1h = bf16_hi_to_f32(aw[e]);
          const float x2l = bf16_lo_to_f32(bw[e]), x2h = bf16_hi_to_f32(bw[e]);
          split_bf16x2(x1l * c0.x - x2l * c0.y, x1h * c1.x - x2h * c1.y, h1[e], l1[e]);
          split_bf16x2(x2l * c0.x + x1l * c0.y, x2h * c1.x + x1h * c1.y, h2[e], l2[e]);
        }
        *(uint4*)(k_hi + r * KSTRIDE + i0) = make_uint4(h1[0], h1[1], h1[2], h1[3]);
        *(uint4*)(k_lo + r * KSTRIDE + i0) = make_uint4(l1[0], l1[1], l1[2], l1[3]);
        *(uint4*)(k_hi + r * KSTRIDE + HALF + i0) = make_uint4(h2[0], h2[1], h2[2], h2[3]);
        *(uint4*)(k_lo + r * KSTRIDE + HALF + i0) = make_uint4(l2[0], l2[1], l2[2], l2[3]);
        if (pre) {
          // the hi halves are the rotated key rounded to bf16: the cache row and its K image granules
          const int row = key0 + r;
          const bool in_seq = row < a.L;
          const uint4 oa = in_seq ? make_uint4(h1[0], h1[1], h1[2], h1[3]) : make_uint4(0, 0, 0, 0);
          const uint4 ob = in_seq ? make_uint4(h2[0], h2[1], h2[2], h2[3]) : make_uint4(0, 0, 0, 0);
          if (in_seq && a.k_rope != nullptr) {
            uint16_t* dst = a.k_rope + (((long long)c * a.L + row) * a.n_kv_heads + g) * D;
            pc_store_once((uint4*)(dst + i0), oa);
            pc_store_once((uint4*)(dst + HALF + i0), ob);
          }
          if (row < a.Lp) {
            uint16_t* img = a.k_img + (img_cg + row / 64) * (64LL * D);
            pc_store_once((uint4*)(img + ((i0 / 8) * 64 + row % 64) * 8), oa);
            pc_store_once((uint4*)(img + (((HALF + i0) / 8) * 64 + row % 64) * 8), ob);
          }
        }
        // (cos, sin) of the thread's next row: angle + RP theta
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float cn = cs_cur[e].x * cs_step[e].x - cs_cur[e].y * cs_step[e].y;
          const float sn = cs_cur[e].y * cs_step[e].x + cs_cur[e].x * cs_step[e].y;
          cs_cur[e] = make_float2(cn, sn);
        }
      }
    };
    if (kblock * a.kb_keys < a.L) fetch(kblock * a.kb_keys);

    // one loop body (not unrolled): leaves room for the prefetch registers
    const int n_tiles = a.kb_keys / TILE;
#pragma unroll 1
    for (int t = 0; t < n_tiles; ++t) {
      const int key0 = kblock * a.kb_keys + t * TILE;
      if (key0 >= a.L) break;                               // uniform over the workgroup
      __syncthreads();                                      // previous tile fully consumed
      stage(key0);
      __syncthreads();
      if (t + 1 < n_tiles && key0 + TILE < a.L) fetch(key0 + TILE);
      if (!active) continue;
      // every key of the tile is visible to every voting row: no causal mask (all but the last
      // tiles of a sequence; the voting rows sit at its end)
      const bool unmasked = key0 + TILE - 1 <= first_obs;

#pragma unroll
      for (int kq = 0; kq < NSUB / WPC; ++kq) {
        const int kb = kb0 + kq * WPC;
        floatx16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
        const uint16_t* ph = k_hi + (32 * kb + n) * KSTRIDE + 8 * hf;
        const uint16_t* pl = k_lo + (32 * kb + n) * KSTRIDE + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 kh = *(const bf16x8*)(ph + 16 * ks);
          const bf16x8 kl = *(const bf16x8*)(pl + 16 * ks);
          if (PASS == 1) {     // rows = keys, columns = voting rows
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kl, qhi[ks], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kh, qlo[ks], s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kh, qhi[ks], s, 0, 0, 0);
          } else {             // rows = voting rows, columns = keys
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qhi[ks], kl, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qlo[ks], kh, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qhi[ks], kh, s, 0, 0, 0);
          }
        }
        if (PASS == 1) {
          float sv[16], tmax = -INFINITY;
          if (unmasked) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { sv[r] = s[r]; tmax = fmaxf(tmax, sv[r]); }
          } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = key0 + 32 * kb + 8 * (r / 4) + 4 * hf + (r % 4);
              sv[r] = (key <= my_qrow) ? s[r] : -INFINITY;
              tmax = fmaxf(tmax, sv[r]);
            }
          }
          const float m_new = fmaxf(m_run, tmax);
          if (m_new > -INFINITY) {
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(sv[r] - m_new);
            l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + sum;
            m_run = m_new;
          }
        } else {
          const int key = key0 + 32 * kb + n;
          float sum = 0.f;
          if (unmasked) {       // padding columns carry lse = +inf: their p is 0 without a mask
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(s[r] - lse_r[r]);
          } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float p = __builtin_amdgcn_exp2f(s[r] - lse_r[r]);
              sum += (key <= qrow_r[r]) ? p : 0.f;
            }
          }
          sum += __shfl_xor(sum, 32);
          if (hf == 0) tok_part[wave][t * TILE + 32 * kb + n] += sum;
        }
      }
    }

    if (PASS == 1) {
      // the lane halves hold disjoint keys of the same column; then the WPC wavefronts of the
      // column block (disjoint keys again) are combined in wavefront order
      const float m_o = __shfl_xor(m_run, 32), l_o = __shfl_xor(l_run, 32);
      float M = fmaxf(m_run, m_o);
      float l = 0.f;
      if (l_run > 0.f) l += l_run * exp2f(m_run - M);
      if (l_o > 0.f) l += l_o * exp2f(m_o - M);
      if (WPC > 1) {
        if (hf == 0) ml_part[wave][n] = make_float2(M, l);
        __syncthreads();
        if (kb0 == 0) {
          M = -INFINITY;
#pragma unroll
          for (int i = 0; i < WPC; ++i) M = fmaxf(M, ml_part[wave + i][n].x);
          l = 0.f;
#pragma unroll
          for (int i = 0; i < WPC; ++i) {
            const float2 v = ml_part[wave + i][n];
            if (v.y > 0.f) l += v.y * exp2f(v.x - M);
          }
        }
        __syncthreads();                               // ml_part free for the next round
      }
      const int cc = 32 * cb + n;
      if (active && kb0 == 0 && hf == 0 && cc < a.n_cols)
        a.ml[ml_base + (long long)kblock * a.n_cols + cc] = make_float2(M, l);
    }
  }

  if (PASS == 2) {
    __syncthreads();
    float blk = 0.f;                                         // this thread's share of the block's sum
    for (int i = tid; i < a.kb_keys; i += PC_SC_THREADS) {
      const int key = kblock * a.kb_keys + i;
      if (key < a.w) {
        float x = 0.f;
#pragma unroll
        for (int wv = 0; wv < PC_SC_WAVES; ++wv) x += tok_part[wv][i];
        x = key < ctx_len ? x : 0.f;
        a.tok_score[((long long)c * a.n_kv_heads + g) * a.w + key] = x;
        blk += x;
      }
    }
    // block sum in a fixed order: lanes (xor tree), then the wavefronts in order
#pragma unroll
    for (int off = PC_WAVE / 2; off > 0; off >>= 1) blk += __shfl_xor(blk, off);
    __syncthreads();                                         // tok_part is read no more: reuse its first floats
    if (lane == 0) tok_part[0][wave] = blk;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
#pragma unroll
      for (int wv = 0; wv < PC_SC_WAVES; ++wv) tot += tok_part[0][wv];
      a.blk_sum[((long long)c * a.n_kv_heads + g) * a.n_kb + kblock] = tot;
    }
  }
}

// Row logsumexp (log2 units) of every voting row from the per-key-block (max, sum) of pass 1,
// combined in block order.  One thread per column; the loads of a batch of blocks are
// independent, so a thread waits for memory n_kb / 8 times, not n_kb times.
__global__ __launch_bounds__(128) void scores_lse_kernel(const float2* __restrict__ ml,
                                                         float* __restrict__ lse2, int n_kb,
                                                         int n_cols) {
  const int col = blockIdx.y * 128 + threadIdx.x;
  if (col >= n_cols) return;
  const float2* src = ml + (long long)blockIdx.x * n_kb * n_cols + col;
  float M = -INFINITY;
  for (int kb0 = 0; kb0 < n_kb; kb0 += 8) {
    float2 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = src[(long long)min(kb0 + i, n_kb - 1) * n_cols];
#pragma unroll
    for (int i = 0; i < 8; ++i) M = fmaxf(M, v[i].x);
  }
  float sum = 0.f;
  for (int kb0 = 0; kb0 < n_kb; kb0 += 8) {
    float2 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = src[(long long)min(kb0 + i, n_kb - 1) * n_cols];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (kb0 + i < n_kb && v[i].y > 0.f) sum += v[i].y * exp2f(v[i].x - M);
  }
  lse2[(long long)blockIdx.x * n_cols + col] = M + log2f(sum);
}

// chunk_score[c] = sum of tok_score[c, :, :] = sum of the chunk's pass-2 block sums, added in a
// fixed order (thread-strided partial sums, then a tree), so the result does not depend on timing.
__global__ __launch_bounds__(256) void chunk_score_kernel(const float* __restrict__ blk_sum,
                                                          float* __restrict__ chunk_score,
                                                          int per_chunk) {
  __shared__ float red[256];
  const float* src = blk_sum + (long long)blockIdx.x * per_chunk;
  float x = 0.f;
  for (int i = threadIdx.x; i < per_chunk; i += 256) x += src[i];
  red[threadIdx.x] = x;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) chunk_score[blockIdx.x] = red[0];
}

template <int PASS>
static void launch_scores_pass(int head_dim, int wpc, dim3 grid, dim3 block, hipStream_t st,
                               const PcScoreArgs& a) {
  if (head_dim == 128) {
    if (wpc == 4) hipLaunchKernelGGL((scores_kernel<128, PASS, 4>), grid, block, 0, st, a);
    else if (wpc == 2) hipLaunchKernelGGL((scores_kernel<128, PASS, 2>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((scores_kernel<128, PASS, 1>), grid, block, 0, st, a);
  } else {
    if (wpc == 4) hipLaunchKernelGGL((scores_kernel<64, PASS, 4>), grid, block, 0, st, a);
    else if (wpc == 2) hipLaunchKernelGGL((scores_kernel<64, PASS, 2>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((scores_kernel<64, PASS, 1>), grid, block, 0, st, a);
  }
}

size_t pc_scores_ml_bytes(const pc_shape* s) {
  const size_t L = (size_t)s->chunk_len + s->query_len;
  const size_t n_kb = (L + PC_SC_KB - 1) / PC_SC_KB;
  const size_t n_cols = (size_t)(s->n_q_heads / s->n_kv_heads) * s->obs_window;
  const size_t cg = (size_t)s->n_chunks * s->n_kv_heads;
  // per-block (max, sum) of pass 1, the combined row logsumexp, the block sums of pass 2
  return cg * n_kb * n_cols * sizeof(float2) + cg * n_cols * sizeof(float) + cg * n_kb * sizeof(float);
}

int pc_launch_scores(const pc_shape* s, const void* q, const void* k, const int32_t* chunk_lens, const float2* table,
                     void* ml_ws, float* tok_score, float* chunk_score, const PcPrepassOut* pre,
                     hipStream_t st) {
  PcScoreArgs a = {};
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.table = table; a.chunk_lens = chunk_lens;
  a.ml = (float2*)ml_ws; a.tok_score = tok_score;
  a.L = s->chunk_len + s->query_len; a.w = s->chunk_len; a.w_obs = s->obs_window;
  a.n_q_heads = s->n_q_heads; a.n_kv_heads = s->n_kv_heads;
  a.n_cols = (s->n_q_heads / s->n_kv_heads) * s->obs_window;
  const int n_cb = (a.n_cols + 31) / 32;
  const int wpc = n_cb == 1 ? 4 : (n_cb == 2 ? 2 : 1);
  // keys per workgroup: double while at least 512 workgroups (one full round of two per CU)
  // remain: fewer, longer workgroups spread their start-up over more keys (measured: 4 and 8
  // chunks of 8192 rows 10 % faster than with twice as many workgroups of half the keys)
  a.kb_keys = PC_SC_KB;
  const int kb_cap = wpc == 4 ? PC_SC_KB_MAX / 2 : PC_SC_KB_MAX;
  while (a.kb_keys < kb_cap &&
         (long long)s->n_chunks * s->n_kv_heads * ((a.L + 2 * a.kb_keys - 1) / (2 * a.kb_keys)) >= 512)
    a.kb_keys *= 2;
  a.n_kb = (a.L + a.kb_keys - 1) / a.kb_keys;
  const float scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
  a.scale_log2 = scale * PC_SC_LOG2E;
  const size_t cg = (size_t)s->n_chunks * s->n_kv_heads;
  a.lse2 = (float*)(a.ml + cg * a.n_kb * a.n_cols);
  a.blk_sum = a.lse2 + cg * a.n_cols;
  if ((long long)a.n_kb > 65535 || (long long)s->n_kv_heads > 65535) return PC_ERR_SHAPE;   // grid limits
  dim3 grid(s->n_chunks, s->n_kv_heads, a.n_kb), block(PC_SC_THREADS);
  if (pre) {
    a.v = (const uint16_t*)pre->v; a.k_rope = (uint16_t*)pre->k_rope; a.k_img = (uint16_t*)pre->k_img;
    a.v_img = (uint16_t*)pre->v_img; a.Lp = pre->Lp;
    PcProfScope prof(PC_KERNEL_PREPASS_SCORES, st);
    launch_scores_pass<1>(s->head_dim, wpc, grid, block, st, a);
  } else {
    PcProfScope prof(PC_KERNEL_SCORES_P1, st);
    launch_scores_pass<1>(s->head_dim, wpc, grid, block, st, a);
  }
  PC_LAUNCH_CHECK();
  {
    PcProfScope prof(PC_KERNEL_SCORES_LSE, st);
    hipLaunchKernelGGL(scores_lse_kernel, dim3(s->n_chunks * s->n_kv_heads, (a.n_cols + 127) / 128),
                       dim3(128), 0, st, a.ml, a.lse2, a.n_kb, a.n_cols);
  }
  {
    PcProfScope prof(PC_KERNEL_SCORES_P2, st);
    launch_scores_pass<2>(s->head_dim, wpc, grid, block, st, a);
  }
  PC_LAUNCH_CHECK();
  if (chunk_score) {
    PcProfScope prof(PC_KERNEL_CHUNK_SCORE, st);
    hipLaunchKernelGGL(chunk_score_kernel, dim3(s->n_chunks), dim3(256), 0, st, a.blk_sum,
                       chunk_score, s->n_kv_heads * a.n_kb);
    PC_LAUNCH_CHECK();
  }
  return PC_OK;
}
