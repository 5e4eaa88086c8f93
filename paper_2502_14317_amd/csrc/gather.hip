// KV compaction gather (Eq. 7: K_r = K_x[kept], V_r = V_x[kept]).
//
// HBM-bound byte copy.  One head row is D bf16 = 128 or 256 bytes; a lane moves one 16-byte
// piece of a K row and the matching piece of the V row, so D/8 adjacent lanes read one
// contiguous row and a wavefront writes 1 KiB of contiguous destination per store.  Each
// thread handles PC_GATHER_UNROLL rows so that several independent loads are in flight.  Both
// sides are touched once, so loads and stores carry the non-temporal hint (64 -> 70 % of peak).
#include "pc_common.h"

#define PC_GATHER_UNROLL 4

// largest bf16 magnitude (15-bit pattern) among the 8 values of a 16-byte piece
__device__ __forceinline__ uint32_t pc_piece_amax(uint4 x) {
  const uint32_t w[4] = {x.x, x.y, x.z, x.w};
  uint32_t m = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) m = max(m, max(w[e] & 0x7fffu, (w[e] >> 16) & 0x7fffu));
  return m;
}

// AMAX: also leave, per destination segment (b, s, g), the largest |value| of its K rows and of
// its V rows (as fp32 bit patterns, so an integer maximum orders them): what a later
// quantisation of the compacted cache needs, taken while the rows are in flight.  The maxima
// must start at zero (amax_clear_kernel); an integer maximum does not depend on the order of
// the updates, so the result is deterministic.
template <int LANES_PER_ROW, bool AMAX>
__global__ __launch_bounds__(256) void gather_kv_kernel(
    const uint4* __restrict__ k_src, const uint4* __restrict__ v_src,
    const int32_t* __restrict__ chunk_idx, const int32_t* __restrict__ tok_idx,
    uint4* __restrict__ k_dst, uint4* __restrict__ v_dst,
    int n_chunks, int rows, int n_sel, int n_kv_heads, int k, long long n_dst_rows,
    uint32_t* __restrict__ k_amax, uint32_t* __restrict__ v_amax) {
  constexpr int ROWS_PER_BLOCK = 256 / LANES_PER_ROW;
  const int piece = threadIdx.x % LANES_PER_ROW;
  const int row_in_block = threadIdx.x / LANES_PER_ROW;
  const long long base = ((long long)blockIdx.x * PC_GATHER_UNROLL) * ROWS_PER_BLOCK + row_in_block;

  uint4 kv[PC_GATHER_UNROLL], vv[PC_GATHER_UNROLL];
  bool skip[PC_GATHER_UNROLL];                                  // destination segment without a source chunk
#pragma unroll
  for (int u = 0; u < PC_GATHER_UNROLL; ++u) {
    const long long r = base + (long long)u * ROWS_PER_BLOCK;   // destination row id
    kv[u] = make_uint4(0, 0, 0, 0);
    vv[u] = make_uint4(0, 0, 0, 0);
    skip[u] = false;
    if (r < n_dst_rows) {
      // r = ((b * n_sel + s) * H_kv + g) * k + t
      const long long bsg = r / k;
      const int g = (int)(bsg % n_kv_heads);
      const long long bs = bsg / n_kv_heads;
      const int s = (int)(bs % n_sel);
      const long long b = bs / n_sel;
      const int c = chunk_idx ? chunk_idx[bs] : s;
      skip[u] = c < 0;
      const int t = skip[u] ? -1 : tok_idx[r];
      if (c >= 0 && c < n_chunks && t >= 0 && t < rows) {
        const long long src_row = ((b * n_chunks + c) * rows + t) * n_kv_heads + g;
        kv[u] = pc_load_once(k_src + src_row * LANES_PER_ROW + piece);
        vv[u] = pc_load_once(v_src + src_row * LANES_PER_ROW + piece);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < PC_GATHER_UNROLL; ++u) {
    const long long r = base + (long long)u * ROWS_PER_BLOCK;
    if (r < n_dst_rows && !skip[u]) {
      pc_store_once(k_dst + r * LANES_PER_ROW + piece, kv[u]);
      pc_store_once(v_dst + r * LANES_PER_ROW + piece, vv[u]);
    }
  }
  if (AMAX) {
    // The block's rows are consecutive destination rows: where they all lie in one segment (the
    // usual case, k being much larger than a block) the maxima are reduced over the thread's
    // rows, then over the wavefront, and one lane updates the segment; otherwise every row
    // updates its own segment.
    const long long r_first = ((long long)blockIdx.x * PC_GATHER_UNROLL) * ROWS_PER_BLOCK;
    const long long r_last = min(r_first + (long long)PC_GATHER_UNROLL * ROWS_PER_BLOCK, n_dst_rows) - 1;
    if (r_first / k == r_last / k) {
      uint32_t mk = 0, mv = 0;
      bool any = false;
#pragma unroll
      for (int u = 0; u < PC_GATHER_UNROLL; ++u) {
        const long long r = base + (long long)u * ROWS_PER_BLOCK;
        if (r < n_dst_rows && !skip[u]) { mk = max(mk, pc_piece_amax(kv[u])); mv = max(mv, pc_piece_amax(vv[u])); any = true; }
      }
#pragma unroll
      for (int off = PC_WAVE / 2; off > 0; off >>= 1) {
        mk = max(mk, (uint32_t)__shfl_xor((int)mk, off));
        mv = max(mv, (uint32_t)__shfl_xor((int)mv, off));
      }
      if (__any(any) && threadIdx.x % PC_WAVE == 0) {
        const long long bsg = r_first / k;
        if (mk) atomicMax(k_amax + bsg, mk << 16);
        if (mv) atomicMax(v_amax + bsg, mv << 16);
      }
    } else {
#pragma unroll
      for (int u = 0; u < PC_GATHER_UNROLL; ++u) {
        const long long r = base + (long long)u * ROWS_PER_BLOCK;
        if (r < n_dst_rows && !skip[u]) {
          const uint32_t mk = pc_piece_amax(kv[u]), mv = pc_piece_amax(vv[u]);
          if (mk) atomicMax(k_amax + r / k, mk << 16);
          if (mv) atomicMax(v_amax + r / k, mv << 16);
        }
      }
    }
  }
}

// zero the maxima of the segments the gather is about to fill (those with a source chunk)
__global__ void amax_clear_kernel(const int32_t* __restrict__ chunk_idx, long long n_bs, int n_kv_heads,
                                  uint32_t* __restrict__ k_amax, uint32_t* __restrict__ v_amax) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;      // (b, s, g)
  if (i >= n_bs * n_kv_heads) return;
  if (chunk_idx && chunk_idx[i / n_kv_heads] < 0) return;
  k_amax[i] = 0u; v_amax[i] = 0u;
}

int pc_launch_gather(const void* k_src, const void* v_src, const int32_t* chunk_idx,
                     const int32_t* tok_idx, int batch, int n_chunks, int rows, int n_sel,
                     int n_kv_heads, int k, int head_dim, void* k_dst, void* v_dst,
                     float* k_amax, float* v_amax, hipStream_t st) {
  const long long n_dst_rows = (long long)batch * n_sel * n_kv_heads * k;
  if (n_dst_rows == 0) return PC_OK;
  const bool amax = k_amax != nullptr;
  if (amax) {
    const long long n = (long long)batch * n_sel * n_kv_heads;
    hipLaunchKernelGGL(amax_clear_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, chunk_idx,
                       (long long)batch * n_sel, n_kv_heads, (uint32_t*)k_amax, (uint32_t*)v_amax);
    PC_LAUNCH_CHECK();
  }
  const int lanes = head_dim / 8;
  const int rows_per_block = (256 / lanes) * PC_GATHER_UNROLL;
  const long long blocks = (n_dst_rows + rows_per_block - 1) / rows_per_block;
  if (blocks > 0x7fffffffLL) return PC_ERR_SHAPE;
  dim3 grid((unsigned)blocks), block(256);
  PcProfScope prof(PC_KERNEL_GATHER, st);
#define PC_GATHER_LAUNCH(LANES, AMAX)                                                              \
  hipLaunchKernelGGL((gather_kv_kernel<LANES, AMAX>), grid, block, 0, st, (const uint4*)k_src,        \
                     (const uint4*)v_src, chunk_idx, tok_idx, (uint4*)k_dst, (uint4*)v_dst, n_chunks, \
                     rows, n_sel, n_kv_heads, k, n_dst_rows, (uint32_t*)k_amax, (uint32_t*)v_amax)
  if (lanes == 16) {
    if (amax) PC_GATHER_LAUNCH(16, true); else PC_GATHER_LAUNCH(16, false);
  } else {
    if (amax) PC_GATHER_LAUNCH(8, true); else PC_GATHER_LAUNCH(8, false);
  }
#undef PC_GATHER_LAUNCH
  PC_LAUNCH_CHECK();
  return PC_OK;
}
