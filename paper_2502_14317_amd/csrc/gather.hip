// KV compaction gather (Eq. 7: K_r = K_x[kept], V_r = V_x[kept]).
//
// HBM-bound byte copy.  One head row is D bf16 = 128 or 256 bytes; a lane moves one 16-byte
// piece of a K row and the matching piece of the V row, so D/8 adjacent lanes read one
// contiguous row and a wavefront writes 1 KiB of contiguous destination per store.  Each
// thread handles PC_GATHER_UNROLL rows so that several independent loads are in flight.  Both
// sides are touched once, so loads and stores carry the non-temporal hint (64 -> 70 % of peak).
#include "pc_common.h"

#define PC_GATHER_UNROLL 4

template <int LANES_PER_ROW>
__global__ __launch_bounds__(256) void gather_kv_kernel(
    const uint4* __restrict__ k_src, const uint4* __restrict__ v_src,
    const int32_t* __restrict__ chunk_idx, const int32_t* __restrict__ tok_idx,
    uint4* __restrict__ k_dst, uint4* __restrict__ v_dst,
    int n_chunks, int rows, int n_sel, int n_kv_heads, int k, long long n_dst_rows) {
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
}

int pc_launch_gather(const void* k_src, const void* v_src, const int32_t* chunk_idx,
                     const int32_t* tok_idx, int batch, int n_chunks, int rows, int n_sel,
                     int n_kv_heads, int k, int head_dim, void* k_dst, void* v_dst,
                     hipStream_t st) {
  const long long n_dst_rows = (long long)batch * n_sel * n_kv_heads * k;
  if (n_dst_rows == 0) return PC_OK;
  const int lanes = head_dim / 8;
  const int rows_per_block = (256 / lanes) * PC_GATHER_UNROLL;
  const long long blocks = (n_dst_rows + rows_per_block - 1) / rows_per_block;
  if (blocks > 0x7fffffffLL) return PC_ERR_SHAPE;
  dim3 grid((unsigned)blocks), block(256);
  PcProfScope prof(PC_KERNEL_GATHER, st);
  if (lanes == 16) {
    hipLaunchKernelGGL(gather_kv_kernel<16>, grid, block, 0, st, (const uint4*)k_src,
                       (const uint4*)v_src, chunk_idx, tok_idx, (uint4*)k_dst, (uint4*)v_dst,
                       n_chunks, rows, n_sel, n_kv_heads, k, n_dst_rows);
  } else {
    hipLaunchKernelGGL(gather_kv_kernel<8>, grid, block, 0, st, (const uint4*)k_src,
                       (const uint4*)v_src, chunk_idx, tok_idx, (uint4*)k_dst, (uint4*)v_dst,
                       n_chunks, rows, n_sel, n_kv_heads, k, n_dst_rows);
  }
  PC_LAUNCH_CHECK();
  return PC_OK;
}
