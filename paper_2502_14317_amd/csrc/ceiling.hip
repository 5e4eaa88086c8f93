// Measurement aid: what the matrix pipe of this machine sustains, to put the attention kernel's
// roofline fraction in context.  A loop of nothing but independent 32x32x16 bf16 MFMAs, two
// wavefronts per SIMD on every CU, on constant or on random operands (the shader clock, and with
// it the throughput, depends on how many bits toggle: the part is power-limited).  A third mode
// adds, per MFMA, what a flash-attention loop cannot avoid at 32 queries per wavefront: one
// 16-byte-per-lane LDS read that supplies the A operand and one softmax element on the vector ALU
// (exponential, add, multiply).  Its throughput is the power-limited ceiling of that instruction
// mix, whatever the schedule.
#include "pc_common.h"

__device__ __forceinline__ uint32_t pc_mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

template <int RND, int MIX>
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(float* out, int iters) {
  __shared__ u32x4 lds_ops[MIX ? 2048 : 1];   // 32 KiB of random operands, read by every wavefront
  if (MIX) {
    for (int i = threadIdx.x; i < 2048; i += 512) {
      u32x4 x;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t h = pc_mix(i * 4 + e + blockIdx.x * 977u);
        x[e] = (h & 0x807f807fu) | 0x3f003f00u | ((h >> 3) & 0x00800080u);
      }
      lds_ops[i] = x;
    }
    __syncthreads();
  }
  float xv[8], xsum = 0.f;                    // softmax-like elements in [-4.2, 0)
#pragma unroll
  for (int r = 0; r < 8; ++r) xv[r] = -(float)(pc_mix(threadIdx.x * 8 + r) & 1023) * (4.f / 1024.f);
  const int lane = threadIdx.x & 63;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    u32x4 x, y;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (RND) {   // bf16 pairs with random sign and mantissa, magnitude in [0.5, 2)
        const uint32_t h1 = pc_mix(threadIdx.x * 131u + j * 17u + e + blockIdx.x * 7919u), h2 = pc_mix(h1 + 12345u);
        x[e] = (h1 & 0x807f807fu) | 0x3f003f00u | ((h1 >> 3) & 0x00800080u);
        y[e] = (h2 & 0x807f807fu) | 0x3f003f00u | ((h2 >> 3) & 0x00800080u);
      } else {
        x[e] = 0x3f803f80u; y[e] = 0x3f803f80u;   // 1.0
      }
    }
    a[j] = *(bf16x8*)&x; b[j] = *(bf16x8*)&y;
  }
  floatx16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      if (MIX) {
        const u32x4 t = lds_ops[lane + (((it * 8 + m) & 31) << 6)];
        a[m & 3] = *(const bf16x8*)&t;
      }
      acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m & 3], b[(m + (m >> 2)) & 3], acc[m], 0, 0, 0);
      if (MIX) {
        const float p = __builtin_amdgcn_exp2f(xv[m]);
        xsum += p;
        xv[m] = p * -4.2f;
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  float s = xsum;
#pragma unroll
  for (int r = 0; r < 8; ++r) s += xv[r];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

extern "C" int pc_mfma_ceiling(int mode, int n_cus, int iters, float* scratch,
                               size_t scratch_bytes, double* flops, void* stream) {
  if (!scratch || !flops) return PC_ERR_NULL;
  if (mode < 0 || mode > 2 || n_cus < 1 || n_cus > 4096 || iters < 1 || iters > (1 << 22)) return PC_ERR_SHAPE;
  if (scratch_bytes < (size_t)n_cus * 512 * sizeof(float)) return PC_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  if (mode == 2) hipLaunchKernelGGL((mfma_ceiling_kernel<1, 1>), dim3(n_cus), dim3(512), 0, st, scratch, iters);
  else if (mode == 1) hipLaunchKernelGGL((mfma_ceiling_kernel<1, 0>), dim3(n_cus), dim3(512), 0, st, scratch, iters);
  else hipLaunchKernelGGL((mfma_ceiling_kernel<0, 0>), dim3(n_cus), dim3(512), 0, st, scratch, iters);
  PC_LAUNCH_CHECK();
  *flops = (double)n_cus * 8.0 /* wavefronts */ * 8.0 * iters * 32768.0;
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
// Copy ceiling: what a bare read-and-write loop sustains, to put the gather's fraction of the
// HBM peak in context.  Every thread moves 16-byte pieces, four loads in flight, a wavefront
// covering 1 KiB of consecutive bytes per instruction; mode 0 ordinary loads and stores, mode 1
// with the non-temporal hint on both sides (the gather's own instructions).
template <int NT>
__global__ __launch_bounds__(256) void copy_ceiling_kernel(const u32x4* __restrict__ src,
                                                           u32x4* __restrict__ dst, long long n) {
  const long long stride = (long long)gridDim.x * 256;
  for (long long i0 = (long long)blockIdx.x * 256 + threadIdx.x; i0 < n; i0 += 4 * stride) {
    u32x4 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long i = i0 + u * stride;
      if (i < n) x[u] = NT ? __builtin_nontemporal_load(src + i) : src[i];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long i = i0 + u * stride;
      if (i < n) { if (NT) __builtin_nontemporal_store(x[u], dst + i); else dst[i] = x[u]; }
    }
  }
}

extern "C" int pc_copy_ceiling(int mode, const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return PC_ERR_NULL;
  if (mode < 0 || mode > 1 || bytes < 16 || bytes % 16 != 0 || !pc_aligned(src, 16) || !pc_aligned(dst, 16))
    return PC_ERR_SHAPE;
  const long long n = (long long)(bytes / 16);
  long long blocks = (n + 4 * 256 - 1) / (4 * 256);
  if (blocks > 8192) blocks = 8192;                       // 32 workgroups per CU, grid-stride beyond
  hipStream_t st = (hipStream_t)stream;
  if (mode == 1) hipLaunchKernelGGL(copy_ceiling_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, st, (const u32x4*)src, (u32x4*)dst, n);
  else hipLaunchKernelGGL(copy_ceiling_kernel<0>, dim3((unsigned)blocks), dim3(256), 0, st, (const u32x4*)src, (u32x4*)dst, n);
  PC_LAUNCH_CHECK();
  return PC_OK;
}
