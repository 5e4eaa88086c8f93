// Chunk self-information (Eq. 3):  I_c = -log P(X^q | X^c) = sum_t ( lse(logits[c, t, :]) - logits[c, t, target_t] )
// from the language model's logits for the query tokens after each chunk.  One streaming pass over
// the logits (HBM-bound: every logit is read once, 16 bytes per lane per load), online
// max / sum-of-exponentials per lane, then a fixed-order reduction over the workgroup, so the
// result does not depend on timing.  A second small kernel sums the per-token terms per chunk.
#include "pc_common.h"
#include <math.h>

#define PC_SI_THREADS 1024
#define PC_SI_LOG2E 1.4426950408889634f
#define PC_SI_LN2 0.6931471805599453f

// one workgroup per (chunk, token) row of `vocab` bf16 logits, vocab % 8 == 0
__global__ __launch_bounds__(PC_SI_THREADS) void self_info_rows_kernel(
    const uint16_t* __restrict__ logits, const int32_t* __restrict__ targets, int n_tokens,
    int vocab, float* __restrict__ token_nll) {
  __shared__ float red_m[PC_SI_THREADS / PC_WAVE], red_l[PC_SI_THREADS / PC_WAVE];
  const long long row = blockIdx.x;
  const int t = (int)(row % n_tokens);
  const uint16_t* src = logits + row * vocab;
  // running maximum m (log2 units) and sum l of 2^(x - m) over this lane's elements; four
  // independent 16-byte loads per round, one update of the running maximum per round
  float m = -INFINITY, l = 0.f;
  const int n_vec = vocab / 8;
  constexpr int U = 4;
  for (int i0 = threadIdx.x; i0 < n_vec; i0 += U * PC_SI_THREADS) {
    u32x4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * PC_SI_THREADS;
      // behind the row's end: the first vector again, masked below
      x[u] = __builtin_nontemporal_load((const u32x4*)(src + 8 * (long long)(i < n_vec ? i : i0)));
    }
    float f[U][8], vm = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = i0 + u * PC_SI_THREADS < n_vec;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f[u][2 * e] = in ? bf16_lo_to_f32(x[u][e]) : -INFINITY;
        f[u][2 * e + 1] = in ? bf16_hi_to_f32(x[u][e]) : -INFINITY;
      }
#pragma unroll
      for (int e = 0; e < 8; e += 2) vm = fmaxf(fmaxf(vm, f[u][e]), f[u][e + 1]);
    }
    const float m_new = fmaxf(m, vm * PC_SI_LOG2E);       // log2(e) > 0: the maximum commutes with it
    // a lane that has seen nothing but -inf logits so far (masked vocabulary entries) keeps
    // m = -inf, l = 0: the reference 0 turns its terms into exp2(-inf) = 0 instead of NaN
    const float ref = (m_new == -INFINITY) ? 0.f : m_new;
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) s += __builtin_amdgcn_exp2f(fmaf(f[u][e], PC_SI_LOG2E, -ref));
    l = ((m == -INFINITY) ? 0.f : l * __builtin_amdgcn_exp2f(m - m_new)) + s;
    m = m_new;
  }
  // fixed-order tree over the wavefront, then over the wavefronts
#pragma unroll
  for (int off = 1; off < PC_WAVE; off <<= 1) {
    const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
    const float mn = fmaxf(m, mo);
    const float a = (m == -INFINITY) ? 0.f : l * __builtin_amdgcn_exp2f(m - mn);
    const float b = (mo == -INFINITY) ? 0.f : lo * __builtin_amdgcn_exp2f(mo - mn);
    // both lanes of a pair must add in the same order to get the same bits: lower lane's term first
    l = ((threadIdx.x & off) == 0) ? a + b : b + a;
    m = mn;
  }
  const int wave = threadIdx.x / PC_WAVE;
  if (threadIdx.x % PC_WAVE == 0) { red_m[wave] = m; red_l[wave] = l; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = red_m[0], Lsum = red_l[0];
    for (int w = 1; w < PC_SI_THREADS / PC_WAVE; ++w) {
      const float mn = fmaxf(M, red_m[w]);
      const float a = (M == -INFINITY) ? 0.f : Lsum * __builtin_amdgcn_exp2f(M - mn);
      const float b = (red_m[w] == -INFINITY) ? 0.f : red_l[w] * __builtin_amdgcn_exp2f(red_m[w] - mn);
      Lsum = a + b; M = mn;
    }
    const int tgt = min(max(targets[t], 0), vocab - 1);
    const float xt = bf16_bits_to_f32(src[tgt]);
    token_nll[row] = (M + log2f(Lsum)) * PC_SI_LN2 - xt;
  }
}

// info[c] = (+/-) sum_t token_nll[c, t], summed in a fixed order
__global__ __launch_bounds__(256) void self_info_sum_kernel(const float* __restrict__ token_nll,
                                                            int n_tokens, float sign,
                                                            float* __restrict__ info) {
  __shared__ float red[256];
  const float* src = token_nll + (long long)blockIdx.x * n_tokens;
  float x = 0.f;
  for (int i = threadIdx.x; i < n_tokens; i += 256) x += src[i];
  red[threadIdx.x] = x;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) info[blockIdx.x] = sign * red[0];
}

int pc_launch_self_info(const void* logits, const int32_t* targets, int n_chunks, int n_tokens,
                        int vocab, int negate, float* token_nll, float* info, hipStream_t st) {
  {
    PcProfScope prof(PC_KERNEL_SELF_INFO, st);
    hipLaunchKernelGGL(self_info_rows_kernel, dim3((unsigned)(n_chunks * n_tokens)), dim3(PC_SI_THREADS),
                       0, st, (const uint16_t*)logits, targets, n_tokens, vocab, token_nll);
    PC_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(self_info_sum_kernel, dim3(n_chunks), dim3(256), 0, st, token_nll, n_tokens,
                     negate ? -1.0f : 1.0f, info);
  PC_LAUNCH_CHECK();
  return PC_OK;
}
