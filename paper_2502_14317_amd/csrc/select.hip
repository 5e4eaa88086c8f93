// Top-k selection of chunks (Eq. 3-4: a fixed number of best chunks) and of tokens per KV
// head (Eq. 7), under the total order (score descending, index ascending): of equal scores
// the lower index wins.  Scores are mapped to unsigned keys whose integer order is the float
// order, so every comparison is exact integer work.
#include "pc_common.h"
#include <atomic>

// ------------------------------------------------------------------------------------------
// Chunks: n <= 4096.  One workgroup; rank by counting.  rank(i) = #{j : key_j > key_i or
// (key_j == key_i and j < i)}; item i is kept iff rank(i) < k and lands at out[rank(i)].
__global__ __launch_bounds__(256) void select_chunks_kernel(const float* __restrict__ score, int n,
                                                            int k, int32_t* __restrict__ out_idx,
                                                            float* __restrict__ out_score) {
  __shared__ uint32_t keys[4096];
  for (int i = threadIdx.x; i < n; i += blockDim.x) keys[i] = pc_order_key(score[i]);
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const uint32_t ki = keys[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const uint32_t kj = keys[j];
      rank += (kj > ki) || (kj == ki && j < i);
    }
    if (rank < k) {
      out_idx[rank] = i;
      if (out_score) out_score[rank] = score[i];
    }
  }
}

int pc_launch_select_chunks(const float* score, int n, int k, int32_t* out_idx, float* out_score,
                            hipStream_t st) {
  PcProfScope prof(PC_KERNEL_SELECT_CHUNKS, st);
  hipLaunchKernelGGL(select_chunks_kernel, dim3(1), dim3(256), 0, st, score, n, k, out_idx,
                     out_score);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
// The fixed-size priority queue of chunks (sec. 3.1 "Chunk eviction"), updated with one batch
// of newly encoded chunks.  The queue lives on the device: ids in rank order (-1 = empty
// entry), their scores, and the KV slot each entry owns.  One workgroup ranks the resident
// entries and the batch together by counting, under (score descending, earlier chunk first;
// NaN lowest, empty entries last); the best `cap` stay.  A chunk that stays keeps its slot; the
// entrants, in rank order, take the free slots in ascending order.  slot_src[s] names, for the
// later selection / gather launches, the batch-local index of the chunk that enters slot s, or
// -1 where the slot keeps its content.
#define PC_QUEUE_MAX 1024              // capacity and batch size limit (each)
__global__ __launch_bounds__(256) void chunk_queue_kernel(
    const float* __restrict__ batch_score, int n_batch, int chunk_id0, int cap,
    int32_t* __restrict__ queue_id, float* __restrict__ queue_score,
    int32_t* __restrict__ queue_slot, int32_t* __restrict__ slot_src) {
  __shared__ uint32_t key[2 * PC_QUEUE_MAX];
  __shared__ int32_t id[2 * PC_QUEUE_MAX], slot[2 * PC_QUEUE_MAX];
  __shared__ float val[2 * PC_QUEUE_MAX];
  __shared__ int32_t new_id[PC_QUEUE_MAX], new_slot[PC_QUEUE_MAX];
  __shared__ float new_val[PC_QUEUE_MAX];
  __shared__ uint8_t used[PC_QUEUE_MAX];
  const int n = cap + n_batch;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    if (i < cap) {
      id[i] = queue_id[i]; val[i] = queue_score[i]; slot[i] = queue_slot[i];
    } else {
      id[i] = chunk_id0 + (i - cap); val[i] = batch_score[i - cap]; slot[i] = -1;
    }
    key[i] = pc_order_key(val[i]);
  }
  for (int i = threadIdx.x; i < cap; i += blockDim.x) { new_id[i] = -1; new_slot[i] = -1; new_val[i] = 0.f; used[i] = 0; slot_src[i] = -1; }
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    if (id[i] < 0) continue;                                   // an empty entry ranks behind every chunk
    const uint32_t ki = key[i];
    const int ii = id[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const uint32_t kj = key[j];
      rank += (id[j] >= 0) && ((kj > ki) || (kj == ki && id[j] < ii));
    }
    if (rank < cap) {
      new_id[rank] = ii; new_val[rank] = val[i]; new_slot[rank] = slot[i];
      if (slot[i] >= 0 && slot[i] < cap) used[slot[i]] = 1;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int f = 0;                                                  // next candidate free slot
    for (int r = 0; r < cap; ++r) {
      if (new_id[r] < 0 || new_slot[r] >= 0) continue;          // empty, or a resident chunk
      while (f < cap && used[f]) ++f;
      if (f >= cap) break;                                      // cannot happen: at most cap entries hold slots
      new_slot[r] = f; used[f] = 1;
      slot_src[f] = new_id[r] - chunk_id0;
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < cap; i += blockDim.x) {
    queue_id[i] = new_id[i]; queue_score[i] = new_val[i]; queue_slot[i] = new_slot[i];
  }
}

int pc_launch_chunk_queue(const float* batch_score, int n_batch, int chunk_id0, int cap,
                          int32_t* queue_id, float* queue_score, int32_t* queue_slot,
                          int32_t* slot_src, hipStream_t st) {
  PcProfScope prof(PC_KERNEL_CHUNK_QUEUE, st);
  hipLaunchKernelGGL(chunk_queue_kernel, dim3(1), dim3(256), 0, st, batch_score, n_batch, chunk_id0,
                     cap, queue_id, queue_score, queue_slot, slot_src);
  PC_LAUNCH_CHECK();
  return PC_OK;
}

// ------------------------------------------------------------------------------------------
// Tokens: one workgroup per (selected chunk, KV head).  The n keys sit in LDS.
//  1. Radix select, 4 passes of 8 bits from the top: after the passes T is the k-th largest
//     key and `need_eq` the number of keys equal to T that still fit (1 <= need_eq).
//  2. Ordered compaction: each wavefront owns a contiguous index range; it counts its keys
//     above T and equal to T, the counts are prefix-summed over wavefronts, and a second sweep
//     emits index i iff key_i > T, or key_i == T and fewer than need_eq equal keys precede it.
//     Output is ascending by construction and ties go to the lower index.
// Attention calibration (Eq. 8) is a predicate on the keys: a token of the position class
// [cls_lo, cls_hi) whose score is above lambda gets key 0, below every candidate (a NaN score
// is a candidate with key 1), and k shrinks to the number of candidates when fewer are left;
// the unused tail of the output is filled with -1 and the kept count is reported.
#define PC_SEL_THREADS 512
#define PC_SEL_WAVES (PC_SEL_THREADS / PC_WAVE)

__global__ __launch_bounds__(PC_SEL_THREADS) void select_tokens_kernel(
    const float* __restrict__ tok_score, const int32_t* __restrict__ chunk_idx, int n_kv_heads,
    int n, int k, float lambda, int cls_lo, int cls_hi, const int32_t* __restrict__ chunk_lens,
    int32_t* __restrict__ out_idx, int32_t* __restrict__ out_cnt) {
  extern __shared__ uint32_t keys[];   // n
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_bin, sh_need, sh_evicted;
  __shared__ uint32_t wave_tot[256 / PC_WAVE];
  __shared__ uint32_t wave_gt[PC_SEL_WAVES], wave_eq[PC_SEL_WAVES];

  const int s = blockIdx.x / n_kv_heads;
  const int g = blockIdx.x % n_kv_heads;
  const int c = chunk_idx ? chunk_idx[s] : s;
  if (c < 0) return;                               // no chunk for this entry: its outputs stay as they are
  const float* src = tok_score + ((long long)c * n_kv_heads + g) * n;
  int32_t* dst = out_idx + (long long)blockIdx.x * k;

  const int n_valid = chunk_lens ? min(max(chunk_lens[c], 0), n) : n;   // a short chunk has fewer tokens
  if (threadIdx.x == 0) sh_evicted = 0;
  __syncthreads();
  uint32_t my_evicted = 0;
  for (int i = threadIdx.x; i < n; i += PC_SEL_THREADS) {
    const float x = src[i];
    uint32_t key = pc_order_key(x);
    key = key == 0u ? 1u : key;
    if ((i >= cls_lo && i < cls_hi && x > lambda) || i >= n_valid) { key = 0u; ++my_evicted; }
    keys[i] = key;
  }
  if (my_evicted) atomicAdd(&sh_evicted, my_evicted);
  __syncthreads();
  const int k_eff = min(k, n - (int)sh_evicted);
  for (int i = k_eff + threadIdx.x; i < k; i += PC_SEL_THREADS) dst[i] = -1;
  if (threadIdx.x == 0 && out_cnt) out_cnt[blockIdx.x] = k_eff;
  if (k_eff == 0) return;                          // uniform over the workgroup

  uint32_t prefix = 0, mask = 0, need = (uint32_t)k_eff;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (threadIdx.x < 256) hist[threadIdx.x] = 0;
    __syncthreads();
    // Histogram of the next 8 bits over the keys that still match the prefix.  Scores of one
    // chunk are close to each other, so in the upper passes nearly all keys of a wavefront fall
    // into one bin: the lanes that share the first active lane's bin are counted with a ballot
    // and added once, the others add one each.
    for (int i0 = 0; i0 < n; i0 += PC_SEL_THREADS) {
      const int i = i0 + threadIdx.x;
      const uint32_t key = i < n ? keys[i] : 0u;
      const bool live = i < n && (key & mask) == prefix;
      const uint32_t bin = (key >> shift) & 255u;
      const unsigned long long todo = __ballot(live);
      if (todo) {
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t lead_bin = (uint32_t)__shfl((int)bin, leader);
        const bool with_leader = live && bin == lead_bin;
        const unsigned long long same = __ballot(with_leader);
        if ((int)(threadIdx.x % PC_WAVE) == leader) atomicAdd(&hist[lead_bin], (uint32_t)__popcll(same));
        if (live && !with_leader) atomicAdd(&hist[bin], 1u);
      }
    }
    __syncthreads();
    // The bin that holds the need-th largest key: every bin's count of keys above it by a
    // suffix sum over the 256 bins (4 wavefronts x 64 bins), instead of one thread walking them.
    {
      const int t = threadIdx.x, ln = t % PC_WAVE;
      const uint32_t h = t < 256 ? hist[t] : 0u;
      uint32_t suf = h;                              // inclusive suffix sum inside the wavefront
#pragma unroll
      for (int off = 1; off < PC_WAVE; off <<= 1) {
        const uint32_t up = (uint32_t)__shfl_down((int)suf, off);
        if (ln + off < PC_WAVE) suf += up;
      }
      if (t < 256 && ln == 0) wave_tot[t / PC_WAVE] = suf;
      __syncthreads();
      if (t < 256) {
        uint32_t above = suf - h;                    // keys in higher bins
        for (int w = t / PC_WAVE + 1; w < 256 / PC_WAVE; ++w) above += wave_tot[w];
        if (h > 0 && above < need && above + h >= need) { sh_bin = (uint32_t)t; sh_need = need - above; }
      }
    }
    __syncthreads();
    prefix |= sh_bin << shift;
    mask |= 255u << shift;
    need = sh_need;
  }
  const uint32_t T = prefix;       // k-th largest key
  const uint32_t need_eq = need;   // how many keys equal to T are admitted

  const int wave = threadIdx.x / PC_WAVE, lane = threadIdx.x % PC_WAVE;
  const int per_wave = ((n + PC_SEL_WAVES - 1) / PC_SEL_WAVES + PC_WAVE - 1) / PC_WAVE * PC_WAVE;
  const int begin = wave * per_wave;
  const int end = min(n, begin + per_wave);

  uint32_t cnt_gt = 0, cnt_eq = 0;
  for (int i0 = begin; i0 < end; i0 += PC_WAVE) {
    const int i = i0 + lane;
    const uint32_t key = (i < end) ? keys[i] : 0u;
    const bool gt = (i < end) && key > T, eq = (i < end) && key == T;
    cnt_gt += (uint32_t)__popcll(__ballot(gt));
    cnt_eq += (uint32_t)__popcll(__ballot(eq));
  }
  if (lane == 0) { wave_gt[wave] = cnt_gt; wave_eq[wave] = cnt_eq; }
  __syncthreads();
  uint32_t base_gt = 0, base_eq = 0;
  for (int w = 0; w < wave; ++w) { base_gt += wave_gt[w]; base_eq += wave_eq[w]; }

  for (int i0 = begin; i0 < end; i0 += PC_WAVE) {
    const int i = i0 + lane;
    const uint32_t key = (i < end) ? keys[i] : 0u;
    const bool gt = (i < end) && key > T, eq = (i < end) && key == T;
    const unsigned long long bg = __ballot(gt), be = __ballot(eq);
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    const uint32_t gt_before = base_gt + (uint32_t)__popcll(bg & below);
    const uint32_t eq_before = base_eq + (uint32_t)__popcll(be & below);
    if (gt || (eq && eq_before < need_eq)) {
      const uint32_t pos = gt_before + min(eq_before, need_eq);
      dst[pos] = i;
    }
    base_gt += (uint32_t)__popcll(bg);
    base_eq += (uint32_t)__popcll(be);
  }
}

int pc_launch_select_tokens(const float* tok_score, const int32_t* chunk_idx, int n_sel,
                            int n_kv_heads, int chunk_len, int k, float lambda, int cls_lo,
                            int cls_hi, const int32_t* chunk_lens, int32_t* out_idx,
                            int32_t* out_cnt, hipStream_t st) {
  const size_t lds = (size_t)chunk_len * sizeof(uint32_t);
  if (lds > 48 * 1024) {      // raised once per device, to the largest chunk the entry point accepts
    static std::atomic<uint64_t> raised{0};
    const int rc = pc_raise_dynamic_lds((const void*)select_tokens_kernel, 32768 * (int)sizeof(uint32_t), raised);
    if (rc != PC_OK) return rc;
  }
  PcProfScope prof(PC_KERNEL_SELECT_TOKENS, st);
  hipLaunchKernelGGL(select_tokens_kernel, dim3(n_sel * n_kv_heads), dim3(PC_SEL_THREADS), lds, st,
                     tok_score, chunk_idx, n_kv_heads, chunk_len, k, lambda, cls_lo, cls_hi,
                     chunk_lens, out_idx, out_cnt);
  PC_LAUNCH_CHECK();
  return PC_OK;
}
