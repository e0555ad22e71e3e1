// Whole-shot selection under the token budget and the copy plan for compaction
// (Section 5.1, Eq. 5-6; Algorithm 1 phase 1: rank by score, keep shots in descending order while the
// budget holds).  One workgroup per problem; ranking is a bitonic sort in LDS on the key
// (score descending, shot index ascending), the budget walk is a prefix sum of shot lengths in rank
// order, and the copy plan - the original position of every retained row, ascending - comes from a
// prefix sum of kept lengths in position order.
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kSelThreads = 256;

// block-wide exclusive scan over `n` ints stored in LDS array `a` (in place), returns the total.
// `tmp` is kSelThreads ints of LDS.
__device__ int block_exclusive_scan(int* a, int n, int* tmp) {
  const int tid = threadIdx.x;
  const int per = (n + kSelThreads - 1) / kSelThreads;
  const int lo = min(tid * per, n), hi = min(lo + per, n);
  int sum = 0;
  for (int i = lo; i < hi; ++i) sum += a[i];
  tmp[tid] = sum;
  __syncthreads();
  for (int o = 1; o < kSelThreads; o <<= 1) {
    const int add = (tid >= o) ? tmp[tid - o] : 0;
    __syncthreads();
    tmp[tid] += add;
    __syncthreads();
  }
  const int total = tmp[kSelThreads - 1];
  int run = tmp[tid] - sum;
  for (int i = lo; i < hi; ++i) {
    const int v = a[i];
    a[i] = run;
    run += v;
  }
  __syncthreads();
  return total;
}

__device__ __forceinline__ bool ranks_before(float sa, int ia, float sb, int ib) {
  return (sa > sb) || (sa == sb && ia < ib);
}

__global__ __launch_bounds__(kSelThreads) void select_plan_kernel(
    const float* __restrict__ shot_scores, const int32_t* __restrict__ shot_offsets,
    const int32_t* __restrict__ budget_tokens, int share, int n_shots, int n_tokens, int window, int cap,
    int select_mode, int32_t* __restrict__ kept_count, uint8_t* __restrict__ shot_selected,
    int32_t* __restrict__ status, int32_t* __restrict__ kept_positions) {
  const int p = blockIdx.x, tid = threadIdx.x;
  const int32_t* off = shot_offsets + static_cast<size_t>(p / share) * (n_shots + 1);
  const float* scores = shot_scores + static_cast<size_t>(p) * n_shots;
  uint8_t* sel = shot_selected ? shot_selected + static_cast<size_t>(p) * n_shots : nullptr;
  int32_t* kept_pos = kept_positions + static_cast<size_t>(p) * cap;

  __shared__ float s_score[SHOTKV_MAX_SHOTS];
  __shared__ uint16_t s_idx[SHOTKV_MAX_SHOTS];
  __shared__ int s_a[SHOTKV_MAX_SHOTS + 2];    // scan array
  __shared__ uint8_t s_keep[SHOTKV_MAX_SHOTS];
  __shared__ int s_tmp[kSelThreads];
  __shared__ int s_flag;

  // ---- validation (same rules as the chunk planner, so this kernel can run on its own) ---------
  if (tid == 0) s_flag = 0;
  __syncthreads();
  int local_bad = 0;
  for (int i = tid; i <= n_shots; i += kSelThreads) {
    const int o = off[i];
    if (o < 0 || o > n_tokens) local_bad = 1;
    if (i > 0 && o <= off[i - 1]) local_bad = 1;
  }
  if (local_bad) atomicOr(&s_flag, 1);
  __syncthreads();
  int st = s_flag ? SHOTKV_ST_BAD_OFFSETS : SHOTKV_ST_OK;
  int shot_budget = 0, n_prefix = 0, n_tail = 0;
  if (st == SHOTKV_ST_OK) {
    n_prefix = off[0];
    n_tail = n_tokens - off[n_shots];
    shot_budget = min(budget_tokens[p / share], cap) - n_prefix - n_tail;
    if (shot_budget < 0) st = SHOTKV_ST_BUDGET_TOO_SMALL;
  }
  if (st != SHOTKV_ST_OK) {
    if (tid == 0) { status[p] = st; kept_count[p] = 0; }
    if (sel) for (int i = tid; i < n_shots; i += kSelThreads) sel[i] = 0;
    return;
  }

  // ---- rank: bitonic sort of (score, index) ------------------------------------------------------
  int n_pad = 1;
  while (n_pad < n_shots) n_pad <<= 1;
  for (int i = tid; i < n_pad; i += kSelThreads) {
    s_score[i] = (i < n_shots) ? scores[i] : -INFINITY;
    s_idx[i] = static_cast<uint16_t>(i);  // padding carries indices >= n_shots, so it ranks after every real -inf score
  }
  __syncthreads();
  for (int size = 2; size <= n_pad; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < (n_pad >> 1); t += kSelThreads) {
        const int lo = ((t / stride) * stride << 1) + (t % stride);
        const int hi = lo + stride;
        const bool ascending = ((lo & size) == 0);  // "ascending" = rank order
        const float sa = s_score[lo], sb = s_score[hi];
        const int ia = s_idx[lo], ib = s_idx[hi];
        const bool in_order = ranks_before(sa, ia, sb, ib);
        if (in_order != ascending) {
          s_score[lo] = sb; s_score[hi] = sa;
          s_idx[lo] = static_cast<uint16_t>(ib); s_idx[hi] = static_cast<uint16_t>(ia);
        }
      }
      __syncthreads();
    }
  }

  // ---- budget walk in rank order ------------------------------------------------------------------
  for (int i = tid; i < n_shots; i += kSelThreads) {
    const int shot = s_idx[i];
    s_a[i] = off[shot + 1] - off[shot];
    s_keep[i] = 0;
  }
  __syncthreads();
  if (select_mode == SHOTKV_SELECT_PREFIX) {
    block_exclusive_scan(s_a, n_shots, s_tmp);
    // s_a[r] = tokens used by the shots ranked above r; lengths are positive, so the inclusive sums
    // are increasing and the kept ranks are exactly those whose inclusive sum fits
    for (int r = tid; r < n_shots; r += kSelThreads) {
      const int shot = s_idx[r];
      const int inclusive = s_a[r] + (off[shot + 1] - off[shot]);
      if (inclusive <= shot_budget) s_keep[shot] = 1;
    }
  } else if (tid == 0) {  // first-fit: inherently sequential over the ranking
    int used = 0;
    for (int r = 0; r < n_shots; ++r) {
      const int shot = s_idx[r];
      const int len = s_a[r];
      if (used + len <= shot_budget) { used += len; s_keep[shot] = 1; }
    }
  }
  __syncthreads();

  // ---- copy plan in position order: segment 0 = prefix, 1..n = shots, n+1 = tail ----------------
  const int n_seg = n_shots + 2;
  auto segment = [&](int s, int& src, int& len) {
    if (s == 0) { src = 0; len = n_prefix; }
    else if (s == n_seg - 1) { src = off[n_shots]; len = n_tail; }
    else { src = off[s - 1]; len = s_keep[s - 1] ? (off[s] - off[s - 1]) : 0; }
  };
  for (int s = tid; s < n_seg; s += kSelThreads) {
    int src, len;
    segment(s, src, len);
    s_a[s] = len;
  }
  __syncthreads();
  const int total = block_exclusive_scan(s_a, n_seg, s_tmp);  // s_a[s] = first output row of segment s
  // every retained row's original position; one wave per segment, lanes along the rows
  for (int s = tid / kWave; s < n_seg; s += kSelThreads / kWave) {
    int src, len;
    segment(s, src, len);
    const int dst = s_a[s];
    for (int i = tid % kWave; i < len; i += kWave) kept_pos[dst + i] = src + i;
  }
  if (sel) for (int i = tid; i < n_shots; i += kSelThreads) sel[i] = s_keep[i];
  if (tid == 0) { status[p] = SHOTKV_ST_OK; kept_count[p] = total; }
}

}  // namespace

hipError_t launch_select_plan(const PrefillDims& d, const float* shot_scores,
                              const int32_t* shot_offsets, const int32_t* budget_tokens, int cap,
                              int32_t* kept_count, uint8_t* shot_selected, int32_t* status,
                              int32_t* kept_positions, hipStream_t s) {
  KernelTimer timer(kKernelSelect, s);
  hipLaunchKernelGGL(select_plan_kernel, dim3(d.P), dim3(kSelThreads), 0, s, shot_scores, shot_offsets,
                     budget_tokens, d.share, d.n_shots, d.n_tokens, d.W, cap, d.select_mode, kept_count,
                     shot_selected, status, kept_positions);
  return hipGetLastError();
}

}  // namespace shotkv
