// Per-shot scores from the chunk masses, whole-shot selection under the token budget and the copy plan
// for compaction (Section 5.1, Eq. 3-6; Algorithm 1 phase 1: score every shot, rank by score, keep
// shots in descending order while the budget holds).  One workgroup per problem does all of it:
//
//   scores    Score(s_i) = (sum of the masses of the shot's chunks) / k_i;
//   ranking   bitonic sort in LDS on the key (score descending, shot index ascending);
//   budget    prefix sum of shot lengths in rank order (or the sequential first-fit walk);
//   plan      prefix sum of kept lengths in position order gives every retained row's output slot;
//             the original position of each output row is written in ascending order.
//
// The two halves can also run alone: scores only, or selection from caller-supplied scores.  All sums
// run in a fixed order (no atomics), so results are reproducible run to run.
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;

// block-wide exclusive scan over `n` ints stored in LDS array `a` (in place), returns the total.
// `tmp` is kSelWaves + 1 ints of LDS.
__device__ int block_exclusive_scan(int* a, int n, int* tmp) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int per = (n + kSelThreads - 1) / kSelThreads;
  const int lo = min(tid * per, n), hi = min(lo + per, n);
  int sum = 0;
  for (int i = lo; i < hi; ++i) sum += a[i];
  int incl = sum;  // inclusive scan of the per-thread sums inside the wave
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += up;
  }
  if (lane == kWave - 1) tmp[wave] = incl;
  __syncthreads();
  int before = 0, total = 0;
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = tmp[w];
    if (w < wave) before += t;
    total += t;
  }
  int run = before + incl - sum;
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

template <bool MASS, bool SELECT>
__global__ __launch_bounds__(kSelThreads) void reduce_select_kernel(
    const int32_t* __restrict__ seg_first, const float* __restrict__ chunk_mass, int max_c,
    float* __restrict__ shot_scores,
    const int32_t* __restrict__ shot_offsets, const int32_t* __restrict__ budget_tokens, int share,
    int n_shots, int n_tokens, int cap, int select_mode, int32_t* __restrict__ kept_count,
    uint8_t* __restrict__ shot_selected, int32_t* __restrict__ status,
    int32_t* __restrict__ kept_positions) {
  const int p = blockIdx.x, tid = threadIdx.x;
  const int lane = tid % kWave, wave = tid / kWave;
  const int32_t* off_g = shot_offsets + static_cast<size_t>(p / share) * (n_shots + 1);
  float* scores = shot_scores + static_cast<size_t>(p) * n_shots;

  __shared__ int s_off[SHOTKV_MAX_SHOTS + 1];
  __shared__ int s_a[SHOTKV_MAX_SHOTS + 2];   // shot scores (as float bits) while ranking, then the scan array
  __shared__ uint16_t s_idx[SHOTKV_MAX_SHOTS];
  __shared__ uint8_t s_keep[SHOTKV_MAX_SHOTS];
  __shared__ int s_tmp[kSelWaves + 1];
  __shared__ int s_flag;
  float* s_score = reinterpret_cast<float*>(s_a);

  // ---- shot boundaries into LDS, validated: 0 <= off[0], strictly increasing, off[n] <= n_tokens --
  if (tid == 0) s_flag = 0;
  __syncthreads();
  int local_bad = 0;
  for (int i = tid; i <= n_shots; i += kSelThreads) {
    const int o = off_g[i];
    s_off[i] = o;
    if (o < 0 || o > n_tokens) local_bad = 1;
    if (i > 0 && o <= off_g[i - 1]) local_bad = 1;
  }
  if (local_bad) atomicOr(&s_flag, 1);
  __syncthreads();
  const bool bad = s_flag != 0;

  // ---- Eq. 3: one score per shot from the masses of its chunks ----------------------------------
  if (MASS) {
    if (!bad) {
      const float* mass = chunk_mass + static_cast<size_t>(p) * max_c;
      const int32_t* sf = seg_first + static_cast<size_t>(p) * (n_shots + 3);
      for (int i = tid; i < n_shots; i += kSelThreads) {
        float sum = 0.f;
        for (int c = sf[i + 1]; c < sf[i + 2]; ++c) sum += mass[c];
        const float sc = sum / static_cast<float>(s_off[i + 1] - s_off[i]);
        scores[i] = sc;
        if (SELECT) s_score[i] = sc;
      }
    } else {
      for (int i = tid; i < n_shots; i += kSelThreads) scores[i] = 0.f;
    }
  } else if (!bad) {
    for (int i = tid; i < n_shots; i += kSelThreads) s_score[i] = scores[i];
  }
  if (!SELECT) return;

  uint8_t* sel = shot_selected ? shot_selected + static_cast<size_t>(p) * n_shots : nullptr;
  int32_t* kept_pos = kept_positions + static_cast<size_t>(p) * cap;
  int st = bad ? SHOTKV_ST_BAD_OFFSETS : SHOTKV_ST_OK;
  int shot_budget = 0, n_prefix = 0, n_tail = 0;
  if (st == SHOTKV_ST_OK) {
    n_prefix = s_off[0];
    n_tail = n_tokens - s_off[n_shots];
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
    if (i >= n_shots) s_score[i] = -INFINITY;
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

  // ---- budget walk in rank order (the scores are no longer needed: s_a becomes the scan array) ----
  for (int i = tid; i < n_shots; i += kSelThreads) {
    const int shot = s_idx[i];
    s_a[i] = s_off[shot + 1] - s_off[shot];
    s_keep[i] = 0;
  }
  __syncthreads();
  if (select_mode == SHOTKV_SELECT_PREFIX) {
    block_exclusive_scan(s_a, n_shots, s_tmp);
    // s_a[r] = tokens used by the shots ranked above r; lengths are positive, so the inclusive sums
    // are increasing and the kept ranks are exactly those whose inclusive sum fits
    for (int r = tid; r < n_shots; r += kSelThreads) {
      const int shot = s_idx[r];
      const int inclusive = s_a[r] + (s_off[shot + 1] - s_off[shot]);
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
    else if (s == n_seg - 1) { src = s_off[n_shots]; len = n_tail; }
    else { src = s_off[s - 1]; len = s_keep[s - 1] ? (s_off[s] - s_off[s - 1]) : 0; }
  };
  for (int s = tid; s < n_seg; s += kSelThreads) {
    int src, len;
    segment(s, src, len);
    s_a[s] = len;
  }
  __syncthreads();
  const int total = block_exclusive_scan(s_a, n_seg, s_tmp);  // s_a[s] = first output row of segment s
  // every retained row's original position; one wave per segment, lanes along the rows
  for (int s = wave; s < n_seg; s += kSelWaves) {
    int src, len;
    segment(s, src, len);
    const int dst = s_a[s];
    for (int i = lane; i < len; i += kWave) kept_pos[dst + i] = src + i;
  }
  if (sel) for (int i = tid; i < n_shots; i += kSelThreads) sel[i] = s_keep[i];
  if (tid == 0) { status[p] = SHOTKV_ST_OK; kept_count[p] = total; }
}

}  // namespace

hipError_t launch_reduce_select(const PrefillDims& d, bool with_mass, bool with_select, float* shot_scores,
                                const int32_t* shot_offsets, const int32_t* budget_tokens, int cap,
                                int32_t* kept_count, uint8_t* shot_selected, int32_t* status,
                                int32_t* kept_positions, const PrefillWorkspace& w, hipStream_t s) {
  KernelTimer timer(d.timing, kKernelReduceSelect, s);
#define SHOTKV_LAUNCH_RS(M, S)                                                                          \
  hipLaunchKernelGGL((reduce_select_kernel<M, S>), dim3(d.P), dim3(kSelThreads), 0, s, w.seg_first,     \
                     w.chunk_mass, w.max_c, shot_scores,                                                \
                     shot_offsets, budget_tokens, d.share, d.n_shots, d.n_tokens, cap, d.select_mode,   \
                     kept_count, shot_selected, status, kept_positions)
  if (with_mass && with_select) SHOTKV_LAUNCH_RS(true, true);
  else if (with_mass) SHOTKV_LAUNCH_RS(true, false);
  else if (with_select) SHOTKV_LAUNCH_RS(false, true);
  else return hipErrorInvalidValue;
#undef SHOTKV_LAUNCH_RS
  return hipGetLastError();
}

}  // namespace shotkv
