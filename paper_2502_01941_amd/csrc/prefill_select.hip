// Per-shot scores from the chunk masses, whole-shot selection under the token budget and the copy plan
// for compaction (Section 5.1, Eq. 3-6; Algorithm 1 phase 1: score every shot, rank by score, keep
// shots in descending order while the budget holds).  One workgroup per problem does all of it:
//
//   scores    Score(s_i) = (sum of the masses of the shot's chunks) / k_i;
//   ranking   bitonic sort on one 64-bit key per shot (score descending, shot index ascending): keys
//             live in registers, partners less than 64 apart are exchanged between lanes without LDS
//             (DPP moves inside a row of 16, row and half swaps beyond), and for the larger strides the keys pass through LDS into a transposed layout in which
//             those strides are lane distances too - two LDS round trips per merge level instead of
//             one per compare-exchange step;
//   budget    prefix sum of shot lengths in rank order (or the sequential first-fit walk);
//   plan      prefix sum of kept lengths in position order gives every retained row's output slot;
//             the original position of each output row is written in ascending order.
//
// The two halves can also run alone: scores only, or selection from caller-supplied scores.  All sums
// run in a fixed order (no atomics), so results are reproducible run to run.
#include "common.hpp"

#include <type_traits>

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

constexpr int kMaxPad = SHOTKV_MAX_SHOTS;            // keys sorted at most (a power of two)
constexpr int kKeySlots = kMaxPad + kMaxPad / 64;    // one pad slot per 64 keys: transposed reads hit all banks
static_assert((kMaxPad & (kMaxPad - 1)) == 0 && kMaxPad <= 4 * kSelThreads, "up to four keys per thread");

// One key per shot whose descending order is the ranking: score descending, then index ascending.
// The float's bits are mapped to an unsigned integer with the same order (-0 ranks with +0); entry i
// of the padding (i >= n_shots) gets the smallest score word and therefore ranks after every shot.
__device__ __forceinline__ uint64_t rank_key(float score, int idx) {
  uint32_t b = __float_as_uint(score);
  if ((b << 1) == 0u) b = 0u;
  const uint32_t u = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return (static_cast<uint64_t>(u) << 32) | (0xFFFFFFFFu - static_cast<uint32_t>(idx));
}
__device__ __forceinline__ uint64_t padding_key(int idx) { return 0xFFFFFFFFu - static_cast<uint32_t>(idx); }

// Value of lane (own lane ^ MASK), MASK a power of two below 64, without a trip through the LDS pipe:
// data-parallel-primitive moves inside a row of 16 lanes (1, 2: quad permutations; 4: the mirror of 8
// lanes followed by the mirror of 4; 8: a rotation of the row by 8), row swaps for 16 and half swaps for 32.
template <int MASK>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
  static_assert(MASK == 1 || MASK == 2 || MASK == 4 || MASK == 8 || MASK == 16 || MASK == 32, "one lane bit");
  if constexpr (MASK == 1) {
    return __builtin_amdgcn_update_dpp(0u, v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  } else if constexpr (MASK == 2) {
    return __builtin_amdgcn_update_dpp(0u, v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  } else if constexpr (MASK == 4) {
    const uint32_t m = __builtin_amdgcn_update_dpp(0u, v, 0x141, 0xf, 0xf, false);  // row_half_mirror: lane ^ 7
    return __builtin_amdgcn_update_dpp(0u, m, 0x1B, 0xf, 0xf, false);               // quad_perm [3,2,1,0]: ^ 3
  } else if constexpr (MASK == 8) {
    return __builtin_amdgcn_update_dpp(0u, v, 0x128, 0xf, 0xf, false);  // row_ror:8
  } else if constexpr (MASK == 16) {
    // first result: own even rows, the other operand's even rows in the odd rows; second: the odd rows
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return (threadIdx.x & 16) ? r[0] : r[1];
  } else {
    // first result: the lower half in both halves; second: the upper half in both
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (threadIdx.x & 32) ? r[0] : r[1];
  }
}

template <int MASK>
__device__ __forceinline__ uint64_t lane_xor64(uint64_t v) {
  const uint32_t lo = lane_xor<MASK>(static_cast<uint32_t>(v));
  const uint32_t hi = lane_xor<MASK>(static_cast<uint32_t>(v >> 32));
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// Sorts n_pad keys (a power of two, 64 <= n_pad <= E * 1024) into descending order.  Thread tid holds
// array elements tid + 1024 * j in k[j]; on return k[j] is the key of rank tid + 1024 * j.  All 1024
// threads must call it (barriers); threads whose elements lie past n_pad carry dummies.
// Layouts: "natural" - element t = tid + 1024 j is array index t; "transposed" - it is array index
// ((t mod 2^hb) << 6) | (t >> hb) with hb = log2(n_pad) - 6, which puts index bits 6.. on the low lane
// bits.  keys[] holds kKeySlots entries; array index a lives in slot a + a/64.  With n_pad <= 2048 two
// alternating buffers make one barrier per layout change enough; 4096 keys need a second one.
template <int E>
__device__ void sort_keys_descending(uint64_t (&k)[E], int n_pad, uint64_t* keys) {
  const int tid = threadIdx.x;
  const int hb = (31 - __clz(n_pad)) - 6;
  const int low_mask = (1 << hb) - 1;
  const int second = n_pad <= kMaxPad / 2 ? kKeySlots / 2 : 0;
  int buf = 0;
  auto natural = [&](int j) { return tid + kSelThreads * j; };
  auto transposed = [&](int j) {
    const int t = tid + kSelThreads * j;
    return ((t & low_mask) << 6) | (t >> hb);
  };
  auto slot = [](int a) { return a + (a >> 6); };
  // one compare-exchange step with the partner LANE_MASK lanes away: array distance LANE_MASK in the
  // natural layout, 64 * LANE_MASK in the transposed one
  auto stage = [&](int size, auto lane_mask_c, bool in_transposed) {
    constexpr int LANE_MASK = decltype(lane_mask_c)::value;
    const int stride = in_transposed ? LANE_MASK << 6 : LANE_MASK;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const int a = in_transposed ? transposed(j) : natural(j);
      const uint64_t other = lane_xor64<LANE_MASK>(k[j]);
      const bool want_max = ((a & size) == 0) == ((a & stride) == 0);
      const bool take = want_max ? other > k[j] : other < k[j];
      k[j] = take ? other : k[j];
    }
  };
  // the steps of one merge level whose partners are at most `top` lanes away, widest first
  auto lane_stages = [&](int size, int top, bool in_transposed) {
    if (top >= 32) stage(size, std::integral_constant<int, 32>{}, in_transposed);
    if (top >= 16) stage(size, std::integral_constant<int, 16>{}, in_transposed);
    if (top >= 8) stage(size, std::integral_constant<int, 8>{}, in_transposed);
    if (top >= 4) stage(size, std::integral_constant<int, 4>{}, in_transposed);
    if (top >= 2) stage(size, std::integral_constant<int, 2>{}, in_transposed);
    stage(size, std::integral_constant<int, 1>{}, in_transposed);
  };
  auto relayout = [&](bool to_transposed) {
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const int t = natural(j);
      if (t < n_pad) keys[buf + slot(to_transposed ? t : transposed(j))] = k[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const int t = natural(j);
      if (t < n_pad) k[j] = keys[buf + slot(to_transposed ? transposed(j) : t)];
    }
    if (second) buf ^= second;
    else __syncthreads();
  };
  for (int size = 2; size <= n_pad; size <<= 1) {
    if (size > kWave) {
      relayout(true);
      lane_stages(size, size >> 7, true);   // array distances size/2 .. 64
      relayout(false);
    }
    lane_stages(size, min(size >> 1, kWave / 2), false);
  }
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
  const int32_t* off_g = shot_offsets + static_cast<size_t>(p / share) * (n_shots + 1);
  float* scores = shot_scores + static_cast<size_t>(p) * n_shots;

  __shared__ int s_off[SHOTKV_MAX_SHOTS + 1];
  __shared__ uint64_t s_key[kKeySlots];       // the sort's exchange buffer, then (as ints) the scan array
  __shared__ uint16_t s_idx[SHOTKV_MAX_SHOTS];
  __shared__ uint8_t s_keep[SHOTKV_MAX_SHOTS];
  __shared__ int s_tmp[kSelWaves + 1];
  __shared__ int s_flag;
  int* s_a = reinterpret_cast<int*>(s_key);   // SHOTKV_MAX_SHOTS + 2 ints
  static_assert(sizeof(uint64_t) * kKeySlots >= sizeof(int) * (SHOTKV_MAX_SHOTS + 2), "scan array fits");

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
  // thread tid takes shots tid, tid + 1024, ...: the layout the sort starts from
  constexpr int kMaxPerThread = kMaxPad / kSelThreads;
  float my_score[kMaxPerThread];
#pragma unroll
  for (int j = 0; j < kMaxPerThread; ++j) {
    const int i = tid + kSelThreads * j;
    my_score[j] = 0.f;
    if (i >= n_shots) continue;
    if (MASS) {
      if (!bad) {
        const float* mass = chunk_mass + static_cast<size_t>(p) * max_c;
        const int32_t* sf = seg_first + static_cast<size_t>(p) * (n_shots + 3);
        float sum = 0.f;
        for (int c = sf[i + 1]; c < sf[i + 2]; ++c) sum += mass[c];
        my_score[j] = sum / static_cast<float>(s_off[i + 1] - s_off[i]);
      }
      scores[i] = my_score[j];
    } else if (!bad) {
      my_score[j] = scores[i];
    }
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

  // ---- rank: sort one key per shot, descending ----------------------------------------------------
  int n_pad = kWave;
  while (n_pad < n_shots) n_pad <<= 1;
  {
    uint64_t key[kMaxPerThread];
#pragma unroll
    for (int j = 0; j < kMaxPerThread; ++j) {
      const int i = tid + kSelThreads * j;
      key[j] = i < n_shots ? rank_key(my_score[j], i) : padding_key(i);
    }
    if (n_pad <= kSelThreads) {
      uint64_t k1[1] = {key[0]};
      sort_keys_descending<1>(k1, n_pad, s_key);
      key[0] = k1[0];
    } else if (n_pad <= 2 * kSelThreads) {
      uint64_t k2[2] = {key[0], key[1]};
      sort_keys_descending<2>(k2, n_pad, s_key);
      key[0] = k2[0];
      key[1] = k2[1];
    } else {
      sort_keys_descending<kMaxPerThread>(key, n_pad, s_key);
    }
#pragma unroll
    for (int j = 0; j < kMaxPerThread; ++j) {
      const int r = tid + kSelThreads * j;  // rank
      if (r < n_shots) s_idx[r] = static_cast<uint16_t>(0xFFFFFFFFu - static_cast<uint32_t>(key[j]));
    }
  }
  __syncthreads();  // the ranking is complete, and the exchange buffer is free to become the scan array

  // ---- budget walk in rank order ---------------------------------------------------------------------
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
  // every retained row's original position: a group of lanes per segment, lanes along the rows; the
  // group is as wide as an average shot is long (a wave for shots of hundreds of tokens, 8..32 lanes for
  // sentence-sized units), so that most lanes have a row to write
  int group_w = 8;
  {
    const int avg = n_shots > 0 ? (s_off[n_shots] - s_off[0]) / n_shots : kWave;
    while (group_w < kWave && group_w < avg) group_w <<= 1;
  }
  const int n_groups = kSelThreads / group_w, gid = tid / group_w, gl = tid % group_w;
  constexpr int kSegBatch = 4;  // segments whose LDS lookups are in flight together
  for (int s0 = gid; s0 < n_seg; s0 += n_groups * kSegBatch) {
    int src[kSegBatch], len[kSegBatch], dst[kSegBatch];
#pragma unroll
    for (int b = 0; b < kSegBatch; ++b) {
      const int s = s0 + b * n_groups;
      src[b] = 0; len[b] = 0; dst[b] = 0;
      if (s < n_seg) {
        segment(s, src[b], len[b]);
        dst[b] = s_a[s];
      }
    }
#pragma unroll
    for (int b = 0; b < kSegBatch; ++b)
      for (int i = gl; i < len[b]; i += group_w) kept_pos[dst[b] + i] = src[b] + i;
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
