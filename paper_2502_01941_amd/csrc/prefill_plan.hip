// Chunk planning for the prefill score pass (Section 5.1, Eq. 3: shots are the pooling units).
//
// The key range [0, n_tokens) of a problem is cut into segments - the region before the first shot,
// each shot, the region after the last shot - and every segment into chunks of at most chunk_keys
// keys.  Because a chunk never crosses a shot boundary, the score pass needs no per-key segment
// bookkeeping: a chunk's softmax partial belongs to one shot or to the always-kept region.
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / kWave;

__device__ __forceinline__ void segment_span(const int32_t* off, int n_shots, int n_tokens, int s,
                                             int& start, int& len) {
  // s = 0: prefix, 1..n: shots, n+1: tail
  const int lo = (s == 0) ? 0 : off[s - 1];
  const int hi = (s == n_shots + 1) ? n_tokens : off[s];
  start = lo;
  len = hi - lo;
}

__device__ __forceinline__ int chunks_of(int len, int chunk_keys) {
  return len <= 0 ? 0 : (len + chunk_keys - 1) / chunk_keys;
}

__device__ __forceinline__ int chunk_stride(int len, int nc) {
  // equal split rounded up to whole 32-key blocks; never more than chunk_keys because
  // len <= nc * chunk_keys and chunk_keys is a multiple of 32
  const int per = (len + nc - 1) / nc;
  return (per + 31) & ~31;
}

__global__ __launch_bounds__(kPlanThreads) void plan_chunks_kernel(
    const int32_t* __restrict__ shot_offsets, int share, int n_shots, int n_tokens, int chunk_keys, int max_c,
    int32_t* __restrict__ status, int32_t* __restrict__ n_chunks, int32_t* __restrict__ chunk_start,
    int32_t* __restrict__ chunk_len, int32_t* __restrict__ seg_first, int group_keys, int n_groups,
    int32_t* __restrict__ group_first, uint32_t* __restrict__ v_absmax, int n_kv_heads) {
  const int p = blockIdx.x;
  const int tid = threadIdx.x;
  const int32_t* off = shot_offsets + static_cast<size_t>(p / share) * (n_shots + 1);
  int32_t* c_start = chunk_start + static_cast<size_t>(p) * max_c;
  int32_t* c_len = chunk_len + static_cast<size_t>(p) * max_c;
  int32_t* s_first = seg_first + static_cast<size_t>(p) * (n_shots + 3);

  __shared__ int bad;
  __shared__ int wave_total[kPlanWaves];
  if (tid == 0) bad = 0;
  // the fused attention path collects the largest |v| of every KV-head plane with atomic maxima: start at 0
  if (v_absmax && tid < n_kv_heads) v_absmax[static_cast<size_t>(p) * n_kv_heads + tid] = 0u;
  __syncthreads();

  // validation: 0 <= off[0], off strictly increasing, off[n] <= n_tokens
  int local_bad = 0;
  for (int i = tid; i <= n_shots; i += kPlanThreads) {
    const int o = off[i];
    if (o < 0 || o > n_tokens) local_bad = 1;
    if (i > 0 && o <= off[i - 1]) local_bad = 1;
  }
  if (local_bad) atomicOr(&bad, 1);
  __syncthreads();
  int32_t* g_first = group_first ? group_first + static_cast<size_t>(p) * (n_groups + 1) : nullptr;
  if (bad) {
    if (tid == 0) { status[p] = SHOTKV_ST_BAD_OFFSETS; n_chunks[p] = 0; }
    for (int s = tid; s < n_shots + 3; s += kPlanThreads) s_first[s] = 0;
    if (g_first)
      for (int gi = tid; gi <= n_groups; gi += kPlanThreads) g_first[gi] = 0;
    return;
  }
  if (tid == 0) status[p] = SHOTKV_ST_OK;

  const int n_seg = n_shots + 2;
  const int lane = tid % kWave, wave = tid / kWave;
  int carry = 0;  // chunks of the segments before this tile; the same in every thread
  for (int base = 0; base < n_seg; base += kPlanThreads) {
    const int s = base + tid;
    int start = 0, len = 0, nc = 0;
    if (s < n_seg) {
      segment_span(off, n_shots, n_tokens, s, start, len);
      nc = chunks_of(len, chunk_keys);
    }
    // inclusive scan of nc over the tile: lane shuffles inside a wave, wave totals through LDS
    int incl = nc;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(incl, o, kWave);
      if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) wave_total[wave] = incl;
    __syncthreads();
    int before = 0, tile_total = 0;
#pragma unroll
    for (int w = 0; w < kPlanWaves; ++w) {
      const int t = wave_total[w];
      if (w < wave) before += t;
      tile_total += t;
    }
    const int first = carry + before + incl - nc;
    if (s < n_seg) {
      s_first[s] = first;
      if (nc > 0) {
        const int per = chunk_stride(len, nc);
        for (int j = 0; j < nc; ++j) {
          c_start[first + j] = start + j * per;
          c_len[first + j] = min(per, len - j * per);
        }
      }
    }
    carry += tile_total;
    __syncthreads();  // wave_total is rewritten by the next tile; the chunk table is complete after the last
  }
  if (tid == 0) {
    s_first[n_seg] = carry;
    n_chunks[p] = carry;
  }
  if (g_first) {
    // Group g of the score pass owns the chunks that start in key slice [g * group_keys, (g + 1) *
    // group_keys): group_first[g] = first chunk starting at or after the slice's first key.  Chunk
    // starts increase, so chunk c opens every group after its predecessor's up to its own.
    const int nc = carry;  // final since the barrier that ended the loop above
    for (int c = tid; c <= nc; c += kPlanThreads) {
      const int g_hi = (c < nc) ? c_start[c] / group_keys : n_groups;
      const int g_lo = (c == 0) ? 0 : c_start[c - 1] / group_keys + 1;
      for (int gi = g_lo; gi <= g_hi; ++gi) g_first[gi] = c;
    }
  }
}

}  // namespace

hipError_t launch_plan_chunks(const PrefillDims& d, const int32_t* shot_offsets, int32_t* status,
                              const PrefillWorkspace& w, hipStream_t s) {
  KernelTimer timer(d.timing, kKernelPlan, s);
  hipLaunchKernelGGL(plan_chunks_kernel, dim3(d.P), dim3(kPlanThreads), 0, s, shot_offsets, d.share, d.n_shots,
                     d.n_tokens, w.chunk_keys, w.max_c, status, w.n_chunks, w.chunk_start, w.chunk_len,
                     w.seg_first, w.group_keys, w.n_groups, w.group_first, w.v_absmax, d.H_kv);
  return hipGetLastError();
}

}  // namespace shotkv
