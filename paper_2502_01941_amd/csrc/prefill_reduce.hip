// Normalisation of the window-softmax partials (Section 5.1, Eq. 3).
//
//   row_stats  : per (problem, KV head, query row) the log2 of the softmax denominator over all of the
//                row's keys, combined from the per-workgroup statistics the score kernel wrote
//   chunk_mass : per (problem, chunk) the attention mass sum_{heads, rows} 2^(lse_chunk - lse_row)
// All sums are in fixed order (no atomics), so results are reproducible run to run.
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kStatThreads = 1024;

__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(const float* __restrict__ group_stat,
                                                                 const int32_t* __restrict__ n_chunks,
                                                                 int H_kv, int R, size_t problem_stride,
                                                                 size_t head_stride, size_t group_stride,
                                                                 int n_groups,
                                                                 float* __restrict__ row_stat) {
  const int g = blockIdx.x, p = blockIdx.y;
  const int nl = kStatThreads / R;  // group lanes
  const int tid = threadIdx.x;
  const int r = tid % R, gl = tid / R;
  // entries to combine: every score workgroup's statistic (-inf from one without chunks), or on the
  // generic path the partial of every chunk
  const int ng = n_groups > 0 ? (n_chunks[p] > 0 ? n_groups : 0) : n_chunks[p];
  const float* base = group_stat + p * problem_stride + g * head_stride;
  // two passes over the lane's share (second one out of cache): the maximum first, then the sum of
  // 2^(x - max) with independent loads
  float M = -INFINITY;
  if (gl < nl)
    for (int c = gl; c < ng; c += nl) M = fmaxf(M, base[c * group_stride + r]);
  float L = 0.f;
  if (gl < nl && M > -INFINITY)
    for (int c = gl; c < ng; c += nl) L += exp2f(base[c * group_stride + r] - M);  // 2^-inf = 0
  __shared__ float sM[kStatThreads];
  __shared__ float sL[kStatThreads];
  sM[tid] = M;
  sL[tid] = L;
  __syncthreads();
  if (tid < R) {
    float Mt = -INFINITY;
    for (int i = 0; i < nl; ++i) Mt = fmaxf(Mt, sM[i * R + tid]);
    float Lt = 0.f;
    if (Mt > -INFINITY)
      for (int i = 0; i < nl; ++i) Lt += sL[i * R + tid] * exp2f(sM[i * R + tid] - Mt);
    // log2 of the row's softmax denominator; +inf for a row without keys so that its weights vanish
    row_stat[(static_cast<size_t>(p) * H_kv + g) * R + tid] = Lt > 0.f ? Mt + log2f(Lt) : INFINITY;
  }
}

constexpr int kMassThreads = 256;
constexpr int kMassWaves = kMassThreads / kWave;
constexpr int kMassPerWave = 4;  // chunks a wave has in flight
constexpr int kMassPerBlock = kMassWaves * kMassPerWave;

__global__ __launch_bounds__(kMassThreads) void chunk_mass_kernel(const float* __restrict__ partial,
                                                                  const float* __restrict__ row_stat,
                                                                  const int32_t* __restrict__ n_chunks,
                                                                  int H_kv, int R, int max_c,
                                                                  float* __restrict__ chunk_mass) {
  const int p = blockIdx.y;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int c0 = blockIdx.x * kMassPerBlock + wave;  // this wave's chunks: c0, c0 + kMassWaves, ...
  const int nc = n_chunks[p];
  if (blockIdx.x * kMassPerBlock >= nc) return;
  // a chunk's statistics of all KV heads are contiguous and line up with the row denominators
  const float* stat = row_stat + static_cast<size_t>(p) * H_kv * R;
  const int E = H_kv * R;
  float acc[kMassPerWave];
#pragma unroll
  for (int j = 0; j < kMassPerWave; ++j) acc[j] = 0.f;
  for (int e = lane; e < E; e += kWave) {
    const float st = stat[e];
    float x[kMassPerWave];
#pragma unroll
    for (int j = 0; j < kMassPerWave; ++j) {  // independent loads first
      const int c = min(c0 + j * kMassWaves, nc - 1);
      x[j] = partial[(static_cast<size_t>(p) * max_c + c) * E + e];
    }
#pragma unroll
    for (int j = 0; j < kMassPerWave; ++j) acc[j] += exp2f(x[j] - st);  // 2^-inf = 0
  }
#pragma unroll
  for (int j = 0; j < kMassPerWave; ++j) {
    const float total = wave_sum(acc[j]);
    const int c = c0 + j * kMassWaves;
    if (lane == 0 && c < nc) chunk_mass[static_cast<size_t>(p) * max_c + c] = total;
  }
}

}  // namespace

hipError_t launch_chunk_mass(const PrefillDims& d, const PrefillWorkspace& w, hipStream_t s) {
  KernelTimer timer(d.timing, kKernelChunkMass, s);
  hipLaunchKernelGGL(chunk_mass_kernel, dim3(ceil_div(w.max_c, kMassPerBlock), d.P), dim3(kMassThreads), 0, s,
                     w.partial, w.row_stat, w.n_chunks, d.H_kv, d.R, w.max_c, w.chunk_mass);
  return hipGetLastError();
}

hipError_t launch_row_stats(const PrefillDims& d, const PrefillWorkspace& w, hipStream_t s) {
  KernelTimer timer(d.timing, kKernelRowStats, s);
  // per-workgroup statistics are [P][H_kv][n_groups][R]; without them (one chunk per score workgroup)
  // the per-chunk partials [P][max_c][H_kv][R] are read in their place
  const bool own = w.group_stat != w.partial;
  const size_t R = d.R, heads = d.H_kv;
  const size_t problem_stride = own ? heads * w.n_groups * R : static_cast<size_t>(w.max_c) * heads * R;
  const size_t head_stride = own ? w.n_groups * R : R;
  const size_t group_stride = own ? R : heads * R;
  hipLaunchKernelGGL(row_stats_kernel, dim3(d.H_kv, d.P), dim3(kStatThreads), 0, s, w.group_stat, w.n_chunks,
                     d.H_kv, d.R, problem_stride, head_stride, group_stride, own ? w.n_groups : 0, w.row_stat);
  return hipGetLastError();
}

}  // namespace shotkv
