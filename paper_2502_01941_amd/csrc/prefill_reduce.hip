// Segmented per-shot reduction of the softmax partials (Section 5.1, Eq. 3).
//
//   row_stats   : per (problem, KV head, query row) log2 of the softmax denominator over all chunks
//   chunk_mass  : per (problem, chunk) the attention mass sum_{heads, rows} 2^(lse_chunk - lse_row)
//   shot_scores : Score(s_i) = (sum of the masses of the shot's chunks) / k_i
// All sums are in fixed order (no atomics), so results are reproducible run to run.
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kStatThreads = 1024;

// log2(2^a + 2^b) style accumulation of (max, sum) with a partial given as log2 of a sum
__device__ __forceinline__ void lse_accumulate(float& M, float& L, float x) {
  if (x > -INFINITY) {
    const float Mn = fmaxf(M, x);
    L = L * exp2f(M - Mn) + exp2f(x - Mn);
    M = Mn;
  }
}

__global__ __launch_bounds__(kStatThreads) void row_stats_kernel(const float* __restrict__ partial,
                                                                 const int32_t* __restrict__ n_chunks,
                                                                 int H_kv, int R, int max_c,
                                                                 float* __restrict__ row_stat) {
  const int g = blockIdx.x, p = blockIdx.y;
  const int nl = kStatThreads / R;  // chunk lanes
  const int tid = threadIdx.x;
  const int r = tid % R, cl = tid / R;
  const int nc = n_chunks[p];
  const float* base = partial + (static_cast<size_t>(p) * H_kv + g) * max_c * R;
  float M = -INFINITY, L = 0.f;
  if (cl < nl)
    for (int c = cl; c < nc; c += nl) lse_accumulate(M, L, base[static_cast<size_t>(c) * R + r]);
  __shared__ float sM[kStatThreads];
  __shared__ float sL[kStatThreads];
  sM[tid] = M;
  sL[tid] = L;
  __syncthreads();
  if (tid < R) {
    float Mt = -INFINITY, Lt = 0.f;
    for (int i = 0; i < nl; ++i) {
      const float m = sM[i * R + tid], l = sL[i * R + tid];
      if (l > 0.f) {
        const float Mn = fmaxf(Mt, m);
        Lt = Lt * exp2f(Mt - Mn) + l * exp2f(m - Mn);
        Mt = Mn;
      }
    }
    // log2 of the row's softmax denominator; +inf for a row without keys so that its weights vanish
    row_stat[(static_cast<size_t>(p) * H_kv + g) * R + tid] = Lt > 0.f ? Mt + log2f(Lt) : INFINITY;
  }
}

constexpr int kMassThreads = 256;

__global__ __launch_bounds__(kMassThreads) void chunk_mass_kernel(const float* __restrict__ partial,
                                                                  const float* __restrict__ row_stat,
                                                                  const int32_t* __restrict__ n_chunks,
                                                                  int H_kv, int R, int max_c,
                                                                  float* __restrict__ chunk_mass) {
  const int p = blockIdx.y;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int c = blockIdx.x * (kMassThreads / kWave) + wave;
  if (c >= n_chunks[p]) return;
  const float* stat = row_stat + static_cast<size_t>(p) * H_kv * R;
  float acc = 0.f;
  for (int g = 0; g < H_kv; ++g) {
    const float* part = partial + ((static_cast<size_t>(p) * H_kv + g) * max_c + c) * R;
    for (int r = lane; r < R; r += kWave) acc += exp2f(part[r] - stat[g * R + r]);  // 2^-inf = 0
  }
  acc = wave_sum(acc);
  if (lane == 0) chunk_mass[static_cast<size_t>(p) * max_c + c] = acc;
}

__global__ void shot_scores_kernel(const float* __restrict__ chunk_mass,
                                   const int32_t* __restrict__ seg_first,
                                   const int32_t* __restrict__ shot_offsets,
                                   const int32_t* __restrict__ status, int share, int n_shots,
                                   int max_c, float* __restrict__ shot_scores) {
  const int p = blockIdx.y;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_shots) return;
  float score = 0.f;
  if (status[p] == SHOTKV_ST_OK) {
    const int32_t* sf = seg_first + static_cast<size_t>(p) * (n_shots + 3);
    const int32_t* off = shot_offsets + static_cast<size_t>(p / share) * (n_shots + 1);
    const float* mass = chunk_mass + static_cast<size_t>(p) * max_c;
    float sum = 0.f;
    for (int c = sf[i + 1]; c < sf[i + 2]; ++c) sum += mass[c];
    score = sum / static_cast<float>(off[i + 1] - off[i]);
  }
  shot_scores[static_cast<size_t>(p) * n_shots + i] = score;
}

}  // namespace

hipError_t launch_reduce_scores(const PrefillDims& d, const int32_t* shot_offsets,
                                const int32_t* status, float* shot_scores, const PrefillWorkspace& w,
                                hipStream_t s) {
  {
    KernelTimer timer(kKernelRowStats, s);
    hipLaunchKernelGGL(row_stats_kernel, dim3(d.H_kv, d.P), dim3(kStatThreads), 0, s, w.partial,
                       w.n_chunks, d.H_kv, d.R, w.max_c, w.row_stat);
  }
  {
    KernelTimer timer(kKernelChunkMass, s);
    hipLaunchKernelGGL(chunk_mass_kernel, dim3(ceil_div(w.max_c, kMassThreads / kWave), d.P),
                       dim3(kMassThreads), 0, s, w.partial, w.row_stat, w.n_chunks, d.H_kv, d.R,
                       w.max_c, w.chunk_mass);
  }
  if (d.n_shots > 0) {
    KernelTimer timer(kKernelShotScores, s);
    hipLaunchKernelGGL(shot_scores_kernel, dim3(ceil_div(d.n_shots, 256), d.P), dim3(256), 0, s,
                       w.chunk_mass, w.seg_first, shot_offsets, status, d.share, d.n_shots, w.max_c,
                       shot_scores);
  }
  return hipGetLastError();
}

}  // namespace shotkv
