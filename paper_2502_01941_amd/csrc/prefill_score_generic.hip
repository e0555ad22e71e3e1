// Window-attention softmax partials, shape-generic path (Section 5.1, Eq. 3: alpha_{t,h}).
//
// One workgroup takes one chunk of at most 64 keys of one KV head and, for each of the R = G*W query
// rows attached to that head, produces the chunk-local softmax statistic log2(sum of exponentials)
// (logits in the log2 domain).  The global normalisation happens in the reduction kernels.  This path serves
// fp32 inputs and shapes the matrix-core kernel does not cover; it is plain vector arithmetic.
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxD = 128;

template <typename T>
__global__ __launch_bounds__(kThreads) void score_partials_generic_kernel(
    const T* __restrict__ q_obs, const T* __restrict__ k, int n_tokens, int H, int H_kv, int G, int D,
    int W, float scale_log2e, const int32_t* __restrict__ n_chunks,
    const int32_t* __restrict__ chunk_start, const int32_t* __restrict__ chunk_len, int max_c,
    float* __restrict__ partial) {
  const int c = blockIdx.x, g = blockIdx.y, p = blockIdx.z;
  if (c >= n_chunks[p]) return;
  const int start = chunk_start[static_cast<size_t>(p) * max_c + c];
  const int len = chunk_len[static_cast<size_t>(p) * max_c + c];
  const int R = G * W;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;

  __shared__ float ks[kChunkKeysGeneric * (kMaxD + 1)];
  const T* kbase = k + (static_cast<size_t>(p) * H_kv + g) * n_tokens * D + static_cast<size_t>(start) * D;
  for (int idx = tid; idx < len * D; idx += kThreads) {
    const int key = idx / D, dd = idx - key * D;
    ks[key * (D + 1) + dd] = to_f32(kbase[idx]);
  }
  __syncthreads();

  const T* qbase = q_obs + (static_cast<size_t>(p) * H + static_cast<size_t>(g) * G) * W * D;
  float* out = partial + ((static_cast<size_t>(p) * max_c + c) * H_kv + g) * R;
  for (int r = wave; r < R; r += kThreads / kWave) {
    const int j = r % W;
    const int last_visible = n_tokens - W + j;  // the query's own position
    const T* qrow = qbase + static_cast<size_t>(r) * D;
    float z = -INFINITY;
    if (lane < len && start + lane <= last_visible) {
      float acc = 0.f;
      const float* krow = ks + lane * (D + 1);
      for (int dd = 0; dd < D; ++dd) acc = fmaf(to_f32(qrow[dd]), krow[dd], acc);
      z = acc * scale_log2e;
    }
    const float m = wave_max(z);
    const float e = (z == -INFINITY) ? 0.f : exp2f(z - m);
    const float l = wave_sum(e);
    if (lane == 0) out[r] = (m == -INFINITY) ? -INFINITY : m + log2f(l);  // log2 sum_k 2^z_k
  }
}

}  // namespace

hipError_t launch_score_partials_generic(const PrefillDims& d, const void* q_obs, const void* k,
                                         const PrefillWorkspace& w, hipStream_t s) {
  const dim3 grid(w.max_c, d.H_kv, d.P), block(kThreads);
  const float c = d.sm_scale * kLog2e;
  KernelTimer timer(d.timing, kKernelScore, s);
  if (d.dtype == SHOTKV_BF16) {
    hipLaunchKernelGGL(score_partials_generic_kernel<bf16_t>, grid, block, 0, s,
                       static_cast<const bf16_t*>(q_obs), static_cast<const bf16_t*>(k), d.n_tokens,
                       d.H, d.H_kv, d.G, d.D, d.W, c, w.n_chunks, w.chunk_start, w.chunk_len, w.max_c,
                       w.partial);
  } else {
    hipLaunchKernelGGL(score_partials_generic_kernel<float>, grid, block, 0, s,
                       static_cast<const float*>(q_obs), static_cast<const float*>(k), d.n_tokens, d.H,
                       d.H_kv, d.G, d.D, d.W, c, w.n_chunks, w.chunk_start, w.chunk_len, w.max_c,
                       w.partial);
  }
  return hipGetLastError();
}

}  // namespace shotkv
