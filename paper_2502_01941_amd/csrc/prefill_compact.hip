// Gather-compaction of the retained K/V rows into the dense compressed cache
// (Section 5.1, Eq. 4: KV^C_prefill = Compress({s_i in S*}); Section 3: compression keeps a subset of
// the original rows, so this is a bit-exact copy).
//
// Destination-centric: a workgroup owns kRowsPerBlock consecutive output rows of one (problem, KV
// head, K-or-V) plane, finds each row's source through the copy plan (runs sorted by destination) and
// moves it with 16-byte lanes, so stores are fully coalesced and loads are contiguous within a run.
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kCopyThreads = 256;
constexpr int kRowsPerBlock = 64;

// index of the last run whose destination start is <= row
__device__ __forceinline__ int find_run(const int32_t* __restrict__ run_dst, int n_runs, int row) {
  int lo = 0, hi = n_runs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (run_dst[mid] <= row) lo = mid; else hi = mid - 1;
  }
  return lo;
}

template <int kRowBytes>
__global__ __launch_bounds__(kCopyThreads) void compact_kernel(
    const char* __restrict__ k, const char* __restrict__ v, char* __restrict__ k_out,
    char* __restrict__ v_out, int n_tokens, int H_kv, int cap, const int32_t* __restrict__ kept_count,
    const int32_t* __restrict__ n_runs, const int32_t* __restrict__ run_src,
    const int32_t* __restrict__ run_dst, int max_runs, int32_t* __restrict__ kept_positions) {
  constexpr int kLanesPerRow = kRowBytes / 16;
  constexpr int kRowsPerPass = kCopyThreads / kLanesPerRow;
  const int g = blockIdx.y;
  const int p = blockIdx.z >> 1;
  const bool is_v = blockIdx.z & 1;
  const int kept = kept_count[p];
  const int row0 = blockIdx.x * kRowsPerBlock;
  if (row0 >= kept) return;
  const int nr = n_runs[p];
  const int32_t* r_src = run_src + static_cast<size_t>(p) * max_runs;
  const int32_t* r_dst = run_dst + static_cast<size_t>(p) * max_runs;
  const char* src_plane = (is_v ? v : k) + (static_cast<size_t>(p) * H_kv + g) * n_tokens * kRowBytes;
  char* dst_plane = (is_v ? v_out : k_out) + (static_cast<size_t>(p) * H_kv + g) * cap * kRowBytes;
  const int sub = threadIdx.x / kLanesPerRow;
  const int lane = threadIdx.x % kLanesPerRow;

  constexpr int kPasses = kRowsPerBlock / kRowsPerPass;
  int src_row[kPasses];
  uint4 data[kPasses];
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int row = row0 + i * kRowsPerPass + sub;
    src_row[i] = -1;
    if (row < kept) {
      const int r = find_run(r_dst, nr, row);
      src_row[i] = r_src[r] + (row - r_dst[r]);
    }
  }
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    if (src_row[i] >= 0)
      data[i] = *reinterpret_cast<const uint4*>(src_plane + static_cast<size_t>(src_row[i]) * kRowBytes +
                                                lane * 16);
  }
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int row = row0 + i * kRowsPerPass + sub;
    if (src_row[i] >= 0) {
      *reinterpret_cast<uint4*>(dst_plane + static_cast<size_t>(row) * kRowBytes + lane * 16) = data[i];
      if (g == 0 && !is_v && lane == 0) kept_positions[static_cast<size_t>(p) * cap + row] = src_row[i];
    }
  }
}

}  // namespace

hipError_t launch_compact(const PrefillDims& d, const void* k, const void* v, void* k_out, void* v_out,
                          int cap, int32_t* kept_positions, const int32_t* kept_count,
                          const PrefillWorkspace& w, hipStream_t s) {
  const int row_bytes = d.D * (d.dtype == SHOTKV_BF16 ? 2 : 4);
  const dim3 grid(ceil_div(cap, kRowsPerBlock), d.H_kv, d.P * 2), block(kCopyThreads);
  const int max_runs = d.n_shots + 2;
  KernelTimer timer(kKernelCompact, s);
#define SHOTKV_LAUNCH_COMPACT(RB)                                                                      \
  hipLaunchKernelGGL(compact_kernel<RB>, grid, block, 0, s, static_cast<const char*>(k),               \
                     static_cast<const char*>(v), static_cast<char*>(k_out), static_cast<char*>(v_out), \
                     d.n_tokens, d.H_kv, cap, kept_count, w.n_runs, w.run_src, w.run_dst, max_runs,     \
                     kept_positions)
  switch (row_bytes) {
    case 128: SHOTKV_LAUNCH_COMPACT(128); break;
    case 256: SHOTKV_LAUNCH_COMPACT(256); break;
    case 512: SHOTKV_LAUNCH_COMPACT(512); break;
    default: return hipErrorInvalidValue;
  }
#undef SHOTKV_LAUNCH_COMPACT
  return hipGetLastError();
}

}  // namespace shotkv
