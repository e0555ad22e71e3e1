// Gather-compaction of the retained K/V rows into the dense compressed cache
// (Section 5.1, Eq. 4: KV^C_prefill = Compress({s_i in S*}); Section 3: compression keeps a subset of
// the original rows, so this is a bit-exact copy).
//
// Destination-centric: a workgroup owns a few dozen consecutive output rows of one (problem, KV
// head, K-or-V) plane, reads each row's source position from kept_positions (written by the
// selection kernel) and moves it with 16-byte lanes, so stores are fully coalesced and loads are
// contiguous within a kept shot.  A thread moves only kPasses x 16 bytes: many small workgroups
// measured faster than deep per-thread batches, which put too many DRAM pages in play at once.
// Loads and stores carry the non-temporal hint: nothing here is read twice, and rows that do not linger
// in the caches leave them to the kernels that run before and after (measured: this kernel 9 % faster,
// the scoring kernel of the next call 2 % faster).
#include "common.hpp"

namespace shotkv {

namespace {

constexpr int kCopyThreads = 256;
#ifndef SHOTKV_COPY_PASSES
#define SHOTKV_COPY_PASSES 1
#endif
constexpr int kPasses = SHOTKV_COPY_PASSES;  // rows per thread

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int rows_per_block(int row_bytes) { return kPasses * (kCopyThreads / (row_bytes / 16)); }

template <int kRowBytes>
__global__ __launch_bounds__(kCopyThreads) void compact_kernel(
    const char* __restrict__ k, const char* __restrict__ v, char* __restrict__ k_out,
    char* __restrict__ v_out, int n_tokens, int H_kv, int cap, const int32_t* __restrict__ kept_count,
    const int32_t* __restrict__ kept_positions) {
  constexpr int kLanesPerRow = kRowBytes / 16;
  constexpr int kRowsPerPass = kCopyThreads / kLanesPerRow;
  constexpr int kRowsPerBlock = rows_per_block(kRowBytes);
  const int g = blockIdx.y;
  const int p = blockIdx.z >> 1;
  const bool is_v = blockIdx.z & 1;
  const int kept = kept_count[p];
  const int row0 = blockIdx.x * kRowsPerBlock;
  if (row0 >= kept) return;
  const int32_t* pos = kept_positions + static_cast<size_t>(p) * cap;
  const char* src_plane = (is_v ? v : k) + (static_cast<size_t>(p) * H_kv + g) * n_tokens * kRowBytes;
  char* dst_plane = (is_v ? v_out : k_out) + (static_cast<size_t>(p) * H_kv + g) * cap * kRowBytes;
  const int sub = threadIdx.x / kLanesPerRow;
  const int lane = threadIdx.x % kLanesPerRow;

  int src_row[kPasses];
  u32x4 data[kPasses];
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int row = row0 + i * kRowsPerPass + sub;
    src_row[i] = row < kept ? pos[row] : -1;
  }
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    if (src_row[i] >= 0)
      data[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(
          src_plane + static_cast<size_t>(src_row[i]) * kRowBytes + lane * 16));
  }
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int row = row0 + i * kRowsPerPass + sub;
    if (src_row[i] >= 0)
      __builtin_nontemporal_store(
          data[i], reinterpret_cast<u32x4*>(dst_plane + static_cast<size_t>(row) * kRowBytes + lane * 16));
  }
}

}  // namespace

hipError_t launch_compact(const PrefillDims& d, const void* k, const void* v, void* k_out, void* v_out,
                          int cap, const int32_t* kept_positions, const int32_t* kept_count,
                          hipStream_t s) {
  const int row_bytes = d.D * (d.dtype == SHOTKV_BF16 ? 2 : 4);
  const dim3 grid(ceil_div(cap, rows_per_block(row_bytes)), d.H_kv, d.P * 2), block(kCopyThreads);
  KernelTimer timer(d.timing, kKernelCompact, s);
#define SHOTKV_LAUNCH_COMPACT(RB)                                                                      \
  hipLaunchKernelGGL(compact_kernel<RB>, grid, block, 0, s, static_cast<const char*>(k),               \
                     static_cast<const char*>(v), static_cast<char*>(k_out), static_cast<char*>(v_out), \
                     d.n_tokens, d.H_kv, cap, kept_count, kept_positions)
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
