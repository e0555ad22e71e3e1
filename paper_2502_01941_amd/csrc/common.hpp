// Shared device/host helpers for the ShotKV gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "shotkv.h"

namespace shotkv {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

// Keys per scoring chunk.  A chunk never straddles a shot boundary, so a chunk's softmax partial can
// be credited to exactly one shot (or to the always-kept region).
constexpr int kChunkKeys = 256;       // MFMA path: one wave walks a chunk in 32-key blocks
constexpr int kChunkKeysGeneric = 64; // generic path: one 64-key block per workgroup

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t x) {
  return __uint_as_float(static_cast<uint32_t>(x) << 16);
}
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x); }
__device__ __forceinline__ float to_f32(float x) { return x; }

template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, kWave));
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Combining a value with the one held 32 (or 16) lanes away without a trip through the LDS pipe: the
// half swap returns the lower half of the wave in both halves of its first result and the upper half in
// both halves of the second, the row swap does the same for each pair of 16-lane rows.
__device__ __forceinline__ float sum_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_row_pairs(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__host__ __device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Upper bound on the number of chunks one problem can be cut into: every segment (n_shots shots plus
// the prefix and tail regions) adds at most one partially filled chunk.
__host__ __device__ __forceinline__ int max_chunks(int n_tokens, int n_shots, int chunk_keys) {
  return ceil_div(n_tokens, chunk_keys) + n_shots + 2;
}

// ---- optional per-kernel timing (host) -----------------------------------------------------------

enum KernelKind {
  kKernelPlan = 0, kKernelScore, kKernelRowStats, kKernelChunkMass, kKernelReduceSelect, kKernelCompact,
  kKernelDecodePartial, kKernelDecodeFinish, kKernelPackVt, kKernelAttention, kKernelKinds
};
static_assert(kKernelKinds == SHOTKV_KERNEL_KINDS, "kernel kinds");

// Brackets one kernel launch with the caller's HIP events for that kind, if the caller passed any.
class KernelTimer {
 public:
  KernelTimer(void* const* events, KernelKind kind, hipStream_t stream)
      : stop_(events ? static_cast<hipEvent_t>(events[2 * kind + 1]) : nullptr), stream_(stream) {
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[2 * kind]), stream);
  }
  ~KernelTimer() {
    if (stop_) (void)hipEventRecord(stop_, stream_);
  }
  KernelTimer(const KernelTimer&) = delete;
  KernelTimer& operator=(const KernelTimer&) = delete;

 private:
  hipEvent_t stop_;
  hipStream_t stream_;
};

// ---- workspace carving (host) -------------------------------------------------------------------

struct PrefillWorkspace {
  // chunk table, one row per problem
  int32_t* n_chunks;      // [P]
  int32_t* chunk_start;   // [P][maxC] first key of the chunk
  int32_t* chunk_len;     // [P][maxC] keys in the chunk (<= chunk_keys)
  int32_t* seg_first;     // [P][n_shots+3] first chunk of segment s; segment 0 = prefix, 1..n = shots,
                          //                n+1 = tail, entry n+2 = n_chunks
  // softmax partial per (problem, chunk, kv head, row): log2 of the chunk's sum of exponentials
  // (-inf for a row that sees none of the chunk's keys)
  float*   partial;       // [P][maxC][H_kv][R]
  // matrix-core score path: a score workgroup ("group") takes the chunks that start inside one slice
  // of group_keys keys; group g of a problem owns chunks [group_first[g], group_first[g + 1])
  int32_t* group_first;   // [P][n_groups + 1]
  // the same statistic over all chunks of a group, which is what the row denominators are built
  // from; on the generic path (one chunk per workgroup) it is the partial array itself
  float*   group_stat;    // [P][H_kv][n_groups][R]
  float*   row_stat;      // [P][H_kv][R]  log2 of the row's sum of exponentials over all chunks
  float*   chunk_mass;    // [P][maxC]
  float*   scores;        // [P][n_shots]
  void*    vt;            // fused attention path only: V packed into 32-key blocks [P][H_kv][blocks][D][32], fp16
  uint32_t* v_absmax;     // fused attention path only: [P][H_kv] largest finite |v| of the plane, as bf16 bits
  int32_t  max_c;
  int32_t  chunk_keys;
  int32_t  group_keys;    // keys per slice of the key axis, 0 on the generic path
  int32_t  n_groups;      // ceil(n_tokens / group_keys); max_c on the generic path
  size_t   bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int score_group_keys(int P, int H_kv, int n_tokens, int n_shots);  // keys per workgroup of the matrix-core score kernel

inline PrefillWorkspace carve_prefill(void* base, int P, int H_kv, int R, int n_tokens, int n_shots,
                                      bool mfma_score, size_t vt_bytes = 0) {
  PrefillWorkspace w{};
  w.chunk_keys = mfma_score ? kChunkKeys : kChunkKeysGeneric;
  w.max_c = max_chunks(n_tokens, n_shots, w.chunk_keys);
  w.group_keys = mfma_score ? score_group_keys(P, H_kv, n_tokens, n_shots) : 0;
  w.n_groups = mfma_score ? ceil_div(n_tokens, w.group_keys) : w.max_c;
  size_t off = 0;
  char* b = static_cast<char*>(base);
  auto take = [&](size_t bytes) {
    char* p = b ? b + off : nullptr;
    off = align_up(off + bytes, 256);
    return p;
  };
  const size_t P_ = P, C = w.max_c, S = n_shots;
  w.n_chunks = reinterpret_cast<int32_t*>(take(P_ * 4));
  w.chunk_start = reinterpret_cast<int32_t*>(take(P_ * C * 4));
  w.chunk_len = reinterpret_cast<int32_t*>(take(P_ * C * 4));
  w.seg_first = reinterpret_cast<int32_t*>(take(P_ * (S + 3) * 4));
  w.group_first = mfma_score ? reinterpret_cast<int32_t*>(take(P_ * (w.n_groups + 1) * 4)) : nullptr;
  w.partial = reinterpret_cast<float*>(take(P_ * H_kv * C * R * 4));
  w.group_stat = mfma_score ? reinterpret_cast<float*>(take(P_ * H_kv * w.n_groups * R * 4)) : w.partial;
  w.row_stat = reinterpret_cast<float*>(take(P_ * H_kv * R * 4));
  w.chunk_mass = reinterpret_cast<float*>(take(P_ * C * 4));
  w.scores = reinterpret_cast<float*>(take(P_ * S * 4 + 4));
  w.vt = vt_bytes ? take(vt_bytes) : nullptr;
  w.v_absmax = vt_bytes ? reinterpret_cast<uint32_t*>(take(P_ * H_kv * 4)) : nullptr;
  w.bytes = off;
  return w;
}

// ---- launchers implemented in the kernel files --------------------------------------------------

struct PrefillDims {
  int P, n_tokens, n_shots, H, H_kv, G, D, W;
  int R;       // row stride of the per-row workspace arrays: G * W, padded to 32/64/128/192/256 on the matrix-core score path
  int R_rows;  // G * W query rows per KV head that really exist
  int dtype;
  float sm_scale;
  int select_mode;
  int share;  // consecutive problems that read one row of shot_offsets / budget_tokens
  void* const* timing;  // the caller's timing events, or null
};

hipError_t launch_plan_chunks(const PrefillDims& d, const int32_t* shot_offsets, int32_t* status,
                              const PrefillWorkspace& w, hipStream_t s);
hipError_t launch_score_partials(const PrefillDims& d, const void* q_obs, const void* k,
                                 const PrefillWorkspace& w, hipStream_t s);
hipError_t launch_row_stats(const PrefillDims& d, const PrefillWorkspace& w, hipStream_t s);
hipError_t launch_chunk_mass(const PrefillDims& d, const PrefillWorkspace& w, hipStream_t s);
// Shot scores from the chunk masses (with_mass), the selection and copy plan (with_select), or both in
// one launch.  with_mass writes shot_scores; otherwise shot_scores is read.
hipError_t launch_reduce_select(const PrefillDims& d, bool with_mass, bool with_select, float* shot_scores,
                                const int32_t* shot_offsets, const int32_t* budget_tokens, int cap,
                                int32_t* kept_count, uint8_t* shot_selected, int32_t* status,
                                int32_t* kept_positions, const PrefillWorkspace& w, hipStream_t s);
hipError_t launch_compact(const PrefillDims& d, const void* k, const void* v, void* k_out, void* v_out,
                          int cap, const int32_t* kept_positions, const int32_t* kept_count,
                          hipStream_t s);

bool score_uses_mfma(const PrefillDims& d);

// causal attention forward that also writes the window rows' softmax partials and row denominators
bool attention_supported(const PrefillDims& d);
int attention_key_blocks(int n_tokens);
hipError_t launch_pack_vt(const PrefillDims& d, const void* v, const PrefillWorkspace& w, hipStream_t s);
hipError_t launch_attention_scores(const PrefillDims& d, const void* q, const void* k, const void* vt,
                                   float* attn_out, const PrefillWorkspace& w, hipStream_t s);

struct DecodeDims {
  int S, H, H_kv, G, D, dtype, cap, n_slots, budget, step, n_splits, split_tokens;
  float sm_scale;
  void* const* timing;  // the caller's timing events, or null
};

struct DecodeWorkspace {
  float2* part_ml;   // [S][H][n_splits] (max in log2 domain, sum)
  float*  part_o;    // [S][H][n_splits][D]
  float*  z_dec;     // [S][H][n_slots] scaled logits (log2 domain) of decode slots, -inf when free
  int32_t* new_slot;  // [S] slot chosen for the new token this step, -1 if the pool is full
  size_t  bytes;
};

inline DecodeWorkspace carve_decode(void* base, int S, int H, int H_kv, int D, int n_slots,
                                    int n_splits) {
  DecodeWorkspace w{};
  size_t off = 0;
  char* b = static_cast<char*>(base);
  auto take = [&](size_t bytes) {
    char* p = b ? b + off : nullptr;
    off = align_up(off + bytes, 256);
    return p;
  };
  const size_t S_ = S;
  w.part_ml = reinterpret_cast<float2*>(take(S_ * H * n_splits * 8));
  w.part_o = reinterpret_cast<float*>(take(S_ * H * n_splits * D * 4));
  w.z_dec = reinterpret_cast<float*>(take(S_ * H * n_slots * 4));
  w.new_slot = reinterpret_cast<int32_t*>(take(S_ * 4));
  w.bytes = off;
  return w;
}

// Tokens per workgroup the matrix-core decode kernel can hold logits for in LDS.
#ifndef SHOTKV_DEC_MAX_RANGE
#define SHOTKV_DEC_MAX_RANGE 1024
#endif
constexpr int kDecodeMaxRange = SHOTKV_DEC_MAX_RANGE;
constexpr int kDecodeMaxSplits = 1024;  // token ranges per (sequence, KV head) the finish kernel can merge

// query heads per KV head rounded up to 1, 2, 4 or 8: what the decode kernels are instantiated for
inline int padded_group(int G) { return G <= 1 ? 1 : G <= 2 ? 2 : G <= 4 ? 4 : G <= 8 ? 8 : 0; }

int decode_splits(int S, int H_kv, int total_tokens);
bool decode_uses_mfma(const DecodeDims& d);
hipError_t launch_decode_partial_mfma(const DecodeDims& d, const shotkv_decode_state& st, const void* q_new,
                                      const void* k_new, const void* v_new, const DecodeWorkspace& w,
                                      hipStream_t s);

hipError_t launch_decode_partial(const DecodeDims& d, const shotkv_decode_state& st, const void* q_new,
                                 const void* k_new, const void* v_new, const DecodeWorkspace& w,
                                 hipStream_t s);
hipError_t launch_decode_finish(const DecodeDims& d, const shotkv_decode_state& st, float* out,
                                float* token_scores, int32_t* evicted_pos, int32_t* status,
                                const DecodeWorkspace& w, hipStream_t s);

}  // namespace shotkv
